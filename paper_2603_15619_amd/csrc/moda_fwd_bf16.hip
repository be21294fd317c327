// MoDA attention forward, bf16 inputs, fp32 online-softmax state, gfx950 MFMA.
//
// One workgroup = 8 waves (two per SIMD) = one tile of 256 (position, query head) pairs of
// one key/value head (256 positions of one head without grouped queries); each wave owns 32
// of them.  (A second geometry, 4 waves and 2-stage rings, serves small grids.)  Two waves
// per SIMD matter: a single wave issues a vector-ALU
// instruction only every ~8 cycles and an exp2 every ~24, two waves together reach
// ~5.7 and ~9.4 (measured), and the softmax arithmetic of this operator needs about as
// many vector-ALU cycles as its matrix products need matrix-pipe cycles.
// Sequence K/V tiles of 64 keys are copied global -> LDS without passing through
// registers, into rings of 4 stages each, two iterations ahead of their use, and
// consumed by v_mfma_f32_32x32x16_bf16:
//   S^T = K Q^T   (keys on the MFMA M axis, queries on N): a lane then holds 16
//                 scores of ONE query per 32x32 block, so the row max / row sum
//                 are in-lane reductions plus one exchange with lane ^ 32;
//   O^T += V^T P^T with P^T taken straight from the S^T accumulators (no layout
//                 round trip); the V^T operand comes from ds_read_b64_tr_b16.
// The key loop is software pipelined: while tile kt-1's P V and tile kt+1's K Q^T run
// on the matrix pipe, the vector ALUs take the row max of tile kt and exponentiate it,
// a fixed slice after every MFMA.  The loop body is unrolled over the 4 ring stages, so
// every LDS address is a per-lane base register plus an immediate.  K / V^T fragments
// are read from LDS straight into named accumulation registers a fixed number of MFMAs
// ahead of their use (moda_fwd_regs.h), next to the Q fragments and the output
// accumulators; score tiles, P and the softmax state live in the 128 vector registers.
// Tiles above the diagonal are never loaded; only the diagonal tile is masked
// (Algorithm 1's split into fully visible and boundary blocks).
// The depth slots of the query's own position -- one contiguous L*d block in the
// [B,H,T,L,d] layout -- are handled in a row-major mapping (d/8 lanes x 8 channels per
// query): scored with packed dot products and a DPP reduction over those lanes and folded
// into the SAME running max / normaliser / output (Algorithm 1's third loop and its single
// final division).  Every other workgroup does this after the sequence loop (the
// accumulators pass through LDS into the row-major mapping), the others before it (the
// row-major state passes through LDS into the accumulators): the result is the same, and the
// compute units then do not all stream from HBM at the same time.  O / LSE are stored with
// 128-bit accesses.
#include <type_traits>
#include <utility>

#include "moda_launch.h"
#include "moda_fwd_regs.h"

namespace moda {

constexpr int kQPerWave = 32;            // one 32-query MFMA block per wave
constexpr int kBN = 64;                  // keys per LDS tile
constexpr int kUnroll = 4;               // the key loop is unrolled over 4 steps (a multiple of every ring depth)
// cache policy of loads whose data is used exactly once (depth K/V): non-temporal, so
// that the stream does not push the re-used sequence K/V tiles out of the L2
constexpr int kStreamOnce = 2;
constexpr int kDepthChunk = 5;           // depth slots per work item of the depth phase
constexpr int kAhead = 4;                // fragments read from LDS ahead of the MFMA that consumes them
static_assert(kAhead < kSlots - 1, "a slot is refilled only after the MFMA that read it was issued");

// Two geometries:
//   W = 8: one workgroup of 8 waves (256 queries) per compute unit, K and V rings of 4 stages
//          (128 KB at d = 128); copies run two steps ahead of their use.
//   W = 4: workgroups of 4 waves (128 queries), rings of 2 stages (64 KB), so that TWO
//          workgroups share a compute unit (still two waves per SIMD): while one of them is in
//          its depth phase, which is bound by memory latency, the other keeps the matrix pipe
//          busy.  Copies run one step ahead; every K/V tile is fetched from L2 twice as often.
template <int D, int W>
struct FwdCfg {
  static constexpr int kD = D;
  static constexpr int kWaves = W;
  static constexpr int kThreads = W * 64;
  static constexpr int kBM = W * kQPerWave;        // queries per workgroup
  static constexpr int kStages = W == 8 ? 4 : 2;   // LDS ring depth, K and V each
  static constexpr int kVAhead = W == 8 ? 2 : 1;   // V tile kt + kVAhead is requested in step kt
  static_assert(kUnroll % kStages == 0, "ring stage of a step is a compile-time constant");
  static constexpr int kChunks = D / 8;          // 16-byte chunks per K/V row
  static constexpr int kRowBytes = D * 2;
  static constexpr int kGTileBytes = kBN * kRowBytes;  // a tile in global memory
  // A tile in LDS is made of 1 KB pieces (what one wave copy instruction moves: 4 rows at
  // d = 128, 8 at d = 64); the pieces of a K tile at d = 128 are 64 bytes apart (see the
  // layout comment), all others adjacent.
  static constexpr int kPieceRows = 1024 / kRowBytes;
  static constexpr int kKPieceStride = 1024 + (D == 128 ? 64 : 0);
  static constexpr int kVPieceStride = 1024;
  static constexpr int kKTileBytes = kBN / kPieceRows * kKPieceStride;  // a K tile (ring stage) in LDS
  static constexpr int kVTileBytes = kBN / kPieceRows * kVPieceStride;  // a V tile (ring stage) in LDS
  static constexpr int kKRegs = D == 128 ? 2 : D / 16;  // per-lane K fragment base addresses
  static constexpr int kDSteps = D / 16;         // MFMA k-steps over the head dim
  static constexpr int kDBlocks = D / 32;        // 32-wide output blocks over the head dim
  static constexpr int kNFK = kDSteps * 2;       // K fragments (= MFMAs of S^T = K Q^T) per tile
  static constexpr int kNFV = 4 * kDBlocks;      // V^T fragments (= MFMAs of O^T += V^T P^T) per tile
  static_assert(kNFK % kSlots == 0 && kNFV % kSlots == 0, "fragment f always uses slot f % kSlots");
  // fp32 exchange buffer: 32 query rows x D floats per wave, rows padded by 16 B
  static constexpr int kXRow = D * 4 + 16;
  static constexpr int kXWave = 32 * kXRow + 32 * 8;  // + (m, l) per row
  static constexpr int kXBytes = kWaves * kXWave;
  static constexpr int kVBase = kStages * kKTileBytes;  // V ring follows the K ring
  static constexpr int kRingBytes = kStages * (kKTileBytes + kVTileBytes);
  static constexpr int kLds = kRingBytes > kXBytes ? kRingBytes : kXBytes;
  static_assert((W == 8 ? 1 : 2) * kLds <= 160 * 1024, "workgroups per compute unit x LDS");
  static constexpr int kInstPerWave = kBN / kPieceRows / kWaves;  // copy instructions (pieces) per wave per tile
  // copy instructions of a wave that may still be in flight at a step's barrier: with 4 stages
  // the copies of the step before (needed one step later), with 2 stages none
  static constexpr int kPending = W == 8 ? 2 * kInstPerWave : 0;
  // V tile: segment permutation of row r (see the layout comment below)
  static constexpr int kSegs = kRowBytes / 64;        // 64-byte segments per row (4 or 2)
  static constexpr int kRowsPer256 = 256 / kRowBytes; // rows per sweep over all banks (1 or 2)
  __device__ __host__ static constexpr int vswz(int r) { return (r / kRowsPer256) & (kSegs - 1); }
  static_assert(kInstPerWave >= 1, "every wave copies part of every tile");
};

// Compile-time loop: f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>).
template <class F, int... Is>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, Is...>) {
  (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(f, std::make_integer_sequence<int, N>{});
}

typedef __attribute__((address_space(3))) void* lds_ptr;

// Nothing may be moved across this point by the instruction scheduler.
#define MODA_PIN() __builtin_amdgcn_sched_barrier(0)
// Keeps the computation of x where it is written: the empty volatile statement "uses"
// x there, and volatile statements (the MFMAs among them) are never reordered, so
// the compiler can neither sink the arithmetic below the following MFMAs nor hoist it.
#define MODA_ANCHOR(x) asm volatile("" : "+v"(x))
// n+1 idle issue slots (n <= 15)
#define MODA_NOP(n) asm volatile("s_nop " #n ::: "memory")

// Lane index within the wave, recomputed where it is needed (2 instructions) instead of
// being kept in a register across the key loop: volatile, so it is neither hoisted nor merged.
__device__ __forceinline__ int lane_id() {
  int x;
  asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(x));
  return x;
}

// 16 bytes per lane, global -> LDS, no register staging: lane i's bytes land at
// lds_addr + 16 i.  The source is a raw buffer (base, size in bytes): lanes whose
// offset voff + soff falls outside it fetch nothing and write zeros, so ragged and
// non-existent tiles need no special case.  Issued through inline assembly so that
// the compiler does not serialise later LDS reads of OTHER ring stages against it;
// completion is awaited explicitly (s_waitcnt vmcnt) before the barrier that
// publishes the stage.
__device__ __forceinline__ i32x4 make_raw_buffer(const void* base, unsigned bytes) {
  const unsigned long long b = (unsigned long long)base;
  i32x4 r;
  r[0] = __builtin_amdgcn_readfirstlane((int)(unsigned)(b & 0xffffffffu));
  r[1] = __builtin_amdgcn_readfirstlane((int)(unsigned)((b >> 32) & 0xffffu));  // stride 0
  r[2] = __builtin_amdgcn_readfirstlane((int)bytes);
  r[3] = 0x00020000;  // 32-bit untyped data
  return r;
}
// The LDS address is lds_base + LDS_CONST + IMM + 16 i and the global offset voff + soff + IMM:
// the instruction's immediate offset IMM (< 4096) advances both sides.  lds_base and soff
// are wave-uniform; LDS_CONST is a compile-time constant, added inside the statement so
// that the compiler does not keep one precomputed address per (stage, piece) in a
// scalar register.
// SOFF_CONST is added to soff the same way (the V copies of a step address their tile
// relative to the K tile of the same step).
template <int LDS_CONST, int IMM, int SOFF_CONST>
__device__ __forceinline__ void copy16_to_lds(const i32x4& rsrc, int voff, int soff, int lds_base) {
  static_assert(IMM >= 0 && IMM < 4096, "12-bit immediate offset");
  if constexpr (SOFF_CONST == 0) {
    asm volatile("s_add_u32 m0, %0, %c4\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen offset:%c5 lds"
                 :
                 : "s"(lds_base), "v"(voff), "s"(rsrc), "s"(soff), "n"(LDS_CONST), "n"(IMM)
                 : "memory", "scc");
  } else {
    int tmp;
    asm volatile("s_add_u32 m0, %1, %c5\n\ts_add_i32 %0, %4, %c7\n\tbuffer_load_dwordx4 %2, %3, %0 offen offset:%c6 lds"
                 : "=&s"(tmp)
                 : "s"(lds_base), "v"(voff), "s"(rsrc), "s"(soff), "n"(LDS_CONST), "n"(IMM), "n"(SOFF_CONST)
                 : "memory", "scc");
  }
}
template <int N>
__device__ __forceinline__ void wait_copies_but() {  // all but the N most recent copies are complete
  static_assert(N >= 0 && N < 16, "vmcnt immediate");
  __builtin_amdgcn_s_waitcnt(0x0F70 | N);
}

// LDS layout of a K or V tile.  Row r (one key, kRowBytes long) is row r % kPieceRows of
// piece r / kPieceRows; a piece is 1 KB, contiguous (the global -> LDS copy writes it with
// one instruction), and pieces are kPieceStride bytes apart.  Inside a row the 16-byte
// chunks are permuted so that fragment reads spread over all 64 banks (256 B):
//   K tile, d = 128: chunk c of row r sits at chunk position c ^ (r & 3) (only the two
//           low bits are permuted), and pieces are 1024 + 64 bytes apart.  The MFMA
//           A-operand read (16 consecutive lanes = 16 consecutive rows = 4 pieces x 4 rows,
//           same c) then touches 64-byte bank group (piece + c / 4) mod 4 and, inside it,
//           chunk (c ^ row) & 3: 16 different 16-byte bank groups, conflict free.  Because
//           only two chunk bits depend on the lane, the address of fragment (st, kb) is one
//           of TWO per-lane registers (st even / odd) plus an immediate.
//   K tile, d = 64:  chunk c of row r at chunk position c ^ ((r >> 1) & 7), pieces adjacent
//           (two 128-byte rows span the banks, so 16 consecutive rows need 8 different
//           positions per row parity); one per-lane register per k-step.
//   V tile: the 64-byte segment (c >> 2) sits at segment position (c >> 2) ^ vswz(r).  The
//           transposing read takes 2 cycles of 32 lanes; in one cycle the lanes read 4
//           consecutive rows x one 64-byte segment, and vswz spreads those 4 rows over the
//           4 groups of 16 banks (measured: the 32-byte-pair permutation used before cost a
//           2-way conflict on every transposing read).  Same pieces as the K tile.
// Every fragment address is a per-lane base register plus stage offset + constant in
// the instruction's immediate.
template <class C>
struct FragBase {
  int k[C::kKRegs];    // K ring
  int v[C::kDBlocks];  // V ring: (lane base ^ (db << 6)) + offset of the V ring
  __device__ __forceinline__ void init(int lane, int smem_addr) {
    const int l32 = lane & 31, hi = lane >> 5;
    // K fragment (st, kb): row kb*32 + l32, logical chunk 2*st + hi
    if constexpr (C::kD == 128) {
      const int j = l32 & 3;
      const int kbase = (l32 >> 2) * C::kKPieceStride + j * C::kRowBytes;
#pragma unroll
      for (int e = 0; e < 2; ++e) k[e] = smem_addr + kbase + ((((e << 1) | hi) ^ j) << 4);
    } else {
      const int kbase = l32 * C::kRowBytes + ((((l32 >> 1) & (C::kChunks - 1)) ^ hi) << 4);
#pragma unroll
      for (int st = 0; st < C::kDSteps; ++st) k[st] = smem_addr + (kbase ^ (st << 5));
    }
    // V fragment (ks, db): transposing read, see read_vfrag
    const int r8 = hi * 4 + ((lane & 15) >> 2);  // row inside the 16-key group (first read)
    const int grp = (lane >> 4) & 1;             // which 16 channels of the 32-channel block
#pragma unroll
    for (int db = 0; db < C::kDBlocks; ++db) {
      // (the XOR only touches bits 6..7 of the offset inside the piece)
      const int in_piece = ((r8 % C::kPieceRows) * C::kRowBytes + grp * 32 + (lane & 3) * 8) ^
                           ((C::vswz(r8) ^ db) << 6);
      v[db] = smem_addr + C::kVBase + (r8 / C::kPieceRows) * C::kVPieceStride + in_piece;
    }
  }
};

// K fragment F = st*2 + kb of the tile in ring stage KS: 32 keys x 16 channels; this
// lane reads 8 channels of one key.
template <class C, int KS, int F>
__device__ __forceinline__ void read_kfrag(const FragBase<C>& fb) {
  constexpr int st = F >> 1, kb = F & 1;
  constexpr int blk = KS * C::kKTileBytes + kb * (32 / C::kPieceRows) * C::kKPieceStride;
  if constexpr (C::kD == 128) read_k_slot<F % kSlots, blk + (st >> 1) * 64>(fb.k[st & 1]);
  else read_k_slot<F % kSlots, blk>(fb.k[st]);
}
// V^T fragment F = ks*kDBlocks + db of the tile in ring stage VS: 16 keys x 32 channels.
// Transposing read: within 16 lanes, lane i supplies row (i/4), 8-byte piece (i%4)
// of a 4-key x 16-channel block and receives channel i of the 4 keys.  MFMA k-slots
// 0..7 (lanes < 32) are keys {0..3, 8..11} of the 16-key group and slots 8..15
// (lanes >= 32) keys {4..7, 12..15}: how the S^T accumulators hold P^T.
template <class C, int VS, int F>
__device__ __forceinline__ void read_vfrag(const FragBase<C>& fb) {
  constexpr int ks = F / C::kDBlocks, db = F % C::kDBlocks;
  read_v_slot<F % kSlots, VS * C::kVTileBytes + ks * (16 / C::kPieceRows) * C::kVPieceStride,
              8 / C::kPieceRows * C::kVPieceStride>(fb.v[db]);
}

// One wave's share of a 64-key x 32-query score tile (vector registers).
struct STile {
  f32x16 a[2];  // [key block of 32]
};
// P^T (packed bf16) of one tile as MFMA B operands.
struct PTile {
  i32x4 a[2][2];  // [key block of 32][16-key half]
};

// Values that are not produced on some control path are declared overwritten there
// (with unspecified contents that nothing reads), so that the compiler does not have
// to keep their stale contents alive.
__device__ __forceinline__ void clear(STile& s) { asm volatile("" : "=v"(s.a[0]), "=v"(s.a[1])); }
__device__ __forceinline__ void clear(PTile& t) {
  asm volatile("" : "=v"(t.a[0][0]), "=v"(t.a[0][1]), "=v"(t.a[1][0]), "=v"(t.a[1][1]));
}
// All-zero P (multiplied with the zero-filled V stage that stands in for "tile -1").
__device__ __forceinline__ void zero(PTile& t) {
#pragma unroll
  for (int kb = 0; kb < 2; ++kb)
#pragma unroll
    for (int hf = 0; hf < 2; ++hf)
#pragma unroll
      for (int i = 0; i < 4; ++i) asm volatile("v_mov_b32 %0, 0" : "=v"(t.a[kb][hf][i]));
}

// exp2 of two adjacent scores: pair Q of a tile, Q = kb*8 + j.
template <int Q>
__device__ __forceinline__ void exp_pair(const STile& s, PTile& pt, float mc, float& l_run, float c2) {
  constexpr int kb = Q / 8, j = Q % 8;
  const float e0 = fast_exp2(s.a[kb][2 * j] * c2 - mc);
  const float e1 = fast_exp2(s.a[kb][2 * j + 1] * c2 - mc);
  float l = l_run + (e0 + e1);
  int pk = (int)pack_bf16(e0, e1);
  MODA_ANCHOR(l);
  MODA_ANCHOR(pk);
  l_run = l;
  pt.a[kb][j >> 2][j & 3] = pk;
}

// The LDS reads form one stream per wave: V^T fragments 0..NFV-1 of a tile, then K
// fragments 0..NFK-1 of the next score tile, then V^T fragments again, ...; the read
// of the fragment kAhead places further on is issued just before each MFMA, and every
// fragment lands in slot (its index % kSlots).  LDS operations issued after the read of
// the fragment that MFMA number F of a phase consumes (kAhead fragments, of 1 or 2
// reads each):
template <int F, int NF, int OPS_THIS, int OPS_NEXT>
constexpr int ops_after() {
  int n = 0;
  for (int j = 1; j <= kAhead; ++j) n += (F + j < NF) ? OPS_THIS : OPS_NEXT;
  return n;
}

// ---- matrix phase 1: S^T(next) = K Q^T over the 64-key tile in K stage KS (kNFK
// MFMAs), with exp2 of the CURRENT tile's second key block (pairs 8..15) spread
// between the MFMAs when WITH_EXP.  The first kAhead K fragments were requested by the
// phase before; this one requests the first V^T fragments of stage VSN for the phase
// after.  The hardware does not interlock a matrix result against a vector-ALU reader:
// the caller keeps at least 12 issue slots between the end of this function and the
// first read of `nxt` (an MFMA of the next phase counts 8).
// `hook(integral_constant<m>)` runs after MFMA number m: the caller spreads its
// global->LDS copy instructions there, one at a time, so that their issue time is
// hidden behind matrix work as well.
struct NoHook {
  template <class I>
  __device__ __forceinline__ void operator()(I) const {}
};
template <class C, int KS, int VSN, bool WITH_EXP, class Hook = NoHook>
__device__ __forceinline__ void qk_phase(STile& nxt, const STile& cur, PTile& pcur, float mc,
                                         float& l_run, float c2, const FragBase<C>& fb,
                                         Hook hook = Hook{}) {
  constexpr int NF = C::kNFK;
  static_for<NF>([&](auto F) {
    constexpr int f = decltype(F)::value;
    constexpr int st = f >> 1, kb = f & 1;
    constexpr int pf = f + kAhead;
    if constexpr (pf < NF) read_kfrag<C, KS, (pf < NF ? pf : 0)>(fb);
    else read_vfrag<C, VSN, (pf < NF ? 0 : pf - NF)>(fb);
    lds_wait<ops_after<f, NF, 1, 2>()>();
    mfma_s<f % kSlots, st, st == 0>(nxt.a[kb]);
    if constexpr (WITH_EXP) {
      constexpr int lo = 8 + (f * 8) / NF, up = 8 + ((f + 1) * 8) / NF;
      static_for<up - lo>([&](auto Q) { exp_pair<lo + decltype(Q)::value>(cur, pcur, mc, l_run, c2); });
    }
    hook(F);
    MODA_PIN();
  });
}

// ---- matrix phase 2: O^T += V^T P^T over the 64-key tile in V stage VS, V^T fragments
// FIRST..LAST-1 (one MFMA each); requests the first K fragments of stage KSN for the
// phase after.  MODE 0: nothing else.  MODE 1 (head, fragments of the first 16 keys):
// the row max of the current score tile is taken between the MFMAs, starting after the
// second one (see qk_phase).  MODE 2 (tail): exp2 of the current tile's first key block
// (pairs 0..7) is spread between the MFMAs.
// `before_k(...)` runs just before the first K fragment of stage KSN is requested (all V^T
// fragments of this tile have been requested by then): where the 2-stage geometry awaits
// the copies of that K tile and synchronises the workgroup.
template <class C, int VS, int KSN, int FIRST, int LAST, int MODE, class BeforeK = NoHook>
__device__ __forceinline__ void pv_phase(const PTile& pin, const STile& s, PTile& pout, float mc,
                                         float& l_run, float& mx, float c2, const FragBase<C>& fb,
                                         BeforeK before_k = BeforeK{}) {
  static_assert((FIRST <= C::kNFV - kAhead && LAST > C::kNFV - kAhead) || std::is_same<BeforeK, NoHook>::value,
                "only the call that requests the first K fragment takes the hook");
  constexpr int DB = C::kDBlocks;
  constexpr int NF = C::kNFV;
  constexpr int NM = LAST - FIRST;  // MFMAs in this call
  float vmax[2];                    // MODE 1: two independent chains of partial maxima
  static_for<NM>([&](auto FI) {
    constexpr int m = decltype(FI)::value;
    constexpr int f = FIRST + m;
    constexpr int ks = f / DB, db = f % DB;
    constexpr int kb = ks >> 1, hf = ks & 1;
    constexpr int pf = f + kAhead;
    if constexpr (pf == NF) before_k(FI);
    if constexpr (pf < NF) read_vfrag<C, VS, (pf < NF ? pf : 0)>(fb);
    else read_kfrag<C, KSN, (pf < NF ? 0 : pf - NF)>(fb);
    lds_wait<ops_after<f, NF, 2, 1>()>();
    mfma_o<db, f % kSlots>(pin.a[kb][hf]);
    if constexpr (MODE == 1 && m >= 1) {
      // 32 score registers folded 2 at a time (v_max3): 16 steps spread over NM-1 slots
      constexpr int lo = ((m - 1) * 16) / (NM - 1), up = (m * 16) / (NM - 1);
      static_for<up - lo>([&](auto Z) {
        constexpr int w = lo + decltype(Z)::value;  // step w folds registers 2w, 2w+1 of the 32
        constexpr int kb2 = w >> 3, i0 = (w & 7) * 2;
        constexpr int ch = w & 1;
        if constexpr (w < 2) vmax[ch] = fmaxf(s.a[kb2][i0], s.a[kb2][i0 + 1]);
        else vmax[ch] = fmaxf(fmaxf(vmax[ch], s.a[kb2][i0]), s.a[kb2][i0 + 1]);
        MODA_ANCHOR(vmax[ch]);
      });
    }
    if constexpr (MODE == 2) {
      constexpr int lo = (m * 8) / NM, up = ((m + 1) * 8) / NM;
      static_for<up - lo>([&](auto Q) { exp_pair<lo + decltype(Q)::value>(s, pout, mc, l_run, c2); });
    }
    MODA_PIN();
  });
  if constexpr (MODE == 1) mx = pair_max(fmaxf(vmax[0], vmax[1]));
}

template <int D, int W>
__global__ __launch_bounds__(W * 64) __attribute__((amdgpu_waves_per_eu(2, 2))) void moda_fwd_bf16_kernel(FwdParams p) {
  using C = FwdCfg<D, W>;
  constexpr int kThreads = C::kThreads, kBM = C::kBM, kStages = C::kStages;
  __shared__ __attribute__((aligned(16))) unsigned char smem[C::kLds];
  reserve_acc_registers();

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

  // ---- What this workgroup computes.  A tile is kBM (position, query head) pairs of one
  // key/value head: kBM / GT consecutive positions x GT query heads of its group (GT a power of
  // two up to 32 that divides the group size; GT = 1 without grouped queries).  All rows of the
  // tile read the same sequence K/V tiles and, position by position, the same depth slots (the
  // paper flattens the G heads of a group into the row axis for the same reason).  Wave w owns
  // the 32 / GT positions w * 32 / GT ... and all GT heads: its query l (a column of the matrix
  // products) is position l / GT, head l % GT, so that the depth slots of a position, which only
  // the queries at that position attend, are needed by one wave only.
  // Heavy (late) tiles first; consecutive workgroup ids walk over (batch, key/value head,
  // head subset), so that, with ids dealt round-robin to the 8 dies, one die keeps serving the
  // same heads and its L2 sees each K/V tile from several workgroups.
  const int G = p.Hq / p.Hk;
  const int GT = p.heads_per_tile;
  const int sub = G / GT;                 // head subsets per group
  const int NBH = p.B * p.Hk * sub;
  // A die (equal id mod 8) does not walk all its heads tile by tile at once: it takes
  // head_group of them at a time, heavy tiles first, then the next head_group, so that the
  // K/V of the heads in progress fit its L2 (measured at T = 65536, 2 heads per die: one at
  // a time -4 %; at T = 4096, 16 heads per die: two at a time -4 %, one at a time slower
  // again, because the heaviest tiles of a head then start late).
  int tbh = blockIdx.x % NBH;
  int tile_idx = blockIdx.x / NBH;
  if (p.head_group > 0 && NBH % (8 * p.head_group) == 0) {
    const int die = blockIdx.x & 7, r = blockIdx.x >> 3;       // r-th workgroup of this die
    const int per_group = p.head_group * p.n_qtiles;
    const int grp = r / per_group, w = r % per_group;
    tile_idx = w / p.head_group;
    tbh = (grp * p.head_group + w % p.head_group) * 8 + die;
  }
  if (sub > 1 && NBH % (8 * sub) == 0) {
    // the head subsets of one group read the same K/V: the ids that land on one die (equal id
    // mod 8) walk over the subsets of one group first, so that one L2 serves the group
    const int die = tbh & 7, m = tbh >> 3;
    tbh = ((m / sub) * 8 + die) * sub + m % sub;
  }
  const int qt = p.n_qtiles - 1 - tile_idx;
  const int bg = tbh / sub;               // (batch, key/value head)
  const int b = bg / p.Hk;
  const int g = bg - b * p.Hk;
  const int hb = b * p.Hq + g * G + (tbh - bg * sub) * GT;  // first head of the tile, as an index into [B*Hq]
  const int T = p.T;
  const int tile_pos = kBM / GT;          // positions per tile
  const int q0 = qt * tile_pos;
  const int PW = kQPerWave / GT;          // positions per wave
  const int gt_shift = __builtin_ctz(GT);
  const int qw0 = q0 + wave * PW;         // the wave's first position

  const char* Kb = (const char*)p.Kseq + (size_t)bg * T * C::kRowBytes;
  const char* Vb = (const char*)p.Vseq + (size_t)bg * T * C::kRowBytes;

  const int L = p.depth_count;
  const float c2 = p.scale_log2;

  // ---- The depth slots of the tile's own positions, folded into the running (m, l, o) of
  // every query row, in a row-major mapping: d/8 lanes x 8 channels per row, 64 / (d/8) rows
  // per wave step.  Three uses:
  //   kDepthLast  (after the key loop): rows start from the exchange buffer (the key loop's
  //               state), are folded with the depth slots, normalised and stored;
  //   kDepthFirst (before the key loop): rows start empty, are folded with the depth slots
  //               and written to the exchange buffer, from where the key loop picks them up;
  //   kPlainStore: no depth slots (or already folded in): rows from the exchange buffer are
  //               normalised and stored.
  // Work items (row step, chunk of kDepthChunk slots) are walked in order with the loads of
  // the next TWO items in flight while the current item is folded: the phase is bound by
  // memory latency, i.e. by the bytes a compute unit keeps in flight, and the 128
  // accumulation registers that the key loop does not need at that time hold most of them.
  constexpr std::integral_constant<int, 0> kDepthLast{};
  constexpr std::integral_constant<int, 1> kDepthFirst{};
  constexpr std::integral_constant<int, 2> kPlainStore{};
  auto depth_phase = [&](auto MODE_T) {
    constexpr int MODE = decltype(MODE_T)::value;
    const int lane = lane_id();
    constexpr int LPR = C::kChunks;   // lanes per query row: each owns 8 channels (16 B)
    constexpr int RPS = 64 / LPR;     // query rows per wave step
    constexpr int NIT = 32 / RPS;     // row steps of the wave's 32 rows
    const int rg = lane / LPR;
    const int l16 = lane % LPR;       // owns channels 8*l16 .. 8*l16+7
    const size_t drow = (size_t)p.depth_alloc * C::kRowBytes;  // bytes of one position's slots
    // The depth slots are addressed from the tile's first position (a 64-bit base per tile) with
    // 32-bit offsets inside the tile: the depth tensors may be of any size.
    const size_t dtile = ((size_t)bg * T + q0) * drow;
    const char* Kdb = (const char*)p.Kdepth + dtile;
    const char* Vdb = (const char*)p.Vdepth + dtile;
    // As in the key loop, wave w takes 32 / GT positions x all GT heads of the tile, heads
    // fastest: the rows of one load instruction that share a position fetch the same depth slots,
    // so a group's slots come from memory once per tile, not once per head.  Row r of the wave
    // is column r of its matrix products: its state is row r of the wave's own exchange buffer.
    struct Row {
      int head;  // within the tile
      int pos;   // within the tile
    };
    auto row_at = [&](int it) {
      const int r = it * RPS + rg;
      return Row{r % GT, wave * (kQPerWave / GT) + r / GT};
    };
    auto state_of = [&](Row) { return smem + wave * C::kXWave; };
    auto row_in_wave = [&](Row r) { return (r.pos - wave * PW) * GT + r.head; };

    // row state in the row-major mapping
    float o[8], m = 0.f, l = 1.f;
    auto begin_row = [&](Row rw) {
      unsigned char* xw = state_of(rw);
      float* ml = (float*)(xw + 32 * C::kXRow);
      const int row = row_in_wave(rw);
      if constexpr (MODE == 1) {
#pragma unroll
        for (int k = 0; k < 8; ++k) o[k] = 0.f;
        m = -INFINITY;
        l = 0.f;
      } else {
        const f32x4 o0 = *(const f32x4*)(xw + row * C::kXRow + l16 * 32);
        const f32x4 o1 = *(const f32x4*)(xw + row * C::kXRow + l16 * 32 + 16);
        o[0] = o0[0]; o[1] = o0[1]; o[2] = o0[2]; o[3] = o0[3];
        o[4] = o1[0]; o[5] = o1[1]; o[6] = o1[2]; o[7] = o1[3];
        m = ml[2 * row];
        l = ml[2 * row + 1];
      }
    };
    auto end_row = [&](Row rw) {
      unsigned char* xw = state_of(rw);
      float* ml = (float*)(xw + 32 * C::kXRow);
      const int row = row_in_wave(rw);
      if constexpr (MODE == 1) {
        *(f32x4*)(xw + row * C::kXRow + l16 * 32) = (f32x4){o[0], o[1], o[2], o[3]};
        *(f32x4*)(xw + row * C::kXRow + l16 * 32 + 16) = (f32x4){o[4], o[5], o[6], o[7]};
        if (l16 == 0) {
          ml[2 * row] = m;
          ml[2 * row + 1] = l;
        }
      } else {
        const int t = q0 + rw.pos;
        if (t < T) {
          const float inv = 1.0f / l;
          u32x4 ov = {pack_bf16(o[0] * inv, o[1] * inv), pack_bf16(o[2] * inv, o[3] * inv),
                      pack_bf16(o[4] * inv, o[5] * inv), pack_bf16(o[6] * inv, o[7] * inv)};
          const size_t orow = (size_t)(hb + rw.head) * T + t;
          *(u32x4*)((char*)p.O + orow * C::kRowBytes + l16 * 16) = ov;
          if (l16 == 0) p.LSE[orow] = m * p.scale + __logf(l);
        }
      }
    };
    if constexpr (MODE == 2) {
      for (int it = 0; it < NIT; ++it) {
        begin_row(row_at(it));
        end_row(row_at(it));
      }
      return;
    }

    struct DepthBuf {
      u32x4 q;
      u32x4 k[kDepthChunk], v[kDepthChunk];
    };
    const int nch = (L + kDepthChunk - 1) / kDepthChunk;
    // ... through raw buffers that end with the (batch, head) slab (clamped to what 32 bits hold;
    // a tile never reaches that far).
    const size_t left = (size_t)(T - q0) * drow;
    const size_t slab_bytes = left < 0xffffffffull ? left : 0xffffffffull;
    const __amdgpu_buffer_rsrc_t kd_buf = __builtin_amdgcn_make_buffer_rsrc(
        (void*)Kdb, 0, (int)(unsigned)slab_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t vd_buf = __builtin_amdgcn_make_buffer_rsrc(
        (void*)Vdb, 0, (int)(unsigned)slab_bytes, 0x00020000);
    auto issue = [&](int it, int c, DepthBuf& buf) {
      const Row rw = row_at(it);
      const int tc = min(q0 + rw.pos, T - 1);  // rows past the end use row T-1, never stored
      buf.q = *(const u32x4*)((const char*)p.Q + ((size_t)(hb + rw.head) * T + tc) * C::kRowBytes + l16 * 16);
      const int voff = (int)((unsigned)(tc - q0) * (unsigned)drow + (unsigned)l16 * 16u);  // a tile's slots stay far below 4 GiB (depth_alloc is limited by the host)
      // slots of the chunk past depth_count re-read the last attended slot (a cache hit, ignored)
      // rather than fetching bytes that nothing uses
#pragma unroll
      for (int i = 0; i < kDepthChunk; ++i)
        buf.k[i] = __builtin_amdgcn_raw_buffer_load_b128(kd_buf, voff, min(c * kDepthChunk + i, L - 1) * C::kRowBytes,
                                                         kStreamOnce);
#pragma unroll
      for (int i = 0; i < kDepthChunk; ++i)
        buf.v[i] = __builtin_amdgcn_raw_buffer_load_b128(vd_buf, voff, min(c * kDepthChunk + i, L - 1) * C::kRowBytes,
                                                         kStreamOnce);
    };
    auto fold = [&](int c, const DepthBuf& buf) {
      float sc[kDepthChunk];
      float mx2 = m;
#pragma unroll
      for (int i = 0; i < kDepthChunk; ++i) {
        float a = dot2_bf16(buf.q[0], buf.k[i][0], 0.f);
        a = dot2_bf16(buf.q[1], buf.k[i][1], a);
        a = dot2_bf16(buf.q[2], buf.k[i][2], a);
        a = dot2_bf16(buf.q[3], buf.k[i][3], a);
        a = group_sum<LPR>(a);
        sc[i] = (c * kDepthChunk + i < L) ? a : -INFINITY;
        mx2 = fmaxf(mx2, sc[i]);
      }
      // (a chunk always holds at least one attended slot, so mx2 is finite; with m = -inf,
      //  the state of an empty row, the factor is exp2(-inf) = 0)
      const float al = fast_exp2((m - mx2) * c2);
      const float mc = mx2 * c2;
      m = mx2;
      l *= al;
#pragma unroll
      for (int k = 0; k < 8; ++k) o[k] *= al;
#pragma unroll
      for (int i = 0; i < kDepthChunk; ++i) {
        // (uniform) slots past depth_count may hold anything, NaN included (a cache that is
        // still being filled): their values must not even be multiplied by a zero weight
        if (c * kDepthChunk + i >= L) break;
        const float pw = fast_exp2(sc[i] * c2 - mc);
        l += pw;
        // weight rounded to bf16 (as P is for the sequence keys) and placed in the low or
        // the high half of a pair: one packed dot product per output channel
        const uint32_t w_lo = pack_bf16(pw, 0.f);
        const uint32_t w_hi = w_lo << 16;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          o[2 * k] = dot2_bf16(w_lo, buf.v[i][k], o[2 * k]);
          o[2 * k + 1] = dot2_bf16(w_hi, buf.v[i][k], o[2 * k + 1]);
        }
      }
    };
    // Item cursors: (it, c) is the item being folded, (iti, ci) the next one whose loads
    // are to be issued (two items ahead).  Past the end the issue cursor stays on the last
    // item (its loads are repeated and ignored): a conditional issue would make the
    // compiler wait for the older loads as if the newer ones were not there.
    int it = 0, c = 0;
    int iti = 0, ci = 0;
    auto advance = [&](int& i_, int& c_) {
      if (++c_ == nch) {
        c_ = 0;
        ++i_;
      }
    };
    auto issue_next = [&](DepthBuf& buf) {
      issue(iti, ci, buf);
      int i2 = iti, c2n = ci;
      advance(i2, c2n);
      if (i2 < NIT) {
        iti = i2;
        ci = c2n;
      }
      MODA_PIN();  // these loads are issued before anything below waits for older ones
    };
    // fold the current item from `cur`; false when it was the last one
    auto one = [&](const DepthBuf& cur, DepthBuf& refill) -> bool {
      issue_next(refill);
      if (c == 0) begin_row(row_at(it));
      fold(c, cur);
      if (c == nch - 1) end_row(row_at(it));
      advance(it, c);
      return it < NIT;
    };
    DepthBuf bufA, bufB, bufC;
    issue_next(bufA);
    issue_next(bufB);
    while (true) {
      if (!one(bufA, bufC)) break;
      if (!one(bufB, bufA)) break;
      if (!one(bufC, bufB)) break;
    }
  };

  // ---- Which end of the kernel takes the depth slots.  The depth phase leaves the matrix
  // pipe idle and is bound by what ONE compute unit can pull from HBM (about 50 GB/s
  // measured, where the chip's 8 TB/s shared by all 256 units would be about 30 GB/s each).
  // When every workgroup streams its depth slots after its key loop, the compute units
  // of a short-sequence launch all stream at the same time, at the shared rate, and all
  // compute at the same time, with HBM idle.  Every other workgroup therefore takes its
  // depth slots FIRST: half of the units stream, at the full per-unit rate, while the other
  // half computes.  The result does not depend on the order (one softmax over the union).
  // Workgroup ids are dealt round-robin to the 8 dies: the role alternates within a die.
  const bool depth_first = L > 0 && ((blockIdx.x >> 3) & 1) != 0;
  // Two implementations of the depth slots: on the vector ALUs in the row-major mapping
  // (depth_phase above), or on the matrix pipe as extra key blocks (depth_blocks below).
  const bool depth_on_mfma = p.depth_mfma != 0;
  if (depth_first && !depth_on_mfma) {
    depth_phase(kDepthFirst);
    __syncthreads();  // rows were written into the buffers of the waves that own them
  }
  // From here to the release marker the accumulation registers are owned by name.
  asm volatile("; MODA_ACC_REGISTERS_ACQUIRED" ::: "memory");

  // ---- Q fragments (MFMA B operand of S^T = K Q^T), resident in accumulation registers
  {
    i32x4 qtmp[C::kDSteps];  // all loads are issued before the first one is consumed
    const int lane = lane_id(), l32 = lane & 31, hi = lane >> 5;
    const int row = min(qw0 + (l32 >> gt_shift), T - 1);
    const char* Qb = (const char*)p.Q + ((size_t)(hb + (l32 & (GT - 1))) * T + row) * C::kRowBytes;
#pragma unroll
    for (int st = 0; st < C::kDSteps; ++st)
      qtmp[st] = *(const i32x4*)(Qb + st * 32 + hi * 16);
    MODA_PIN();
    static_for<C::kDSteps>([&](auto ST) { set_q<decltype(ST)::value>(qtmp[decltype(ST)::value]); });
  }
  float m_run = -INFINITY;  // reference max of the raw scores <q,k>
  float l_run = 0.f;        // this lane's share of the normaliser
  if (depth_first && !depth_on_mfma) {
    // state left by the depth slots, from the row-major exchange buffer into the accumulator
    // layout (the inverse of the epilogue's exchange); the lane pair (l, l ^ 32) shares a row:
    // both hold its reference max, one of them its normaliser
    const int lane = lane_id(), l32 = lane & 31, hi = lane >> 5;
    const unsigned char* xw = smem + wave * C::kXWave;
    const float* ml = (const float*)(xw + 32 * C::kXRow);
    static_for<C::kDBlocks>([&](auto DBI) {
      constexpr int db = decltype(DBI)::value;
      static_for<4>([&](auto BQ) {
        constexpr int bq = decltype(BQ)::value;
        constexpr int r0 = kAccO + db * 16 + bq * 4;
        const f32x4 v = *(const f32x4*)(xw + l32 * C::kXRow + (db * 32 + bq * 8 + hi * 4) * 4);
        write_acc<r0>(v[0]);
        write_acc<r0 + 1>(v[1]);
        write_acc<r0 + 2>(v[2]);
        write_acc<r0 + 3>(v[3]);
      });
    });
    m_run = ml[2 * l32];
    l_run = hi == 0 ? ml[2 * l32 + 1] : 0.f;
    __syncthreads();  // every wave has its state: the buffer becomes the K/V rings
  } else {
    static_for<C::kDBlocks * 16>([&](auto R) { zero_acc<kAccO + decltype(R)::value>(); });
  }

  // number of key tiles this workgroup walks, and the last one this wave needs
  const int n_keys = p.causal ? min(T, q0 + tile_pos) : T;
  const int nt = (n_keys + kBN - 1) / kBN;
  const int wave_last = p.causal ? min(nt - 1, qw0 / kBN) : nt - 1;

  // ---- global -> LDS copies of one K or V tile.  One wave instruction moves one 1 KB
  // piece, so the chunk permutation is applied by choosing which global chunk each lane
  // fetches; one per-lane offset serves all K copies and one all V copies (at d = 128 the
  // permutations only look at the row index inside a piece; at d = 64 the K permutation also
  // looks at the parity of the piece, a constant XOR for a wave's odd pieces).
  // A wave copies pieces wave * kInstPerWave + i, i < kInstPerWave, of every tile.
  int k_goff, v_goff;
  {
    const int lane = tid & 63;
    const int j = lane / C::kChunks;   // row inside the piece
    const int pc = lane % C::kChunks;  // chunk position this lane fills
    const int piece0 = wave * C::kInstPerWave;  // the wave's first piece
    const int kc = C::kD == 128 ? (pc ^ (j & 3)) : (pc ^ ((((piece0 & 1) * C::kPieceRows + j) >> 1) & (C::kChunks - 1)));
    const int vc = (((pc >> 2) ^ C::vswz(j)) << 2) | (pc & 3);
    k_goff = j * C::kRowBytes + kc * 16;
    v_goff = j * C::kRowBytes + vc * 16;
  }
  static_assert(C::vswz(0) == C::vswz(C::kPieceRows) && C::vswz(1) == C::vswz(1 + C::kPieceRows),
                "the V permutation repeats from piece to piece");
  const unsigned smem_addr = (unsigned)(size_t)(lds_ptr)smem;
  const i32x4 k_buf = make_raw_buffer(Kb, (unsigned)T * C::kRowBytes);
  const i32x4 v_buf = make_raw_buffer(Vb, (unsigned)T * C::kRowBytes);
  // Copy instruction I (of kInstPerWave) of this wave's share of tile kt into the ring stage at
  // byte offset STAGE_OFF: piece wave * kInstPerWave + I.  The wave-dependent parts of both
  // addresses are two scalars; everything else is a compile-time constant.
  const int wave_lds = __builtin_amdgcn_readfirstlane((int)smem_addr + wave * C::kInstPerWave * C::kKPieceStride);
  const int wave_lds_v = __builtin_amdgcn_readfirstlane((int)smem_addr + wave * C::kInstPerWave * C::kVPieceStride);
  const int wave_goff = __builtin_amdgcn_readfirstlane(wave * C::kInstPerWave * 1024);
  // `kt` is the K tile index of the step; the V tile copied in the same step is
  // kStages - kVAhead tiles behind it.
  auto issue_one = [&](auto IS_K, auto I, auto STAGE_OFF, const i32x4& buf, int kt) {
    constexpr bool is_k = decltype(IS_K)::value;
    constexpr int i = decltype(I)::value;
    constexpr int stride = is_k ? C::kKPieceStride : C::kVPieceStride;
    const int soff = __builtin_amdgcn_readfirstlane(kt * C::kGTileBytes) + wave_goff;
    int goff = is_k ? k_goff : v_goff;
    if constexpr (is_k && C::kD == 64 && (i & 1) != 0) {
      // odd piece of an even first piece (kInstPerWave is even whenever it is not 1): the row
      // index has bit 3 set, which flips bit 2 of the chunk permutation
      static_assert(C::kInstPerWave % 2 == 0, "a wave's first piece is even");
      asm volatile("v_xor_b32 %0, %1, %2" : "=v"(goff) : "n"(4 << 4), "v"(k_goff));
    }
    copy16_to_lds<decltype(STAGE_OFF)::value + i * (stride - 1024), i * 1024,
                  is_k ? 0 : -(kStages - C::kVAhead) * C::kGTileBytes>(
        buf, goff, soff, is_k ? wave_lds : wave_lds_v);
  };
  auto issue_tile = [&](auto IS_K, auto STAGE_OFF, const i32x4& buf, int kt) {
    static_for<C::kInstPerWave>([&](auto I) { issue_one(IS_K, I, STAGE_OFF, buf, kt); });
  };
  constexpr std::true_type kIsK{};
  constexpr std::false_type kIsV{};
  // tile kt of K sits in K stage kt % kStages, tile kt of V in V stage kt % kStages
  // (tile -1: the last stage)
  auto k_stage_off = [](auto STAGE) { return std::integral_constant<int, decltype(STAGE)::value * C::kKTileBytes>{}; };
  auto v_stage_off = [](auto STAGE) {
    return std::integral_constant<int, C::kVBase + decltype(STAGE)::value * C::kVTileBytes>{};
  };

  auto mask_tile = [&](STile& s, int kt) {
    const int k0 = kt * kBN;
    const int lane = lane_id(), l32 = lane & 31, hi = lane >> 5;
    const int qi = qw0 + (l32 >> gt_shift);
    const int lim = p.causal ? min(qi, T - 1) : T - 1;  // last visible key
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int key = k0 + kb * 32 + (i >> 2) * 8 + hi * 4 + (i & 3);
        if (key > lim) s.a[kb][i] = -INFINITY;
      }
  };
  auto needs_mask = [&](int kt) { return (p.causal && kt * kBN + kBN - 1 > qw0) || (kt * kBN + kBN > T); };

  FragBase<C> fb;
  fb.init(tid & 63, (int)smem_addr);
  float mx = 0.f;

  // ---- The depth slots on the matrix pipe.  A wave's 32 queries are PW = 32 / GT consecutive
  // positions x GT heads; the attended depth slots of those positions, enumerated position by
  // position, are PW * L keys that only THIS wave needs, key kk belonging to position kk / L
  // (and attended by the GT queries at that position: the matrix instructions do 32 / GT times
  // the work a dense product would need).  They are taken
  // 32 keys at a time exactly like a block of sequence keys - S^T = K Q^T, the same running
  // (max, normaliser, output) in the same registers, O^T += V^T P^T - with the mask "key and query
  // belong to the same position" (Algorithm 1's depth mask) in place of the causal one.  Each wave
  // copies its own blocks global -> LDS into a private region of the (idle) K/V rings and waits
  // for them alone: no workgroup barrier inside the phase, and the 8 waves together keep 8
  // blocks in flight, which is what a compute unit can pull from HBM.  Slots >= depth_count are
  // never fetched (a lane whose row is not an attended slot points outside the buffer and
  // receives zeros), so they may hold anything.  Runs before the key loop (on an empty state) or
  // after it.
  auto depth_blocks = [&]() {
    constexpr int PR = C::kPieceRows, NP = 32 / PR;  // rows per 1 KB piece, pieces per block
    constexpr int kDK = NP * C::kKPieceStride, kDV = NP * C::kVPieceStride, kDWave = kDK + kDV;
    static_assert(W * kDWave <= C::kLds, "one block per wave fits the rings");
    static_assert(C::kDSteps <= kSlots && 2 * C::kDBlocks <= kSlots, "a block's fragments fit the slots");
    const int lane = lane_id(), l32 = lane & 31, hi = lane >> 5;
    const int nkeys = PW * L;
    const int nblk = (nkeys + 31) >> 5;
    const size_t drow = (size_t)p.depth_alloc * C::kRowBytes;
    // raw buffers that start at the wave's first position (64-bit base) and end with the
    // (batch, head) slab; a wave whose positions all lie past the end gets an empty buffer
    const bool any = qw0 < T;
    const size_t dbase = ((size_t)bg * T + (any ? qw0 : 0)) * drow;
    const size_t left = any ? (size_t)(T - qw0) * drow : 0;
    const unsigned recs = left < 0xffffff00ull ? (unsigned)left : 0xffffff00u;
    const i32x4 kd_buf = make_raw_buffer((const char*)p.Kdepth + dbase, recs);
    const i32x4 vd_buf = make_raw_buffer((const char*)p.Vdepth + dbase, recs);
    const int dlds = __builtin_amdgcn_readfirstlane((int)smem_addr + wave * kDWave);
    const int dwave = wave * kDWave;  // the same, as an addend to the per-lane fragment bases
    // this lane's part of a copy: row j of the piece, chunk position pc (see the tile layouts)
    const int j = lane / C::kChunks, pc = lane % C::kChunks;
    const int vc = (((pc >> 2) ^ C::vswz(j)) << 2) | (pc & 3);
    // K and V pieces of a block are requested separately: the K region is refilled as soon as the
    // block's K fragments have been read (while its scores are still being computed), the V region
    // as soon as its V^T fragments have been read, so that a wave always has the next block's
    // other half in flight.  IS_K picks the tensor.
    auto copy_half = [&](auto IS_K, int blk) {
      constexpr bool is_k = decltype(IS_K)::value;
      static_for<NP>([&](auto P) {
        constexpr int pi = decltype(P)::value;
        const int kc = C::kD == 128 ? (pc ^ (j & 3)) : (pc ^ (((pi & 1) * 4 + (j >> 1)) & (C::kChunks - 1)));
        const unsigned kk = (unsigned)(blk * 32 + pi * PR + j);          // key in the wave's enumeration
        const unsigned pos = L == 1 ? kk : __umulhi(kk, p.depth_magic);  // kk / L (exact for kk * L < 2^32)
        const unsigned slot = kk - pos * (unsigned)L;
        const unsigned rowoff = (pos * (unsigned)p.depth_alloc + slot) * (unsigned)C::kRowBytes;
        const bool ok = kk < (unsigned)nkeys;
        const int vo = ok ? (int)(rowoff + (is_k ? kc : vc) * 16) : (int)0xffffff80u;  // outside every buffer: zeros
        if constexpr (is_k) copy16_to_lds<pi * C::kKPieceStride, 0, 0>(kd_buf, vo, 0, dlds);
        else copy16_to_lds<kDK + pi * C::kVPieceStride, 0, 0>(vd_buf, vo, 0, dlds);
      });
    };
    constexpr std::true_type kHalfK{};
    constexpr std::false_type kHalfV{};
    if (nblk > 0) {
      copy_half(kHalfK, 0);
      copy_half(kHalfV, 0);
    }
    for (int blk = 0; blk < nblk; ++blk) {
      const bool more = blk + 1 < nblk;
      // S^T = K Q^T over the block's 32 keys (the V copies of this block were issued after its K copies)
      wait_copies_but<NP>();
      STile sd;
      static_for<C::kDSteps>([&](auto ST) {
        constexpr int st = decltype(ST)::value;
        if constexpr (C::kD == 128) read_k_slot<st % kSlots, (st >> 1) * 64>(fb.k[st & 1] + dwave);
        else read_k_slot<st % kSlots, 0>(fb.k[st] + dwave);
      });
      lds_wait<0>();
      static_for<C::kDSteps>([&](auto ST) {
        constexpr int st = decltype(ST)::value;
        mfma_s<st % kSlots, st, st == 0>(sd.a[0]);
      });
      if (more) copy_half(kHalfK, blk + 1);  // the K region has been read
      MODA_PIN();
      MODA_NOP(15);  // the matrix results have landed before the vector ALUs read them
      MODA_NOP(15);
      // mask: key r of the block is attended by this lane's query iff it is a slot of its position
      const unsigned lo = (unsigned)((l32 >> gt_shift) * L - blk * 32);  // first key of the position, relative to the block
      float vmax = -INFINITY;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const unsigned r = (unsigned)((i >> 2) * 8 + hi * 4 + (i & 3));
        const bool vis = (r - lo) < (unsigned)L;
        sd.a[0][i] = vis ? sd.a[0][i] : -INFINITY;
        vmax = fmaxf(vmax, sd.a[0][i]);
      }
      const float mxd = pair_max(vmax);
      const bool raise = (mxd - m_run) * c2 > 8.f;  // false when the query has no key in this block
      if (__builtin_amdgcn_ballot_w64(raise) != 0) {
        const float m_new = fmaxf(m_run, mxd);
        // (a query that has seen no key yet keeps its empty state: -inf - -inf must not become NaN)
        const float alpha = m_new == m_run ? 1.0f : fast_exp2((m_run - m_new) * c2);
        m_run = m_new;
        l_run *= alpha;
        static_for<C::kDBlocks * 16>([&](auto R) { scale_acc<kAccO + decltype(R)::value>(alpha); });
        MODA_PIN();
        MODA_NOP(7);
      }
      const float mc = m_run == -INFINITY ? 0.f : m_run * c2;
      PTile pd;
      float lsum = 0.f;
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const float e0 = fast_exp2(sd.a[0][2 * q] * c2 - mc);
        const float e1 = fast_exp2(sd.a[0][2 * q + 1] * c2 - mc);
        lsum += e0 + e1;
        pd.a[0][q >> 2][q & 3] = (int)pack_bf16(e0, e1);
      }
      l_run += lsum;
      // O^T += V^T P^T (the next block's K copies, if any, were issued after this block's V copies)
      if (more) wait_copies_but<NP>();
      else wait_copies_but<0>();
      static_for<2 * C::kDBlocks>([&](auto F) {
        constexpr int f = decltype(F)::value, ks = f / C::kDBlocks, db = f % C::kDBlocks;
        read_v_slot<f % kSlots, ks * (16 / PR) * C::kVPieceStride, 8 / PR * C::kVPieceStride>(
            fb.v[db] + (dwave + kDK - C::kVBase));
      });
      lds_wait<0>();
      static_for<2 * C::kDBlocks>([&](auto F) {
        constexpr int f = decltype(F)::value, ks = f / C::kDBlocks, db = f % C::kDBlocks;
        mfma_o<db, f % kSlots>(pd.a[0][ks]);
      });
      if (more) copy_half(kHalfV, blk + 1);  // the V region has been read
      MODA_PIN();
    }
    MODA_NOP(15);
    lds_wait<0>();
  };
  if (depth_first && depth_on_mfma) {
    depth_blocks();
    __syncthreads();  // every wave is done with its region: the rings may be filled
  }

  // ---- prologue: fill the rings, zero the V stage that stands in for "tile -1"
  // (its P is zero too, but 0 * garbage could be NaN), S(0) = K(0) Q^T.
  static_for<kStages>([&](auto J) { issue_tile(kIsK, k_stage_off(J), k_buf, decltype(J)::value); });
  static_for<C::kVAhead>([&](auto J) {
    issue_tile(kIsV, v_stage_off(J), v_buf, decltype(J)::value + kStages - C::kVAhead);
  });
  for (int i = tid * 16; i < C::kVTileBytes; i += kThreads * 16)
    *(i32x4*)(smem + C::kVBase + (kStages - 1) * C::kVTileBytes + i) = (i32x4){0, 0, 0, 0};
  wait_copies_but<0>();
  __syncthreads();

  STile sA, sB;
  PTile pA, pB;
  zero(pA);
  clear(pB);
  {
    static_for<kAhead>([&](auto I) { read_kfrag<C, 0, decltype(I)::value>(fb); });
    qk_phase<C, 0, kStages - 1, false>(sA, sA, pA, 0.f, l_run, c2, fb);
    MODA_PIN();
    MODA_NOP(15);
    if (wave_last == 0 && needs_mask(0)) mask_tile(sA, 0);
  }

  // ---- steady state.  Step kt, kt % 4 == S (scores of tile kt are in `cur`, P of tile
  // kt-1 in `pprev`):
  //   matrix pipe : O += P V (tile kt-1)            | S(next) = K Q^T (tile kt+1)
  //   vector ALUs : row max of tile kt, exp2 of its | exp2 of its second key block
  //                 first key block                 |
  //   in between  : wait for the copies issued two steps ago, barrier; the copies of
  //                 K tile kt+4 and V tile kt+2 into the stages just vacated ride along
  //                 with the second matrix phase.
  // The reference max is only raised when some row's tile max exceeds it by more than
  // 2^8 in the exp2 domain; P may then exceed 1 (bounded by 256), which fp32 sums and
  // bf16 P hold without loss, and the final division is unchanged.  Raising it is the
  // rare path: the pending P V is finished first, then the accumulators are rescaled.
  auto step = [&](auto SI, int kt, STile& cur, STile& nxt, const PTile& pprev, PTile& pcur) {
    constexpr int S = decltype(SI)::value;
    constexpr int VS_PREV = (S + kStages - 1) % kStages;  // V tile kt-1
    constexpr int KS_NEXT = (S + 1) % kStages;            // K tile kt+1
    constexpr int VS_CUR = S % kStages;                   // V tile kt
    constexpr int NFV = C::kNFV;
    constexpr int HEAD = C::kDBlocks;  // V fragments of the first 16 keys
    // Await this wave's copies and synchronise the workgroup.  With 4 stages this stands
    // between the two matrix phases.  With 2 stages K tile kt+1 was only requested in step
    // kt-1, and its first fragments are read at the end of the first matrix phase: the
    // synchronisation point moves to just before that read.  All V^T fragment reads of tile
    // kt-1 have been issued by then (LDS serves requests in order, and a copy into that
    // stage is only requested after the barrier, so it lands after them).
    constexpr bool kEarlySync = kStages == 2;
    auto sync_copies = [&]() {
      if (kt < nt) {
        wait_copies_but<C::kPending>();
        __syncthreads();
      }
    };
    auto before_k = [&](auto) {
      if constexpr (kEarlySync) sync_copies();
    };
    if (kt <= wave_last) {
      pv_phase<C, VS_PREV, KS_NEXT, 0, HEAD, 1>(pprev, cur, pcur, 0.f, l_run, mx, c2, fb);
      const bool raise = (mx - m_run) * c2 > 8.f;
      if (__builtin_amdgcn_ballot_w64(raise) != 0) {
        // Rare path (always taken for the first tile, where m_run = -inf).
        pv_phase<C, VS_PREV, KS_NEXT, HEAD, NFV, 0>(pprev, cur, pcur, 0.f, l_run, mx, c2, fb, before_k);
        MODA_PIN();
        MODA_NOP(15);  // every MFMA above has retired
        const float m_new = fmaxf(m_run, mx);
        const float alpha = fast_exp2((m_run - m_new) * c2);  // 0 when m_run = -inf
        m_run = m_new;
        l_run *= alpha;
        static_for<C::kDBlocks * 16>([&](auto R) { scale_acc<kAccO + decltype(R)::value>(alpha); });
        MODA_PIN();
        MODA_NOP(7);  // register writes settle before the next MFMA
        const float mc = m_run * c2;
        static_for<8>([&](auto Q) { exp_pair<decltype(Q)::value>(cur, pcur, mc, l_run, c2); });
      } else {
        const float mc = m_run * c2;
        pv_phase<C, VS_PREV, KS_NEXT, HEAD, NFV, 2>(pprev, cur, pcur, mc, l_run, mx, c2, fb, before_k);
      }
      // (for this wave's last tile the next K tile is not needed; it is read and
      //  multiplied all the same, which keeps the loop body free of branches)
    } else if (kt == wave_last + 1) {
      // this wave's last tile: only its P V is left (the K fragments it requests are never used)
      pv_phase<C, VS_PREV, KS_NEXT, 0, NFV, 0>(pprev, cur, pcur, 0.f, l_run, mx, c2, fb, before_k);
      clear(pcur);
    } else {
      clear(pcur);
      if constexpr (kEarlySync) sync_copies();
    }

    // Every step issues the same number of copies (tiles past the end of the tensor are
    // out of range of the raw buffer: nothing is fetched), so "all but the newest
    // kPending copies have landed" always means: K tile kt+1 and V tile kt, which are
    // read next, are complete (with 4 stages K tile kt+2 too: one step of slack).
    // The stages written are those of K tile kt (its scores were taken in step kt-1) and,
    // with 4 stages, of V tile kt-2, with 2 stages of V tile kt-1 (consumed in the first
    // half of this step): every wave is past those reads once it has passed the barrier.
    const int kt_k = kt + kStages;  // the V tile of this step is kt + kVAhead
    constexpr auto so_k = k_stage_off(std::integral_constant<int, S % kStages>{});
    constexpr auto so_v = v_stage_off(std::integral_constant<int, (S + C::kVAhead) % kStages>{});
    if constexpr (!kEarlySync) sync_copies();
    // every wave is past the reads of the stages that this step's copies overwrite
    if (kt < nt && kt > wave_last) {
      issue_tile(kIsK, so_k, k_buf, kt_k);
      issue_tile(kIsV, so_v, v_buf, kt_k);
    }

    if (kt <= wave_last) {
      const float mc = m_run * c2;
      // this step's copies ride along, spread evenly over the MFMAs of the phase
      auto hook = [&](auto M) {
        constexpr int m = decltype(M)::value;
        constexpr int every = C::kNFK / (2 * C::kInstPerWave) >= 4 ? 4 : C::kNFK / (2 * C::kInstPerWave);
        static_assert(every >= 1, "at most one copy per MFMA");
        if constexpr (m % every == every / 2 && m / every < 2 * C::kInstPerWave) {
          constexpr int i = m / every;
          if constexpr (i < C::kInstPerWave)
            issue_one(kIsK, std::integral_constant<int, i>{}, so_k, k_buf, kt_k);
          else
            issue_one(kIsV, std::integral_constant<int, (i < C::kInstPerWave ? 0 : i - C::kInstPerWave)>{}, so_v,
                      v_buf, kt_k);
        }
      };
      qk_phase<C, KS_NEXT, VS_CUR, true>(nxt, cur, pcur, mc, l_run, c2, fb, hook);
      if (kt + 1 == wave_last && needs_mask(kt + 1)) {
        MODA_PIN();
        MODA_NOP(15);
        mask_tile(nxt, kt + 1);
      }
    } else {
      clear(nxt);
    }
  };
  static_assert(kUnroll == 4, "the four steps below");
  for (int kt = 0; kt <= nt; kt += 4) {
    step(std::integral_constant<int, 0>{}, kt, sA, sB, pA, pB);
    if (kt + 1 <= nt) step(std::integral_constant<int, 1>{}, kt + 1, sB, sA, pB, pA);
    if (kt + 2 <= nt) step(std::integral_constant<int, 2>{}, kt + 2, sA, sB, pA, pB);
    if (kt + 3 <= nt) step(std::integral_constant<int, 3>{}, kt + 3, sB, sA, pB, pA);
  }
  MODA_PIN();
  MODA_NOP(15);          // accumulators final before they are read out
  lds_wait<0>();         // fragment reads requested but never used have landed
  wait_copies_but<0>();  // the ring is reused below: no copy may still be landing in it
  __syncthreads();
  if (L > 0 && !depth_first && depth_on_mfma) {
    depth_blocks();
    __syncthreads();     // every wave is done with its region: the exchange buffers may be written
  }

  // ================= epilogue: accumulator layout -> row-major, depth slots, store
  {
    // accumulators -> this wave's exchange buffer, (m, l) per row
    const int lane = lane_id(), l32 = lane & 31, hi = lane >> 5;
    unsigned char* xw = smem + wave * C::kXWave;
    float* ml = (float*)(xw + 32 * C::kXRow);
    const float l_tot = pair_sum(l_run);
    static_for<C::kDBlocks>([&](auto DBI) {
      constexpr int db = decltype(DBI)::value;
      static_for<4>([&](auto BQ) {
        constexpr int bq = decltype(BQ)::value;
        constexpr int r0 = kAccO + db * 16 + bq * 4;
        f32x4 v = {read_acc<r0>(), read_acc<r0 + 1>(), read_acc<r0 + 2>(), read_acc<r0 + 3>()};
        *(f32x4*)(xw + l32 * C::kXRow + (db * 32 + bq * 8 + hi * 4) * 4) = v;
      });
    });
    if (hi == 0) {
      ml[2 * l32] = m_run;
      ml[2 * l32 + 1] = l_tot;
    }
  }
  __syncthreads();  // the depth phase reads rows from the buffers of other waves
  // From here on the accumulation registers are the compiler's (it parks depth K/V
  // loads in them); the build step checks that on the generated code.
  asm volatile("; MODA_ACC_REGISTERS_RELEASED" ::: "memory");
  if (L == 0 || depth_first || depth_on_mfma) depth_phase(kPlainStore);
  else depth_phase(kDepthLast);
}

}  // namespace moda

namespace moda {

int fwd_bf16_tile_rows(int waves) { return waves * kQPerWave; }

hipError_t launch_fwd_bf16(const FwdParams& p, int d, int waves, hipStream_t stream) {
  const int gt = p.heads_per_tile;
  if ((waves != 4 && waves != 8) || gt < 1 || gt > kQPerWave || (gt & (gt - 1)) != 0 || (p.Hq / p.Hk) % gt != 0)
    return hipErrorInvalidValue;
  const int tile_pos = waves * kQPerWave / gt;
  if (p.n_qtiles != (p.T + tile_pos - 1) / tile_pos) return hipErrorInvalidValue;
  const long long blocks = (long long)p.B * (p.Hq / gt) * p.n_qtiles;
  if (!grid_ok(blocks)) return kGridTooLarge;
  dim3 grid((unsigned)blocks), block(waves * 64);
  if (d == 128 && waves == 8) return launch_kernel(moda_fwd_bf16_kernel<128, 8>, grid, block, stream, p);
  if (d == 128) return launch_kernel(moda_fwd_bf16_kernel<128, 4>, grid, block, stream, p);
  if (d == 64 && waves == 8) return launch_kernel(moda_fwd_bf16_kernel<64, 8>, grid, block, stream, p);
  if (d == 64) return launch_kernel(moda_fwd_bf16_kernel<64, 4>, grid, block, stream, p);
  return hipErrorInvalidValue;
}

}  // namespace moda
