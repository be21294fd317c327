// MoDA attention forward, bf16 inputs, fp32 online-softmax state, gfx950 MFMA.
//
// One workgroup = 4 waves = one tile of 256 queries of one (b, h); each wave owns
// 64 queries.  Sequence K/V tiles of 64 keys are copied global -> LDS without
// passing through registers, into rings of 4 (K) and 3 (V) stages, two iterations
// ahead of their use, and consumed by v_mfma_f32_32x32x16_bf16:
//   S^T = K Q^T   (keys on the MFMA M axis, queries on N): a lane then holds 16
//                 scores of ONE query per 32x32 block, so the row max / row sum
//                 are in-lane reductions plus one exchange with lane ^ 32;
//   O^T += V^T P^T with P^T taken straight from the S^T accumulators (no layout
//                 round trip); the V^T operand comes from ds_read_b64_tr_b16.
// The key loop is software pipelined so that the matrix pipe never waits for the
// vector ALUs: while tile kt-1's P V and tile kt+1's K Q^T run on the matrix pipe,
// the vector ALUs take the row max of tile kt and exponentiate it, a fixed slice
// after every MFMA.  The output accumulators and the resident Q fragments sit in
// named accumulation registers (moda_acc_regs.inc), score tiles in vector registers.
// Tiles above the diagonal are never loaded; only the diagonal tile is masked
// (Algorithm 1's split into fully visible and boundary blocks).
// After the sequence loop the accumulators pass through LDS into a row-major
// mapping (d/8 lanes x 8 channels per query).  There the depth slots of the
// query's own position -- one contiguous L*d block in the [B,H,T,L,d] layout --
// are scored with packed dot products and a DPP reduction over those lanes and folded
// into the SAME running max / normaliser / output (Algorithm 1's third loop and
// its single final division), and O / LSE are stored with 128-bit accesses.
#include <type_traits>
#include <utility>

#include "moda_launch.h"

namespace moda {
typedef int i32x4 __attribute__((ext_vector_type(4)));
}
#include "moda_acc_regs.inc"

namespace moda {

constexpr int kWaves = 4;
constexpr int kThreads = kWaves * 64;
constexpr int kQPerWave = 64;
constexpr int kBM = kWaves * kQPerWave;  // 256 queries per workgroup
constexpr int kBN = 64;                  // keys per LDS tile
constexpr int kStagesK = 4;              // LDS ring depth for K tiles
constexpr int kStagesV = 3;              // LDS ring depth for V tiles
// cache policy of loads whose data is used exactly once (depth K/V): non-temporal, so
// that the stream does not push the re-used sequence K/V tiles out of the L2
constexpr int kStreamOnce = 2;
constexpr int kDepthChunk = 8;           // depth slots per work item of the depth phase

template <int D>
struct FwdCfg {
  static constexpr int kChunks = D / 8;          // 16-byte chunks per K/V row
  static constexpr int kRowBytes = D * 2;
  static constexpr int kTileBytes = kBN * kRowBytes;
  static constexpr int kDSteps = D / 16;         // MFMA k-steps over the head dim
  static constexpr int kDBlocks = D / 32;        // 32-wide output blocks over the head dim
  // fp32 exchange buffer: 32 query rows x D floats per wave, rows padded by 16 B
  static constexpr int kXRow = D * 4 + 16;
  static constexpr int kXWave = 32 * kXRow + 32 * 8;  // + (m, l) per row
  static constexpr int kXBytes = kWaves * kXWave;
  static constexpr int kVBase = kStagesK * kTileBytes;  // V ring follows the K ring
  static constexpr int kRingBytes = (kStagesK + kStagesV) * kTileBytes;
  static constexpr int kLds = kRingBytes > kXBytes ? kRingBytes : kXBytes;
  static constexpr int kRowsPerInst = 64 / kChunks;                 // tile rows per wave copy instruction
  static constexpr int kInstPerWave = kBN / kRowsPerInst / kWaves;  // copy instructions per wave per tile
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
__device__ __forceinline__ void copy16_to_lds(const i32x4& rsrc, int voff, int soff, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
               :
               : "s"(__builtin_amdgcn_readfirstlane((int)lds_addr)), "v"(voff), "s"(rsrc),
                 "s"(__builtin_amdgcn_readfirstlane(soff))
               : "memory");
}
template <int N>
__device__ __forceinline__ void wait_copies_but() {  // all but the N most recent copies are complete
  static_assert(N >= 0 && N < 16, "vmcnt immediate");
  __builtin_amdgcn_s_waitcnt(0x0F70 | N);
}

// LDS layout of a K or V tile: row r (one key) is kRowBytes long; its 16-byte chunks
// are permuted by an XOR with the row index so that fragment reads spread over all
// banks:
//   K tile: chunk c of row r sits at chunk position c ^ (r & (chunks-1)); the MFMA
//           A-operand read (consecutive lanes = consecutive rows, same c) is then
//           conflict free.
//   V tile: the 32-byte pair (c >> 1) sits at pair position (c >> 1) ^ (r & (chunks/2-1));
//           the transposing read (16 lanes read 4 rows x 32 B) is then conflict free.
// Every fragment address below is (per-lane base ^ constant) + stage offset + constant;
// the last constant rides in the instructions' immediate offset.
template <int D>
struct FragBase {
  int k[FwdCfg<D>::kDSteps];   // K: lane base ^ (st << 5)
  int v[FwdCfg<D>::kDBlocks];  // V: lane base ^ (db << 6)
  __device__ __forceinline__ void init(int lane) {
    using C = FwdCfg<D>;
    const int l32 = lane & 31, hi = lane >> 5;
    // K fragment (st, kb): row kb*32 + l32, logical chunk 2*st + hi
    const int kbase = l32 * C::kRowBytes + (((l32 & (C::kChunks - 1)) ^ hi) << 4);
#pragma unroll
    for (int st = 0; st < C::kDSteps; ++st) k[st] = kbase ^ (st << 5);
    // V fragment (ks, db): transposing read, see read_vfrag
    const int r8 = hi * 4 + ((lane & 15) >> 2);  // row inside the 16-key group (first read)
    const int grp = (lane >> 4) & 1;             // which 16 channels of the 32-channel block
    const int x = r8 & (C::kChunks / 2 - 1);
    const int vbase = r8 * C::kRowBytes + ((grp ^ x) << 5) + (lane & 3) * 8;
#pragma unroll
    for (int db = 0; db < C::kDBlocks; ++db) v[db] = vbase ^ (db << 6);
  }
};

// K fragment IDX = st*2 + kb: 32 keys x 16 channels; this lane reads 8 channels of one key.
// `stage` = smem + byte offset of the ring stage.
template <int D, int IDX>
__device__ __forceinline__ i32x4 read_kfrag(const unsigned char* stage, const FragBase<D>& fb) {
  constexpr int st = IDX >> 1, kb = IDX & 1;
  return *(const i32x4*)(stage + fb.k[st] + kb * 32 * FwdCfg<D>::kRowBytes);
}

// V^T fragment F = ks*kDBlocks + db of a 64-key tile: 16 keys x 32 channels.
// Transposing read: within 16 lanes, lane i supplies row (i/4), 8-byte piece (i%4)
// of a 4-key x 16-channel block and receives channel i of the 4 keys.  MFMA k-slots
// 0..7 (lanes < 32) are keys {0..3, 8..11} of the 16-key group and slots 8..15
// (lanes >= 32) keys {4..7, 12..15}: how the S^T accumulators hold P^T.
template <int D, int F>
__device__ __forceinline__ i32x4 read_vfrag(const unsigned char* stage, const FragBase<D>& fb) {
  constexpr int DB = FwdCfg<D>::kDBlocks;
  constexpr int ks = F / DB, db = F % DB;
  const unsigned char* a0 = stage + fb.v[db] + ks * 16 * FwdCfg<D>::kRowBytes;
  const unsigned char* a1 = a0 + 8 * FwdCfg<D>::kRowBytes;
  s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)a0);
  s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)a1);
  s16x8 v01 = __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(i32x4, v01);
}

// One wave's share of a 64-key x 64-query score tile (vector registers).
struct STile {
  f32x16 a[2][2];  // [key block of 32][query block of 32]
};
// P^T (packed bf16) of one tile as MFMA B operands.
struct PTile {
  i32x4 a[2][2][2];  // [key block of 32][16-key half][query block]
};
// The first fragments of the next matrix phase, read ahead of it.
constexpr int kAhead = 4;  // fragments read ahead of the MFMA that consumes them
struct Pre3 {
  i32x4 f[kAhead];
};

// Values that are not produced on some control path are set to zero there, so that
// the compiler does not have to keep their stale contents alive.
__device__ __forceinline__ void clear(STile& s) {
#pragma unroll
  for (int kb = 0; kb < 2; ++kb)
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int i = 0; i < 16; ++i) s.a[kb][nb][i] = 0.f;
}
__device__ __forceinline__ void clear(PTile& t) {
#pragma unroll
  for (int kb = 0; kb < 2; ++kb)
#pragma unroll
    for (int hf = 0; hf < 2; ++hf)
#pragma unroll
      for (int nb = 0; nb < 2; ++nb) t.a[kb][hf][nb] = (i32x4){0, 0, 0, 0};
}
__device__ __forceinline__ void clear(Pre3& t) {
#pragma unroll
  for (int i = 0; i < kAhead; ++i) t.f[i] = (i32x4){0, 0, 0, 0};
}

// exp2 of two adjacent scores: pair Q of a tile, Q = kb*16 + nb*8 + j.
template <int Q>
__device__ __forceinline__ void exp_pair(const STile& s, PTile& pt, const float (&mc)[2],
                                         float (&l_run)[2], float c2) {
  constexpr int kb = Q >> 4, nb = (Q >> 3) & 1, j = Q & 7;
  const float e0 = fast_exp2(s.a[kb][nb][2 * j] * c2 - mc[nb]);
  const float e1 = fast_exp2(s.a[kb][nb][2 * j + 1] * c2 - mc[nb]);
  float l = l_run[nb] + (e0 + e1);
  int pk = (int)pack_bf16(e0, e1);
  MODA_ANCHOR(l);
  MODA_ANCHOR(pk);
  l_run[nb] = l;
  pt.a[kb][j >> 2][nb][j & 3] = pk;
}

// ---- matrix phase 1: S^T(next) = K Q^T over one 64-key tile (4*kDSteps MFMAs), with
// exp2 of the CURRENT tile's second key block (pairs 16..31) spread between the MFMAs
// when WITH_EXP.  `pre` holds K fragments 0..2, read before the call.  The hardware
// does not interlock a matrix result against a vector-ALU reader: the caller keeps
// at least 12 issue slots between the end of this function and the first read of
// `nxt` (an MFMA of the next phase counts 8).
// `hook(integral_constant<m>)` runs after MFMA number m: the caller spreads its
// global->LDS copy instructions there, one at a time, so that their issue time is
// hidden behind matrix work as well.
struct NoHook {
  template <class I>
  __device__ __forceinline__ void operator()(I) const {}
};
template <int D, bool WITH_EXP, class Hook = NoHook>
__device__ __forceinline__ void qk_phase(STile& nxt, const unsigned char* kstage, const Pre3& pre,
                                         const i32x4 (&qf)[2][FwdCfg<D>::kDSteps], const STile& cur,
                                         PTile& pcur, const float (&mc)[2], float (&l_run)[2],
                                         float c2, const FragBase<D>& fb, Hook hook = Hook{}) {
  constexpr int NF = FwdCfg<D>::kDSteps * 2;
  constexpr int NM = NF * 2;
  i32x4 kf[NF];
#pragma unroll
  for (int i = 0; i < kAhead; ++i) kf[i] = pre.f[i];
  static_for<NF>([&](auto F) {
    constexpr int f = decltype(F)::value;
    constexpr int st = f >> 1, kb = f & 1;
    if constexpr (f + kAhead < NF) kf[f + kAhead] = read_kfrag<D, (f + kAhead < NF ? f + kAhead : 0)>(kstage, fb);
    static_for<2>([&](auto NB) {
      constexpr int nb = decltype(NB)::value;
      if constexpr (st == 0) mfma_s_init(nxt.a[kb][nb], kf[f], qf[nb][st]);
      else mfma_s_acc(nxt.a[kb][nb], kf[f], qf[nb][st]);
      if constexpr (WITH_EXP) {
        constexpr int m = f * 2 + nb;
        constexpr int lo = 16 + (m * 16) / NM, up = 16 + ((m + 1) * 16) / NM;
        static_for<up - lo>([&](auto Q) { exp_pair<lo + decltype(Q)::value>(cur, pcur, mc, l_run, c2); });
      }
      hook(std::integral_constant<int, f * 2 + nb>{});
      MODA_PIN();
    });
  });
}

// ---- matrix phase 2: O^T += V^T P^T over one 64-key tile, V fragments FIRST..LAST-1
// (2 MFMAs each).  MODE 0: nothing else.  MODE 1 (head, fragments of the first 16
// keys): the row max of the current score tile is taken between the MFMAs, starting
// after the second one (see qk_phase).  MODE 2 (tail): exp2 of the current tile's
// first key block (pairs 0..15) is spread between the MFMAs.
template <int D, int FIRST, int LAST, int MODE>
__device__ __forceinline__ void pv_phase(const unsigned char* vstage, i32x4 (&vf)[4 * FwdCfg<D>::kDBlocks],
                                         const PTile& pin, const STile& s, PTile& pout,
                                         const float (&mc)[2], float (&l_run)[2], float (&mx)[2],
                                         float c2, const FragBase<D>& fb) {
  constexpr int DB = FwdCfg<D>::kDBlocks;
  constexpr int NF = 4 * DB;
  constexpr int NM = (LAST - FIRST) * 2;  // MFMAs in this call
  float vmax[2][2];                        // MODE 1: partial maxima [nb][2 chains]
  static_for<LAST - FIRST>([&](auto FI) {
    constexpr int f = FIRST + decltype(FI)::value;
    constexpr int ks = f / DB, db = f % DB;
    constexpr int kb = ks >> 1, hf = ks & 1;
    if constexpr (f + kAhead < NF) vf[f + kAhead] = read_vfrag<D, (f + kAhead < NF ? f + kAhead : 0)>(vstage, fb);
    static_for<2>([&](auto NB) {
      constexpr int nb = decltype(NB)::value;
      mfma_o<db * 2 + nb>(vf[f], pin.a[kb][hf][nb]);
      constexpr int m = (f - FIRST) * 2 + nb;  // MFMA index within this call
      if constexpr (MODE == 1 && m >= 1) {
        // 64 score registers (2 nb x 32) folded 3 at a time: 32 max3 steps spread over NM-1 slots
        constexpr int lo = ((m - 1) * 32) / (NM - 1), up = (m * 32) / (NM - 1);
        static_for<up - lo>([&](auto Z) {
          constexpr int z = lo + decltype(Z)::value;      // step: nb2 = z / 16, within = z % 16
          constexpr int nb2 = z >> 4, w = z & 15;         // step w folds registers 2w, 2w+1 of the 32
          constexpr int kb2 = w >> 3, i0 = (w & 7) * 2;
          constexpr int ch = w & 1;                        // two independent chains per nb
          if constexpr (w < 2) vmax[nb2][ch] = fmaxf(s.a[kb2][nb2][i0], s.a[kb2][nb2][i0 + 1]);
          else vmax[nb2][ch] = fmaxf(fmaxf(vmax[nb2][ch], s.a[kb2][nb2][i0]), s.a[kb2][nb2][i0 + 1]);
          MODA_ANCHOR(vmax[nb2][ch]);
        });
      }
      if constexpr (MODE == 2) {
        constexpr int lo = (m * 16) / NM, up = ((m + 1) * 16) / NM;
        static_for<up - lo>([&](auto Q) { exp_pair<lo + decltype(Q)::value>(s, pout, mc, l_run, c2); });
      }
      MODA_PIN();
    });
  });
  if constexpr (MODE == 1) {
    mx[0] = pair_max(fmaxf(vmax[0][0], vmax[0][1]));
    mx[1] = pair_max(fmaxf(vmax[1][0], vmax[1][1]));
  }
}

template <int D>
__global__ __launch_bounds__(kThreads, 1) void moda_fwd_bf16_kernel(FwdParams p) {
  using C = FwdCfg<D>;
  __shared__ __attribute__((aligned(16))) unsigned char smem[C::kLds];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31;
  const int hi = lane >> 5;

  // Heavy (late) query tiles first; consecutive workgroup ids walk over (b, h)
  // so that, with ids dealt round-robin to the 8 XCDs, one XCD keeps serving
  // the same heads and its L2 sees each K/V tile from several workgroups.
  const int BH = p.B * p.Hq;
  const int bh = blockIdx.x % BH;
  const int qt = p.n_qtiles - 1 - blockIdx.x / BH;
  const int b = bh / p.Hq;
  const int h = bh - b * p.Hq;
  const int g = h / (p.Hq / p.Hk);
  const int T = p.T;
  const int q0 = qt * kBM;
  const int qw0 = q0 + wave * kQPerWave;

  const char* Qb = (const char*)p.Q + (size_t)bh * T * C::kRowBytes;
  const char* Kb = (const char*)p.Kseq + (size_t)(b * p.Hk + g) * T * C::kRowBytes;
  const char* Vb = (const char*)p.Vseq + (size_t)(b * p.Hk + g) * T * C::kRowBytes;

  // ---- Q fragments (MFMA B operand of S^T = K Q^T), resident in accumulation registers
  i32x4 qf[2][C::kDSteps];
  {
    i32x4 qtmp[2][C::kDSteps];  // all loads are issued before the first one is consumed
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
      const int row = min(qw0 + nb * 32 + l32, T - 1);
#pragma unroll
      for (int st = 0; st < C::kDSteps; ++st)
        qtmp[nb][st] = *(const i32x4*)(Qb + (size_t)row * C::kRowBytes + st * 32 + hi * 16);
    }
    MODA_PIN();
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int st = 0; st < C::kDSteps; ++st) qf[nb][st] = to_acc(qtmp[nb][st]);
  }
  static_for<C::kDBlocks * 2>([&](auto OB) { zero_o<decltype(OB)::value>(); });

  float m_run[2] = {-INFINITY, -INFINITY};  // reference max of the raw scores <q,k>
  float l_run[2] = {0.f, 0.f};              // this lane's share of the normaliser

  // number of key tiles this workgroup walks, and the last one this wave needs
  const int n_keys = p.causal ? min(T, q0 + kBM) : T;
  const int nt = (n_keys + kBN - 1) / kBN;
  const int wave_last = p.causal ? min(nt - 1, qw0 / kBN) : nt - 1;
  const float c2 = p.scale_log2;

  // ---- global -> LDS copies of one K or V tile.  One wave instruction moves 1 KB,
  // so the chunk permutation is applied by choosing which global chunk each lane fetches.
  int k_goff[C::kInstPerWave], v_goff[C::kInstPerWave];
#pragma unroll
  for (int i = 0; i < C::kInstPerWave; ++i) {
    const int r = (wave * C::kInstPerWave + i) * C::kRowsPerInst + lane / C::kChunks;
    const int pc = lane % C::kChunks;  // chunk position this lane fills
    const int kc = pc ^ (r & (C::kChunks - 1));
    const int vc = (((pc >> 1) ^ (r & (C::kChunks / 2 - 1))) << 1) | (pc & 1);
    k_goff[i] = r * C::kRowBytes + kc * 16;
    v_goff[i] = r * C::kRowBytes + vc * 16;
  }
  const unsigned smem_addr = (unsigned)(size_t)(lds_ptr)smem;
  const i32x4 k_buf = make_raw_buffer(Kb, (unsigned)T * C::kRowBytes);
  const i32x4 v_buf = make_raw_buffer(Vb, (unsigned)T * C::kRowBytes);
  // copy instruction i (of kInstPerWave) of this wave's share of tile kt
  auto issue_one = [&](const i32x4& buf, int kt, int stage_off, const int (&goff)[C::kInstPerWave], int i) {
    copy16_to_lds(buf, goff[i], kt * C::kTileBytes,
                  smem_addr + stage_off + (wave * C::kInstPerWave + i) * C::kRowsPerInst * C::kRowBytes);
  };
  auto issue_tile = [&](const i32x4& buf, int kt, int stage_off, const int (&goff)[C::kInstPerWave]) {
#pragma unroll
    for (int i = 0; i < C::kInstPerWave; ++i) issue_one(buf, kt, stage_off, goff, i);
  };
  auto k_stage_off = [&](int kt) { return (kt % kStagesK) * C::kTileBytes; };
  auto v_stage_off = [&](int kt) { return C::kVBase + ((kt + kStagesV) % kStagesV) * C::kTileBytes; };

  auto mask_tile = [&](STile& s, int kt) {
    const int k0 = kt * kBN;
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
      const int qi = qw0 + nb * 32 + l32;
      const int lim = p.causal ? min(qi, T - 1) : T - 1;  // last visible key
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int key = k0 + kb * 32 + (i >> 2) * 8 + hi * 4 + (i & 3);
          if (key > lim) s.a[kb][nb][i] = -INFINITY;
        }
    }
  };
  auto needs_mask = [&](int kt) { return (p.causal && kt * kBN + kBN - 1 > qw0) || (kt * kBN + kBN > T); };

  FragBase<D> fb;
  fb.init(lane);
  const float zero2[2] = {0.f, 0.f};
  float mx[2] = {0.f, 0.f};

  // ---- prologue: fill the rings, zero the V stage that stands in for "tile -1"
  // (its P is zero too, but 0 * garbage could be NaN), S(0) = K(0) Q^T.
  for (int j = 0; j < kStagesK; ++j) issue_tile(k_buf, j, k_stage_off(j), k_goff);
  for (int j = 0; j < kStagesV - 1; ++j) issue_tile(v_buf, j, v_stage_off(j), v_goff);
  for (int i = tid * 16; i < C::kTileBytes; i += kThreads * 16)
    *(i32x4*)(smem + v_stage_off(-1) + i) = (i32x4){0, 0, 0, 0};
  wait_copies_but<0>();
  __syncthreads();

  STile sA, sB;
  PTile pA, pB;
#pragma unroll
  for (int kb = 0; kb < 2; ++kb)
#pragma unroll
    for (int hf = 0; hf < 2; ++hf)
#pragma unroll
      for (int nb = 0; nb < 2; ++nb) pA.a[kb][hf][nb] = pB.a[kb][hf][nb] = (i32x4){0, 0, 0, 0};
  Pre3 kpre, vpre;
  {
    const unsigned char* ks0 = smem + k_stage_off(0);
    static_for<kAhead>([&](auto I) { kpre.f[decltype(I)::value] = read_kfrag<D, decltype(I)::value>(ks0, fb); });
    qk_phase<D, false>(sA, ks0, kpre, qf, sA, pA, zero2, l_run, c2, fb);
    MODA_PIN();
    MODA_NOP(15);
    if (wave_last == 0 && needs_mask(0)) mask_tile(sA, 0);
    const unsigned char* vs = smem + v_stage_off(-1);
    static_for<kAhead>([&](auto I) { vpre.f[decltype(I)::value] = read_vfrag<D, decltype(I)::value>(vs, fb); });
  }

  // ---- steady state.  Step kt (scores of tile kt are in `cur`, P of tile kt-1 in `pprev`):
  //   matrix pipe : O += P V (tile kt-1)            | S(next) = K Q^T (tile kt+1)
  //   vector ALUs : row max of tile kt, exp2 of its | exp2 of its second key block
  //                 first key block                 |
  //   in between  : wait for the copies issued two steps ago, barrier, issue the copies
  //                 of K tile kt+4 and V tile kt+2 into the stages just vacated.
  // The reference max is only raised when some row's tile max exceeds it by more than
  // 2^8 in the exp2 domain; P may then exceed 1 (bounded by 256), which fp32 sums and
  // bf16 P hold without loss, and the final division is unchanged.  Raising it is the
  // rare path: the pending P V is finished first, then the accumulators are rescaled.
  auto step = [&](int kt, STile& cur, STile& nxt, const PTile& pprev, PTile& pcur) {
    constexpr int NFV = 4 * C::kDBlocks;
    constexpr int HEAD = C::kDBlocks;  // V fragments of the first 16 keys
    if (kt <= wave_last) {
      const unsigned char* vs = smem + v_stage_off(kt - 1);
      i32x4 vf[NFV];
      #pragma unroll
      for (int i = 0; i < kAhead; ++i) vf[i] = vpre.f[i];
      pv_phase<D, 0, HEAD, 1>(vs, vf, pprev, cur, pcur, zero2, l_run, mx, c2, fb);
      const bool raise = (mx[0] - m_run[0]) * c2 > 8.f || (mx[1] - m_run[1]) * c2 > 8.f;
      if (__builtin_amdgcn_ballot_w64(raise) != 0) {
        // Rare path (always taken for the first tile, where m_run = -inf).
        pv_phase<D, HEAD, NFV, 0>(vs, vf, pprev, cur, pcur, zero2, l_run, mx, c2, fb);
        MODA_PIN();
        MODA_NOP(15);  // every MFMA above has retired
        float alpha[2];
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) {
          const float m_new = fmaxf(m_run[nb], mx[nb]);
          alpha[nb] = fast_exp2((m_run[nb] - m_new) * c2);  // 0 when m_run = -inf
          m_run[nb] = m_new;
          l_run[nb] *= alpha[nb];
        }
        static_for<C::kDBlocks * 2>([&](auto OB) {
          constexpr int ob = decltype(OB)::value;
          scale_o<ob>(alpha[ob & 1]);
        });
        MODA_PIN();
        MODA_NOP(7);  // register writes settle before the next MFMA
        const float mc[2] = {m_run[0] * c2, m_run[1] * c2};
        static_for<16>([&](auto Q) { exp_pair<decltype(Q)::value>(cur, pcur, mc, l_run, c2); });
      } else {
        const float mc[2] = {m_run[0] * c2, m_run[1] * c2};
        pv_phase<D, HEAD, NFV, 2>(vs, vf, pprev, cur, pcur, mc, l_run, mx, c2, fb);
      }
      // (for this wave's last tile the next K tile is not needed; it is read and
      //  multiplied all the same, which keeps the loop body free of branches)
      const unsigned char* ksn = smem + k_stage_off(kt + 1);
      static_for<kAhead>([&](auto I) { kpre.f[decltype(I)::value] = read_kfrag<D, decltype(I)::value>(ksn, fb); });
    } else if (kt == wave_last + 1) {
      // this wave's last tile: only its P V is left
      const unsigned char* vs = smem + v_stage_off(kt - 1);
      i32x4 vf[NFV];
      #pragma unroll
      for (int i = 0; i < kAhead; ++i) vf[i] = vpre.f[i];
      pv_phase<D, 0, NFV, 0>(vs, vf, pprev, cur, pcur, zero2, l_run, mx, c2, fb);
      clear(kpre);
      clear(pcur);
    } else {
      clear(kpre);
      clear(pcur);
    }

    // Every step issues the same number of copies (tiles past the end of the tensor are
    // out of range of the raw buffer: nothing is fetched), so "all but the newest
    // 2*kInstPerWave copies have landed" always means: K tile kt+2 and V tile kt, which
    // are read next, are complete.
    const int kt_k = kt + kStagesK, kt_v = kt + kStagesV - 1;
    const int so_k = k_stage_off(kt_k), so_v = v_stage_off(kt_v);
    if (kt < nt) {
      wait_copies_but<2 * C::kInstPerWave>();
      __syncthreads();
      // every wave is past the first half of step kt: K tile kt and V tile kt-1 are dead
      if (kt > wave_last) {
        issue_tile(k_buf, kt_k, so_k, k_goff);
        issue_tile(v_buf, kt_v, so_v, v_goff);
      }
    }

    if (kt <= wave_last) {
      const float mc[2] = {m_run[0] * c2, m_run[1] * c2};
      // this step's copies ride along, one after every fourth MFMA
      auto hook = [&](auto M) {
        constexpr int m = decltype(M)::value;
        if constexpr (m % 4 == 1 && m / 4 < 2 * C::kInstPerWave) {
          constexpr int i = m / 4;
          if constexpr (i < C::kInstPerWave) issue_one(k_buf, kt_k, so_k, k_goff, i);
          else issue_one(v_buf, kt_v, so_v, v_goff, i - C::kInstPerWave);
        }
      };
      qk_phase<D, true>(nxt, smem + k_stage_off(kt + 1), kpre, qf, cur, pcur, mc, l_run, c2, fb, hook);
      if (kt + 1 == wave_last && needs_mask(kt + 1)) {
        MODA_PIN();
        MODA_NOP(15);
        mask_tile(nxt, kt + 1);
      }
      const unsigned char* vs = smem + v_stage_off(kt);
      static_for<kAhead>([&](auto I) { vpre.f[decltype(I)::value] = read_vfrag<D, decltype(I)::value>(vs, fb); });
    } else {
      clear(nxt);
      clear(vpre);
    }
  };
  for (int kt = 0; kt <= nt; kt += 2) {
    step(kt, sA, sB, pA, pB);
    if (kt + 1 <= nt) step(kt + 1, sB, sA, pB, pA);
  }
  MODA_PIN();
  MODA_NOP(15);          // accumulators final before they are read out
  wait_copies_but<0>();  // the ring is reused below: no copy may still be landing in it
  __syncthreads();

  // ================= epilogue: accumulator layout -> row-major, depth slots, store
  unsigned char* xw = smem + wave * C::kXWave;
  float* ml = (float*)(xw + 32 * C::kXRow);
  constexpr int LPR = C::kChunks;   // lanes per query row: each owns 8 channels (16 B)
  constexpr int RPS = 64 / LPR;     // query rows per wave step
  const int rg = lane / LPR;
  const int l16 = lane % LPR;       // owns channels 8*l16 .. 8*l16+7
  const int L = p.depth_count;
  const size_t drow = (size_t)p.depth_alloc * C::kRowBytes;  // bytes of one position's slots
  const char* Kdb = (const char*)p.Kdepth + (size_t)(b * p.Hk + g) * T * drow;
  const char* Vdb = (const char*)p.Vdepth + (size_t)(b * p.Hk + g) * T * drow;
  char* Ob = (char*)p.O + (size_t)bh * T * C::kRowBytes;
  float* LSEb = p.LSE + (size_t)bh * T;

  // accumulators of query block NB -> this wave's exchange buffer, (m, l) per row
  auto exchange = [&](auto NB) {
    constexpr int nb = decltype(NB)::value;
    const float l_tot = pair_sum(l_run[nb]);
    static_for<C::kDBlocks>([&](auto DBI) {
      constexpr int db = decltype(DBI)::value;
      float x[16];
      read_o<db * 2 + nb>(x);
#pragma unroll
      for (int bq = 0; bq < 4; ++bq) {
        f32x4 v = {x[4 * bq], x[4 * bq + 1], x[4 * bq + 2], x[4 * bq + 3]};
        *(f32x4*)(xw + l32 * C::kXRow + (db * 32 + bq * 8 + hi * 4) * 4) = v;
      }
    });
    if (hi == 0) {
      ml[2 * l32] = m_run[nb];
      ml[2 * l32 + 1] = l_tot;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  };
  // row state in the row-major mapping
  float o[8], m = 0.f, l = 1.f;
  auto load_row = [&](int row) {
    const f32x4 o0 = *(const f32x4*)(xw + row * C::kXRow + l16 * 32);
    const f32x4 o1 = *(const f32x4*)(xw + row * C::kXRow + l16 * 32 + 16);
    o[0] = o0[0]; o[1] = o0[1]; o[2] = o0[2]; o[3] = o0[3];
    o[4] = o1[0]; o[5] = o1[1]; o[6] = o1[2]; o[7] = o1[3];
    m = ml[2 * row];
    l = ml[2 * row + 1];
  };
  auto store_row = [&](int t) {
    if (t < T) {
      const float inv = 1.0f / l;
      u32x4 ov = {pack_bf16(o[0] * inv, o[1] * inv), pack_bf16(o[2] * inv, o[3] * inv),
                  pack_bf16(o[4] * inv, o[5] * inv), pack_bf16(o[6] * inv, o[7] * inv)};
      *(u32x4*)(Ob + (size_t)t * C::kRowBytes + l16 * 16) = ov;
      if (l16 == 0) LSEb[t] = m * p.scale + __logf(l);
    }
  };
  constexpr int NIT = 32 / RPS;  // row steps per query block

  if (L == 0) {
    static_for<2>([&](auto NB) {
      constexpr int nb = decltype(NB)::value;
      exchange(NB);
      for (int it = 0; it < NIT; ++it) {
        const int row = it * RPS + rg;
        load_row(row);
        store_row(qw0 + nb * 32 + row);
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    });
    return;
  }

  // ---- depth slots.  Work items (query block, row step, chunk of kDepthChunk slots) are
  // walked in order with the NEXT item's loads already in flight while the current
  // item is folded into the row's (m, l, o): the phase is bound by memory latency, so
  // the loads of one item must never wait for the arithmetic of another.
  struct DepthBuf {
    u32x4 q;
    u32x4 k[kDepthChunk], v[kDepthChunk];
  };
  const int nch = (L + kDepthChunk - 1) / kDepthChunk;
  // The depth slabs are read through bounds-checked raw buffers with 32-bit offsets:
  // a chunk's slots past depth_alloc at the very end of the slab read as zero, and no
  // index clamping is needed (slots past depth_count get weight zero below).
  const size_t slab_bytes = (size_t)T * drow;
  const __amdgpu_buffer_rsrc_t kd_buf = __builtin_amdgcn_make_buffer_rsrc(
      (void*)Kdb, 0, (int)(unsigned)slab_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t vd_buf = __builtin_amdgcn_make_buffer_rsrc(
      (void*)Vdb, 0, (int)(unsigned)slab_bytes, 0x00020000);
  auto issue = [&](int nb, int it, int c, DepthBuf& buf) {
    const int tc = min(qw0 + nb * 32 + it * RPS + rg, T - 1);  // rows past the end use row T-1, never stored
    buf.q = *(const u32x4*)(Qb + (size_t)tc * C::kRowBytes + l16 * 16);
    const int voff = (int)((unsigned)tc * (unsigned)drow + (unsigned)l16 * 16u);  // < 4 GiB per slab (checked by the host)
    const int soff = c * kDepthChunk * C::kRowBytes;
#pragma unroll
    for (int i = 0; i < kDepthChunk; ++i)
      buf.k[i] = __builtin_amdgcn_raw_buffer_load_b128(kd_buf, voff + i * C::kRowBytes, soff, kStreamOnce);
#pragma unroll
    for (int i = 0; i < kDepthChunk; ++i)
      buf.v[i] = __builtin_amdgcn_raw_buffer_load_b128(vd_buf, voff + i * C::kRowBytes, soff, kStreamOnce);
  };
  auto fold = [&](int c, const DepthBuf& buf) {
    float sc[kDepthChunk];
    float mx = m;
#pragma unroll
    for (int i = 0; i < kDepthChunk; ++i) {
      float a = dot2_bf16(buf.q[0], buf.k[i][0], 0.f);
      a = dot2_bf16(buf.q[1], buf.k[i][1], a);
      a = dot2_bf16(buf.q[2], buf.k[i][2], a);
      a = dot2_bf16(buf.q[3], buf.k[i][3], a);
      a = group_sum<LPR>(a);
      sc[i] = (c * kDepthChunk + i < L) ? a : -INFINITY;
      mx = fmaxf(mx, sc[i]);
    }
    const float al = fast_exp2((m - mx) * c2);
    const float mc = mx * c2;
    m = mx;
    l *= al;
#pragma unroll
    for (int k = 0; k < 8; ++k) o[k] *= al;
#pragma unroll
    for (int i = 0; i < kDepthChunk; ++i) {
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
  // Item cursors: (nb, it, c) is the item being folded, (nbi, iti, ci) the next one
  // whose loads are to be issued (two items ahead).  Past the end the issue cursor
  // stays on the last item (its loads are repeated and ignored): a conditional issue
  // would make the compiler wait for the older loads as if the newer ones were not there.
  int nb = 0, it = 0, c = 0;
  int nbi = 0, iti = 0, ci = 0;
  auto advance = [&](int& b_, int& i_, int& c_) {
    if (++c_ == nch) {
      c_ = 0;
      if (++i_ == NIT) {
        i_ = 0;
        ++b_;
      }
    }
  };
  auto issue_next = [&](DepthBuf& buf) {
    issue(nbi, iti, ci, buf);
    int b2 = nbi, i2 = iti, c2n = ci;
    advance(b2, i2, c2n);
    if (b2 < 2) {
      nbi = b2;
      iti = i2;
      ci = c2n;
    }
    MODA_PIN();  // these loads are issued before anything below waits for older ones
  };
  // fold the current item from `cur`; false when it was the last one
  auto one = [&](const DepthBuf& cur, DepthBuf& refill) -> bool {
    issue_next(refill);
    if (it == 0 && c == 0) {
      if (nb == 0) {
        exchange(std::integral_constant<int, 0>{});
      } else {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        exchange(std::integral_constant<int, 1>{});
      }
    }
    const int row = it * RPS + rg;
    if (c == 0) load_row(row);
    fold(c, cur);
    if (c == nch - 1) store_row(qw0 + nb * 32 + row);
    advance(nb, it, c);
    return nb < 2;
  };
  DepthBuf bufA, bufB, bufC;
  issue_next(bufA);
  issue_next(bufB);
  while (true) {
    if (!one(bufA, bufC)) break;
    if (!one(bufB, bufA)) break;
    if (!one(bufC, bufB)) break;
  }
}

}  // namespace moda

namespace moda {

int fwd_bf16_tile_rows() { return kBM; }

hipError_t launch_fwd_bf16(const FwdParams& p, int d, hipStream_t stream) {
  const long long blocks = (long long)p.B * p.Hq * p.n_qtiles;
  if (blocks <= 0 || blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  dim3 grid((unsigned)blocks), block(kThreads);
  if (d == 128)
    hipLaunchKernelGGL(moda_fwd_bf16_kernel<128>, grid, block, 0, stream, p);
  else if (d == 64)
    hipLaunchKernelGGL(moda_fwd_bf16_kernel<64>, grid, block, 0, stream, p);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace moda
