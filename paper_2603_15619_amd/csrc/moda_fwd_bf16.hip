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
constexpr int kDepthChunk = 16;          // depth slots whose loads are in flight together

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
// lds_addr + 16 i.  Issued through inline assembly so that the compiler does not
// serialise later LDS reads of OTHER ring stages against it; completion is awaited
// explicitly (s_waitcnt vmcnt) before the barrier that publishes the stage.
__device__ __forceinline__ void copy16_to_lds(const char* gbase, int voff, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :
               : "s"(lds_addr), "v"(voff), "s"(gbase)
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
struct Pre3 {
  i32x4 f[3];
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
  t.f[0] = t.f[1] = t.f[2] = (i32x4){0, 0, 0, 0};
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
template <int D, bool WITH_EXP>
__device__ __forceinline__ void qk_phase(STile& nxt, const unsigned char* kstage, const Pre3& pre,
                                         const i32x4 (&qf)[2][FwdCfg<D>::kDSteps], const STile& cur,
                                         PTile& pcur, const float (&mc)[2], float (&l_run)[2],
                                         float c2, const FragBase<D>& fb) {
  constexpr int NF = FwdCfg<D>::kDSteps * 2;
  constexpr int NM = NF * 2;
  i32x4 kf[NF];
  kf[0] = pre.f[0];
  kf[1] = pre.f[1];
  kf[2] = pre.f[2];
  static_for<NF>([&](auto F) {
    constexpr int f = decltype(F)::value;
    constexpr int st = f >> 1, kb = f & 1;
    if constexpr (f + 3 < NF) kf[f + 3] = read_kfrag<D, (f + 3 < NF ? f + 3 : 0)>(kstage, fb);
    static_for<2>([&](auto NB) {
      constexpr int nb = decltype(NB)::value;
      if constexpr (st == 0) mfma_s_init(nxt.a[kb][nb], kf[f], qf[nb][st]);
      else mfma_s_acc(nxt.a[kb][nb], kf[f], qf[nb][st]);
      if constexpr (WITH_EXP) {
        constexpr int m = f * 2 + nb;
        constexpr int lo = 16 + (m * 16) / NM, up = 16 + ((m + 1) * 16) / NM;
        static_for<up - lo>([&](auto Q) { exp_pair<lo + decltype(Q)::value>(cur, pcur, mc, l_run, c2); });
      }
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
    if constexpr (f + 3 < NF) vf[f + 3] = read_vfrag<D, (f + 3 < NF ? f + 3 : 0)>(vstage, fb);
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
  int k_goff[C::kInstPerWave], v_goff[C::kInstPerWave], ld_row[C::kInstPerWave];
#pragma unroll
  for (int i = 0; i < C::kInstPerWave; ++i) {
    const int r = (wave * C::kInstPerWave + i) * C::kRowsPerInst + lane / C::kChunks;
    const int pc = lane % C::kChunks;  // chunk position this lane fills
    const int kc = pc ^ (r & (C::kChunks - 1));
    const int vc = (((pc >> 1) ^ (r & (C::kChunks / 2 - 1))) << 1) | (pc & 1);
    ld_row[i] = r;
    k_goff[i] = r * C::kRowBytes + kc * 16;
    v_goff[i] = r * C::kRowBytes + vc * 16;
  }
  const unsigned smem_addr = (unsigned)(size_t)(lds_ptr)smem;
  auto issue_tile = [&](const char* gbase, int kt, int stage_off, const int (&goff)[C::kInstPerWave]) {
    const char* gt = gbase + (size_t)kt * C::kTileBytes;
    const int valid = T - kt * kBN;  // rows of this tile that exist
    if (valid >= kBN) {
#pragma unroll
      for (int i = 0; i < C::kInstPerWave; ++i)
        copy16_to_lds(gt, goff[i], smem_addr + stage_off + (wave * C::kInstPerWave + i) * C::kRowsPerInst * C::kRowBytes);
    } else {
      // ragged last tile: rows past the end re-read the last row (their keys are masked later)
#pragma unroll
      for (int i = 0; i < C::kInstPerWave; ++i) {
        const int r = min(ld_row[i], valid - 1);
        copy16_to_lds(gt, goff[i] + (r - ld_row[i]) * C::kRowBytes,
                      smem_addr + stage_off + (wave * C::kInstPerWave + i) * C::kRowsPerInst * C::kRowBytes);
      }
    }
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
  for (int j = 0; j < kStagesK && j < nt; ++j) issue_tile(Kb, j, k_stage_off(j), k_goff);
  for (int j = 0; j < kStagesV - 1 && j < nt; ++j) issue_tile(Vb, j, v_stage_off(j), v_goff);
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
    kpre.f[0] = read_kfrag<D, 0>(ks0, fb);
    kpre.f[1] = read_kfrag<D, 1>(ks0, fb);
    kpre.f[2] = read_kfrag<D, 2>(ks0, fb);
    qk_phase<D, false>(sA, ks0, kpre, qf, sA, pA, zero2, l_run, c2, fb);
    MODA_PIN();
    MODA_NOP(15);
    if (wave_last == 0 && needs_mask(0)) mask_tile(sA, 0);
    const unsigned char* vs = smem + v_stage_off(-1);
    vpre.f[0] = read_vfrag<D, 0>(vs, fb);
    vpre.f[1] = read_vfrag<D, 1>(vs, fb);
    vpre.f[2] = read_vfrag<D, 2>(vs, fb);
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
      vf[0] = vpre.f[0];
      vf[1] = vpre.f[1];
      vf[2] = vpre.f[2];
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
      kpre.f[0] = read_kfrag<D, 0>(ksn, fb);
      kpre.f[1] = read_kfrag<D, 1>(ksn, fb);
      kpre.f[2] = read_kfrag<D, 2>(ksn, fb);
    } else if (kt == wave_last + 1) {
      // this wave's last tile: only its P V is left
      const unsigned char* vs = smem + v_stage_off(kt - 1);
      i32x4 vf[NFV];
      vf[0] = vpre.f[0];
      vf[1] = vpre.f[1];
      vf[2] = vpre.f[2];
      pv_phase<D, 0, NFV, 0>(vs, vf, pprev, cur, pcur, zero2, l_run, mx, c2, fb);
      clear(kpre);
      clear(pcur);
    } else {
      clear(kpre);
      clear(pcur);
    }

    if (kt < nt) {
      // The copies issued at the previous step (K tile kt+3, V tile kt+1) may still be in
      // flight; everything older must have landed: K tile kt+2 and V tile kt are read next.
      const int newer = ((kt + kStagesK - 1 < nt) ? C::kInstPerWave : 0) +
                        ((kt >= 1 && kt + kStagesV - 2 < nt) ? C::kInstPerWave : 0);
      if (newer == 2 * C::kInstPerWave) wait_copies_but<2 * C::kInstPerWave>();
      else if (newer == C::kInstPerWave) wait_copies_but<C::kInstPerWave>();
      else wait_copies_but<0>();
      __syncthreads();
      // every wave is past the first half of step kt: K tile kt and V tile kt-1 are dead
      if (kt + kStagesK < nt) issue_tile(Kb, kt + kStagesK, k_stage_off(kt + kStagesK), k_goff);
      if (kt + kStagesV - 1 < nt) issue_tile(Vb, kt + kStagesV - 1, v_stage_off(kt + kStagesV - 1), v_goff);
    }

    if (kt <= wave_last) {
      const float mc[2] = {m_run[0] * c2, m_run[1] * c2};
      qk_phase<D, true>(nxt, smem + k_stage_off(kt + 1), kpre, qf, cur, pcur, mc, l_run, c2, fb);
      if (kt + 1 == wave_last && needs_mask(kt + 1)) {
        MODA_PIN();
        MODA_NOP(15);
        mask_tile(nxt, kt + 1);
      }
      const unsigned char* vs = smem + v_stage_off(kt);
      vpre.f[0] = read_vfrag<D, 0>(vs, fb);
      vpre.f[1] = read_vfrag<D, 1>(vs, fb);
      vpre.f[2] = read_vfrag<D, 2>(vs, fb);
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
  MODA_NOP(15);  // accumulators final before they are read out
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

#pragma unroll
  for (int nb = 0; nb < 2; ++nb) {
    float l_tot = pair_sum(l_run[nb]);
    static_for<C::kDBlocks>([&](auto DBI) {
      constexpr int db = decltype(DBI)::value;
      float x[16];
      if (nb == 0) read_o<db * 2>(x); else read_o<db * 2 + 1>(x);
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

    for (int it = 0; it < 32 / RPS; ++it) {
      const int row = it * RPS + rg;
      const int t = qw0 + nb * 32 + row;
      const int tc = min(t, T - 1);  // rows past the end compute on row T-1 and are not stored
      f32x4 o0 = *(const f32x4*)(xw + row * C::kXRow + l16 * 32);
      f32x4 o1 = *(const f32x4*)(xw + row * C::kXRow + l16 * 32 + 16);
      float o[8] = {o0[0], o0[1], o0[2], o0[3], o1[0], o1[1], o1[2], o1[3]};
      float m = ml[2 * row];
      float l = ml[2 * row + 1];
      if (L > 0) {
        const u32x4 qv = *(const u32x4*)(Qb + (size_t)tc * C::kRowBytes + l16 * 16);
        const char* kd = Kdb + (size_t)tc * drow + l16 * 16;
        const char* vd = Vdb + (size_t)tc * drow + l16 * 16;
        for (int i0 = 0; i0 < L; i0 += kDepthChunk) {
          // All loads of the chunk are issued before anything waits on them; slots
          // past depth_count re-read the last valid slot and get weight zero.
          u32x4 kv[kDepthChunk], vv[kDepthChunk];
#pragma unroll
          for (int i = 0; i < kDepthChunk; ++i)
            kv[i] = *(const u32x4*)(kd + (size_t)min(i0 + i, L - 1) * C::kRowBytes);
#pragma unroll
          for (int i = 0; i < kDepthChunk; ++i)
            vv[i] = *(const u32x4*)(vd + (size_t)min(i0 + i, L - 1) * C::kRowBytes);
          float sc[kDepthChunk];
          float mx = m;
#pragma unroll
          for (int i = 0; i < kDepthChunk; ++i) {
            float a = dot2_bf16(qv[0], kv[i][0], 0.f);
            a = dot2_bf16(qv[1], kv[i][1], a);
            a = dot2_bf16(qv[2], kv[i][2], a);
            a = dot2_bf16(qv[3], kv[i][3], a);
            a = group_sum<LPR>(a);
            sc[i] = (i0 + i < L) ? a : -INFINITY;
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
#pragma unroll
            for (int k = 0; k < 4; ++k) {
              o[2 * k] += pw * bf16_lo(vv[i][k]);
              o[2 * k + 1] += pw * bf16_hi(vv[i][k]);
            }
          }
        }
      }
      if (t < T) {
        const float inv = 1.0f / l;
        u32x4 ov = {pack_bf16(o[0] * inv, o[1] * inv), pack_bf16(o[2] * inv, o[3] * inv),
                    pack_bf16(o[4] * inv, o[5] * inv), pack_bf16(o[6] * inv, o[7] * inv)};
        *(u32x4*)(Ob + (size_t)t * C::kRowBytes + l16 * 16) = ov;
        if (l16 == 0) LSEb[t] = m * p.scale + __logf(l);
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
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
