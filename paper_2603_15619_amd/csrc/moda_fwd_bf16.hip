// MoDA attention forward, bf16 inputs, fp32 online-softmax state, gfx950 MFMA.
//
// One workgroup = 4 waves = one tile of 256 queries of one (b, h); each wave owns
// 64 queries.  Sequence K/V tiles of 64 keys are copied global -> LDS without
// passing through registers (double buffered) and consumed by
// v_mfma_f32_32x32x16_bf16:
//   S^T = K Q^T   (keys on the MFMA M axis, queries on N): a lane then holds 16
//                 scores of ONE query per 32x32 block, so the row max / row sum
//                 are in-lane reductions plus one exchange with lane ^ 32;
//   O^T += V^T P^T with P^T taken straight from the S^T accumulators (no layout
//                 round trip); the V^T operand comes from ds_read_b64_tr_b16.
// The key loop is software pipelined: while the vector ALUs exponentiate tile kt,
// the matrix pipe accumulates O += P V of tile kt-1.  The output accumulators and
// the resident Q fragments sit in named accumulation registers (moda_acc_regs.inc),
// the score tiles in ordinary vector registers.
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
typedef const __attribute__((address_space(1))) void* gbl_ptr;

// Wait until every global->LDS transfer this wave has issued is complete.
__device__ __forceinline__ void wait_all_vmem() { __builtin_amdgcn_s_waitcnt(0x0F70); }

// Nothing may be moved across this point by the instruction scheduler.
#define MODA_PIN() __builtin_amdgcn_sched_barrier(0)

// LDS layout of a K or V tile: row r (one key) is kRowBytes long; its 16-byte chunks
// are permuted by an XOR with the row index so that fragment reads spread over all
// banks:
//   K tile: chunk c of row r sits at chunk position c ^ (r & (chunks-1)); the MFMA
//           A-operand read (consecutive lanes = consecutive rows, same c) is then
//           conflict free.
//   V tile: the 32-byte pair (c >> 1) sits at pair position (c >> 1) ^ (r & (chunks/2-1));
//           the transposing read (16 lanes read 4 rows x 32 B) is then conflict free.
// Every fragment address below is (per-lane base ^ constant) + constant, so the
// second constant rides in the instructions' immediate offset.
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

// K fragment idx = st*2 + kb: 32 keys x 16 channels; this lane reads 8 channels of one key.
template <int D, int IDX>
__device__ __forceinline__ i32x4 read_kfrag(const unsigned char* kbuf, const FragBase<D>& fb) {
  constexpr int st = IDX >> 1, kb = IDX & 1;
  return *(const i32x4*)(kbuf + fb.k[st] + kb * 32 * FwdCfg<D>::kRowBytes);
}

// V^T fragment F = ks*kDBlocks + db of a 64-key tile: 16 keys x 32 channels.
// Transposing read: within 16 lanes, lane i supplies row (i/4), 8-byte piece (i%4)
// of a 4-key x 16-channel block and receives channel i of the 4 keys.  MFMA k-slots
// 0..7 (lanes < 32) are keys {0..3, 8..11} of the 16-key group and slots 8..15
// (lanes >= 32) keys {4..7, 12..15}: how the S^T accumulators hold P^T.
template <int D, int F>
__device__ __forceinline__ i32x4 read_vfrag(const unsigned char* vbuf, const FragBase<D>& fb) {
  constexpr int DB = FwdCfg<D>::kDBlocks;
  constexpr int ks = F / DB, db = F % DB;
  const unsigned char* a0 = vbuf + fb.v[db] + ks * 16 * FwdCfg<D>::kRowBytes;
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

// S^T = K Q^T for a 64-key tile: 4 * kDSteps MFMAs, K fragments prefetched 3 ahead.
// The hardware does not interlock a matrix result against a vector-ALU reader, so
// the function ends with enough wait states for the last MFMA (8 passes) to retire.
template <int D>
__device__ __forceinline__ void qk_tile(STile& s, const unsigned char* kbuf, const FragBase<D>& fb) {
  constexpr int NF = FwdCfg<D>::kDSteps * 2;
  i32x4 kf[NF];
  kf[0] = read_kfrag<D, 0>(kbuf, fb);
  kf[1] = read_kfrag<D, 1>(kbuf, fb);
  kf[2] = read_kfrag<D, 2>(kbuf, fb);
  static_for<NF>([&](auto F) {
    constexpr int f = decltype(F)::value;
    constexpr int st = f >> 1, kb = f & 1;
    if constexpr (f + 3 < NF) kf[f + 3] = read_kfrag<D, (f + 3 < NF ? f + 3 : 0)>(kbuf, fb);
    if constexpr (st == 0) {
      mfma_s_init<st>(s.a[kb][0], kf[f]);
      mfma_s_init<8 + st>(s.a[kb][1], kf[f]);
    } else {
      mfma_s_acc<st>(s.a[kb][0], kf[f]);
      mfma_s_acc<8 + st>(s.a[kb][1], kf[f]);
    }
    MODA_PIN();
  });
  asm volatile("s_nop 15\n\ts_nop 7" ::: "memory");
  MODA_PIN();
}

// exp2 of two adjacent scores: pair q of a tile, q = kb*16 + nb*8 + j.
template <int Q>
__device__ __forceinline__ void exp_pair(const STile& s, PTile& pt, const float (&mc)[2],
                                         float (&l_run)[2], float c2) {
  constexpr int kb = Q >> 4, nb = (Q >> 3) & 1, j = Q & 7;
  const float e0 = fast_exp2(s.a[kb][nb][2 * j] * c2 - mc[nb]);
  const float e1 = fast_exp2(s.a[kb][nb][2 * j + 1] * c2 - mc[nb]);
  l_run[nb] += e0 + e1;
  pt.a[kb][j >> 2][nb][j & 3] = (int)pack_bf16(e0, e1);
}

// O^T += V^T P^T over a whole tile (8 * kDBlocks MFMAs), optionally interleaved with
// the exponentiation of the NEXT tile's scores: after every MFMA a fixed slice of the
// vector-ALU work is issued and pinned there, so both pipes stay busy.
template <int D, bool WITH_EXP>
__device__ __forceinline__ void pv_tile(const unsigned char* vbuf, const PTile& pin, const STile& s,
                                        PTile& pout, const float (&mc)[2], float (&l_run)[2],
                                        float c2, const FragBase<D>& fb) {
  constexpr int DB = FwdCfg<D>::kDBlocks;
  constexpr int NF = 4 * DB;  // V fragments per tile
  constexpr int NM = NF * 2;  // MFMAs per tile
  i32x4 vf[NF];
  vf[0] = read_vfrag<D, 0>(vbuf, fb);
  vf[1] = read_vfrag<D, 1>(vbuf, fb);
  vf[2] = read_vfrag<D, 2>(vbuf, fb);
  static_for<NF>([&](auto F) {
    constexpr int f = decltype(F)::value;
    constexpr int ks = f / DB, db = f % DB;
    constexpr int kb = ks >> 1, hf = ks & 1;
    if constexpr (f + 3 < NF) vf[f + 3] = read_vfrag<D, (f + 3 < NF ? f + 3 : 0)>(vbuf, fb);
    static_for<2>([&](auto NB) {
      constexpr int nb = decltype(NB)::value;
      mfma_o<db * 2 + nb>(vf[f], pin.a[kb][hf][nb]);
      if constexpr (WITH_EXP) {
        constexpr int m = f * 2 + nb;             // MFMA index
        constexpr int lo = (m * 32) / NM;         // exp pairs done before it
        constexpr int up = ((m + 1) * 32) / NM;   // ... and after it
        static_for<up - lo>([&](auto Q) { exp_pair<lo + decltype(Q)::value>(s, pout, mc, l_run, c2); });
      }
      MODA_PIN();
    });
  });
}

template <int D>
__global__ __launch_bounds__(kThreads, 1) void moda_fwd_bf16_kernel(FwdParams p) {
  using C = FwdCfg<D>;
  // Separate LDS objects per buffer: the compiler then knows that a fragment read of
  // one buffer does not depend on an in-flight global->LDS copy into another, and
  // does not make the read wait for it.
  __shared__ __attribute__((aligned(16))) unsigned char lds_k0[C::kTileBytes];
  __shared__ __attribute__((aligned(16))) unsigned char lds_k1[C::kTileBytes];
  __shared__ __attribute__((aligned(16))) unsigned char lds_v0[C::kTileBytes];
  __shared__ __attribute__((aligned(16))) unsigned char lds_v1[C::kTileBytes];
  __shared__ __attribute__((aligned(16))) unsigned char lds_x[C::kXBytes];

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

  // ---- Q fragments (MFMA B operand of S^T = K Q^T) into their named registers;
  //      fragment index = nb*8 + st
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
    static_for<2>([&](auto NB) {
      constexpr int nb = decltype(NB)::value;
      static_for<C::kDSteps>([&](auto ST) {
        constexpr int st = decltype(ST)::value;
        set_q<nb * 8 + st>(qtmp[nb][st]);
      });
    });
  }
  static_for<C::kDBlocks * 2>([&](auto OB) { zero_o<decltype(OB)::value>(); });

  float m_run[2] = {-INFINITY, -INFINITY};  // reference max of the raw scores <q,k>
  float l_run[2] = {0.f, 0.f};              // this lane's share of the normaliser

  // number of key tiles this workgroup walks, and the last one this wave needs
  const int n_keys = p.causal ? min(T, q0 + kBM) : T;
  const int nt = (n_keys + kBN - 1) / kBN;
  const int wave_last = p.causal ? min(nt - 1, qw0 / kBN) : nt - 1;
  const float c2 = p.scale_log2;

  // ---- global -> LDS transfers of one K or V tile (no register staging).  One
  // wave instruction moves 1 KB: lane i's 16 bytes land at LDS base + 16 i, so the
  // chunk permutation is applied by choosing which global chunk each lane fetches.
  constexpr int kRowsPerInst = 64 / C::kChunks;              // tile rows per wave instruction
  constexpr int kInstPerWave = kBN / kRowsPerInst / kWaves;  // instructions per wave per tile
  int k_goff[kInstPerWave], v_goff[kInstPerWave], ld_row[kInstPerWave];
#pragma unroll
  for (int i = 0; i < kInstPerWave; ++i) {
    const int r = (wave * kInstPerWave + i) * kRowsPerInst + lane / C::kChunks;
    const int pc = lane % C::kChunks;  // chunk position this lane fills
    const int kc = pc ^ (r & (C::kChunks - 1));
    const int vc = (((pc >> 1) ^ (r & (C::kChunks / 2 - 1))) << 1) | (pc & 1);
    ld_row[i] = r;
    k_goff[i] = r * C::kRowBytes + kc * 16;
    v_goff[i] = r * C::kRowBytes + vc * 16;
  }
  auto issue_tile = [&](const char* gbase, int kt, unsigned char* lbuf, const int (&goff)[kInstPerWave]) {
    const char* gt = gbase + (size_t)kt * C::kTileBytes;
    const int valid = T - kt * kBN;  // rows of this tile that exist
#pragma unroll
    for (int i = 0; i < kInstPerWave; ++i) {
      unsigned char* ldst = lbuf + (wave * kInstPerWave + i) * kRowsPerInst * C::kRowBytes;
      int off = goff[i];
      if (valid < kBN) {  // ragged last tile: rows past the end re-read the last row (masked later)
        const int r = min(ld_row[i], valid - 1);
        off += (r - ld_row[i]) * C::kRowBytes;
      }
      __builtin_amdgcn_global_load_lds((gbl_ptr)(gt + off), (lds_ptr)ldst, 16, 0, 0);
    }
  };

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

  // ---- software pipeline over key tiles.  Iteration kt computes S = K Q^T of tile
  // kt on the matrix pipe, then exponentiates it on the vector ALUs WHILE the matrix
  // pipe accumulates O += P V of tile kt-1 (P of one tile is carried to the next
  // iteration as packed bf16).  The reference max is only raised when some row's tile
  // max exceeds it by more than 2^8 in the exp2 domain; P may then exceed 1 (bounded
  // by 256), which fp32 sums and bf16 P hold without loss, and the final division is
  // unchanged.  Raising it is the rare path: the pending P V is flushed first, then
  // the accumulators are rescaled.
  FragBase<D> fb;
  fb.init(lane);
  PTile pA, pB;
#pragma unroll
  for (int kb = 0; kb < 2; ++kb)
#pragma unroll
    for (int hf = 0; hf < 2; ++hf)
#pragma unroll
      for (int nb = 0; nb < 2; ++nb) pA.a[kb][hf][nb] = pB.a[kb][hf][nb] = (i32x4){0, 0, 0, 0};
  const float zero2[2] = {0.f, 0.f};

  issue_tile(Kb, 0, lds_k0, k_goff);
  // One pipeline iteration; `pin` holds P of tile kt-1, `pout` receives P of tile kt.
  auto iteration = [&](int kt, auto parity, const PTile& pin, PTile& pout) {
    constexpr int PAR = decltype(parity)::value;  // kt & 1, known at compile time
    unsigned char* const k_cur = PAR ? lds_k1 : lds_k0;  // K tile kt
    unsigned char* const k_nxt = PAR ? lds_k0 : lds_k1;  // K tile kt+1
    unsigned char* const v_cur = PAR ? lds_v1 : lds_v0;  // V tile kt
    unsigned char* const v_prv = PAR ? lds_v0 : lds_v1;  // V tile kt-1
    // K tile kt and V tile kt-1 were issued one iteration ago
    wait_all_vmem();
    __syncthreads();
    // every wave is past iteration kt-1: K tile kt-1 and V tile kt-2 are dead
    if (kt + 1 < nt) issue_tile(Kb, kt + 1, k_nxt, k_goff);
    if (kt < nt) issue_tile(Vb, kt, v_cur, v_goff);

    if (kt <= wave_last) {
      STile s;
      qk_tile<D>(s, k_cur, fb);
      const int k0 = kt * kBN;
      if ((p.causal && k0 + kBN - 1 > qw0) || (k0 + kBN > T)) mask_tile(s, kt);

      float mx[2];
#pragma unroll
      for (int nb = 0; nb < 2; ++nb) {
        float v = s.a[0][nb][0];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int i = 0; i < 16; ++i) v = fmaxf(v, s.a[kb][nb][i]);
        mx[nb] = pair_max(v);
      }
      const bool raise = (mx[0] - m_run[0]) * c2 > 8.f || (mx[1] - m_run[1]) * c2 > 8.f;
      if (__builtin_amdgcn_ballot_w64(raise) != 0) {
        // Rare path (always taken for the first tile, where m_run = -inf).
        if (kt > 0) pv_tile<D, false>(v_prv, pin, s, pout, zero2, l_run, c2, fb);
        MODA_PIN();
        asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");  // every MFMA above has retired
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
        asm volatile("s_nop 7\n\ts_nop 7" ::: "memory");  // register writes settle before the next MFMA
        const float mc[2] = {m_run[0] * c2, m_run[1] * c2};
        static_for<32>([&](auto Q) { exp_pair<decltype(Q)::value>(s, pout, mc, l_run, c2); });
      } else {
        const float mc[2] = {m_run[0] * c2, m_run[1] * c2};
        pv_tile<D, true>(v_prv, pin, s, pout, mc, l_run, c2, fb);
      }
    } else if (kt == wave_last + 1) {
      // this wave's last tile: only its P V is left
      STile s;
      pv_tile<D, false>(v_prv, pin, s, pout, zero2, l_run, c2, fb);
    }
  };
  for (int kt = 0; kt <= nt; kt += 2) {
    iteration(kt, std::integral_constant<int, 0>{}, pA, pB);
    if (kt + 1 <= nt) iteration(kt + 1, std::integral_constant<int, 1>{}, pB, pA);
  }
  MODA_PIN();
  asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");  // accumulators final before they are read out
  __syncthreads();

  // ================= epilogue: accumulator layout -> row-major, depth slots, store
  unsigned char* xw = lds_x + wave * C::kXWave;
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
