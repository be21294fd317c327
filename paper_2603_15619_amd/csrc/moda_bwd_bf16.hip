// MoDA attention backward, bf16 inputs, fp32 accumulation, gfx950 MFMA.
//
// The paper gives no backward algorithm; this is the derivative of the forward
// definition (one softmax over causal sequence keys and same-position depth slots),
// evaluated by recomputation from Q, K, V, the depth tensors, O and LSE:
//   p_c = exp(scale <q_t, k_c> - LSE_t),  delta_t = <dO_t, O_t>,
//   dV_c += p_c dO_t,  e_c = p_c (<dO_t, v_c> - delta_t),
//   dQ_t = scale sum_c e_c k_c,  dK_c += scale e_c q_t.
// Three kernels, no atomics, every output element written exactly once:
//   delta  : delta_t for every row (row-parallel, vector ALUs).
//   dkdv   : one workgroup per 128 sequence keys; Q / dO tiles stream through LDS;
//            S = Q K^T and dP = dO V^T are recomputed per 32x32 block on the MFMA
//            pipe, P and dS = P (dP - delta) are packed to bf16 straight out of the
//            accumulators and contracted over the queries into dV^T, dK^T.
//   dq     : one workgroup per 128 queries; K / V tiles stream through LDS; S^T, dP^T
//            are recomputed in the transposed orientation (a lane owns one query),
//            dQ^T += K^T dS^T; then, in a row-major epilogue, the depth slots of the
//            query's own position give dKdepth, dVdepth (row-local, written once)
//            and their share of dQ.
// Grouped-query attention (Hq != Hk) is not handled here.
#include "moda_launch.h"
#include "moda_tile.h"

namespace moda {

constexpr float kLog2e = 1.4426950408889634f;

// ---------------------------------------------------------------- delta_t = <dO_t, O_t>
template <int D>
__global__ __launch_bounds__(256) void moda_bwd_delta_kernel(const void* dO, const void* O, float* delta,
                                                             long long rows) {
  constexpr int LPR = D / 8;  // lanes per row, 8 channels each
  const long long row = ((long long)blockIdx.x * 256 + threadIdx.x) / LPR;
  const int l = threadIdx.x % LPR;
  const long long rc = row < rows ? row : rows - 1;
  const u32x4 a = *(const u32x4*)((const char*)dO + (size_t)rc * D * 2 + l * 16);
  const u32x4 b = *(const u32x4*)((const char*)O + (size_t)rc * D * 2 + l * 16);
  float s = 0.f;
#pragma unroll
  for (int k = 0; k < 4; ++k) s = dot2_bf16(a[k], b[k], s);
  s = group_sum<LPR>(s);
  if (l == 0 && row < rows) delta[row] = s;
}

template <int D>
struct BwdCfg {
  static constexpr int kXRow = D * 4 + 16;        // fp32 exchange row, padded
  static constexpr int kXWave = 32 * kXRow;       // 32 rows per wave
  static constexpr int kXBytes = 4 * kXWave;
  static constexpr int kStageBytes = 2 * Tile<D>::kBytes;  // two tiles per stage
  static constexpr int kAux = 2 * 2 * 64 * 4;     // per stage: lse2[64], delta[64] (dkdv only)
  static constexpr int kRing = 2 * kStageBytes;
  static constexpr int kLds = (kRing > kXBytes ? kRing : kXBytes) + kAux;
};

__device__ __forceinline__ bf16x8 pack8(const float (&x)[8]) {
  u32x4 t = {pack_bf16(x[0], x[1]), pack_bf16(x[2], x[3]), pack_bf16(x[4], x[5]), pack_bf16(x[6], x[7])};
  return __builtin_bit_cast(bf16x8, t);
}

// ---------------------------------------------------------------- dK, dV
// Workgroup = 128 keys (4 waves x 32 keys).  Accumulators hold dK^T, dV^T
// ([channel][key]: a lane owns one key and 64 of its channels).
template <int D>
__global__ __launch_bounds__(256, 2) void moda_bwd_dkdv_kernel(BwdParams p) {
  using Tl = Tile<D>;
  using C = BwdCfg<D>;
  __shared__ __attribute__((aligned(16))) unsigned char smem[C::kLds];
  float* aux = (float*)(smem + C::kLds - C::kAux);

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, hi = lane >> 5;
  const int T = p.T;
  const int BH = p.B * p.Hq;
  const int bh = blockIdx.x % BH;
  const int jt = blockIdx.x / BH;  // key tiles in natural order: the first ones see the most queries
  const int j0 = jt * 128;
  const int kw0 = j0 + wave * 32;

  const char* Qb = (const char*)p.Q + (size_t)bh * T * Tl::kRowBytes;
  const char* Kb = (const char*)p.Kseq + (size_t)bh * T * Tl::kRowBytes;
  const char* Vb = (const char*)p.Vseq + (size_t)bh * T * Tl::kRowBytes;
  const char* dOb = (const char*)p.dO + (size_t)bh * T * Tl::kRowBytes;
  const float* LSEb = p.LSE + (size_t)bh * T;
  const float* Db = p.delta + (size_t)bh * T;

  // resident K and V fragments of this wave's 32 keys (MFMA B operands: N = key, K = channels)
  bf16x8 kf[Tl::kDSteps], vf[Tl::kDSteps];
  {
    const int row = min(kw0 + l32, T - 1);
#pragma unroll
    for (int st = 0; st < Tl::kDSteps; ++st) {
      kf[st] = *(const bf16x8*)(Kb + (size_t)row * Tl::kRowBytes + st * 32 + hi * 16);
      vf[st] = *(const bf16x8*)(Vb + (size_t)row * Tl::kRowBytes + st * 32 + hi * 16);
    }
  }
  f32x16 dk[Tl::kDBlocks], dv[Tl::kDBlocks];
#pragma unroll
  for (int db = 0; db < Tl::kDBlocks; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) dk[db][i] = dv[db][i] = 0.f;

  const int nq = (T + 63) / 64;
  const int qt0 = p.causal ? j0 / 64 : 0;
  const float c2 = p.scale_log2;
  const unsigned smem_addr = (unsigned)(size_t)(lds_ptr)smem;
  TileLoader<D> ld;
  ld.init(wave, lane);

  auto issue = [&](int qt, int stage) {
    ld.issue(Qb, qt * 64, T, smem_addr + stage * C::kStageBytes);
    ld.issue(dOb, qt * 64, T, smem_addr + stage * C::kStageBytes + Tl::kBytes);
    if (tid < 64) {
      const int r = min(qt * 64 + tid, T - 1);
      aux[stage * 128 + tid] = LSEb[r] * kLog2e;
      aux[stage * 128 + 64 + tid] = Db[r];
    }
  };

  issue(qt0, 0);
  for (int qt = qt0; qt < nq; ++qt) {
    const int stage = (qt - qt0) & 1;
    wait_copies();
    __syncthreads();
    if (qt + 1 < nq) issue(qt + 1, stage ^ 1);

    const int q0 = qt * 64;
    if (p.causal && q0 + 63 < kw0) continue;  // every query of the tile precedes this wave's keys
    const unsigned char* qtile = smem + stage * C::kStageBytes;
    const unsigned char* dotile = qtile + Tl::kBytes;
    const float* lse_s = aux + stage * 128;
    const float* del_s = lse_s + 64;

    const int key = kw0 + l32;
    // one 32-query block at a time: S, dP (recomputed), P and dS for this lane's key and
    // 16 queries, then dV^T += dO^T P and dK^T += Q^T dS over those 32 queries
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      f32x16 s, dp;
#pragma unroll
      for (int i = 0; i < 16; ++i) s[i] = dp[i] = 0.f;
#pragma unroll
      for (int st = 0; st < Tl::kDSteps; ++st) {
        s = mfma_bf16(Tl::row_frag(qtile, qb, st, lane), kf[st], s);
        dp = mfma_bf16(Tl::row_frag(dotile, qb, st, lane), vf[st], dp);
      }
      bf16x8 pb[2], dsb[2];  // [16-query half]
      float pv[16], dsv[16];
#pragma unroll
      for (int b4 = 0; b4 < 4; ++b4) {
        const f32x4 l4 = *(const f32x4*)(lse_s + qb * 32 + b4 * 8 + hi * 4);
        const f32x4 d4 = *(const f32x4*)(del_s + qb * 32 + b4 * 8 + hi * 4);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int i = b4 * 4 + r;
          const int q = q0 + qb * 32 + b4 * 8 + hi * 4 + r;
          const bool vis = q < T && (!p.causal || key <= q);
          const float pe = vis ? fast_exp2(s[i] * c2 - l4[r]) : 0.f;
          pv[i] = pe;
          dsv[i] = pe * (dp[i] - d4[r]);
        }
      }
#pragma unroll
      for (int hf = 0; hf < 2; ++hf) {
        float a[8], b[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          a[k] = pv[hf * 8 + k];
          b[k] = dsv[hf * 8 + k];
        }
        pb[hf] = pack8(a);
        dsb[hf] = pack8(b);
      }
#pragma unroll
      for (int hf = 0; hf < 2; ++hf)
#pragma unroll
        for (int db = 0; db < Tl::kDBlocks; ++db) {
          dv[db] = mfma_bf16(Tl::tr_frag(dotile, qb * 2 + hf, db, lane), pb[hf], dv[db]);
          dk[db] = mfma_bf16(Tl::tr_frag(qtile, qb * 2 + hf, db, lane), dsb[hf], dk[db]);
        }
    }
  }
  __syncthreads();

  // ---- write out: accumulator layout -> row-major through LDS, 16-byte stores
  unsigned char* xw = smem + wave * C::kXWave;
  constexpr int LPR = Tl::kChunks, RPS = 64 / LPR;
  const int rg = lane / LPR, l16 = lane % LPR;
#pragma unroll
  for (int which = 0; which < 2; ++which) {
#pragma unroll
    for (int db = 0; db < Tl::kDBlocks; ++db)
#pragma unroll
      for (int bq = 0; bq < 4; ++bq) {
        const f32x16& acc = which ? dv[db] : dk[db];
        f32x4 v = {acc[4 * bq], acc[4 * bq + 1], acc[4 * bq + 2], acc[4 * bq + 3]};
        *(f32x4*)(xw + l32 * C::kXRow + (db * 32 + bq * 8 + hi * 4) * 4) = v;
      }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    char* outb = (char*)(which ? p.dVseq : p.dKseq) + (size_t)bh * T * Tl::kRowBytes;
    const float f = which ? 1.0f : p.scale;
    for (int it = 0; it < 32 / RPS; ++it) {
      const int row = it * RPS + rg;
      const int key = kw0 + row;
      const f32x4 o0 = *(const f32x4*)(xw + row * C::kXRow + l16 * 32);
      const f32x4 o1 = *(const f32x4*)(xw + row * C::kXRow + l16 * 32 + 16);
      if (key < T) {
        u32x4 ov = {pack_bf16(o0[0] * f, o0[1] * f), pack_bf16(o0[2] * f, o0[3] * f),
                    pack_bf16(o1[0] * f, o1[1] * f), pack_bf16(o1[2] * f, o1[3] * f)};
        *(u32x4*)(outb + (size_t)key * Tl::kRowBytes + l16 * 16) = ov;
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  }
}

// ---------------------------------------------------------------- dQ, dKdepth, dVdepth
// Workgroup = 128 queries (4 waves x 32 queries).  Accumulators hold dQ^T
// ([channel][query]: a lane owns one query).
template <int D>
__global__ __launch_bounds__(256, 2) void moda_bwd_dq_kernel(BwdParams p) {
  using Tl = Tile<D>;
  using C = BwdCfg<D>;
  __shared__ __attribute__((aligned(16))) unsigned char smem[C::kLds];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, hi = lane >> 5;
  const int T = p.T;
  const int BH = p.B * p.Hq;
  const int bh = blockIdx.x % BH;
  const int n_qt = (T + 127) / 128;
  const int qt = n_qt - 1 - blockIdx.x / BH;  // heavy (late) query tiles first
  const int q0 = qt * 128;
  const int qw0 = q0 + wave * 32;

  const char* Qb = (const char*)p.Q + (size_t)bh * T * Tl::kRowBytes;
  const char* Kb = (const char*)p.Kseq + (size_t)bh * T * Tl::kRowBytes;
  const char* Vb = (const char*)p.Vseq + (size_t)bh * T * Tl::kRowBytes;
  const char* dOb = (const char*)p.dO + (size_t)bh * T * Tl::kRowBytes;
  const float* LSEb = p.LSE + (size_t)bh * T;
  const float* Db = p.delta + (size_t)bh * T;

  // resident Q and dO fragments of this wave's 32 queries (MFMA B operands)
  bf16x8 qf[Tl::kDSteps], dof[Tl::kDSteps];
  const int qi = qw0 + l32;
  const int qrow = min(qi, T - 1);
#pragma unroll
  for (int st = 0; st < Tl::kDSteps; ++st) {
    qf[st] = *(const bf16x8*)(Qb + (size_t)qrow * Tl::kRowBytes + st * 32 + hi * 16);
    dof[st] = *(const bf16x8*)(dOb + (size_t)qrow * Tl::kRowBytes + st * 32 + hi * 16);
  }
  const float lse2 = LSEb[qrow] * kLog2e;
  const float delta = Db[qrow];

  f32x16 dq[Tl::kDBlocks];
#pragma unroll
  for (int db = 0; db < Tl::kDBlocks; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) dq[db][i] = 0.f;

  const int n_keys = p.causal ? min(T, q0 + 128) : T;
  const int nt = (n_keys + 63) / 64;
  const int wave_last = p.causal ? min(nt - 1, (qw0 + 31) / 64) : nt - 1;
  const int lim = p.causal ? min(qi, T - 1) : T - 1;  // last visible key of this lane's query
  const float c2 = p.scale_log2;
  const unsigned smem_addr = (unsigned)(size_t)(lds_ptr)smem;
  TileLoader<D> ld;
  ld.init(wave, lane);
  auto issue = [&](int kt, int stage) {
    ld.issue(Kb, kt * 64, T, smem_addr + stage * C::kStageBytes);
    ld.issue(Vb, kt * 64, T, smem_addr + stage * C::kStageBytes + Tl::kBytes);
  };

  issue(0, 0);
  for (int kt = 0; kt < nt; ++kt) {
    const int stage = kt & 1;
    wait_copies();
    __syncthreads();
    if (kt + 1 < nt) issue(kt + 1, stage ^ 1);
    if (kt > wave_last) continue;
    const unsigned char* ktile = smem + stage * C::kStageBytes;
    const unsigned char* vtile = ktile + Tl::kBytes;

    f32x16 s[2], dp[2];  // S^T, dP^T: [key block]; a lane holds 16 keys of its query
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int i = 0; i < 16; ++i) s[kb][i] = dp[kb][i] = 0.f;
#pragma unroll
      for (int st = 0; st < Tl::kDSteps; ++st) {
        s[kb] = mfma_bf16(Tl::row_frag(ktile, kb, st, lane), qf[st], s[kb]);
        dp[kb] = mfma_bf16(Tl::row_frag(vtile, kb, st, lane), dof[st], dp[kb]);
      }
    }
    bf16x8 dsb[2][2];
    const int k0 = kt * 64;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      float dsv[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int key = k0 + kb * 32 + (i >> 2) * 8 + hi * 4 + (i & 3);
        const float pe = key <= lim ? fast_exp2(s[kb][i] * c2 - lse2) : 0.f;
        dsv[i] = pe * (dp[kb][i] - delta);
      }
#pragma unroll
      for (int hf = 0; hf < 2; ++hf) {
        float a[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) a[k] = dsv[hf * 8 + k];
        dsb[kb][hf] = pack8(a);
      }
    }
    // dQ^T += K^T dS^T  (contraction over the tile's 64 keys)
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
#pragma unroll
      for (int db = 0; db < Tl::kDBlocks; ++db)
        dq[db] = mfma_bf16(Tl::tr_frag(ktile, ks, db, lane), dsb[ks >> 1][ks & 1], dq[db]);
  }
  __syncthreads();

  // ---- epilogue: accumulator layout -> row-major; depth slots; stores
  unsigned char* xw = smem + wave * C::kXWave;
#pragma unroll
  for (int db = 0; db < Tl::kDBlocks; ++db)
#pragma unroll
    for (int bq = 0; bq < 4; ++bq) {
      f32x4 v = {dq[db][4 * bq], dq[db][4 * bq + 1], dq[db][4 * bq + 2], dq[db][4 * bq + 3]};
      *(f32x4*)(xw + l32 * C::kXRow + (db * 32 + bq * 8 + hi * 4) * 4) = v;
    }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

  constexpr int LPR = Tl::kChunks, RPS = 64 / LPR;
  const int rg = lane / LPR, l16 = lane % LPR;
  const int L = p.depth_count, La = p.depth_alloc;
  const size_t drow = (size_t)La * Tl::kRowBytes;
  const char* Kdb = (const char*)p.Kdepth + (size_t)bh * T * drow;
  const char* Vdb = (const char*)p.Vdepth + (size_t)bh * T * drow;
  char* dKdb = (char*)p.dKdepth + (size_t)bh * T * drow;
  char* dVdb = (char*)p.dVdepth + (size_t)bh * T * drow;
  char* dQb = (char*)p.dQ + (size_t)bh * T * Tl::kRowBytes;
  constexpr int CH = 8;  // depth slots whose loads are in flight together

  for (int it = 0; it < 32 / RPS; ++it) {
    const int row = it * RPS + rg;
    const int t = qw0 + row;
    const int tc = min(t, T - 1);
    const bool live = t < T;
    const f32x4 a0 = *(const f32x4*)(xw + row * C::kXRow + l16 * 32);
    const f32x4 a1 = *(const f32x4*)(xw + row * C::kXRow + l16 * 32 + 16);
    float acc[8] = {a0[0], a0[1], a0[2], a0[3], a1[0], a1[1], a1[2], a1[3]};
    if (La > 0) {
      const u32x4 qv = *(const u32x4*)(Qb + (size_t)tc * Tl::kRowBytes + l16 * 16);
      const u32x4 gv = *(const u32x4*)(dOb + (size_t)tc * Tl::kRowBytes + l16 * 16);
      const float l2 = LSEb[tc] * kLog2e;
      const float dl = Db[tc];
      float qx[8], gx[8];
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        qx[2 * k] = bf16_lo(qv[k]);
        qx[2 * k + 1] = bf16_hi(qv[k]);
        gx[2 * k] = bf16_lo(gv[k]);
        gx[2 * k + 1] = bf16_hi(gv[k]);
      }
      const char* kd = Kdb + (size_t)tc * drow + l16 * 16;
      const char* vd = Vdb + (size_t)tc * drow + l16 * 16;
      char* dkd = dKdb + (size_t)tc * drow + l16 * 16;
      char* dvd = dVdb + (size_t)tc * drow + l16 * 16;
      for (int i0 = 0; i0 < L; i0 += CH) {
        u32x4 kv[CH], vv[CH];
#pragma unroll
        for (int i = 0; i < CH; ++i) kv[i] = *(const u32x4*)(kd + (size_t)min(i0 + i, L - 1) * Tl::kRowBytes);
#pragma unroll
        for (int i = 0; i < CH; ++i) vv[i] = *(const u32x4*)(vd + (size_t)min(i0 + i, L - 1) * Tl::kRowBytes);
#pragma unroll
        for (int i = 0; i < CH; ++i) {
          float sdot = 0.f, gdot = 0.f;
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            sdot = dot2_bf16(qv[k], kv[i][k], sdot);
            gdot = dot2_bf16(gv[k], vv[i][k], gdot);
          }
          sdot = group_sum<LPR>(sdot);
          gdot = group_sum<LPR>(gdot);
          if (i0 + i < L) {  // uniform: slots past depth_count only re-read the last slot
            const float pe = fast_exp2(sdot * c2 - l2);
            const float e = pe * (gdot - dl);
            const float es = e * p.scale;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
              acc[2 * k] += e * bf16_lo(kv[i][k]);
              acc[2 * k + 1] += e * bf16_hi(kv[i][k]);
            }
            if (live) {
              u32x4 o1 = {pack_bf16(pe * gx[0], pe * gx[1]), pack_bf16(pe * gx[2], pe * gx[3]),
                          pack_bf16(pe * gx[4], pe * gx[5]), pack_bf16(pe * gx[6], pe * gx[7])};
              u32x4 o2 = {pack_bf16(es * qx[0], es * qx[1]), pack_bf16(es * qx[2], es * qx[3]),
                          pack_bf16(es * qx[4], es * qx[5]), pack_bf16(es * qx[6], es * qx[7])};
              *(u32x4*)(dvd + (size_t)(i0 + i) * Tl::kRowBytes) = o1;
              *(u32x4*)(dkd + (size_t)(i0 + i) * Tl::kRowBytes) = o2;
            }
          }
        }
      }
      if (live) {
        const u32x4 z = {0u, 0u, 0u, 0u};
        for (int i = L; i < La; ++i) {  // allocated but unattended slots get zero gradients
          *(u32x4*)(dvd + (size_t)i * Tl::kRowBytes) = z;
          *(u32x4*)(dkd + (size_t)i * Tl::kRowBytes) = z;
        }
      }
    }
    if (live) {
      const float f = p.scale;
      u32x4 ov = {pack_bf16(acc[0] * f, acc[1] * f), pack_bf16(acc[2] * f, acc[3] * f),
                  pack_bf16(acc[4] * f, acc[5] * f), pack_bf16(acc[6] * f, acc[7] * f)};
      *(u32x4*)(dQb + (size_t)t * Tl::kRowBytes + l16 * 16) = ov;
    }
  }
}

// ---------------------------------------------------------------- launchers
size_t bwd_bf16_workspace_bytes(const BwdParams& p) { return (size_t)p.B * p.Hq * p.T * sizeof(float); }

hipError_t launch_bwd_bf16(const BwdParams& p, int d, hipStream_t stream) {
  const long long rows = (long long)p.B * p.Hq * p.T;
  const int BH = p.B * p.Hq;
  const long long g_delta = (rows * (d / 8) + 255) / 256;
  const long long g_dkdv = (long long)BH * ((p.T + 127) / 128);
  const long long g_dq = g_dkdv;
  if (g_delta > 0x7fffffffLL || g_dkdv > 0x7fffffffLL) return hipErrorInvalidValue;
  if (d == 128) {
    hipLaunchKernelGGL(moda_bwd_delta_kernel<128>, dim3((unsigned)g_delta), dim3(256), 0, stream, p.dO, p.O, p.delta, rows);
    hipLaunchKernelGGL(moda_bwd_dkdv_kernel<128>, dim3((unsigned)g_dkdv), dim3(256), 0, stream, p);
    hipLaunchKernelGGL(moda_bwd_dq_kernel<128>, dim3((unsigned)g_dq), dim3(256), 0, stream, p);
  } else if (d == 64) {
    hipLaunchKernelGGL(moda_bwd_delta_kernel<64>, dim3((unsigned)g_delta), dim3(256), 0, stream, p.dO, p.O, p.delta, rows);
    hipLaunchKernelGGL(moda_bwd_dkdv_kernel<64>, dim3((unsigned)g_dkdv), dim3(256), 0, stream, p);
    hipLaunchKernelGGL(moda_bwd_dq_kernel<64>, dim3((unsigned)g_dq), dim3(256), 0, stream, p);
  } else {
    return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace moda
