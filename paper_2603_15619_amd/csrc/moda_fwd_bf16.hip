// MoDA attention forward, bf16 inputs, fp32 online-softmax state, gfx950 MFMA.
//
// One workgroup = 4 waves = one tile of 256 queries of one (b, h); each wave owns
// 64 queries.  Sequence K/V tiles of 64 keys are streamed through LDS (double
// buffered) and consumed by v_mfma_f32_32x32x16_bf16:
//   S^T = K Q^T   (keys on the MFMA M axis, queries on N): a lane then holds 16
//                 scores of ONE query per 32x32 block, so the row max / row sum
//                 are in-lane reductions plus one exchange with lane ^ 32;
//   O^T += V^T P^T with P^T taken straight from the S^T accumulators (no layout
//                 round trip); the V^T operand comes from ds_read_b64_tr_b16.
// Tiles above the diagonal are never loaded; only the diagonal tile is masked
// (Algorithm 1's split into fully visible and boundary blocks).
// After the sequence loop the accumulators pass through LDS into a row-major
// mapping (d/8 lanes x 8 channels per query).  There the depth slots of the
// query's own position -- one contiguous L*d block in the [B,H,T,L,d] layout --
// are scored with packed dot products and a DPP reduction over those lanes and folded
// into the SAME running max / normaliser / output (Algorithm 1's third loop and
// its single final division), and O / LSE are stored with 128-bit accesses.
#include "moda_launch.h"

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
  static constexpr int kLoads = kBN * kChunks / kThreads;  // 16 B loads per thread per tile
  static constexpr int kRowsPerPass = kThreads / kChunks;  // tile rows covered per load pass
  // fp32 exchange buffer: 32 query rows x D floats per wave, rows padded by 16 B
  static constexpr int kXRow = D * 4 + 16;
  static constexpr int kXWave = 32 * kXRow + 32 * 8;  // + (m, l) per row
  static constexpr int kKVBytes = 4 * kTileBytes;      // K, V double buffered
  static constexpr int kXBytes = kWaves * kXWave;
  static constexpr int kLds = kKVBytes > kXBytes ? kKVBytes : kXBytes;
};

// LDS placement of the 16-byte chunk c of tile row r.
//  K tile: chunk index XOR row  -> the MFMA A-operand read (consecutive lanes =
//          consecutive rows, same chunk) spreads over all banks.
//  V tile: 32-byte pair index XOR row -> the transposing read (a 16-lane group
//          reads 4 rows x 32 B) spreads over all banks.
template <int D>
__device__ __forceinline__ int k_off(int r, int c) {
  return r * FwdCfg<D>::kRowBytes + ((c ^ (r & (FwdCfg<D>::kChunks - 1))) << 4);
}
template <int D>
__device__ __forceinline__ int v_off(int r, int c) {
  int pair = (c >> 1) ^ (r & (FwdCfg<D>::kChunks / 2 - 1));
  return r * FwdCfg<D>::kRowBytes + (pair << 5) + ((c & 1) << 4);
}

template <int D>
__global__ __launch_bounds__(kThreads, 1) void moda_fwd_bf16_kernel(FwdParams p) {
  using C = FwdCfg<D>;
  __shared__ __attribute__((aligned(16))) unsigned char smem[C::kLds];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
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

  // ---- Q fragments (MFMA B operand of S^T = K Q^T), resident for the whole tile
  bf16x8 qf[2][C::kDSteps];
#pragma unroll
  for (int nb = 0; nb < 2; ++nb) {
    int row = min(qw0 + nb * 32 + l32, T - 1);
#pragma unroll
    for (int st = 0; st < C::kDSteps; ++st)
      qf[nb][st] = *(const bf16x8*)(Qb + (size_t)row * C::kRowBytes + st * 32 + hi * 16);
  }

  f32x16 oacc[C::kDBlocks][2];
#pragma unroll
  for (int db = 0; db < C::kDBlocks; ++db)
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int i = 0; i < 16; ++i) oacc[db][nb][i] = 0.f;
  float m_run[2] = {-INFINITY, -INFINITY};  // running max of the raw scores <q,k>
  float l_run[2] = {0.f, 0.f};              // this lane's share of the normaliser

  // number of key tiles this workgroup walks, and the last one this wave needs
  const int n_keys = p.causal ? min(T, q0 + kBM) : T;
  const int nt = (n_keys + kBN - 1) / kBN;
  const int wave_last = p.causal ? min(nt - 1, qw0 / kBN) : nt - 1;
  const float c2 = p.scale_log2;

  // ---- global -> register -> LDS staging of one K/V tile
  const int ld_c = tid % C::kChunks;
  const int ld_r = tid / C::kChunks;
  u32x4 kst[C::kLoads], vst[C::kLoads];
  auto load_tile = [&](int kt) {
#pragma unroll
    for (int i = 0; i < C::kLoads; ++i) {
      int row = min(kt * kBN + ld_r + i * C::kRowsPerPass, T - 1);
      size_t off = (size_t)row * C::kRowBytes + ld_c * 16;
      kst[i] = *(const u32x4*)(Kb + off);
      vst[i] = *(const u32x4*)(Vb + off);
    }
  };
  auto store_tile = [&](int buf) {
    unsigned char* kbuf = smem + buf * 2 * C::kTileBytes;
    unsigned char* vbuf = kbuf + C::kTileBytes;
#pragma unroll
    for (int i = 0; i < C::kLoads; ++i) {
      int r = ld_r + i * C::kRowsPerPass;
      *(u32x4*)(kbuf + k_off<D>(r, ld_c)) = kst[i];
      *(u32x4*)(vbuf + v_off<D>(r, ld_c)) = vst[i];
    }
  };

  load_tile(0);
  store_tile(0);
  __syncthreads();

  for (int kt = 0; kt < nt; ++kt) {
    const bool more = kt + 1 < nt;
    if (more) load_tile(kt + 1);

    if (kt <= wave_last) {
      const unsigned char* kbuf = smem + (kt & 1) * 2 * C::kTileBytes;
      const unsigned char* vbuf = kbuf + C::kTileBytes;

      // ---- S^T = K Q^T : [2 key blocks][2 query blocks] of 32x32
      f32x16 sacc[2][2];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
          for (int i = 0; i < 16; ++i) sacc[kb][nb][i] = 0.f;
#pragma unroll
      for (int st = 0; st < C::kDSteps; ++st) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
          bf16x8 kf = *(const bf16x8*)(kbuf + k_off<D>(kb * 32 + l32, st * 2 + hi));
#pragma unroll
          for (int nb = 0; nb < 2; ++nb)
            sacc[kb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[nb][st], sacc[kb][nb], 0, 0, 0);
        }
      }

      // ---- mask (diagonal tile under the causal mask, or a ragged last tile)
      const int k0 = kt * kBN;
      const bool need_mask = (p.causal && k0 + kBN - 1 > qw0) || (k0 + kBN > T);
      if (need_mask) {
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) {
          int qi = qw0 + nb * 32 + l32;
          int lim = p.causal ? min(qi, T - 1) : T - 1;  // last visible key
#pragma unroll
          for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
              int key = k0 + kb * 32 + (i >> 2) * 8 + hi * 4 + (i & 3);
              if (key > lim) sacc[kb][nb][i] = -INFINITY;
            }
        }
      }

      // ---- online softmax, one query per lane and query block
      uint32_t pf[2][2][8];  // P^T as packed bf16: [key block][query block][8 regs]
      float alpha[2];
#pragma unroll
      for (int nb = 0; nb < 2; ++nb) {
        float mx = sacc[0][nb][0];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int i = 0; i < 16; ++i) mx = fmaxf(mx, sacc[kb][nb][i]);
        mx = pair_max(mx);
        float m_new = fmaxf(m_run[nb], mx);
        alpha[nb] = fast_exp2((m_run[nb] - m_new) * c2);
        m_run[nb] = m_new;
        float mc = m_new * c2;
        float sum = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int i = 0; i < 16; i += 2) {
            float e0 = fast_exp2(sacc[kb][nb][i] * c2 - mc);
            float e1 = fast_exp2(sacc[kb][nb][i + 1] * c2 - mc);
            sum += e0 + e1;
            pf[kb][nb][i >> 1] = pack_bf16(e0, e1);
          }
        l_run[nb] = l_run[nb] * alpha[nb] + sum;
      }
#pragma unroll
      for (int db = 0; db < C::kDBlocks; ++db)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
          for (int i = 0; i < 16; ++i) oacc[db][nb][i] *= alpha[nb];

      // ---- O^T += V^T P^T.  MFMA k-slots 0..7 (lanes < 32) are keys
      // {0..3, 8..11} of a 16-key group and slots 8..15 (lanes >= 32) keys
      // {4..7, 12..15}: exactly how the S^T accumulators hold them.
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const int kb = ks >> 1, s = ks & 1;
        bf16x8 pb[2];
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) {
          u32x4 t = {pf[kb][nb][4 * s], pf[kb][nb][4 * s + 1], pf[kb][nb][4 * s + 2], pf[kb][nb][4 * s + 3]};
          pb[nb] = __builtin_bit_cast(bf16x8, t);
        }
#pragma unroll
        for (int db = 0; db < C::kDBlocks; ++db) {
          // transposing read: within 16 lanes, lane i supplies row (i/4), 8-byte
          // piece (i%4) of a 4-key x 16-channel block and receives channel i of
          // the 4 keys.
          const int rr = ks * 16 + hi * 4 + ((lane & 15) >> 2);
          const int ch = db * 4 + ((lane >> 4) & 1) * 2;  // 16 B chunk holding the lane's 32 B segment
          const int sub = (lane & 3) * 8;                  // byte offset inside the 32 B segment
          const unsigned char* a0 = vbuf + v_off<D>(rr, ch) + sub;
          const unsigned char* a1 = vbuf + v_off<D>(rr + 8, ch) + sub;
          s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)a0);
          s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)a1);
          s16x8 v01 = __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7);
          bf16x8 vf = __builtin_bit_cast(bf16x8, v01);
#pragma unroll
          for (int nb = 0; nb < 2; ++nb)
            oacc[db][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pb[nb], oacc[db][nb], 0, 0, 0);
        }
      }
    }

    if (more) store_tile((kt + 1) & 1);
    __syncthreads();
  }

  // ================= epilogue: accumulator layout -> row-major, depth slots, store
  // (the loop's last barrier guarantees nobody still reads the K/V buffers)
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
#pragma unroll
    for (int db = 0; db < C::kDBlocks; ++db)
#pragma unroll
      for (int bq = 0; bq < 4; ++bq) {
        f32x4 v = {oacc[db][nb][4 * bq], oacc[db][nb][4 * bq + 1], oacc[db][nb][4 * bq + 2],
                   oacc[db][nb][4 * bq + 3]};
        *(f32x4*)(xw + l32 * C::kXRow + (db * 32 + bq * 8 + hi * 4) * 4) = v;
      }
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
