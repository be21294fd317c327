// MoDA attention backward, bf16 inputs, fp32 accumulation, gfx950 MFMA.
//
// The paper gives no backward algorithm; this is the derivative of the forward
// definition (one softmax over causal sequence keys and same-position depth slots),
// evaluated by recomputation from Q, K, V, the depth tensors, O and LSE:
//   p_c = exp(scale <q_t, k_c> - LSE_t),  delta_t = <dO_t, O_t>,
//   dV_c += p_c dO_t,  e_c = p_c (<dO_t, v_c> - delta_t),
//   dQ_t = scale sum_c e_c k_c,  dK_c += scale e_c q_t.
// Three kernels (four with grouped queries), no atomics, every output element written
// exactly once:
//   delta  : (LSE_t log2(e), delta_t) for every row (row-parallel, vector ALUs).
//   dkdv   : one workgroup per 128 sequence keys; Q / dO tiles stream through LDS;
//            S = Q K^T and dP = dO V^T are recomputed per 32x32 block on the MFMA
//            pipe, P and dS = P (dP - delta) are packed to bf16 straight out of the
//            accumulators and contracted over the queries into dV^T, dK^T.  The same
//            workgroup also takes the depth slots of its 128 positions (row-local: dKdepth,
//            dVdepth and the depth share of dQ, left in the workspace in fp32), before or
//            after its key-tile work: that part is bound by HBM, the rest by the matrix pipe.
//   dq     : one workgroup per 128 queries; K / V tiles stream through LDS; S^T, dP^T
//            are recomputed in the transposed orientation (a lane owns one query),
//            dQ^T += K^T dS^T on top of the depth share found in the workspace; every
//            element of dQ is rounded to bf16 once.
// Grouped-query attention (G = Hq / Hk query heads per key/value head, G <= 64): the
// gradients of the shared keys and values sum over the group.  dkdv walks the query
// tiles of all G heads; the depth-slot gradients are computed by a kernel of their own
// (depth_gqa for G <= 8 on the vector ALUs, depth_group above that on the matrix pipe) that holds
// the G heads of a position side by side, sums in fp32 and rounds every depth gradient once.
#include <type_traits>

#include "moda_launch.h"
#include "moda_tile.h"

namespace moda {

constexpr float kLog2e = 1.4426950408889634f;

// ---------------------------------------------------------------- per-row scalars
// rowstat[row] = (LSE_row * log2(e), delta_row = <dO_row, O_row>), interleaved, for the other
// kernels (they exponentiate with exp2; the pairs of a query tile are one contiguous block
// that is copied to LDS without passing through registers).
template <int D>
__global__ __launch_bounds__(256) void moda_bwd_delta_kernel(const void* dO, const void* O, const float* LSE,
                                                             float* rowstat, long long rows) {
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
  if (l == 0 && row < rows) *(f32x2*)(rowstat + 2 * row) = (f32x2){LSE[row] * kLog2e, s};
}

template <int D, int NW = 4>
struct BwdCfg {
  static constexpr int kXRow = D * 4 + 16;        // fp32 exchange row, padded
  static constexpr int kXWave = 32 * kXRow;       // 32 rows per wave
  static constexpr int kXBytes = NW * kXWave;
  static constexpr int kStageBytes = 2 * Tile<D>::kBytes;  // two tiles per stage
  static constexpr int kAux = 2 * 2 * 64 * 4;     // per stage: (lse2, delta) of 64 queries (dkdv only)
  static constexpr int kRing = 2 * kStageBytes;
  static constexpr int kLds = (kRing > kXBytes ? kRing : kXBytes) + kAux;
};

// 16 bytes per lane to a raw buffer (non-temporal), followed by two wait states in the same
// statement.  Measured on this chip: a vector-ALU instruction that overwrites the last data
// register of a 128-bit buffer store in the very next issue slot can still change what is
// stored (the last lanes of each row of 16 read their data last), also when the store takes its
// offset from a scalar register, the one case for which the compiler inserts no wait state.
__device__ __forceinline__ void buffer_store16_nt(const u32x4& v, const i32x4& rsrc, int voff, int soff) {
  asm volatile("buffer_store_dwordx4 %0, %1, %2, %3 offen nt\n\ts_nop 1" : : "v"(v), "v"(voff), "s"(rsrc), "s"(soff) : "memory");
}

// ---------------------------------------------------------------- depth-slot gradients (G = 1)
// The depth slots of 32 consecutive positions (row0 ...) of one head, handled by one wave in a
// row-major mapping (d/8 lanes x 8 channels per row, 64 / (d/8) rows per wave step): dKdepth,
// dVdepth (row-local, written once) and the depth share of dQ, which is left in the workspace
// (fp32, not yet multiplied by the softmax scale) for the dQ kernel to start from.
// Work items (row step, chunk of kChunk slots) are walked with the loads of the next two
// items in flight (the phase is bound by memory latency).  Uses no LDS.
template <int D>
__device__ __forceinline__ void depth_grad_rows(const BwdParams& p, int bh, int row0, int lane) {
  using Tl = Tile<D>;
  constexpr int LPR = Tl::kChunks, RPS = 64 / LPR, NIT = 32 / RPS;
  constexpr int kChunk = 5;
  const int T = p.T, L = p.depth_count, La = p.depth_alloc;
  const int bg = bh, qw0 = row0;
  const float c2 = p.scale_log2;
  const char* Qb = (const char*)p.Q + (size_t)bh * T * Tl::kRowBytes;
  const char* dOb = (const char*)p.dO + (size_t)bh * T * Tl::kRowBytes;
  const float* statb = p.rowstat + (size_t)bh * T * 2;
  const int rg = lane / LPR, l16 = lane % LPR;
  const size_t drow = (size_t)La * Tl::kRowBytes;
  // (this phase only runs when every key/value head serves one query head: bg == bh)
  // The depth tensors are addressed from the first of the wave's 32 positions (a 64-bit base)
  // with 32-bit offsets from there, so they may be of any size; `slab` is what is left of the
  // (batch, head) slab from that position on, clamped to what 32 bits hold.
  const int rbase = min(qw0, T - 1);
  const size_t dbase = ((size_t)bg * T + rbase) * drow;
  const size_t left = (size_t)(T - rbase) * drow;
  const size_t slab = left < 0xffffffffull ? left : 0xffffffffull;
  const char* Kdb = (const char*)p.Kdepth + dbase;
  const char* Vdb = (const char*)p.Vdepth + dbase;
  char* dKdb = (char*)p.dKdepth + dbase;
  char* dVdb = (char*)p.dVdepth + dbase;
  float* dQd = p.dq_depth + (size_t)bh * T * D;
  const __amdgpu_buffer_rsrc_t kd_buf = __builtin_amdgcn_make_buffer_rsrc((void*)Kdb, 0, (int)(unsigned)slab, 0x00020000);
  const __amdgpu_buffer_rsrc_t vd_buf = __builtin_amdgcn_make_buffer_rsrc((void*)Vdb, 0, (int)(unsigned)slab, 0x00020000);
  const i32x4 dkd_buf = make_tile_buffer(dKdb, (unsigned)slab);
  const i32x4 dvd_buf = make_tile_buffer(dVdb, (unsigned)slab);
  const int nch = (L + kChunk - 1) / kChunk;

  struct Item {
    u32x4 q, g;   // the row's Q and dO channels of this lane
    float l2, dl;  // LSE * log2(e), delta
    u32x4 k[kChunk], v[kChunk];
  };
  float acc[8];
  auto begin_row = [&]() {
#pragma unroll
    for (int k = 0; k < 8; ++k) acc[k] = 0.f;
  };
  auto end_row = [&](int row) {
    const int t = qw0 + row;
    if (t < T) {
      float* dst = dQd + (size_t)t * D + l16 * 8;
      *(f32x4*)dst = (f32x4){acc[0], acc[1], acc[2], acc[3]};
      *(f32x4*)(dst + 4) = (f32x4){acc[4], acc[5], acc[6], acc[7]};
    }
  };
  if (L == 0) {  // no attended slots: a zero share of dQ, zero gradients for allocated slots
    for (int it = 0; it < NIT; ++it) {
      const int row = it * RPS + rg, t = qw0 + row;
      begin_row();
      end_row(row);
      if (t < T) {
        const u32x4 z = {0u, 0u, 0u, 0u};
        for (int i = 0; i < La; ++i) {
          *(u32x4*)(dVdb + (size_t)(t - rbase) * drow + (size_t)i * Tl::kRowBytes + l16 * 16) = z;
          *(u32x4*)(dKdb + (size_t)(t - rbase) * drow + (size_t)i * Tl::kRowBytes + l16 * 16) = z;
        }
      }
    }
    return;
  }
  auto issue = [&](int it, int c, Item& b) {
    const int tc = min(qw0 + it * RPS + rg, T - 1);  // rows past the end use row T-1; nothing of them is stored
    b.q = *(const u32x4*)(Qb + (size_t)tc * Tl::kRowBytes + l16 * 16);
    b.g = *(const u32x4*)(dOb + (size_t)tc * Tl::kRowBytes + l16 * 16);
    const f32x2 st = *(const f32x2*)(statb + 2 * tc);
    b.l2 = st[0];
    b.dl = st[1];
    const int voff = (int)((unsigned)(tc - rbase) * (unsigned)drow + (unsigned)l16 * 16u);  // 32 positions' slots: far below 4 GiB
    // slots of the chunk past depth_count re-read the last attended slot (a cache hit, ignored)
#pragma unroll
    for (int i = 0; i < kChunk; ++i)
      b.k[i] = __builtin_amdgcn_raw_buffer_load_b128(kd_buf, voff, min(c * kChunk + i, L - 1) * Tl::kRowBytes, 2);
#pragma unroll
    for (int i = 0; i < kChunk; ++i)
      b.v[i] = __builtin_amdgcn_raw_buffer_load_b128(vd_buf, voff, min(c * kChunk + i, L - 1) * Tl::kRowBytes, 2);
  };
  auto fold = [&](int it, int c, const Item& b) {
    const int t = qw0 + it * RPS + rg;
    const bool live = t < T;  // rows past the end compute on row T-1 and store nothing
    const int voff = (int)((unsigned)(min(t, T - 1) - rbase) * (unsigned)drow + (unsigned)l16 * 16u);
    const int soff = c * kChunk * Tl::kRowBytes;
    float qx[8], gx[8];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      qx[2 * k] = bf16_lo(b.q[k]);
      qx[2 * k + 1] = bf16_hi(b.q[k]);
      gx[2 * k] = bf16_lo(b.g[k]);
      gx[2 * k + 1] = bf16_hi(b.g[k]);
    }
    // The common case, every slot of the chunk attended and every row of the wave inside the
    // sequence, has no branch per slot: the slots' chains of dependent instructions (dot
    // products, lane sums, exponential) then overlap.
    if ((c + 1) * kChunk <= L && qw0 + 32 <= T) {  // (uniform)
      float pe[kChunk], e[kChunk];
#pragma unroll
      for (int i = 0; i < kChunk; ++i) {
        float sdot = 0.f, gdot = 0.f;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          sdot = dot2_bf16(b.q[k], b.k[i][k], sdot);
          gdot = dot2_bf16(b.g[k], b.v[i][k], gdot);
        }
        sdot = group_sum<LPR>(sdot);
        gdot = group_sum<LPR>(gdot);
        pe[i] = fast_exp2(sdot * c2 - b.l2);
        e[i] = pe[i] * (gdot - b.dl);
      }
#pragma unroll
      for (int i = 0; i < kChunk; ++i) {
        const float es = e[i] * p.scale;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          acc[2 * k] += e[i] * bf16_lo(b.k[i][k]);
          acc[2 * k + 1] += e[i] * bf16_hi(b.k[i][k]);
        }
        const u32x4 o1 = {pack_bf16(pe[i] * gx[0], pe[i] * gx[1]), pack_bf16(pe[i] * gx[2], pe[i] * gx[3]),
                          pack_bf16(pe[i] * gx[4], pe[i] * gx[5]), pack_bf16(pe[i] * gx[6], pe[i] * gx[7])};
        const u32x4 o2 = {pack_bf16(es * qx[0], es * qx[1]), pack_bf16(es * qx[2], es * qx[3]),
                          pack_bf16(es * qx[4], es * qx[5]), pack_bf16(es * qx[6], es * qx[7])};
        buffer_store16_nt(o1, dvd_buf, voff + i * Tl::kRowBytes, soff);
        buffer_store16_nt(o2, dkd_buf, voff + i * Tl::kRowBytes, soff);
      }
      return;
    }
#pragma unroll
    for (int i = 0; i < kChunk; ++i) {
      float sdot = 0.f, gdot = 0.f;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        sdot = dot2_bf16(b.q[k], b.k[i][k], sdot);
        gdot = dot2_bf16(b.g[k], b.v[i][k], gdot);
      }
      sdot = group_sum<LPR>(sdot);
      gdot = group_sum<LPR>(gdot);
      const int slot = c * kChunk + i;
      if (slot >= L) {  // uniform
        // slots past depth_count may hold anything (NaN included) and take no part; those
        // that are allocated get zero gradients
        if (slot < La && live) {
          const u32x4 z = {0u, 0u, 0u, 0u};
          buffer_store16_nt(z, dvd_buf, voff + i * Tl::kRowBytes, soff);
          buffer_store16_nt(z, dkd_buf, voff + i * Tl::kRowBytes, soff);
        }
      } else {
        const float pe = fast_exp2(sdot * c2 - b.l2);
        const float e = pe * (gdot - b.dl);
        const float es = e * p.scale;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          acc[2 * k] += e * bf16_lo(b.k[i][k]);
          acc[2 * k + 1] += e * bf16_hi(b.k[i][k]);
        }
        const u32x4 o1 = {pack_bf16(pe * gx[0], pe * gx[1]), pack_bf16(pe * gx[2], pe * gx[3]),
                          pack_bf16(pe * gx[4], pe * gx[5]), pack_bf16(pe * gx[6], pe * gx[7])};
        const u32x4 o2 = {pack_bf16(es * qx[0], es * qx[1]), pack_bf16(es * qx[2], es * qx[3]),
                          pack_bf16(es * qx[4], es * qx[5]), pack_bf16(es * qx[6], es * qx[7])};
        if (live) {
          buffer_store16_nt(o1, dvd_buf, voff + i * Tl::kRowBytes, soff);
          buffer_store16_nt(o2, dkd_buf, voff + i * Tl::kRowBytes, soff);
        }
      }
    }
  };
  int it = 0, c = 0, iti = 0, ci = 0;
  auto advance = [&](int& i_, int& c_) {
    if (++c_ == nch) {
      c_ = 0;
      ++i_;
    }
  };
  // (past the end the issue cursor stays on the last item: its loads are repeated and ignored)
  auto issue_next = [&](Item& b) {
    issue(iti, ci, b);
    int i2 = iti, c2n = ci;
    advance(i2, c2n);
    if (i2 < NIT) {
      iti = i2;
      ci = c2n;
    }
    __builtin_amdgcn_sched_barrier(0);
  };
  auto one = [&](const Item& cur, Item& refill) -> bool {
    issue_next(refill);
    const int row = it * RPS + rg;
    if (c == 0) begin_row();
    fold(it, c, cur);
    if (c == nch - 1) {
      end_row(row);
      // allocated slots beyond the last chunk (depth_alloc > depth_count rounded up to a chunk)
      const int t = qw0 + row;
      if (t < T) {
        const u32x4 z = {0u, 0u, 0u, 0u};
        for (int i = nch * kChunk; i < La; ++i) {
          *(u32x4*)(dVdb + (size_t)(t - rbase) * drow + (size_t)i * Tl::kRowBytes + l16 * 16) = z;
          *(u32x4*)(dKdb + (size_t)(t - rbase) * drow + (size_t)i * Tl::kRowBytes + l16 * 16) = z;
        }
      }
    }
    advance(it, c);
    return it < NIT;
  };
  Item bufA, bufB, bufC;
  issue_next(bufA);
  issue_next(bufB);
  while (true) {
    if (!one(bufA, bufC)) break;
    if (!one(bufB, bufA)) break;
    if (!one(bufC, bufB)) break;
  }
}

// ---------------------------------------------------------------- depth-slot gradients, grouped queries (2 <= G <= 8)
// One row = one (batch, key/value head, position); d/8 lanes x 8 channels per row, `row` is
// (b * Hk + g) * T + t of this thread's row (rows that do not exist: `live` false, they compute on
// a clamped row and store nothing).  The GT (>= G) query heads of the group are resident (their Q
// and dO rows, LSE, delta, and their depth share of dQ); the row's slots stream by, one prefetched
// ahead.  Per slot i:
//   dVdepth_i = sum_h p_{h,i} dO_h,  dKdepth_i = scale sum_h e_{h,i} q_h  (summed in fp32, one
//                                    rounding each),
//   dQ_h     += e_{h,i} k_i          (left in the workspace, fp32, unscaled, for the dQ kernel).
// Groups of up to 4 heads: runs inside the dK/dV kernel, for the 128 positions of a workgroup's
// key tile, before or after its key-tile work: the phase is then bound by HBM (the slots read
// once, their gradients written once), the key-tile work by the matrix pipe.
template <int D, int GT>
__device__ __forceinline__ void depth_gqa_row(const BwdParams& p, long long row, bool live, int l16) {
  constexpr int LPR = D / 8, RB = D * 2;
  const int T = p.T, L = p.depth_count, La = p.depth_alloc, G = p.Hq / p.Hk;
  const long long rc = row;
  const int t = (int)(rc % T);
  const int bg = (int)(rc / T);
  const int bh0 = (bg / p.Hk) * p.Hq + (bg % p.Hk) * G;
  const float c2 = p.scale_log2;
  u32x4 q[GT], g[GT];
  float l2[GT], dl[GT], dq[GT][8];
#pragma unroll
  for (int j = 0; j < GT; ++j) {
    const int bh = bh0 + min(j, G - 1);  // heads past the group repeat the last one with weight zero
    q[j] = *(const u32x4*)((const char*)p.Q + ((size_t)bh * T + t) * RB + l16 * 16);
    g[j] = *(const u32x4*)((const char*)p.dO + ((size_t)bh * T + t) * RB + l16 * 16);
    const f32x2 st = *(const f32x2*)(p.rowstat + ((size_t)bh * T + t) * 2);
    l2[j] = st[0];
    dl[j] = st[1];
#pragma unroll
    for (int k = 0; k < 8; ++k) dq[j][k] = 0.f;
  }
  const size_t drow = (size_t)La * RB;
  const char* kd = (const char*)p.Kdepth + (size_t)rc * drow + l16 * 16;
  const char* vd = (const char*)p.Vdepth + (size_t)rc * drow + l16 * 16;
  char* dkd = (char*)p.dKdepth + (size_t)rc * drow + l16 * 16;
  char* dvd = (char*)p.dVdepth + (size_t)rc * drow + l16 * 16;

  u32x4 kn = {0u, 0u, 0u, 0u}, vn = kn;
  if (L > 0) {
    kn = __builtin_nontemporal_load((const u32x4*)kd);
    vn = __builtin_nontemporal_load((const u32x4*)vd);
  }
  for (int i = 0; i < L; ++i) {
    const u32x4 kv = kn, vv = vn;
    const int inext = min(i + 1, L - 1);
    kn = __builtin_nontemporal_load((const u32x4*)(kd + (size_t)inext * RB));
    vn = __builtin_nontemporal_load((const u32x4*)(vd + (size_t)inext * RB));
    float kx[8], ak[8], av[8];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      kx[2 * k] = bf16_lo(kv[k]);
      kx[2 * k + 1] = bf16_hi(kv[k]);
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) ak[k] = av[k] = 0.f;
#pragma unroll
    for (int j = 0; j < GT; ++j) {
      float sdot = 0.f, gdot = 0.f;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        sdot = dot2_bf16(q[j][k], kv[k], sdot);
        gdot = dot2_bf16(g[j][k], vv[k], gdot);
      }
      sdot = group_sum<LPR>(sdot);
      gdot = group_sum<LPR>(gdot);
      const float pe = j < G ? fast_exp2(sdot * c2 - l2[j]) : 0.f;
      const float e = pe * (gdot - dl[j]);
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        av[2 * k] += pe * bf16_lo(g[j][k]);
        av[2 * k + 1] += pe * bf16_hi(g[j][k]);
        ak[2 * k] += e * bf16_lo(q[j][k]);
        ak[2 * k + 1] += e * bf16_hi(q[j][k]);
      }
#pragma unroll
      for (int k = 0; k < 8; ++k) dq[j][k] += e * kx[k];
    }
    if (live) {
      const float f = p.scale;
      const u32x4 o1 = {pack_bf16(av[0], av[1]), pack_bf16(av[2], av[3]), pack_bf16(av[4], av[5]), pack_bf16(av[6], av[7])};
      const u32x4 o2 = {pack_bf16(ak[0] * f, ak[1] * f), pack_bf16(ak[2] * f, ak[3] * f),
                        pack_bf16(ak[4] * f, ak[5] * f), pack_bf16(ak[6] * f, ak[7] * f)};
      __builtin_nontemporal_store(o1, (u32x4*)(dvd + (size_t)i * RB));
      __builtin_nontemporal_store(o2, (u32x4*)(dkd + (size_t)i * RB));
    }
  }
  if (live) {
    const u32x4 z = {0u, 0u, 0u, 0u};
    for (int i = L; i < La; ++i) {  // allocated but unattended slots get zero gradients
      *(u32x4*)(dvd + (size_t)i * RB) = z;
      *(u32x4*)(dkd + (size_t)i * RB) = z;
    }
#pragma unroll
    for (int j = 0; j < GT; ++j)
      if (j < G) {
        float* dst = p.dq_depth + ((size_t)(bh0 + j) * T + t) * D + l16 * 8;
        *(f32x4*)dst = (f32x4){dq[j][0], dq[j][1], dq[j][2], dq[j][3]};
        *(f32x4*)(dst + 4) = (f32x4){dq[j][4], dq[j][5], dq[j][6], dq[j][7]};
      }
  }
}

// The same rows as a kernel of its own: groups of 5 to 8 heads, where the arithmetic per fetched
// byte (it grows with the group) makes the phase a vector-ALU job that the dK/dV kernel cannot
// hide (measured at 8 heads: inside dK/dV it costs what it costs alone).
template <int D, int GT>
__global__ __launch_bounds__(256, 2) void moda_bwd_depth_gqa_kernel(BwdParams p) {
  constexpr int LPR = D / 8, ROWS = 256 / LPR;
  const long long row = (long long)blockIdx.x * ROWS + threadIdx.x / LPR;  // (b * Hk + g) * T + t
  const long long n_rows = (long long)p.B * p.Hk * p.T;
  depth_gqa_row<D, GT>(p, row < n_rows ? row : n_rows - 1, row < n_rows, threadIdx.x % LPR);
}

// ---------------------------------------------------------------- dK, dV
// Workgroup = 128 keys (4 waves x 32 keys).  Accumulators hold dK^T, dV^T
// ([channel][key]: a lane owns one key and 64 of its channels).
// GT: 0 = one query head per key/value head, more than 4 heads per group, or no depth slots;
// 2, 4 = the depth-slot gradients of a group of up to GT heads are taken here as well
// (depth_gqa_row).
template <int D, int GT>
__global__ __launch_bounds__(256, 2) void moda_bwd_dkdv_kernel(BwdParams p) {
  using Tl = Tile<D>;
  using C = BwdCfg<D>;
  __shared__ __attribute__((aligned(1024))) unsigned char smem[C::kLds];
  float* aux = (float*)(smem + C::kLds - C::kAux);

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, hi = lane >> 5;
  const int T = p.T;
  const int BHk = p.B * p.Hk;
  int bg, jt;  // (batch, key/value head); key tiles in natural order: the first ones see the most queries
  head_blocked_id((int)blockIdx.x, BHk, (T + 127) / 128, bg, jt, p.head_group);
  const int j0 = jt * 128;
  const int kw0 = j0 + wave * 32;
  const int G = p.Hq / p.Hk;        // query heads per key/value head: their gradients add up here
  const int bh0 = (bg / p.Hk) * p.Hq + (bg % p.Hk) * G;  // first query head of the group

  const char* Kb = (const char*)p.Kseq + (size_t)bg * T * Tl::kRowBytes;
  const char* Vb = (const char*)p.Vseq + (size_t)bg * T * Tl::kRowBytes;

  // ---- Depth-slot gradients (one query head per key/value head; grouped queries have a kernel
  // of their own): row-local, bound by HBM (every depth slot read once, every gradient written
  // once), and independent of everything else this kernel does, which is bound by the matrix
  // pipe and leaves HBM idle.  Each workgroup takes the 128 positions of its key tile, before
  // its key-tile work (every other workgroup) or after it, so that at any time some compute
  // units stream while others compute.
  const bool own_depth = G == 1 && p.depth_alloc > 0;
  const bool depth_first = ((blockIdx.x >> 3) & 1) != 0;
  if (own_depth && depth_first) depth_grad_rows<D>(p, bg, kw0, lane);
  // grouped queries: the workgroup's 128 positions, 256 / (d/8) at a time
  auto group_depth = [&]() {
    if constexpr (GT > 0) {
      constexpr int LPR = D / 8, ROWS = 256 / LPR;
      for (int r0 = 0; r0 < 128; r0 += ROWS) {
        const int t = j0 + r0 + tid / LPR;
        depth_gqa_row<D, GT>(p, (long long)bg * T + min(t, T - 1), t < T, tid % LPR);
      }
    }
  };
  if (GT > 0 && depth_first) group_depth();

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
  const int span = nq - qt0;   // query tiles that see this key tile, per query head
  const int n_items = G * span;  // work items: (query head of the group, query tile)
  const float c2 = p.scale_log2;
  const unsigned smem_addr = (unsigned)(size_t)(lds_ptr)smem;
  TileLoader<D> ld;
  ld.init(wave, lane);
  FragAddr<D> fa;
  fa.init(lane);

  auto issue = [&](int item, int stage) {
    const int bh = bh0 + item / span, qt = qt0 + item % span;
    const i32x4 q_buf = make_tile_buffer((const char*)p.Q + (size_t)bh * T * Tl::kRowBytes, (unsigned)T * Tl::kRowBytes);
    const i32x4 do_buf = make_tile_buffer((const char*)p.dO + (size_t)bh * T * Tl::kRowBytes, (unsigned)T * Tl::kRowBytes);
    ld.issue(q_buf, qt * 64, smem_addr + stage * C::kStageBytes);
    ld.issue(do_buf, qt * 64, smem_addr + stage * C::kStageBytes + Tl::kBytes);
    // (lse2, delta) of the tile's 64 queries: 512 contiguous bytes, copied like the tiles (no
    // load whose result a wave would have to wait for while the tile copies are in flight:
    // memory operations complete in order); waves 0 and 1 copy 256 bytes each
    if (wave < 2) {
      const i32x4 st_buf = make_tile_buffer(p.rowstat + (size_t)bh * T * 2, (unsigned)T * 8);
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, %3 offen lds"
                   :
                   : "s"(__builtin_amdgcn_readfirstlane((int)(smem_addr + (unsigned)(C::kLds - C::kAux) +
                                                               stage * 512 + wave * 256))),
                     "v"(lane * 4), "s"(st_buf), "s"(__builtin_amdgcn_readfirstlane(qt * 512 + wave * 256))
                   : "memory");
    }
  };

  if (n_items > 0) issue(0, 0);
  for (int item = 0; item < n_items; ++item) {
    const int stage = item & 1;
    const int qt = qt0 + item % span;
    wait_copies();
    __syncthreads();
    if (item + 1 < n_items) issue(item + 1, stage ^ 1);

    const int q0 = qt * 64;
    if (p.causal && q0 + 63 < kw0) continue;  // every query of the tile precedes this wave's keys
    // per-lane fragment bases inside this stage (Q tile; the dO tile sits Tl::kBytes after it)
    const unsigned qtile = smem_addr + stage * C::kStageBytes;
    const unsigned b_row = fa.row + qtile, b_tr = fa.tr + qtile, b_tr8 = fa.tr8 + qtile;
    const float* stat_s = aux + stage * 128;  // (lse2, delta) pairs of the tile's queries

    const int key = kw0 + l32;
    // all 64 queries exist and (when causal) none precedes any of this wave's 32 keys
    const bool all_visible = q0 + 64 <= T && (!p.causal || q0 >= kw0 + 31);
    // one 32-query block at a time: S, dP (recomputed), P and dS for this lane's key and
    // 16 queries, then dV^T += dO^T P and dK^T += Q^T dS over those 32 queries
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      f32x16 s, dp;
#pragma unroll
      for (int i = 0; i < 16; ++i) s[i] = dp[i] = 0.f;
#pragma unroll
      for (int st = 0; st < Tl::kDSteps; ++st) {
        const unsigned x = (unsigned)xor_here((int)b_row, st << 5);
        s = mfma_bf16(fa.row_frag(x, qb, 0), kf[st], s);
        dp = mfma_bf16(fa.row_frag(x, qb, Tl::kBytes), vf[st], dp);
      }
      // Order for the scheduler: LDS reads run one step (two fragments) ahead of the matrix
      // instructions that consume them, no further (the kernel has no registers to spare).
      __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
      for (int st = 0; st < Tl::kDSteps - 2; ++st) {
        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
      __builtin_amdgcn_sched_barrier(0);
      // Scores of (query, key) pairs that are not visible become -inf, i.e. weight zero.  Only
      // the diagonal tile and rows past the end have such pairs: everywhere else this block is
      // skipped (a uniform branch around the comparisons, not a second copy of the loop body).
      if (!all_visible) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int q = q0 + qb * 32 + (i >> 2) * 8 + hi * 4 + (i & 3);
          const bool vis = q < T && (!p.causal || key <= q);
          s[i] = vis ? s[i] : -INFINITY;
        }
      }
      // one 16-query half at a time: P and dS packed to bf16, then straight into the products
      // that contract over those 16 queries (keeps few temporaries alive)
#pragma unroll
      for (int hf = 0; hf < 2; ++hf) {
        float pv[8], dsv[8];
#pragma unroll
        for (int b2 = 0; b2 < 2; ++b2) {
          const int b4 = hf * 2 + b2;
          const float* st4 = stat_s + (qb * 32 + b4 * 8 + hi * 4) * 2;
          const f32x4 ld01 = *(const f32x4*)st4, ld23 = *(const f32x4*)(st4 + 4);
          const float l4[4] = {ld01[0], ld01[2], ld23[0], ld23[2]};
          const float d4[4] = {ld01[1], ld01[3], ld23[1], ld23[3]};
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int i = b4 * 4 + r;
            const float pe = fast_exp2(s[i] * c2 - l4[r]);
            pv[b2 * 4 + r] = pe;
            dsv[b2 * 4 + r] = pe * (dp[i] - d4[r]);
          }
        }
        const bf16x8 pb = pack8(pv), dsb = pack8(dsv);
#pragma unroll
        for (int db = 0; db < Tl::kDBlocks; ++db) {
          const unsigned x0 = (unsigned)xor_here((int)b_tr, db << 6), x8 = (unsigned)xor_here((int)b_tr8, db << 6);
          dv[db] = mfma_bf16(fa.tr_frag(x0, x8, qb * 2 + hf, Tl::kBytes), pb, dv[db]);
          dk[db] = mfma_bf16(fa.tr_frag(x0, x8, qb * 2 + hf, 0), dsb, dk[db]);
        }

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
    char* outb = (char*)(which ? p.dVseq : p.dKseq) + (size_t)bg * T * Tl::kRowBytes;
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
  if (own_depth && !depth_first) depth_grad_rows<D>(p, bg, kw0, lane);
  if (GT > 0 && !depth_first) group_depth();
}

// ---------------------------------------------------------------- dQ
// Workgroup = NW waves x 32 queries.  Accumulators hold dQ^T ([channel][query]: a lane owns
// one query).  Launched with NW = 4 (two workgroups per compute unit); NW = 8 (one workgroup
// per unit, a K/V tile serving twice as many queries) measured 6 % slower at B=8 H=16 T=4096.
template <int D, int NW>
__global__ __launch_bounds__(NW * 64, 2) void moda_bwd_dq_kernel(BwdParams p) {
  using Tl = Tile<D>;
  using C = BwdCfg<D, NW>;
  constexpr int kQT = NW * 32;  // queries per workgroup
  __shared__ __attribute__((aligned(1024))) unsigned char smem[C::kLds];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, hi = lane >> 5;
  const int T = p.T;
  const int n_qt = (T + kQT - 1) / kQT;
  // Ids are dealt to the dies by key/value head (see head_blocked_id): the G query heads of a
  // group stream the same K/V, so a die takes a group's heads one right after the other, query
  // tile by query tile (heavy, i.e. late, tiles first).
  const int G = p.Hq / p.Hk;
  int bg, tile_idx;  // (batch, key/value head); position in the walk over (query tile, head of the group)
  head_blocked_id((int)blockIdx.x, p.B * p.Hk, n_qt * G, bg, tile_idx, p.head_group);
  const int qt = n_qt - 1 - tile_idx / G;
  const int bh = (bg / p.Hk) * p.Hq + (bg % p.Hk) * G + tile_idx % G;
  const int q0 = qt * kQT;
  const int qw0 = q0 + wave * 32;

  const char* Qb = (const char*)p.Q + (size_t)bh * T * Tl::kRowBytes;
  const char* Kb = (const char*)p.Kseq + (size_t)bg * T * Tl::kRowBytes;
  const char* Vb = (const char*)p.Vseq + (size_t)bg * T * Tl::kRowBytes;
  const char* dOb = (const char*)p.dO + (size_t)bh * T * Tl::kRowBytes;
  const float* statb = p.rowstat + (size_t)bh * T * 2;  // (LSE * log2(e), delta) per row

  const int qi = qw0 + l32;
  const int qrow = min(qi, T - 1);

  const float c2 = p.scale_log2;
  unsigned char* xw = smem + wave * C::kXWave;  // this wave's fp32 exchange buffer (overlaps the ring)
  constexpr int LPR = Tl::kChunks, RPS = 64 / LPR, NIT = 32 / RPS;
  const int La = p.depth_alloc;

  // The depth-slot gradients and the depth share of dQ were computed before this kernel (by
  // the dK/dV kernel, or by the depth_gqa kernels with grouped queries); the share is in the
  // workspace, in fp32, not yet multiplied by the softmax scale.
  f32x16 dq[Tl::kDBlocks];
  if (La > 0) {
    const float* src = p.dq_depth + ((size_t)bh * T + qrow) * D;
#pragma unroll
    for (int db = 0; db < Tl::kDBlocks; ++db)
#pragma unroll
      for (int bq = 0; bq < 4; ++bq) {
        const f32x4 v = *(const f32x4*)(src + db * 32 + bq * 8 + hi * 4);
        dq[db][4 * bq] = v[0]; dq[db][4 * bq + 1] = v[1];
        dq[db][4 * bq + 2] = v[2]; dq[db][4 * bq + 3] = v[3];
      }
  } else {
#pragma unroll
    for (int db = 0; db < Tl::kDBlocks; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) dq[db][i] = 0.f;
  }

  // resident Q and dO fragments of this wave's 32 queries (MFMA B operands)
  bf16x8 qf[Tl::kDSteps], dof[Tl::kDSteps];
#pragma unroll
  for (int st = 0; st < Tl::kDSteps; ++st) {
    qf[st] = *(const bf16x8*)(Qb + (size_t)qrow * Tl::kRowBytes + st * 32 + hi * 16);
    dof[st] = *(const bf16x8*)(dOb + (size_t)qrow * Tl::kRowBytes + st * 32 + hi * 16);
  }
  const f32x2 stat = *(const f32x2*)(statb + 2 * qrow);
  const float lse2 = stat[0], delta = stat[1];

  const int n_keys = p.causal ? min(T, q0 + kQT) : T;
  const int nt = (n_keys + 63) / 64;
  const int wave_last = p.causal ? min(nt - 1, (qw0 + 31) / 64) : nt - 1;
  const int lim = p.causal ? min(qi, T - 1) : T - 1;  // last visible key of this lane's query
  const unsigned smem_addr = (unsigned)(size_t)(lds_ptr)smem;
  TileLoader<D, NW> ld;
  ld.init(wave, lane);
  FragAddr<D> fa;
  fa.init(lane);
  const i32x4 k_buf = make_tile_buffer(Kb, (unsigned)T * Tl::kRowBytes);
  const i32x4 v_buf = make_tile_buffer(Vb, (unsigned)T * Tl::kRowBytes);
  auto issue = [&](int kt, int stage) {
    ld.issue(k_buf, kt * 64, smem_addr + stage * C::kStageBytes);
    ld.issue(v_buf, kt * 64, smem_addr + stage * C::kStageBytes + Tl::kBytes);
  };

  // One key tile: S^T, dP^T, dS^T and dQ^T += K^T dS^T for this wave's 32 queries.
  auto tile = [&](int kt, int stage) {
    // per-lane fragment bases inside this stage (K tile; the V tile sits Tl::kBytes after it)
    const unsigned ktile = smem_addr + stage * C::kStageBytes;
    const unsigned b_row = fa.row + ktile, b_tr = fa.tr + ktile, b_tr8 = fa.tr8 + ktile;

    f32x16 s[2], dp[2];  // S^T, dP^T: [key block]; a lane holds 16 keys of its query
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i) s[kb][i] = dp[kb][i] = 0.f;
    // four independent accumulation chains per channel step
#pragma unroll
    for (int st = 0; st < Tl::kDSteps; ++st) {
      const unsigned x = (unsigned)xor_here((int)b_row, st << 5);
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        s[kb] = mfma_bf16(fa.row_frag(x, kb, 0), qf[st], s[kb]);
        dp[kb] = mfma_bf16(fa.row_frag(x, kb, Tl::kBytes), dof[st], dp[kb]);
      }
    }
    // Order for the scheduler: the LDS reads run one channel step (four fragments) ahead of the
    // matrix instructions that consume them.
    __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
    for (int st = 0; st < Tl::kDSteps - 1; ++st) {
      __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
    __builtin_amdgcn_sched_barrier(0);

    bf16x8 dsb[2][2];
    const int k0 = kt * 64;
    // every key of the tile exists and is visible to every query of the wave
    const bool all_visible = k0 + 64 <= T && (!p.causal || k0 + 63 <= qw0);
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      float dsv[16];
      if (!all_visible) {  // (uniform) diagonal tile, keys past the end: invisible pairs get weight zero
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int key = k0 + kb * 32 + (i >> 2) * 8 + hi * 4 + (i & 3);
          s[kb][i] = key <= lim ? s[kb][i] : -INFINITY;
        }
      }
#pragma unroll
      for (int i = 0; i < 16; ++i) dsv[i] = fast_exp2(s[kb][i] * c2 - lse2) * (dp[kb][i] - delta);
#pragma unroll
      for (int hf = 0; hf < 2; ++hf) {
        float a[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) a[k] = dsv[hf * 8 + k];
        dsb[kb][hf] = pack8(a);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    // dQ^T += K^T dS^T  (contraction over the tile's 64 keys); transposed fragments two
    // matrix instructions ahead
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
#pragma unroll
      for (int db = 0; db < Tl::kDBlocks; ++db)
        dq[db] = mfma_bf16(fa.tr_frag((unsigned)xor_here((int)b_tr, db << 6), (unsigned)xor_here((int)b_tr8, db << 6), ks, 0),
                           dsb[ks >> 1][ks & 1], dq[db]);
    constexpr int NM = 4 * Tl::kDBlocks;
    __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
    for (int m = 0; m < NM - 2; ++m) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
    __builtin_amdgcn_sched_barrier(0);
  };

  // Every wave takes part in the copies and barriers of all nt tiles, but computes only on the
  // tiles its queries see: first those (no branch around the products inside the loop, which
  // made the compiler copy the accumulators from one register block to another every tile),
  // then the rest.
  issue(0, 0);
  int kt = 0;
  for (; kt <= wave_last; ++kt) {
    const int stage = kt & 1;
    wait_copies();
    __syncthreads();
    if (kt + 1 < nt) issue(kt + 1, stage ^ 1);
    tile(kt, stage);
  }
  for (; kt < nt; ++kt) {
    wait_copies();
    __syncthreads();
    if (kt + 1 < nt) issue(kt + 1, (kt & 1) ^ 1);
  }
  __syncthreads();

  // ---- epilogue: accumulator layout -> row-major; depth slots (unless taken first); stores
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
  {
    const int rg = lane / LPR, l16 = lane % LPR;
    char* dQb = (char*)p.dQ + (size_t)bh * T * Tl::kRowBytes;
    for (int it = 0; it < NIT; ++it) {
      const int row = it * RPS + rg, t = qw0 + row;
      const f32x4 a0 = *(const f32x4*)(xw + row * C::kXRow + l16 * 32);
      const f32x4 a1 = *(const f32x4*)(xw + row * C::kXRow + l16 * 32 + 16);
      if (t < T) {
        const float f = p.scale;
        u32x4 ov = {pack_bf16(a0[0] * f, a0[1] * f), pack_bf16(a0[2] * f, a0[3] * f),
                    pack_bf16(a1[0] * f, a1[1] * f), pack_bf16(a1[2] * f, a1[3] * f)};
        *(u32x4*)(dQb + (size_t)t * Tl::kRowBytes + l16 * 16) = ov;
      }
    }
  }
}

// ---------------------------------------------------------------- depth-slot gradients of a large group, matrix pipe
// Groups of more than 8 query heads (8 < G <= 64; the G * T rows of Q of a group must fit 32-bit
// byte offsets, else the call is rejected as unsupported).
// With that many heads per position the depth-slot gradients of ONE position are small dense
// products (the paper's group-aware depth calculation, here for the backward):
//   S  = Q_p Kd_p^T   [G x L]    dP = dO_p Vd_p^T
//   P  = exp2(S c2 - lse2_h),    E  = P (dP - delta_h)
//   dVd_p = P^T dO_p  [L x d],   dKd_p = scale E^T Q_p,   dQ_p (depth share) = E Kd_p  [G x d]
// One workgroup of ONE wave per (batch, key/value head, position).  The G heads' Q and dO rows
// of the position (rows of different heads, gathered) and 64 slots at a time of Kd_p, Vd_p are
// copied global -> LDS into four 64-row tiles of the layout the other backward kernels use;
// the score products are formed in both orientations (slots x heads for the product that
// contracts over slots, heads x slots for the two that contract over heads), exactly as the
// dK/dV and dQ kernels do for sequence keys.  Rows of the tiles beyond G heads / beyond
// depth_count slots are filled with zeros by the bounds-checked copies (unattended slots are
// never fetched) and get weight zero.  Sums in fp32 on the matrix pipe, one rounding per
// gradient element.  Several such workgroups share a compute unit (32 KB of LDS each at d = 64),
// which is what hides the latency of the copies.
template <int D, int NG>
__global__ __launch_bounds__(64) void moda_bwd_depth_group_kernel(BwdParams p) {
  using Tl = Tile<D>;
  constexpr int RB = D * 2;
  constexpr int kRowsPerInst = 1024 / RB;       // rows one copy instruction moves
  constexpr int kInst = 64 / kRowsPerInst;      // copy instructions per tile
  constexpr int kStatOff = 4 * Tl::kBytes;      // (lse2, delta) per head row, after the four tiles
  __shared__ __attribute__((aligned(1024))) unsigned char smem[4 * Tl::kBytes + 64 * 8];
  const int lane = threadIdx.x, l32 = lane & 31, hi = lane >> 5;
  const int T = p.T, L = p.depth_count, La = p.depth_alloc, G = p.Hq / p.Hk;
  const long long row = blockIdx.x;  // (b * Hk + g) * T + t
  const int t = (int)(row % T);
  const int bg = (int)(row / T);
  const int bh0 = (bg / p.Hk) * p.Hq + (bg % p.Hk) * G;
  const float c2 = p.scale_log2;
  const unsigned smem_addr = (unsigned)(size_t)(lds_ptr)smem;
  const unsigned q_tile = smem_addr, g_tile = smem_addr + Tl::kBytes, k_tile = smem_addr + 2 * Tl::kBytes,
                 v_tile = smem_addr + 3 * Tl::kBytes;
  float* stat = (float*)(smem + kStatOff);
  FragAddr<D> fa;
  fa.init(lane);

  // ---- the heads' rows of this position: row h of the tile = head h of the group
  const int j = lane / Tl::kChunks, pc = lane % Tl::kChunks;  // this lane's row in a piece, chunk position
  {
    const size_t base = ((size_t)bh0 * T + t) * RB;
    const unsigned bytes = (unsigned)(((size_t)(G - 1) * T + 1) * RB);  // (< 0xffffff00, below the offset that stands for "no row": checked by the host)
    const i32x4 q_buf = make_tile_buffer((const char*)p.Q + base, bytes);
    const i32x4 g_buf = make_tile_buffer((const char*)p.dO + base, bytes);
#pragma unroll
    for (int q = 0; q < kInst; ++q) {
      const int h = q * kRowsPerInst + j;
      const int c = pc ^ Tl::swz(h);
      const int voff = h < G ? (int)((unsigned)h * (unsigned)T * (unsigned)RB + (unsigned)c * 16u) : (int)0xffffff80u;
      tile_copy16(q_buf, voff, 0, q_tile + q * 1024);
      tile_copy16(g_buf, voff, 0, g_tile + q * 1024);
    }
    // heads past the group get lse2 = +inf: weight zero
    const int h = lane;
    f32x2 st = {INFINITY, 0.f};
    if (h < G) st = *(const f32x2*)(p.rowstat + ((size_t)(bh0 + h) * T + t) * 2);
    *(f32x2*)(stat + 2 * h) = st;
  }
  f32x16 dqa[NG][Tl::kDBlocks];  // dQ^T (depth share): [head block][channel block], lane = head
#pragma unroll
  for (int hb = 0; hb < NG; ++hb)
#pragma unroll
    for (int cb = 0; cb < Tl::kDBlocks; ++cb)
#pragma unroll
      for (int i = 0; i < 16; ++i) dqa[hb][cb][i] = 0.f;

  const size_t drow = (size_t)La * RB;
  const char* kd = (const char*)p.Kdepth + (size_t)row * drow;
  const char* vd = (const char*)p.Vdepth + (size_t)row * drow;
  char* dkd = (char*)p.dKdepth + (size_t)row * drow;
  char* dvd = (char*)p.dVdepth + (size_t)row * drow;

  for (int c0 = 0; c0 < L; c0 += 64) {
    // ---- 64 slots of this position (rows past depth_count: zeros)
    __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): the fragment reads of the chunk before are complete
    __builtin_amdgcn_wave_barrier();
    {
      const unsigned bytes = (unsigned)(min(64, L - c0) * RB);
      const i32x4 k_buf = make_tile_buffer(kd + (size_t)c0 * RB, bytes);
      const i32x4 v_buf = make_tile_buffer(vd + (size_t)c0 * RB, bytes);
#pragma unroll
      for (int q = 0; q < kInst; ++q) {
        const int r = q * kRowsPerInst + j;
        const int voff = r * RB + ((pc ^ Tl::swz(r)) << 4);
        tile_copy16(k_buf, voff, 0, k_tile + q * 1024);
        tile_copy16(v_buf, voff, 0, v_tile + q * 1024);
      }
    }
    wait_copies();
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const unsigned bq_row = fa.row + q_tile, bq_tr = fa.tr + q_tile, bq_tr8 = fa.tr8 + q_tile;
    const unsigned bk_row = fa.row + k_tile, bk_tr = fa.tr + k_tile, bk_tr8 = fa.tr8 + k_tile;
    constexpr int kGOff = Tl::kBytes;  // the dO tile follows the Q tile, the Vd tile the Kd tile

#pragma unroll
    for (int sb = 0; sb < 2; ++sb) {
      if (c0 + sb * 32 >= L) break;  // (uniform) no attended slot in this block
      // dVd^T, dKd^T of the block's 32 slots: [channel block], lane = slot
      f32x16 dva[Tl::kDBlocks], dka[Tl::kDBlocks];
#pragma unroll
      for (int cb = 0; cb < Tl::kDBlocks; ++cb)
#pragma unroll
        for (int i = 0; i < 16; ++i) dva[cb][i] = dka[cb][i] = 0.f;
#pragma unroll
      for (int hb = 0; hb < NG; ++hb) {
        if (hb * 32 >= G) break;  // (uniform)
        // ---- slots x heads: S^T, dP^T (lane = head, registers = slots) -> E^T -> dQ^T += Kd^T E^T
        {
          f32x16 s, dp;
#pragma unroll
          for (int i = 0; i < 16; ++i) s[i] = dp[i] = 0.f;
#pragma unroll
          for (int st = 0; st < Tl::kDSteps; ++st) {
            const unsigned xk = (unsigned)xor_here((int)bk_row, st << 5), xq = (unsigned)xor_here((int)bq_row, st << 5);
            s = mfma_bf16(FragAddr<D>::row_frag(xk, sb, 0), FragAddr<D>::row_frag(xq, hb, 0), s);
            dp = mfma_bf16(FragAddr<D>::row_frag(xk, sb, kGOff), FragAddr<D>::row_frag(xq, hb, kGOff), dp);
          }
          const f32x2 st_h = *(const f32x2*)(stat + 2 * (hb * 32 + l32));  // this lane's head
          float ev[16];
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int slot = c0 + sb * 32 + (i >> 2) * 8 + hi * 4 + (i & 3);
            const float pe = slot < L ? fast_exp2(s[i] * c2 - st_h[0]) : 0.f;
            ev[i] = pe * (dp[i] - st_h[1]);
          }
#pragma unroll
          for (int hf = 0; hf < 2; ++hf) {
            float a8[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) a8[k] = ev[hf * 8 + k];
            const bf16x8 eb = pack8(a8);
#pragma unroll
            for (int cb = 0; cb < Tl::kDBlocks; ++cb)
              dqa[hb][cb] = mfma_bf16(FragAddr<D>::tr_frag((unsigned)xor_here((int)bk_tr, cb << 6),
                                                           (unsigned)xor_here((int)bk_tr8, cb << 6), sb * 2 + hf, 0),
                                      eb, dqa[hb][cb]);
          }
        }
        // ---- heads x slots: S, dP (lane = slot, registers = heads) -> P, E -> dVd^T += dO^T P, dKd^T += Q^T E
        {
          f32x16 s, dp;
#pragma unroll
          for (int i = 0; i < 16; ++i) s[i] = dp[i] = 0.f;
#pragma unroll
          for (int st = 0; st < Tl::kDSteps; ++st) {
            const unsigned xk = (unsigned)xor_here((int)bk_row, st << 5), xq = (unsigned)xor_here((int)bq_row, st << 5);
            s = mfma_bf16(FragAddr<D>::row_frag(xq, hb, 0), FragAddr<D>::row_frag(xk, sb, 0), s);
            dp = mfma_bf16(FragAddr<D>::row_frag(xq, hb, kGOff), FragAddr<D>::row_frag(xk, sb, kGOff), dp);
          }
          const bool live = c0 + sb * 32 + l32 < L;  // this lane's slot is attended
#pragma unroll
          for (int hf = 0; hf < 2; ++hf) {
            float pv[8], evv[8];
#pragma unroll
            for (int b2 = 0; b2 < 2; ++b2) {
              const int b4 = hf * 2 + b2;
              const float* st4 = stat + (hb * 32 + b4 * 8 + hi * 4) * 2;
              const f32x4 ld01 = *(const f32x4*)st4, ld23 = *(const f32x4*)(st4 + 4);
              const float l4[4] = {ld01[0], ld01[2], ld23[0], ld23[2]};
              const float d4[4] = {ld01[1], ld01[3], ld23[1], ld23[3]};
#pragma unroll
              for (int r = 0; r < 4; ++r) {
                const int i = b4 * 4 + r;
                const float pe = live ? fast_exp2(s[i] * c2 - l4[r]) : 0.f;
                pv[b2 * 4 + r] = pe;
                evv[b2 * 4 + r] = pe * (dp[i] - d4[r]);
              }
            }
            const bf16x8 pb = pack8(pv), eb = pack8(evv);
#pragma unroll
            for (int cb = 0; cb < Tl::kDBlocks; ++cb) {
              const unsigned x0 = (unsigned)xor_here((int)bq_tr, cb << 6), x8 = (unsigned)xor_here((int)bq_tr8, cb << 6);
              dva[cb] = mfma_bf16(FragAddr<D>::tr_frag(x0, x8, hb * 2 + hf, kGOff), pb, dva[cb]);
              dka[cb] = mfma_bf16(FragAddr<D>::tr_frag(x0, x8, hb * 2 + hf, 0), eb, dka[cb]);
            }
          }
        }
      }
      // ---- store the block's dVdepth, dKdepth rows: lane = slot, 4 consecutive channels (8 bytes) at a time
      const int slot = c0 + sb * 32 + l32;
      if (slot < L) {
        const float f = p.scale;
#pragma unroll
        for (int cb = 0; cb < Tl::kDBlocks; ++cb)
#pragma unroll
          for (int bq = 0; bq < 4; ++bq) {
            const size_t off = (size_t)slot * RB + (cb * 32 + bq * 8 + hi * 4) * 2;
            *(u32x2*)(dvd + off) = (u32x2){pack_bf16(dva[cb][4 * bq], dva[cb][4 * bq + 1]),
                                           pack_bf16(dva[cb][4 * bq + 2], dva[cb][4 * bq + 3])};
            *(u32x2*)(dkd + off) = (u32x2){pack_bf16(dka[cb][4 * bq] * f, dka[cb][4 * bq + 1] * f),
                                           pack_bf16(dka[cb][4 * bq + 2] * f, dka[cb][4 * bq + 3] * f)};
          }
      }
    }
  }
  // allocated but unattended slots get zero gradients
  for (int i = L * (RB / 16) + lane; i < La * (RB / 16); i += 64) {
    *(u32x4*)(dvd + (size_t)i * 16) = (u32x4){0u, 0u, 0u, 0u};
    *(u32x4*)(dkd + (size_t)i * 16) = (u32x4){0u, 0u, 0u, 0u};
  }
  // the heads' depth share of dQ: lane = head, 4 consecutive channels (16 bytes of fp32) at a time
#pragma unroll
  for (int hb = 0; hb < NG; ++hb) {
    const int h = hb * 32 + l32;
    if (h < G) {
      float* dst = p.dq_depth + ((size_t)(bh0 + h) * T + t) * D;
#pragma unroll
      for (int cb = 0; cb < Tl::kDBlocks; ++cb)
#pragma unroll
        for (int bq = 0; bq < 4; ++bq)
          *(f32x4*)(dst + cb * 32 + bq * 8 + hi * 4) =
              (f32x4){dqa[hb][cb][4 * bq], dqa[hb][cb][4 * bq + 1], dqa[hb][cb][4 * bq + 2], dqa[hb][cb][4 * bq + 3]};
    }
  }
}

// ---------------------------------------------------------------- launchers
// Workspace: (LSE log2 e, delta) per query row, then - when there are depth slots - the depth
// share of dQ in fp32, [B, Hq, T, d].
static size_t rowstat_bytes(const BwdParams& p) {
  return (((size_t)p.B * p.Hq * p.T * 2 * sizeof(float)) + 255) / 256 * 256;
}
size_t bwd_bf16_workspace_bytes(const BwdParams& p, int d) {
  return rowstat_bytes(p) + (p.depth_alloc > 0 ? (size_t)p.B * p.Hq * p.T * d * sizeof(float) : 0);
}

int bwd_bf16_max_group() { return 64; }

int bwd_bf16_kernels(const BwdParams& p) { return 3 + ((p.Hq / p.Hk > 4 && p.depth_alloc > 0) ? 1 : 0); }

template <int D>
static hipError_t launch_bwd_bf16_d(BwdParams p, hipStream_t stream) {
  const long long rows = (long long)p.B * p.Hq * p.T;
  const int G = p.Hq / p.Hk;
  const long long g_delta = (rows * (D / 8) + 255) / 256;
  const long long n_kt = (p.T + 127) / 128;
  const long long g_dkdv = (long long)p.B * p.Hk * n_kt;
  constexpr int kDqWaves = 4;
  const long long g_dq = (long long)p.B * p.Hq * ((p.T + kDqWaves * 32 - 1) / (kDqWaves * 32));
  const long long kv_rows = (long long)p.B * p.Hk * p.T;
  const long long g_depth = (kv_rows * (D / 8) + 255) / 256;  // 5 <= G <= 8: 256 / (d/8) positions per workgroup
  const long long g_wide = kv_rows;                            // G > 8: one workgroup (of one wave) per position
  // every grid is checked before the first kernel is enqueued
  if (!grid_ok(g_delta) || !grid_ok(g_dkdv) || !grid_ok(g_dq) || !grid_ok(g_depth) || !grid_ok(g_wide))
    return kGridTooLarge;
  if (G > bwd_bf16_max_group()) return hipErrorInvalidValue;
  // the group kernel gathers the G heads' rows of a position with 32-bit offsets from the first head
  if (G > 8 && p.depth_alloc > 0 && (unsigned long long)G * p.T * (D * 2) >= 0xffffff00ull) return kGridTooLarge;
  p.dq_depth = (float*)((char*)p.rowstat + rowstat_bytes(p));
  hipError_t e = launch_kernel(moda_bwd_delta_kernel<D>, dim3((unsigned)g_delta), dim3(256), stream, p.dO, p.O, p.LSE,
                               p.rowstat, rows);
  if (e != hipSuccess) return e;
  if (G > 4 && p.depth_alloc > 0) {
    if (G <= 8) {
      e = launch_kernel(moda_bwd_depth_gqa_kernel<D, 8>, dim3((unsigned)g_depth), dim3(256), stream, p);
    } else {
      // large groups: one wave per position, the group's products on the matrix pipe
      const dim3 gw((unsigned)g_wide);
      if (G <= 32) e = launch_kernel(moda_bwd_depth_group_kernel<D, 1>, gw, dim3(64), stream, p);
      else e = launch_kernel(moda_bwd_depth_group_kernel<D, 2>, gw, dim3(64), stream, p);
    }
    if (e != hipSuccess) return e;
  }
  {
    const dim3 gk((unsigned)g_dkdv), blk(256);
    const bool grouped = G > 1 && G <= 4 && p.depth_alloc > 0;  // the depth-slot gradients of the group run inside dK/dV
    if (!grouped) e = launch_kernel(moda_bwd_dkdv_kernel<D, 0>, gk, blk, stream, p);
    else if (G <= 2) e = launch_kernel(moda_bwd_dkdv_kernel<D, 2>, gk, blk, stream, p);
    else e = launch_kernel(moda_bwd_dkdv_kernel<D, 4>, gk, blk, stream, p);
  }
  if (e != hipSuccess) return e;
  return launch_kernel(moda_bwd_dq_kernel<D, kDqWaves>, dim3((unsigned)g_dq), dim3(kDqWaves * 64), stream, p);
}

hipError_t launch_bwd_bf16(const BwdParams& p, int d, hipStream_t stream) {
  if (d == 128) return launch_bwd_bf16_d<128>(p, stream);
  if (d == 64) return launch_bwd_bf16_d<64>(p, stream);
  return hipErrorInvalidValue;
}

}  // namespace moda
