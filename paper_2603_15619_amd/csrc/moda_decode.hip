// MoDA attention for ONE new token per sequence (decoding; paper Table 1, "Decoding" rows).
// The new token's query attends the T positions of the sequence K/V cache (its own K/V
// included) and the depth slots of its own position, under one softmax (section 2.2); the
// depth cache of a decoding step is therefore only [B, Hk, depth_alloc, d].
//
// The call is bound by reading the sequence cache once (2 * B * Hk * T * d elements), so the
// keys are split over workgroups (one workgroup = one (batch, key/value head, slice of the
// sequence), all G query heads of the group together, so the slice is read once):
//   partial: per slice and head the running (max, normaliser, weighted value sum) in fp32,
//            written to the workspace; the depth slots of the new token's position are one
//            more slice (the last one), read from the depth cache instead of the sequence cache;
//   merge  : per (batch, query head): folds the slices into one softmax, normalises, stores
//            O and LSE.
// Two forms of the partial kernel.  One query head per key/value head: vector ALUs only (one
// query row: no matrix shape to speak of); a lane owns 8 channels, d/8 lanes a key row,
// 64 / (d/8) key rows per wave instruction.  Grouped queries: the G heads of a group are the
// columns of small matrix products (keys x heads), see moda_decode_partial_mfma_kernel.
#include <atomic>

#include "moda_launch.h"
#include "moda_tile.h"

namespace moda {

constexpr int kDecWaves = 4;

// Scratch of the entry point that allocates nothing (moda_attn_decode_noalloc): the partial
// results of the slices, which the caller's workspace holds otherwise.  One copy per GPU, held
// until the process ends.  In host code this name is only a handle for hipGetSymbolAddress:
// kernels get the device address that call returns, never the name.
constexpr size_t kDecodeScratchBytes = 8u << 20;
static __device__ __align__(256) unsigned char scratch[kDecodeScratchBytes];

constexpr int kMaxDevices = 64;
static std::atomic<void*> g_scratch_addr[kMaxDevices];  // device address of `scratch`, per device (0: not looked up yet)

size_t decode_static_scratch_bytes() { return kDecodeScratchBytes; }

// Device address of `scratch` on the CURRENT device: looked up once per device (on the first
// call made with that device current), then served from the table.
hipError_t decode_static_scratch(void** addr) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  void* p = g_scratch_addr[dev].load(std::memory_order_acquire);
  if (!p) {
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_addr[dev].store(p, std::memory_order_release);  // (two threads racing here store the same address)
  }
  *addr = p;
  return hipSuccess;
}

struct DecodeParams {
  const void* Q;       // [B, Hq, d]
  const void* Kseq;    // [B, Hk, T_alloc, d]
  const void* Vseq;
  const void* Kdepth;  // [B, Hk, depth_alloc, d]
  const void* Vdepth;
  void* O;             // [B, Hq, d]
  float* LSE;          // [B, Hq]
  float* ws;           // [B, Hq, n_slices, d + 2]
  int B, Hq, Hk, T, T_alloc;
  int depth_alloc, depth_count;
  int n_split, keys_per_split;  // slices of the sequence
  int n_slices;                 // n_split, plus one for the depth slots when there are any
  float scale, scale_log2;
};

template <int D, int GT>
__global__ __launch_bounds__(kDecWaves * 64) void moda_decode_partial_kernel(DecodeParams p) {
  constexpr int LPR = D / 8, RPS = 64 / LPR, RB = D * 2;
  __shared__ float red[kDecWaves][RPS][GT][D + 2];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int rg = lane / LPR, l16 = lane % LPR;
  const int G = p.Hq / p.Hk;
  const int n_gc = (G + GT - 1) / GT;  // head chunks per group
  int id = blockIdx.x;
  const int split = id % p.n_slices;
  id /= p.n_slices;
  const int gc = id % n_gc;
  const int bg = id / n_gc;  // (batch, key/value head)
  const int b = bg / p.Hk, g = bg - b * p.Hk;
  const int h0 = g * G + gc * GT;  // first query head of this chunk
  const float c2 = p.scale_log2;

  u32x4 q[GT];
  float m[GT], l[GT], o[GT][8];
#pragma unroll
  for (int j = 0; j < GT; ++j) {
    const int h = min(h0 + j, g * G + G - 1);  // heads past the group repeat the last one; never stored
    q[j] = *(const u32x4*)((const char*)p.Q + ((size_t)b * p.Hq + h) * RB + l16 * 16);
    m[j] = -INFINITY;
    l[j] = 0.f;
#pragma unroll
    for (int k = 0; k < 8; ++k) o[j][k] = 0.f;
  }
  // rows [k_begin, k_end) of the sequence cache, or (last slice) the depth slots of the position
  const bool is_depth = split == p.n_split;
  const int k_begin = is_depth ? 0 : split * p.keys_per_split;
  const int k_end = is_depth ? p.depth_count : min(p.T, k_begin + p.keys_per_split);
  const int k_last = k_end - 1;
  const size_t slab = is_depth ? (size_t)bg * p.depth_alloc * RB : (size_t)bg * p.T_alloc * RB;
  const char* Kb = (const char*)(is_depth ? p.Kdepth : p.Kseq) + slab + l16 * 16;
  const char* Vb = (const char*)(is_depth ? p.Vdepth : p.Vseq) + slab + l16 * 16;

  // this lane's keys: k_begin + (wave * RPS + rg) + i * (kDecWaves * RPS), kU at a time with the
  // next kU in flight; the running max is raised (and the state rescaled) once per kU keys
  constexpr int STEP = kDecWaves * RPS;
  constexpr int kU = 4;
  const int key0 = k_begin + wave * RPS + rg;
  auto load = [&](const char* base, int kk) {
    return __builtin_nontemporal_load((const u32x4*)(base + (size_t)min(kk, k_last) * RB));
  };
  u32x4 kn[kU], vn[kU];
#pragma unroll
  for (int u = 0; u < kU; ++u) {
    kn[u] = load(Kb, key0 + u * STEP);
    vn[u] = load(Vb, key0 + u * STEP);
  }
  for (int base = k_begin; base < k_end; base += kU * STEP) {  // uniform trip count over the workgroup
    const int key = key0 + (base - k_begin);
    u32x4 kv[kU], vv[kU];
#pragma unroll
    for (int u = 0; u < kU; ++u) {
      kv[u] = kn[u];
      vv[u] = vn[u];
    }
#pragma unroll
    for (int u = 0; u < kU; ++u) {
      kn[u] = load(Kb, key + (kU + u) * STEP);
      vn[u] = load(Vb, key + (kU + u) * STEP);
    }
#pragma unroll
    for (int j = 0; j < GT; ++j) {
      float sc[kU];
      float mn = m[j];
#pragma unroll
      for (int u = 0; u < kU; ++u) {
        float a = 0.f;
#pragma unroll
        for (int k = 0; k < 4; ++k) a = dot2_bf16(q[j][k], kv[u][k], a);
        a = group_sum<LPR>(a);
        sc[u] = key + u * STEP < k_end ? a : -INFINITY;
        mn = fmaxf(mn, sc[u]);
      }
      // (mn is -inf only while every key so far was past the slice: then nothing is added)
      const bool none = mn == -INFINITY;
      const float al = none ? 0.f : fast_exp2((m[j] - mn) * c2);
      m[j] = mn;
      l[j] *= al;
#pragma unroll
      for (int k = 0; k < 8; ++k) o[j][k] *= al;
#pragma unroll
      for (int u = 0; u < kU; ++u) {
        const float pw = none ? 0.f : fast_exp2((sc[u] - mn) * c2);
        l[j] += pw;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          o[j][2 * k] += pw * bf16_lo(vv[u][k]);
          o[j][2 * k + 1] += pw * bf16_hi(vv[u][k]);
        }
      }
    }
  }

  // ---- combine the (kDecWaves * RPS) row groups of the workgroup, per head
#pragma unroll
  for (int j = 0; j < GT; ++j) {
#pragma unroll
    for (int k = 0; k < 8; ++k) red[wave][rg][j][l16 * 8 + k] = o[j][k];
    if (l16 == 0) {
      red[wave][rg][j][D] = m[j];
      red[wave][rg][j][D + 1] = l[j];
    }
  }
  __syncthreads();
  // thread t < GT * D: head j = t / D, channel t % D
  for (int t = tid; t < GT * D; t += kDecWaves * 64) {
    const int j = t / D, ch = t % D;
    if (h0 + j >= g * G + G) continue;
    float mm = -INFINITY;
    for (int w = 0; w < kDecWaves; ++w)
      for (int r = 0; r < RPS; ++r) mm = fmaxf(mm, red[w][r][j][D]);
    float ll = 0.f, oo = 0.f;
    for (int w = 0; w < kDecWaves; ++w)
      for (int r = 0; r < RPS; ++r) {
        const float mi = red[w][r][j][D];
        const float f = mi == -INFINITY ? 0.f : fast_exp2((mi - mm) * c2);
        ll += f * red[w][r][j][D + 1];
        oo += f * red[w][r][j][ch];
      }
    float* dst = p.ws + (((size_t)b * p.Hq + h0 + j) * p.n_slices + split) * (D + 2);
    dst[ch] = oo;
    if (ch == 0) {
      dst[D] = mm;
      dst[D + 1] = ll;
    }
  }
}

// ---------------------------------------------------------------- grouped queries: slices on the matrix pipe
// With G query heads per key/value head the arithmetic per key row grows G-fold on the vector
// ALUs and bounds the kernel well below the memory rate.  Here the (up to 32) heads of a group
// are the columns of matrix products: per block of 32 keys
//     S^T = K Q^T  (keys x heads),   O^T += V^T P^T  (channels x heads),
// so a lane owns ONE head (column) with 16 of the block's scores in registers: the running
// max / normaliser are per-lane scalars (two lanes per head, combined once at the end) and
// P^T is the second product's B operand straight from the accumulators.  Columns past the
// group hold zero queries and are never stored.
// A workgroup of 4 waves = (batch, key/value head, chunk of 32 heads, 4 consecutive slices):
// every WAVE takes a slice of its own and writes its own partial result; the workgroup only
// shares the Q tile.  A wave walks its slice 32 keys at a time with the K and V rows of the
// next block(s) in flight in registers (fully coalesced, bounds-checked raw-buffer loads:
// rows past the slice read as zeros and fetch nothing).  A block's K and V rows are
// written to the wave's two LDS tiles (the layout the backward kernels use) and read back as
// row fragments (K) and transposed fragments (V).
// Output: the same per-slice partial results as the kernel above.
constexpr int kDecMWaves = 4;   // waves (= slices) per workgroup
constexpr int kDecBlock = 32;   // keys per block
// Measured choices: d = 64: two blocks (8 KB each) in flight per wave and three waves per SIMD
// (146 registers); d = 128: one block (16 KB) and two waves per SIMD.  More waves beat deeper
// prefetch: a block's chain LDS write -> fragment reads -> matrix products -> exponentials ->
// matrix products has little to overlap within one wave.
constexpr int dec_blocks_in_flight(int d) { return d == 64 ? 2 : 1; }
constexpr int dec_waves_per_simd(int d) { return d == 64 ? 3 : 2; }

template <int D>
__global__ __launch_bounds__(kDecMWaves * 64) __attribute__((amdgpu_waves_per_eu(dec_waves_per_simd(D), dec_waves_per_simd(D))))
void moda_decode_partial_mfma_kernel(DecodeParams p) {
  using Tl = Tile<D>;
  constexpr int RB = D * 2;
  constexpr int kSteps = Tl::kDSteps;               // matrix instructions per score block
  constexpr int NB = kDecBlock / 32;                // sub-blocks of 32 keys
  constexpr int kRowsPerInst = 1024 / RB;           // rows one load instruction covers
  constexpr int kInst = kDecBlock / kRowsPerInst;   // load instructions per block of K or V
  constexpr int kHalf = kDecBlock * RB;             // bytes of a block of K or V
  constexpr int kQBytes = 32 * RB;
  constexpr int kPF = dec_blocks_in_flight(D);                            // blocks in flight
  // [Q tile: 32 heads][per wave: K tile, V tile of kDecBlock rows]
  __shared__ __attribute__((aligned(1024))) unsigned char smem[kQBytes + 2 * kDecMWaves * kHalf];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, hi = lane >> 5;
  const int G = p.Hq / p.Hk;
  const int n_gc = (G + 31) / 32;
  const int n_sg = (p.n_slices + kDecMWaves - 1) / kDecMWaves;  // slice groups
  int id = blockIdx.x;
  const int sg = id % n_sg;
  id /= n_sg;
  const int gc = id % n_gc;
  const int bg = id / n_gc;
  const int b = bg / p.Hk, g = bg - b * p.Hk;
  const int h0 = g * G + gc * 32;            // first query head of this chunk
  const int nh = min(32, G - gc * 32);       // heads in this chunk
  const float c2 = p.scale_log2;
  const unsigned smem_addr = (unsigned)(size_t)(lds_ptr)smem;
  const unsigned q_tile = smem_addr, kt = smem_addr + kQBytes + 2 * wave * kHalf, vt = kt + kHalf;
  FragAddr<D> fa;
  fa.init(lane);

  // ---- Q tile: row n = head n of the chunk (zeros past the group)
  {
    const char* qb = (const char*)p.Q + ((size_t)b * p.Hq + h0) * RB;
#pragma unroll
    for (int i = tid; i < 32 * Tl::kChunks; i += kDecMWaves * 64) {
      const int n = i / Tl::kChunks, c = i % Tl::kChunks;
      u32x4 v = *(const u32x4*)(qb + (size_t)min(n, nh - 1) * RB + c * 16);
      if (n >= nh) v = (u32x4){0u, 0u, 0u, 0u};
      *(u32x4*)(smem + Tl::off(n, c)) = v;
    }
  }
  __syncthreads();
  const int split = sg * kDecMWaves + wave;  // this wave's slice
  if (split >= p.n_slices) return;

  f32x16 oa[Tl::kDBlocks];  // O^T: [channel block], lane = head, registers = channels 8 i + 4 hi + j
#pragma unroll
  for (int cb = 0; cb < Tl::kDBlocks; ++cb)
#pragma unroll
    for (int i = 0; i < 16; ++i) oa[cb][i] = 0.f;
  float m = -INFINITY, l = 0.f;
  const float lazy = 8.0f / c2;  // 8 powers of two, in units of the raw scores

  // rows [k_begin, k_end) of the sequence cache, or (last slice) the depth slots of the position
  const bool is_depth = split == p.n_split;
  const int k_begin = is_depth ? 0 : split * p.keys_per_split;
  const int k_end = is_depth ? p.depth_count : min(p.T, k_begin + p.keys_per_split);
  const int n_blocks = (k_end - k_begin + kDecBlock - 1) / kDecBlock;  // (>= 1: no slice is empty)
  const size_t slab = is_depth ? (size_t)bg * p.depth_alloc * RB : ((size_t)bg * p.T_alloc + k_begin) * RB;
  const unsigned bytes = (unsigned)(k_end - k_begin) * (unsigned)RB;
  const __amdgpu_buffer_rsrc_t k_buf = __builtin_amdgcn_make_buffer_rsrc(
      (void*)((const char*)(is_depth ? p.Kdepth : p.Kseq) + slab), 0, (int)bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t v_buf = __builtin_amdgcn_make_buffer_rsrc(
      (void*)((const char*)(is_depth ? p.Vdepth : p.Vseq) + slab), 0, (int)bytes, 0x00020000);
  // The tile-copy mapping: 1 KB per instruction; a lane fetches the chunk that belongs at its
  // place (16 * lane) of the piece of the permuted tile.  The permutation of piece q differs
  // from piece 0's by the swz of the piece's first row.
  const int jr = lane / Tl::kChunks, pc = lane % Tl::kChunks;
  const int g_off = jr * RB + ((pc ^ Tl::swz(jr)) << 4);
  auto piece_xor = [](int q) { return (D == 128 ? (q & 3) : ((q & 1) << 1)) << 4; };
  struct Block {
    u32x4 k[kInst];
    u32x4 v[kInst];
  };
  auto issue = [&](int blk, Block& r) {
    const int soff = blk * kHalf;  // (blocks past the slice: every lane out of range, zeros)
#pragma unroll
    for (int q = 0; q < kInst; ++q)
      r.k[q] = __builtin_amdgcn_raw_buffer_load_b128(k_buf, xor_here(g_off, piece_xor(q)), soff + q * 1024, 2);
#pragma unroll
    for (int q = 0; q < kInst; ++q)
      r.v[q] = __builtin_amdgcn_raw_buffer_load_b128(v_buf, xor_here(g_off, piece_xor(q)), soff + q * 1024, 2);
  };
  const unsigned bq_row = fa.row + q_tile, bk_row = fa.row + kt;
  const unsigned bv_tr = fa.tr + vt, bv_tr8 = fa.tr8 + vt;
  auto fold = [&](int blk, const Block& r) {
    // block -> the wave's LDS tiles (a wave's LDS operations execute in order: these writes
    // follow the fragment reads of the block before)
#pragma unroll
    for (int q = 0; q < kInst; ++q)
      *(u32x4 __attribute__((address_space(3)))*)(size_t)(kt + q * 1024 + lane * 16) = r.k[q];
#pragma unroll
    for (int q = 0; q < kInst; ++q)
      *(u32x4 __attribute__((address_space(3)))*)(size_t)(vt + q * 1024 + lane * 16) = r.v[q];
    f32x16 s[NB];
#pragma unroll
    for (int sb = 0; sb < NB; ++sb)
#pragma unroll
      for (int i = 0; i < 16; ++i) s[sb][i] = 0.f;
#pragma unroll
    for (int st = 0; st < kSteps; ++st) {
      const bf16x8 qf = FragAddr<D>::row_frag((unsigned)xor_here((int)bq_row, st << 5), 0, 0);
      const unsigned xk = (unsigned)xor_here((int)bk_row, st << 5);
#pragma unroll
      for (int sb = 0; sb < NB; ++sb) s[sb] = mfma_bf16(FragAddr<D>::row_frag(xk, sb, 0), qf, s[sb]);
    }
    const int key0 = k_begin + blk * kDecBlock;
    if (key0 + kDecBlock > k_end) {  // (uniform) the slice's last, partial block
#pragma unroll
      for (int sb = 0; sb < NB; ++sb)
#pragma unroll
        for (int i = 0; i < 16; ++i)
          if (key0 + sb * 32 + (i >> 2) * 8 + hi * 4 + (i & 3) >= k_end) s[sb][i] = -INFINITY;
    }
    float bm = s[0][0];
#pragma unroll
    for (int sb = 0; sb < NB; ++sb)
#pragma unroll
      for (int i = 0; i < 16; ++i) bm = fmaxf(bm, s[sb][i]);
    bm = pair_max(bm);
    // The reference m of the exponentials is raised lazily: only when a block's maximum exceeds
    // it by more than 8 powers of two (weights then stay below 2^8, which fp32 sums and bf16
    // weights hold; any reference gives the same quotient).  The first block always raises it
    // (m = -inf; every block holds at least one key of the slice, so bm is finite, and the
    // factor exp2(-inf) = 0 scales the empty state).
    const bool raise = bm > m + lazy || m == -INFINITY;
    if (__builtin_amdgcn_ballot_w64(raise) != 0) {  // (uniform)
      const float mn = raise ? bm : m;
      const float al = fast_exp2((m - mn) * c2);
      m = mn;
      l *= al;
#pragma unroll
      for (int cb = 0; cb < Tl::kDBlocks; ++cb)
#pragma unroll
        for (int i = 0; i < 16; ++i) oa[cb][i] *= al;
    }
    const float mc = m * c2;
#pragma unroll
    for (int sb = 0; sb < NB; ++sb)
#pragma unroll
      for (int hf = 0; hf < 2; ++hf) {
        float pv[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          pv[k] = fast_exp2(s[sb][hf * 8 + k] * c2 - mc);
          l += pv[k];
        }
        const bf16x8 pb = pack8(pv);
#pragma unroll
        for (int cb = 0; cb < Tl::kDBlocks; ++cb)
          oa[cb] = mfma_bf16(FragAddr<D>::tr_frag((unsigned)xor_here((int)bv_tr, cb << 6),
                                                  (unsigned)xor_here((int)bv_tr8, cb << 6), sb * 2 + hf, 0),
                             pb, oa[cb]);
      }
  };

  // Blocks are walked with the loads of the next kPF - 1 in flight; past the end the loads
  // are still issued (out of range: they fetch nothing), so that the wait for an older
  // block's registers never depends on a branch.
  Block buf[kPF];
#pragma unroll
  for (int i = 0; i < kPF - 1; ++i) issue(i, buf[i]);
  for (int blk0 = 0; blk0 < n_blocks; blk0 += kPF) {
#pragma unroll
    for (int i = 0; i < kPF; ++i) {
      const int blk = blk0 + i;
      issue(blk + kPF - 1, buf[(i + kPF - 1) % kPF]);
      if (blk < n_blocks) fold(blk, buf[i]);
    }
  }

  // ---- this slice's partial result of the lane's head: 4 consecutive channels at a time
  const float l_tot = pair_sum(l);
  if (l32 < nh) {
    float* dst = p.ws + (((size_t)b * p.Hq + h0 + l32) * p.n_slices + split) * (D + 2);
#pragma unroll
    for (int cb = 0; cb < Tl::kDBlocks; ++cb)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float* d4 = dst + cb * 32 + i * 8 + hi * 4;
        d4[0] = oa[cb][4 * i];
        d4[1] = oa[cb][4 * i + 1];
        d4[2] = oa[cb][4 * i + 2];
        d4[3] = oa[cb][4 * i + 3];
      }
    if (hi == 0) {
      dst[D] = m;
      dst[D + 1] = l_tot;
    }
  }
}

// One workgroup of D threads per (batch, query head): thread = channel.  The slices are folded
// eight at a time (their loads issued together), with a running reference like any other
// online softmax.
template <int D>
__global__ __launch_bounds__(D) void moda_decode_merge_kernel(DecodeParams p) {
  constexpr int kU = 8;
  const int ch = threadIdx.x;
  const int bh = blockIdx.x;
  const float c2 = p.scale_log2;
  const float* ws = p.ws + (size_t)bh * p.n_slices * (D + 2);
  float mm = -INFINITY, ll = 0.f, oo = 0.f;
  for (int s0 = 0; s0 < p.n_slices; s0 += kU) {
    float mi[kU], li[kU], oi[kU];
#pragma unroll
    for (int u = 0; u < kU; ++u) {
      const float* w = ws + (size_t)min(s0 + u, p.n_slices - 1) * (D + 2);
      mi[u] = w[D];
      li[u] = w[D + 1];
      oi[u] = w[ch];
    }
    float mn = mm;
#pragma unroll
    for (int u = 0; u < kU; ++u)
      if (s0 + u < p.n_slices) mn = fmaxf(mn, mi[u]);
    // (every slice holds at least one key: mn is finite; with mm = -inf the factor is 0)
    const float al = fast_exp2((mm - mn) * c2);
    mm = mn;
    ll *= al;
    oo *= al;
#pragma unroll
    for (int u = 0; u < kU; ++u)
      if (s0 + u < p.n_slices) {
        const float f = fast_exp2((mi[u] - mm) * c2);
        ll += f * li[u];
        oo += f * oi[u];
      }
  }
  ((__bf16*)p.O)[(size_t)bh * D + ch] = (__bf16)(oo / ll);
  if (ch == 0) p.LSE[bh] = mm * p.scale + __logf(ll);
}

// How a call is cut into slices.  One query head per key/value head: workgroups of 4 waves,
// enough of them to fill 256 compute units a few times over, slices of at least 256 keys.
// More than 4 query heads per key/value head (matrix-pipe kernel): one slice per wave.
struct DecodePlan {
  bool mfma;
  int n_split;
  int keys_per_split;
};
static DecodePlan decode_plan(int B, int Hq, int Hk, int T, int d) {
  DecodePlan pl;
  const int G = Hq / Hk;
  // up to 4 heads per group the vector-ALU kernel is at the memory rate and ahead (measured)
  pl.mfma = G > 4;
  const int most = (T + 255) / 256;
  int want, step;
  if (pl.mfma) {
    const int n_gc = (G + 31) / 32;
    // 12 wave-slices per compute unit: all resident at once at d = 64, one and a half rounds
    // at d = 128 (measured better than exactly one round: the second half-round evens out the tail)
    const long long slots = 256ll * 12;
    const long long per = slots / ((long long)B * Hk * n_gc);
    want = per < 1 ? 1 : (int)per;
    step = kDecBlock;
  } else {
    want = (2048 + B * Hk - 1) / (B * Hk);
    step = kDecWaves * (64 / (d / 8));  // key rows a workgroup takes per step (16 or 32)
  }
  int s = want < most ? want : most;
  if (s < 1) s = 1;
  pl.keys_per_split = ((T + s - 1) / s + step - 1) / step * step;
  pl.n_split = (T + pl.keys_per_split - 1) / pl.keys_per_split;
  return pl;
}

size_t decode_workspace_bytes(int B, int Hq, int Hk, int T, int d) {
  // (one slice more than the sequence is cut into: the depth slots)
  return (size_t)B * Hq * (decode_plan(B, Hq, Hk, T, d).n_split + 1) * (d + 2) * sizeof(float);
}

template <int D>
static hipError_t launch_decode_d(DecodeParams p, bool mfma, hipStream_t stream) {
  const int G = p.Hq / p.Hk;
  if (!grid_ok((long long)p.B * p.Hq)) return kGridTooLarge;
  hipError_t e;
  if (mfma) {
    const long long blocks = (long long)p.B * p.Hk * ((G + 31) / 32) * ((p.n_slices + kDecMWaves - 1) / kDecMWaves);
    if (!grid_ok(blocks)) return kGridTooLarge;
    e = launch_kernel(moda_decode_partial_mfma_kernel<D>, dim3((unsigned)blocks), dim3(kDecMWaves * 64), stream, p);
  } else {
    const int gt = G >= 3 ? 4 : G >= 2 ? 2 : 1;  // (3 heads: one chunk of 4 with a padded head, not two chunks)
    const long long blocks = (long long)p.B * p.Hk * ((G + gt - 1) / gt) * p.n_slices;
    if (!grid_ok(blocks)) return kGridTooLarge;
    dim3 grid((unsigned)blocks), block(kDecWaves * 64);
    if (gt == 4) e = launch_kernel(moda_decode_partial_kernel<D, 4>, grid, block, stream, p);
    else if (gt == 2) e = launch_kernel(moda_decode_partial_kernel<D, 2>, grid, block, stream, p);
    else e = launch_kernel(moda_decode_partial_kernel<D, 1>, grid, block, stream, p);
  }
  if (e != hipSuccess) return e;
  return launch_kernel(moda_decode_merge_kernel<D>, dim3((unsigned)(p.B * p.Hq)), dim3(D), stream, p);
}

hipError_t launch_decode_bf16(const void* Q, const void* Kseq, const void* Vseq, const void* Kdepth,
                              const void* Vdepth, void* O, float* LSE, float* ws, int B, int Hq, int Hk, int T,
                              int T_alloc, int d, int depth_alloc, int depth_count, float scale,
                              hipStream_t stream) {
  DecodeParams p;
  p.Q = Q; p.Kseq = Kseq; p.Vseq = Vseq; p.Kdepth = Kdepth; p.Vdepth = Vdepth;
  p.O = O; p.LSE = LSE; p.ws = ws;
  p.B = B; p.Hq = Hq; p.Hk = Hk; p.T = T; p.T_alloc = T_alloc;
  p.depth_alloc = depth_alloc; p.depth_count = depth_count;
  const DecodePlan pl = decode_plan(B, Hq, Hk, T, d);
  p.n_split = pl.n_split;
  p.keys_per_split = pl.keys_per_split;
  p.n_slices = pl.n_split + (depth_count > 0 ? 1 : 0);
  p.scale = scale;
  p.scale_log2 = scale * 1.4426950408889634f;
  if (d == 128) return launch_decode_d<128>(p, pl.mfma, stream);
  if (d == 64) return launch_decode_d<64>(p, pl.mfma, stream);
  return hipErrorInvalidValue;
}

}  // namespace moda
