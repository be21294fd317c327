// libmoda C ABI: argument validation and kernel dispatch (host code only).
#include <math.h>

#include "../../include/moda.h"
#include "moda_launch.h"

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

constexpr int kMaxDepthAlloc = 8192;  // a tile's depth slots are addressed with 32-bit offsets

// Checks shared by every call: dimensions, dtype, head dimension, scale.
moda_status check_dims(const moda_shape* s) {
  if (!s) return MODA_ERR_NULL;
  if (s->B < 0 || s->T < 0 || s->Hq <= 0 || s->Hk <= 0 || s->d <= 0) return MODA_ERR_SHAPE;
  if (s->Hq % s->Hk != 0) return MODA_ERR_SHAPE;
  if (s->depth_count < 0 || s->depth_alloc < s->depth_count) return MODA_ERR_SHAPE;
  if (s->causal != 0 && s->causal != 1) return MODA_ERR_SHAPE;
  if (s->dtype != MODA_F32 && s->dtype != MODA_BF16) return MODA_ERR_UNSUPPORTED;
  if (s->d != 64 && s->d != 128) return MODA_ERR_UNSUPPORTED;
  if (!(s->scale == s->scale) || isinf(s->scale)) return MODA_ERR_SHAPE;  // NaN / inf
  if (s->depth_alloc > kMaxDepthAlloc) return MODA_ERR_UNSUPPORTED;
  // element counts that the kernels keep in 32-bit integers
  if ((long long)s->B * s->Hq > 0x7fffffffLL) return MODA_ERR_UNSUPPORTED;
  return MODA_OK;
}

// One (batch, head) slab of `rows` sequence rows must stay below 4 GiB: the kernels address a
// sequence tensor with 32-bit byte offsets inside a slab.  (The depth tensors are addressed
// from a 64-bit base per tile and have no such limit.)
bool slab_ok(const moda_shape* s, long long rows) {
  const unsigned long long esz = s->dtype == MODA_BF16 ? 2 : 4;
  return (unsigned long long)rows * (unsigned long long)s->d * esz < (1ull << 32);
}

// Shape checks of the calls that take [B, H, T, d] tensors (forward, backward, write step).
moda_status check_shape(const moda_shape* s) {
  const moda_status st = check_dims(s);
  if (st != MODA_OK) return st;
  return slab_ok(s, s->T) ? MODA_OK : MODA_ERR_UNSUPPORTED;
}

moda_status launch_status(hipError_t e) {
  if (e == hipSuccess) return MODA_OK;
  return e == moda::kGridTooLarge ? MODA_ERR_UNSUPPORTED : MODA_ERR_LAUNCH;
}

// Geometry of the bf16 forward kernel (see moda_fwd_bf16.hip): 8 waves (256 queries) per
// workgroup, one workgroup per compute unit, unless that grid would leave compute units
// without work: then 4 waves (128 queries), two workgroups per unit, twice as many
// workgroups.
int fwd_waves_per_workgroup(const moda_shape* s) {
  const long long tiles8 = (long long)s->B * s->Hq * ((s->T + 255) / 256);
  return tiles8 < 256 ? 4 : 8;
}

// Heads that one die (workgroup ids equal mod 8) walks together, tile by tile: as many as have
// their streamed tensors (2 * T * d bf16 elements each: K and V, or Q and dO) in its 4 MB L2, at
// least one; a power of two that divides the heads of a die.  0: the ids cannot be dealt that way.
int heads_per_die_at_a_time(long long n_heads, int T, int d) {
  if (n_heads % 8 != 0) return 0;
  const long long per_die = n_heads / 8;
  const long long fit = (4ll << 20) / (4ll * T * d);
  int hg = 1;
  while (hg * 2 <= fit && per_die % (hg * 2) == 0) hg *= 2;
  return hg;
}

float resolve_scale(const moda_shape* s) {
  return s->scale > 0.f ? s->scale : 1.0f / sqrtf((float)s->d);
}

moda::BwdParams bwd_dims(const moda_shape* s) {
  moda::BwdParams p{};
  p.B = s->B; p.Hq = s->Hq; p.Hk = s->Hk; p.T = s->T;
  p.depth_alloc = s->depth_alloc; p.depth_count = s->depth_count;
  return p;
}

}  // namespace

extern "C" {

const char* moda_status_string(moda_status st) {
  switch (st) {
    case MODA_OK: return "ok";
    case MODA_ERR_NULL: return "a required pointer is NULL";
    case MODA_ERR_SHAPE: return "invalid or inconsistent shape";
    case MODA_ERR_UNSUPPORTED: return "unsupported dtype, head dimension or size";
    case MODA_ERR_ALIGN: return "a base pointer is not 16-byte aligned";
    case MODA_ERR_LAUNCH: return "the HIP runtime refused a kernel launch";
    case MODA_ERR_WORKSPACE: return "workspace missing or too small";
  }
  return "unknown status";
}

int moda_version(void) { return 200; }

int moda_kernels_per_call(const moda_shape* s, int which) {
  if (check_shape(s) != MODA_OK || s->B == 0 || s->T == 0) return 0;
  if (which == 0) return 1;
  if (s->dtype != MODA_BF16 || s->Hq / s->Hk > moda::bwd_bf16_max_group()) return 0;
  return moda::bwd_bf16_kernels(bwd_dims(s));
}

moda_status moda_attn_fwd_tuned(const void* Q, const void* Kseq, const void* Vseq, const void* Kdepth,
                                const void* Vdepth, void* O, float* LSE, const moda_shape* s,
                                const moda_fwd_tuning* tuning, void* hip_stream) {
  moda_status st = check_shape(s);
  if (st != MODA_OK) return st;
  const int G = s->Hq / s->Hk;
  int waves = fwd_waves_per_workgroup(s);
  if (tuning && s->dtype == MODA_BF16) {
    if (tuning->waves != 0 && tuning->waves != 4 && tuning->waves != 8) return MODA_ERR_SHAPE;
    if (tuning->waves != 0) waves = tuning->waves;
    const int gt = tuning->heads_per_tile;
    if (gt < 0 || gt > 32 || (gt & (gt - 1)) != 0 || (gt > 0 && G % gt != 0)) return MODA_ERR_SHAPE;
    if (tuning->head_group < 0) return MODA_ERR_SHAPE;
    if (tuning->depth_path < 0 || tuning->depth_path > 2) return MODA_ERR_SHAPE;
  }
  if (s->B == 0 || s->T == 0) return MODA_OK;
  if (!Q || !Kseq || !Vseq || !O || !LSE) return MODA_ERR_NULL;
  if (s->depth_count > 0 && (!Kdepth || !Vdepth)) return MODA_ERR_NULL;
  if (!aligned16(Q) || !aligned16(Kseq) || !aligned16(Vseq) || !aligned16(O) || !aligned16(LSE) ||
      !aligned16(Kdepth) || !aligned16(Vdepth))
    return MODA_ERR_ALIGN;

  moda::FwdParams p;
  p.Q = Q; p.Kseq = Kseq; p.Vseq = Vseq; p.Kdepth = Kdepth; p.Vdepth = Vdepth;
  p.O = O; p.LSE = LSE;
  p.B = s->B; p.Hq = s->Hq; p.Hk = s->Hk; p.T = s->T;
  p.depth_alloc = s->depth_alloc; p.depth_count = s->depth_count;
  p.causal = s->causal;
  p.scale = resolve_scale(s);
  p.scale_log2 = p.scale * 1.4426950408889634f;
  // grouped queries: as many heads of a group per tile (side by side in every wave) as divide the
  // group, up to 32
  p.heads_per_tile = 1;
  for (int gt = 32; gt > 1; gt /= 2)
    if (G % gt == 0) {
      p.heads_per_tile = gt;
      break;
    }
  // (without depth slots two heads per wave only halve the positions a tile covers: measured 10 %
  //  slower than one head per tile at G = 2, equal or faster from 4 heads on)
  if (s->depth_count == 0 && p.heads_per_tile < 4) p.heads_per_tile = 1;
  if (tuning && tuning->heads_per_tile > 0) p.heads_per_tile = tuning->heads_per_tile;
  p.head_group = heads_per_die_at_a_time((long long)s->B * s->Hk * (G / p.heads_per_tile), s->T, s->d);
  if (tuning && tuning->head_group > 0) p.head_group = tuning->head_group;
  // depth slots: on the matrix pipe when several heads share a position's slots (the block
  // products are then dense enough to beat the vector ALUs), else on the vector ALUs, where the
  // phase already runs at the rate a compute unit can fetch
  p.depth_mfma = (p.heads_per_tile > 1 && s->depth_count > 0) ? 1 : 0;
  if (tuning && s->dtype == MODA_BF16 && tuning->depth_path != 0)
    p.depth_mfma = (tuning->depth_path == 2 && s->depth_count > 0) ? 1 : 0;
  p.depth_magic = s->depth_count > 1 ? (unsigned)((1ull << 32) / (unsigned)s->depth_count) + 1u : 0u;
  const int rows = moda::fwd_bf16_tile_rows(waves) / p.heads_per_tile;  // positions per tile
  p.n_qtiles = (s->T + rows - 1) / rows;

  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  return launch_status((s->dtype == MODA_BF16) ? moda::launch_fwd_bf16(p, s->d, waves, stream)
                                               : moda::launch_fwd_f32(p, s->d, stream));
}

moda_status moda_attn_fwd(const void* Q, const void* Kseq, const void* Vseq, const void* Kdepth,
                          const void* Vdepth, void* O, float* LSE, const moda_shape* s,
                          void* hip_stream) {
  return moda_attn_fwd_tuned(Q, Kseq, Vseq, Kdepth, Vdepth, O, LSE, s, nullptr, hip_stream);
}

moda_status moda_depth_append(const void* K, const void* V, void* Kdepth, void* Vdepth, int32_t slot,
                              const moda_shape* s, void* hip_stream) {
  moda_status st = check_shape(s);
  if (st != MODA_OK) return st;
  if (slot < 0 || slot >= s->depth_alloc) return MODA_ERR_SHAPE;
  if (s->B == 0 || s->T == 0) return MODA_OK;
  if (!K || !V || !Kdepth || !Vdepth) return MODA_ERR_NULL;
  if (!aligned16(K) || !aligned16(V) || !aligned16(Kdepth) || !aligned16(Vdepth)) return MODA_ERR_ALIGN;
  const int esz = s->dtype == MODA_BF16 ? 2 : 4;
  return launch_status(moda::launch_depth_append(K, V, Kdepth, Vdepth, (long long)s->B * s->Hk * s->T, s->d * esz,
                                                 s->depth_alloc, slot, static_cast<hipStream_t>(hip_stream)));
}

// Shape checks of the decoding step: [B, H, d] queries, a sequence cache of kv_alloc rows per
// (batch, head), one position's depth slots.
static moda_status check_decode(const moda_shape* s, int32_t kv_alloc) {
  const moda_status st = check_dims(s);
  if (st != MODA_OK) return st;
  if (s->dtype != MODA_BF16) return MODA_ERR_UNSUPPORTED;
  if (s->T < 1 || kv_alloc < s->T) return MODA_ERR_SHAPE;  // the new token's own key is always attended
  return MODA_OK;  // (the decoding kernels address the caches with 64-bit pointers: no slab limit)
}

size_t moda_attn_decode_workspace_bytes(const moda_shape* s) {
  if (check_dims(s) != MODA_OK || s->dtype != MODA_BF16 || s->B == 0 || s->T < 1) return 0;
  return moda::decode_workspace_bytes(s->B, s->Hq, s->Hk, s->T, s->d);
}

// The decoding step with the slices' partial results in `workspace` (already validated).
static moda_status decode_with(const void* Q, const void* Kseq, const void* Vseq, const void* Kdepth,
                               const void* Vdepth, void* O, float* LSE, int32_t kv_alloc, void* workspace,
                               const moda_shape* s, void* hip_stream);

moda_status moda_attn_decode(const void* Q, const void* Kseq, const void* Vseq, const void* Kdepth,
                             const void* Vdepth, void* O, float* LSE, int32_t kv_alloc, void* workspace,
                             size_t workspace_bytes, const moda_shape* s, void* hip_stream) {
  moda_status st = check_decode(s, kv_alloc);
  if (st != MODA_OK) return st;
  if (s->B == 0) return MODA_OK;
  if (!Q || !Kseq || !Vseq || !O || !LSE) return MODA_ERR_NULL;
  if (s->depth_count > 0 && (!Kdepth || !Vdepth)) return MODA_ERR_NULL;
  const void* ptrs[] = {Q, Kseq, Vseq, Kdepth, Vdepth, O, LSE, workspace};
  for (const void* q : ptrs)
    if (!aligned16(q)) return MODA_ERR_ALIGN;
  if (!workspace || workspace_bytes < moda_attn_decode_workspace_bytes(s)) return MODA_ERR_WORKSPACE;
  return decode_with(Q, Kseq, Vseq, Kdepth, Vdepth, O, LSE, kv_alloc, workspace, s, hip_stream);
}

size_t moda_attn_decode_noalloc_max_bytes(void) { return moda::decode_static_scratch_bytes(); }

moda_status moda_attn_decode_noalloc(const void* Q, const void* Kseq, const void* Vseq, const void* Kdepth,
                                     const void* Vdepth, void* O, float* LSE, int32_t kv_alloc,
                                     const moda_shape* s, void* hip_stream) {
  moda_status st = check_decode(s, kv_alloc);
  if (st != MODA_OK) return st;
  if (moda_attn_decode_workspace_bytes(s) > moda::decode_static_scratch_bytes()) return MODA_ERR_WORKSPACE;
  if (s->B == 0) return MODA_OK;
  if (!Q || !Kseq || !Vseq || !O || !LSE) return MODA_ERR_NULL;
  if (s->depth_count > 0 && (!Kdepth || !Vdepth)) return MODA_ERR_NULL;
  const void* ptrs[] = {Q, Kseq, Vseq, Kdepth, Vdepth, O, LSE};
  for (const void* q : ptrs)
    if (!aligned16(q)) return MODA_ERR_ALIGN;
  void* ws = nullptr;  // this GPU's copy of the library's scratch array (device address)
  if (moda::decode_static_scratch(&ws) != hipSuccess) return MODA_ERR_LAUNCH;
  // Nothing in the scratch has to start at zero: the first kernel writes every partial result
  // that the second one reads.
  return decode_with(Q, Kseq, Vseq, Kdepth, Vdepth, O, LSE, kv_alloc, ws, s, hip_stream);
}

static moda_status decode_with(const void* Q, const void* Kseq, const void* Vseq, const void* Kdepth,
                               const void* Vdepth, void* O, float* LSE, int32_t kv_alloc, void* workspace,
                               const moda_shape* s, void* hip_stream) {
  return launch_status(moda::launch_decode_bf16(Q, Kseq, Vseq, Kdepth, Vdepth, O, LSE, static_cast<float*>(workspace),
                                                s->B, s->Hq, s->Hk, s->T, kv_alloc, s->d, s->depth_alloc,
                                                s->depth_count, resolve_scale(s),
                                                static_cast<hipStream_t>(hip_stream)));
}

size_t moda_calibrate_mfma_operand_bytes(void) { return moda::calibrate_operand_bytes(); }
size_t moda_calibrate_mfma_sink_bytes(int32_t workgroups) {
  return workgroups > 0 ? moda::calibrate_sink_bytes(workgroups) : 0;
}
double moda_calibrate_mfma(const void* operands, float* sink, size_t sink_bytes, int32_t workgroups, int32_t iters,
                           void* hip_stream) {
  if (!operands || !sink || workgroups <= 0 || iters <= 0 || !aligned16(operands) || !aligned16(sink)) return 0.0;
  if (sink_bytes < moda::calibrate_sink_bytes(workgroups)) return 0.0;
  if (moda::launch_calibrate_mfma(operands, sink, workgroups, iters, static_cast<hipStream_t>(hip_stream)) != hipSuccess)
    return 0.0;
  return moda::calibrate_flops(workgroups, iters);
}

size_t moda_attn_bwd_workspace_bytes(const moda_shape* s) {
  if (check_shape(s) != MODA_OK) return 0;
  return moda::bwd_bf16_workspace_bytes(bwd_dims(s), s->d);
}

moda_status moda_attn_bwd(const void* Q, const void* Kseq, const void* Vseq, const void* Kdepth,
                          const void* Vdepth, const void* O, const float* LSE, const void* dO,
                          void* dQ, void* dKseq, void* dVseq, void* dKdepth, void* dVdepth,
                          void* workspace, size_t workspace_bytes, const moda_shape* s,
                          void* hip_stream) {
  moda_status st = check_shape(s);
  if (st != MODA_OK) return st;
  // this build's backward: bf16, at most bwd_bf16_max_group() query heads per key/value head
  if (s->dtype != MODA_BF16 || s->Hq / s->Hk > moda::bwd_bf16_max_group()) return MODA_ERR_UNSUPPORTED;
  if (s->B == 0 || s->T == 0) return MODA_OK;
  if (!Q || !Kseq || !Vseq || !O || !LSE || !dO || !dQ || !dKseq || !dVseq) return MODA_ERR_NULL;
  if (s->depth_count > 0 && (!Kdepth || !Vdepth)) return MODA_ERR_NULL;
  if (s->depth_alloc > 0 && (!dKdepth || !dVdepth)) return MODA_ERR_NULL;
  const void* ptrs[] = {Q, Kseq, Vseq, Kdepth, Vdepth, O, LSE, dO, dQ, dKseq, dVseq, dKdepth, dVdepth, workspace};
  for (const void* q : ptrs)
    if (!aligned16(q)) return MODA_ERR_ALIGN;
  if (!workspace || workspace_bytes < moda_attn_bwd_workspace_bytes(s)) return MODA_ERR_WORKSPACE;

  moda::BwdParams p = bwd_dims(s);
  p.Q = Q; p.Kseq = Kseq; p.Vseq = Vseq; p.Kdepth = Kdepth; p.Vdepth = Vdepth;
  p.O = O; p.LSE = LSE; p.dO = dO;
  p.dQ = dQ; p.dKseq = dKseq; p.dVseq = dVseq; p.dKdepth = dKdepth; p.dVdepth = dVdepth;
  p.rowstat = static_cast<float*>(workspace);
  p.causal = s->causal;
  p.scale = resolve_scale(s);
  p.scale_log2 = p.scale * 1.4426950408889634f;
  p.head_group = heads_per_die_at_a_time((long long)s->B * s->Hk, s->T, s->d);
  return launch_status(moda::launch_bwd_bf16(p, s->d, static_cast<hipStream_t>(hip_stream)));
}

}  // extern "C"
