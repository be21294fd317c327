// libmoda C ABI: argument validation and kernel dispatch (host code only).
#include <math.h>
#include <stdlib.h>

#include "../../include/moda.h"
#include "moda_launch.h"

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Shape checks shared by forward and backward.  Returns MODA_OK if the shape is
// one this build can run.
moda_status check_shape(const moda_shape* s) {
  if (!s) return MODA_ERR_NULL;
  if (s->B < 0 || s->T < 0 || s->Hq <= 0 || s->Hk <= 0 || s->d <= 0) return MODA_ERR_SHAPE;
  if (s->Hq % s->Hk != 0) return MODA_ERR_SHAPE;
  if (s->depth_count < 0 || s->depth_alloc < s->depth_count) return MODA_ERR_SHAPE;
  if (s->causal != 0 && s->causal != 1) return MODA_ERR_SHAPE;
  if (s->dtype != MODA_F32 && s->dtype != MODA_BF16) return MODA_ERR_UNSUPPORTED;
  if (s->d != 64 && s->d != 128) return MODA_ERR_UNSUPPORTED;
  if (!(s->scale == s->scale) || isinf(s->scale)) return MODA_ERR_SHAPE;  // NaN / inf
  // one (b, h) slab of any tensor must stay below 4 GiB (32-bit buffer offsets)
  const unsigned long long esz = s->dtype == MODA_BF16 ? 2 : 4;
  const unsigned long long slots = s->depth_alloc > 0 ? (unsigned long long)s->depth_alloc : 1ull;
  if ((unsigned long long)s->T * slots * (unsigned long long)s->d * esz >= (1ull << 32)) return MODA_ERR_UNSUPPORTED;
  return MODA_OK;
}

// Geometry of the bf16 forward kernel (see moda_fwd_bf16.hip): 8 waves (256 queries) per
// workgroup, one workgroup per compute unit, unless that grid would leave compute units
// without work: then 4 waves (128 queries), two workgroups per unit, twice as many
// workgroups.  MODA_FWD_WAVES = 4 or 8 overrides the choice (for experiments).
int fwd_waves_per_workgroup(const moda_shape* s) {
  if (const char* e = getenv("MODA_FWD_WAVES")) {
    const int w = atoi(e);
    if (w == 4 || w == 8) return w;
  }
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

}  // namespace

extern "C" {

const char* moda_status_string(moda_status st) {
  switch (st) {
    case MODA_OK: return "ok";
    case MODA_ERR_NULL: return "a required pointer is NULL";
    case MODA_ERR_SHAPE: return "invalid or inconsistent shape";
    case MODA_ERR_UNSUPPORTED: return "unsupported dtype or head dimension";
    case MODA_ERR_ALIGN: return "a base pointer is not 16-byte aligned";
    case MODA_ERR_LAUNCH: return "the HIP runtime refused the kernel launch";
    case MODA_ERR_WORKSPACE: return "workspace missing or too small";
  }
  return "unknown status";
}

int moda_version(void) { return 100; }

int moda_kernels_per_call(const moda_shape* s, int which) {
  if (check_shape(s) != MODA_OK || s->B == 0 || s->T == 0) return 0;
  if (which == 0) return 1;
  if (s->dtype != MODA_BF16 || s->Hq / s->Hk > moda::bwd_bf16_max_group()) return 0;
  const int G = s->Hq / s->Hk;
  return 3 + ((G > 1 && s->depth_alloc > 0) ? (G + 7) / 8 : 0);
}

moda_status moda_attn_fwd(const void* Q, const void* Kseq, const void* Vseq, const void* Kdepth,
                          const void* Vdepth, void* O, float* LSE, const moda_shape* s,
                          void* hip_stream) {
  moda_status st = check_shape(s);
  if (st != MODA_OK) return st;
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
  // grouped queries: as many heads of a group per tile as divide both the group and the waves
  const int G = s->Hq / s->Hk;
  const int waves = fwd_waves_per_workgroup(s);
  p.heads_per_tile = 1;
  for (int gt = waves; gt > 1; gt /= 2)
    if (G % gt == 0) {
      p.heads_per_tile = gt;
      break;
    }
  if (const char* e = getenv("MODA_FWD_HEADS_PER_TILE")) {  // experiments
    const int gt = atoi(e);
    if (gt >= 1 && waves % gt == 0 && G % gt == 0) p.heads_per_tile = gt;
  }
  p.head_group = heads_per_die_at_a_time((long long)s->B * s->Hk * (G / p.heads_per_tile), s->T, s->d);
  if (const char* e = getenv("MODA_FWD_HEAD_GROUP")) p.head_group = atoi(e);  // experiments
  const int rows = moda::fwd_bf16_tile_rows(waves) / p.heads_per_tile;  // positions per tile
  p.n_qtiles = (s->T + rows - 1) / rows;

  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  hipError_t e = (s->dtype == MODA_BF16) ? moda::launch_fwd_bf16(p, s->d, waves, stream)
                                         : moda::launch_fwd_f32(p, s->d, stream);
  return e == hipSuccess ? MODA_OK : MODA_ERR_LAUNCH;
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
  hipError_t e = moda::launch_depth_append(K, V, Kdepth, Vdepth, (long long)s->B * s->Hk * s->T, s->d * esz,
                                           s->depth_alloc, slot, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? MODA_OK : MODA_ERR_LAUNCH;
}

size_t moda_attn_decode_workspace_bytes(const moda_shape* s) {
  if (check_shape(s) != MODA_OK || s->dtype != MODA_BF16 || s->B == 0 || s->T == 0) return 0;
  return moda::decode_workspace_bytes(s->B, s->Hq, s->Hk, s->T, s->d);
}

moda_status moda_attn_decode(const void* Q, const void* Kseq, const void* Vseq, const void* Kdepth,
                             const void* Vdepth, void* O, float* LSE, int32_t kv_alloc, void* workspace,
                             size_t workspace_bytes, const moda_shape* s, void* hip_stream) {
  moda_status st = check_shape(s);
  if (st != MODA_OK) return st;
  if (s->dtype != MODA_BF16) return MODA_ERR_UNSUPPORTED;
  if (s->T < 1 || kv_alloc < s->T) return MODA_ERR_SHAPE;  // the new token's own key is always attended
  if ((unsigned long long)kv_alloc * (unsigned long long)s->d * 2ull >= (1ull << 32)) return MODA_ERR_UNSUPPORTED;
  if (s->B == 0) return MODA_OK;
  if (!Q || !Kseq || !Vseq || !O || !LSE) return MODA_ERR_NULL;
  if (s->depth_count > 0 && (!Kdepth || !Vdepth)) return MODA_ERR_NULL;
  const void* ptrs[] = {Q, Kseq, Vseq, Kdepth, Vdepth, O, LSE, workspace};
  for (const void* q : ptrs)
    if (!aligned16(q)) return MODA_ERR_ALIGN;
  if (!workspace || workspace_bytes < moda_attn_decode_workspace_bytes(s)) return MODA_ERR_WORKSPACE;
  hipError_t e = moda::launch_decode_bf16(Q, Kseq, Vseq, Kdepth, Vdepth, O, LSE, static_cast<float*>(workspace),
                                          s->B, s->Hq, s->Hk, s->T, kv_alloc, s->d, s->depth_alloc, s->depth_count,
                                          resolve_scale(s), static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? MODA_OK : MODA_ERR_LAUNCH;
}

size_t moda_attn_bwd_workspace_bytes(const moda_shape* s) {
  if (check_shape(s) != MODA_OK) return 0;
  moda::BwdParams p{};
  p.B = s->B; p.Hq = s->Hq; p.T = s->T;
  return moda::bwd_bf16_workspace_bytes(p);
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

  moda::BwdParams p;
  p.Q = Q; p.Kseq = Kseq; p.Vseq = Vseq; p.Kdepth = Kdepth; p.Vdepth = Vdepth;
  p.O = O; p.LSE = LSE; p.dO = dO;
  p.dQ = dQ; p.dKseq = dKseq; p.dVseq = dVseq; p.dKdepth = dKdepth; p.dVdepth = dVdepth;
  p.rowstat = static_cast<float*>(workspace);
  p.B = s->B; p.Hq = s->Hq; p.Hk = s->Hk; p.T = s->T;
  p.depth_alloc = s->depth_alloc; p.depth_count = s->depth_count;
  p.causal = s->causal;
  p.scale = resolve_scale(s);
  p.scale_log2 = p.scale * 1.4426950408889634f;
  p.head_group = heads_per_die_at_a_time((long long)s->B * s->Hk, s->T, s->d);
  hipError_t e = moda::launch_bwd_bf16(p, s->d, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? MODA_OK : MODA_ERR_LAUNCH;
}

}  // extern "C"
