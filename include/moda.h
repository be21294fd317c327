/*
 * libmoda -- Mixture-of-Depths Attention (MoDA) for AMD MI355X (gfx950).
 *
 * C ABI.  Every data pointer is a DEVICE pointer owned by the caller; the
 * shape struct and the return values live on the host.  The library never
 * allocates, frees or keeps a pointer; its only scratch is the workspace the
 * caller passes to the backward and decoding calls.  Calls are asynchronous on
 * the given HIP stream (NULL = the default stream), never synchronise the
 * device, read no environment variable and hold no global mutable state (one
 * exception, stated at moda_attn_decode_noalloc).
 * Errors are reported by return code only.  Every argument check (pointers,
 * shapes, alignment, workspace size, the size of every kernel grid) is made
 * before the first kernel is enqueued: on any status other than MODA_OK and
 * MODA_ERR_LAUNCH nothing has been launched and no output has been touched.
 * MODA_ERR_LAUNCH means the HIP runtime refused a kernel launch of this call
 * (the code is that launch's own return value, not an error left behind by
 * earlier work of the caller); kernels of the same call that were enqueued
 * before it still run, so the outputs are then unspecified.
 *
 * The operator (paper section 2.2 "Mixture-of-Depths Attention"; Eq. 2 for the
 * sequence part; Algorithm 1 for the index sets and the shared online-softmax
 * state): for batch b, query head h (kv head g = h / (Hq/Hk)) and position t,
 * ONE softmax runs over
 *   - the sequence keys  Kseq[b,g,j],  j <= t  (all j < T when causal == 0;
 *     the diagonal j == t is visible), and
 *   - the depth keys     Kdepth[b,g,t,i],  i < depth_count: the keys that
 *     preceding layers produced at the query's own position t,
 * with logits scale * <Q[b,h,t], key>.  O[b,h,t] is the weighted sum of the
 * matching values (Vseq[b,g,j], Vdepth[b,g,t,i]) under that one normaliser
 * (Algorithm 1's final o / acc), and LSE[b,h,t] = max logit + ln(sum of
 * exp(logit - max)) in natural-log units.  depth_count == 0 is plain
 * (causal) attention.
 *
 * Layouts: contiguous row-major, base pointers 16-byte aligned.
 *   Q, O, dO, dQ                  [B, Hq, T, d]
 *   Kseq, Vseq, dKseq, dVseq      [B, Hk, T, d]
 *   Kdepth, Vdepth, dKdepth, ...  [B, Hk, T, depth_alloc, d]
 *                                 (position-major: the depth_alloc slots of one
 *                                 position are adjacent -- the paper's
 *                                 "flash-compatible depth KV layout" with the
 *                                 flattened T*L axis kept as two indices)
 *   LSE                           [B, Hq, T], always fp32
 * Element type of everything but LSE is `dtype`.  Outputs must not alias
 * inputs.  Kdepth/Vdepth (and their gradients) may be NULL iff
 * depth_count == 0.
 */
#ifndef MODA_H_
#define MODA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  MODA_OK = 0,
  MODA_ERR_NULL = 1,        /* a required pointer is NULL                        */
  MODA_ERR_SHAPE = 2,       /* a dimension is negative / inconsistent            */
  MODA_ERR_UNSUPPORTED = 3, /* valid request this build has no kernel for        */
  MODA_ERR_ALIGN = 4,       /* a base pointer is not 16-byte aligned             */
  MODA_ERR_LAUNCH = 5,      /* the HIP runtime refused the launch                */
  MODA_ERR_WORKSPACE = 6    /* workspace is NULL or smaller than required        */
} moda_status;

typedef enum { MODA_F32 = 0, MODA_BF16 = 1 } moda_dtype;

typedef struct {
  int32_t B;           /* batch, >= 0 (0 is a valid empty call)                           */
  int32_t Hq;          /* query heads, > 0                                                */
  int32_t Hk;          /* key/value heads, > 0, Hq % Hk == 0                              */
  int32_t T;           /* sequence length, T_q == T_kv == T, >= 0                         */
  int32_t d;           /* head dimension: 64 or 128                                       */
  int32_t depth_alloc; /* slots allocated per position in Kdepth/Vdepth (the stride)      */
  int32_t depth_count; /* slots [0, depth_count) are attended; <= depth_alloc             */
  int32_t causal;      /* 1: sequence keys j <= t (Eq. 2's causal mask); 0: all T keys    */
  float scale;         /* softmax scale; <= 0 selects Eq. 2's 1/sqrt(d)                   */
  moda_dtype dtype;    /* type of Q, K, V, depth tensors, O, dO, gradients (a 32-bit enum) */
} moda_shape;

/*
 * Size limits of this build (MODA_ERR_UNSUPPORTED beyond them): d is 64 or 128; one
 * (batch, head) slab of a SEQUENCE tensor, T * d elements, stays below 4 GiB (32-bit byte
 * offsets inside a slab); depth_alloc <= 8192.  The depth tensors themselves are addressed
 * with 64-bit tile bases and may be of any size.
 */

/*
 * Forward pass of the operator defined above (Algorithm 1: sequence blocks,
 * then the depth slots, folded into one running max / normaliser / output,
 * one final division).
 *   in : Q, Kseq, Vseq, Kdepth, Vdepth   device, read-only
 *   out: O (dtype), LSE (fp32)           device, fully overwritten
 * Returns MODA_OK after enqueueing the work on `hip_stream` (a hipStream_t
 * passed as void*).  B == 0 or T == 0 returns MODA_OK without launching.
 */
moda_status moda_attn_fwd(const void* Q, const void* Kseq, const void* Vseq, const void* Kdepth,
                          const void* Vdepth, void* O, float* LSE, const moda_shape* s,
                          void* hip_stream);

/*
 * The same forward pass with the launch geometry of the bf16 kernel chosen by the caller
 * instead of derived from the shape (for experiments and for tests that must reach every
 * code path; the result is the same operator whatever the geometry).  A field that is 0
 * keeps the library's own choice; `tuning` == NULL is moda_attn_fwd.
 *   waves           4 or 8: waves (of 32 queries each) per workgroup
 *   heads_per_tile  query heads of one group that share a tile (side by side in every wave): a
 *                   power of two up to 32 that divides Hq / Hk
 *   head_group      (batch, head) units that one die walks together, tile by tile; >= 1
 *   depth_path      1: depth slots on the vector ALUs (row-major dot products); 2: on the
 *                   matrix pipe (per-wave key blocks)
 * Values that the kernel cannot run are rejected with MODA_ERR_SHAPE.  Ignored for fp32.
 */
typedef struct {
  int32_t waves;
  int32_t heads_per_tile;
  int32_t head_group;
  int32_t depth_path;
} moda_fwd_tuning;
moda_status moda_attn_fwd_tuned(const void* Q, const void* Kseq, const void* Vseq, const void* Kdepth,
                                const void* Vdepth, void* O, float* LSE, const moda_shape* s,
                                const moda_fwd_tuning* tuning, void* hip_stream);

/*
 * Backward pass.  The paper times it (Table 2, "forward&backward") but gives
 * no algorithm; it is the derivative of the forward definition: with softmax
 * weights p over the union, g = dO[b,h,t] and delta = <g, O[b,h,t]>,
 *   dV_c += p_c g;  e_c = p_c (<g, v_c> - delta);
 *   dQ[b,h,t] = scale * sum_c e_c k_c;  dK_c += scale * e_c Q[b,h,t],
 * where a sequence key sums over every query that sees it (and the Hq/Hk query
 * heads of its kv head) and a depth slot (t,i) only over the queries at t.
 *   in : Q, Kseq, Vseq, Kdepth, Vdepth, O, LSE (from moda_attn_fwd), dO
 *   out: dQ, dKseq, dVseq, dKdepth, dVdepth (dtype), fully overwritten; depth
 *        gradient slots >= depth_count are written as zero
 *   workspace: device scratch of at least moda_attn_bwd_workspace_bytes(s)
 *        bytes, 16-byte aligned; contents on entry are ignored.
 * This build: bf16 only, Hq / Hk <= 64 (else MODA_ERR_UNSUPPORTED).
 */
size_t moda_attn_bwd_workspace_bytes(const moda_shape* s);
moda_status moda_attn_bwd(const void* Q, const void* Kseq, const void* Vseq, const void* Kdepth,
                          const void* Vdepth, const void* O, const float* LSE, const void* dO,
                          void* dQ, void* dKseq, void* dVseq, void* dKdepth, void* dVdepth,
                          void* workspace, size_t workspace_bytes, const moda_shape* s,
                          void* hip_stream);

/*
 * The "write" step of the depth stream (paper section 2.2: once a layer has run
 * the operator, its key-value pair is appended to the depth stream so that the
 * following layers can read it; an FFN layer appends the output of its own
 * key-value projection the same way).  Copies the layer's K and V,
 * [B, Hk, T, d], into slot `slot` of Kdepth and Vdepth, [B, Hk, T, depth_alloc, d];
 * no other slot is touched.  A stack of layers allocates the cache once with
 * depth_alloc = number of writers and lets layer l attend depth_count = l slots.
 *   in : K, V                    device, read-only
 *   out: Kdepth, Vdepth          device, slot `slot` of every position overwritten
 * Uses B, Hk, T, d, depth_alloc and dtype of `s` (Hq, depth_count, causal and
 * scale are validated as for the other calls but not used); 0 <= slot <
 * depth_alloc, else MODA_ERR_SHAPE.  K / V must not overlap Kdepth / Vdepth.
 */
moda_status moda_depth_append(const void* K, const void* V, void* Kdepth, void* Vdepth, int32_t slot,
                              const moda_shape* s, void* hip_stream);

/*
 * Decoding step: ONE new token per sequence (paper Table 1, "Decoding" rows).  The
 * operator is the one defined above for the query at the last position: it attends
 * the T positions [0, T) of the sequence cache (the new token's own key/value, which
 * the caller has already written at position T-1, included; no mask is needed) and
 * the depth_count depth slots of ITS OWN position, under one softmax.  During
 * decoding the depth cache therefore holds one position only.
 *   in : Q                 [B, Hq, d]              the new token's queries
 *        Kseq, Vseq        [B, Hk, kv_alloc, d]    sequence cache, kv_alloc >= T rows allocated
 *        Kdepth, Vdepth    [B, Hk, depth_alloc, d] the new token's depth slots (NULL iff depth_count == 0)
 *   out: O                 [B, Hq, d], LSE [B, Hq] fp32
 *   workspace: device scratch of at least moda_attn_decode_workspace_bytes(s) bytes
 *        (partial results of the slices the sequence is split into), 16-byte aligned.
 * `s->T` is the attended length (>= 1), `s->causal` is ignored.  bf16 only.
 */
size_t moda_attn_decode_workspace_bytes(const moda_shape* s);
moda_status moda_attn_decode(const void* Q, const void* Kseq, const void* Vseq, const void* Kdepth,
                             const void* Vdepth, void* O, float* LSE, int32_t kv_alloc, void* workspace,
                             size_t workspace_bytes, const moda_shape* s, void* hip_stream);

/*
 * The decoding step for callers that cannot allocate device memory and have no workspace to
 * pass: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same operator, arguments and results as moda_attn_decode, but the slices' partial results go
 * to a scratch array that is part of the library image (a file-scope device array of
 * moda_attn_decode_noalloc_max_bytes() = 8 MiB; every GPU the library runs on holds its own
 * copy until the process ends).  The call allocates nothing and frees nothing.  A shape whose
 * moda_attn_decode_workspace_bytes() exceeds that size is rejected with MODA_ERR_WORKSPACE
 * before anything is launched (use moda_attn_decode with a workspace then).  All calls on one
 * GPU share that GPU's array: two such calls that overlap in time on the same GPU (different
 * streams, different threads) race and give wrong results; calls on one stream, or otherwise
 * ordered, are safe, and nothing in the array needs clearing between calls.  The array's device
 * address is looked up once per GPU, on the first call made with that GPU current; that per-GPU
 * address table is the only state the library keeps.
 */
size_t moda_attn_decode_noalloc_max_bytes(void);
moda_status moda_attn_decode_noalloc(const void* Q, const void* Kseq, const void* Vseq, const void* Kdepth,
                                     const void* Vdepth, void* O, float* LSE, int32_t kv_alloc,
                                     const moda_shape* s, void* hip_stream);

/*
 * Measurement aid: a kernel whose loop holds nothing but the bf16 matrix instruction the
 * attention kernels use (v_mfma_f32_32x32x16_bf16; eight waves per workgroup, four independent
 * accumulators per wave), for reporting what the matrix pipe of THIS chip sustains next to its
 * published peak.  The operands are read once from `operands`
 * (moda_calibrate_mfma_operand_bytes() bytes of bf16, device, 16-byte aligned): the sustained
 * rate depends on their values (the clock follows the power they draw), so the caller passes
 * zeros, or values distributed like its workload's.  `sink` (device,
 * moda_calibrate_mfma_sink_bytes(workgroups) bytes) receives one float per thread.  Enqueues
 * one launch of `workgroups` workgroups x `iters` loop passes on `hip_stream` and returns the
 * floating-point operations it performs (0 if an argument is bad or the launch is refused);
 * the caller times it with HIP events.
 */
size_t moda_calibrate_mfma_operand_bytes(void);
size_t moda_calibrate_mfma_sink_bytes(int32_t workgroups);
double moda_calibrate_mfma(const void* operands, float* sink, size_t sink_bytes, int32_t workgroups, int32_t iters,
                           void* hip_stream);

/* Static, NUL-terminated description of a status code. */
const char* moda_status_string(moda_status st);

/* Library version: major * 10000 + minor * 100 + patch. */
int moda_version(void);

/*
 * Number of kernels that one forward (which = 0) or backward (which = 1) call
 * enqueues for shape `s` (0 for an empty or unsupported problem), so that a
 * profiler's per-kernel rows can be matched to calls.
 */
int moda_kernels_per_call(const moda_shape* s, int which);

#ifdef __cplusplus
}
#endif
#endif /* MODA_H_ */
