/*
 * gradcache.h - C ABI of the MI355X (gfx950) Gradient Cache hot path.
 *
 * The library computes, for anchor representations Q[B,d] (the paper's
 * f(s_i)), target representations P[P,d] (g(t_j)) and positive indices r_i,
 * the full-batch in-batch-negative contrastive loss (Eq. 1) and its
 * representation gradients dL/dQ, dL/dP (Eq. 4-7): the "Representation
 * Gradient Cache" of Step 2.  It also runs the sub-batch steps around it for a
 * stand-in two-layer MLP encoder: the graph-less forward (Step 1) and the
 * per-sub-batch re-encode + backward of the cached rows (Step 3, Eq. 8-9).
 * The B x P score matrix is never written to device memory.
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers unless marked "host".  Matrices
 *     are row-major and contiguous (leading dimension = number of columns).
 *   - The caller owns every buffer, the workspace included; the library frees
 *     nothing the caller passed.  gc_loss_and_rep_grad_bf16 / _f32 take no
 *     workspace argument: they use a per-device buffer the library allocates
 *     with hipMalloc on first use and grows on demand (growing frees the old
 *     buffer with hipFree, which waits for the device; while `stream` is being
 *     captured into a graph a call that would have to grow it returns
 *     GC_ERR_UNSUPPORTED instead).  Such calls share the buffer, so the library
 *     puts them in order: a call made on another stream than the previous one
 *     first waits (on the GPU, through an event) for that one's kernels.  Calls
 *     made while their stream is being captured are not ordered this way and
 *     must not overlap with other calls.  To run calls side by side use the
 *     *_ex forms with a workspace each, or gc_loss_and_rep_grad_bf16_static
 *     where nothing may be allocated.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  A
 *     call only enqueues work and returns; outputs are valid once the stream
 *     has been synchronised.  No call synchronises the device, except
 *     gc_check_async_error, gc_step_mlp_release and the workspace growth
 *     described above.
 *   - Return value: GC_OK or a negative gc_status.  All argument checks are
 *     made on the host before the first HIP call, so a bad call enqueues
 *     nothing.  pos_idx values cannot be checked on the host: a value outside
 *     [0, P) makes the kernels set loss to NaN and raise the device error word
 *     that gc_check_async_error reads.
 *   - loss, dq, dp, dz, lse, argmax, y are overwritten; gc_mlp_grads buffers are
 *     accumulated into (+=).
 *   - Same inputs give bit-identical outputs from run to run (no atomics, fixed
 *     reduction order).
 */
#ifndef GRADCACHE_H
#define GRADCACHE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  GC_OK = 0,
  GC_ERR_NULL = -1,        /* a required pointer is NULL */
  GC_ERR_SHAPE = -2,       /* a size is <= 0 / too large, or scale/temp is not a positive finite number */
  GC_ERR_UNSUPPORTED = -3, /* dtype, flag or shape combination not implemented */
  GC_ERR_WORKSPACE = -4,   /* workspace NULL, misaligned (256 B) or smaller than the *_workspace_bytes value */
  GC_ERR_POS_IDX = -5,     /* reported by gc_check_async_error: some pos_idx[i] was outside [0, P) */
  GC_ERR_HIP = -6,         /* a HIP runtime call failed (launch, allocation) */
  GC_ERR_TOO_LARGE = -7    /* gc_loss_and_rep_grad_bf16_static: the shape needs more scratch than GC_STATIC_SCRATCH_BYTES */
} gc_status;

/* element types; the entry points take them as int, so that a value outside the list is an error (GC_ERR_UNSUPPORTED),
 * not an invalid enum load */
typedef enum { GC_F32 = 0, GC_BF16 = 1 } gc_dtype;

/* flags of gc_loss_and_rep_grad_ex */
#define GC_MASK_SELF 1u /* s_ii = -inf (needs B == P >= 2): an anchor is never its own target */
/* Which kernel sequence serves a call is chosen from the shape; these two override the choice where both exist
 * (bf16, d a multiple of 128 from 256 to 768, dq asked for) and are ignored elsewhere.  For tests and measurements:
 * the results of the two sequences agree to fp32 rounding, not bit for bit. */
#define GC_PATH_ONLINE 2u     /* the dQ walk forms the row statistics itself, no statistics pass */
#define GC_PATH_STATS_PASS 4u /* statistics pass, then both gradient walks in one launch */
/* The cache in bf16: dq and dp then point to bf16 [rows,d] buffers and receive the fp32 results rounded to nearest
 * even (half the bytes of the cache; the rounding, up to 2^-9 relative per element, is then part of what Step 3 sees).
 * Only where the MFMA kernels run (bf16 inputs, d a multiple of 128 up to 768), else GC_ERR_UNSUPPORTED. */
#define GC_CACHE_BF16 8u

/* Text for a gc_status value (host; static storage, never NULL). */
const char* gc_strerror(int status);

/* Bytes of workspace gc_loss_and_rep_grad_ex needs for this shape (host, pure).
 * Holds per-row softmax statistics and the split partial sums of dq and dp:
 * O((B + P) * d), never O(B * P) (Sec. "Gradient Cache Technique": the cache is
 * (|S| d + |T| d) numbers).  Returns 0 for an invalid shape. */
size_t gc_workspace_bytes(int B, int P, int d, int dt);

/*
 * Loss and representation gradients (Step 2; Eq. 1, 4, 5, 6, 7).
 *   q       [B,d]  anchors, bf16 (or float for _f32)
 *   p       [P,d]  targets, same type
 *   pos_idx [B]    int32, r_i in [0, P); several anchors may share one target
 *   logits  s_ij = (scale / temp) * <q_i, p_j>
 *   loss    [1]    float: (1/B) sum_i (logsumexp_j s_ij - s_{i,r_i})
 *   dq      [B,d]  float: (scale/(temp B)) sum_j (softmax_j(s_i.) - [j = r_i]) p_j
 *   dp      [P,d]  float: (scale/(temp B)) sum_i (softmax_j(s_i.) - [j = r_i]) q_i
 * Any B, P >= 1 and d >= 1 are accepted (ragged sizes are masked); the MFMA
 * kernels serve bf16 with d a multiple of 128 up to 768, other cases take a
 * slower general kernel.  Errors: GC_ERR_NULL, GC_ERR_SHAPE, GC_ERR_HIP.
 */
int gc_loss_and_rep_grad_bf16(const void* q, const void* p, const int32_t* pos_idx, int B, int P, int d,
                              float scale, float temp, float* loss, float* dq, float* dp, void* stream);
int gc_loss_and_rep_grad_f32(const float* q, const float* p, const int32_t* pos_idx, int B, int P, int d,
                             float scale, float temp, float* loss, float* dq, float* dp, void* stream);

/*
 * The same call for callers that cannot allocate: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  Same arguments, same kernels and bit-identical results as gc_loss_and_rep_grad_bf16, but
 * the workspace (row statistics, split partial sums, the error word) is a fixed array of GC_STATIC_SCRATCH_BYTES in
 * the library's device image, one copy per GPU, held until the process ends: the call makes no hipMalloc, hipFree
 * or other allocating call, and its first use on a device only looks the array's address up.  Shapes with
 * gc_workspace_bytes(B, P, d, GC_BF16) > GC_STATIC_SCRATCH_BYTES are rejected with GC_ERR_TOO_LARGE and nothing is
 * enqueued (the limit covers e.g. B = 512, P = 1024, d = 768).  Every call on a GPU uses that GPU's one array,
 * which keeps the previous call's contents (the kernels overwrite what they read): two calls that overlap in time
 * on one GPU, on whatever streams, race; calls on one stream are safe.  A pos_idx outside [0, P) shows as
 * loss = NaN, and gc_check_async_error(NULL) also reads this array's error word.
 * Errors: GC_ERR_NULL, GC_ERR_SHAPE, GC_ERR_TOO_LARGE, GC_ERR_HIP.
 */
#define GC_STATIC_SCRATCH_BYTES (16u << 20)
int gc_loss_and_rep_grad_bf16_static(const void* q, const void* p, const int32_t* pos_idx, int B, int P, int d,
                                     float scale, float temp, float* loss, float* dq, float* dp, void* stream);

/*
 * Extended form of the same computation.
 *   dt         type of q and p, a gc_dtype value
 *   flags      0 or GC_MASK_SELF, optionally with one of GC_PATH_ONLINE / GC_PATH_STATS_PASS, and GC_CACHE_BF16
 *   loss, dq, dp, lse, argmax   each may be NULL (not produced).  lse[B] float is
 *              logsumexp_j s_ij; argmax[B] int32 is the smallest j that attains
 *              max_j s_ij in the kernel's fp32 scores.
 *   workspace  device, 256-byte aligned, at least gc_workspace_bytes(B,P,d,dt)
 */
int gc_loss_and_rep_grad_ex(int dt, const void* q, const void* p, const int32_t* pos_idx, int B, int P, int d,
                            float scale, float temp, unsigned flags, float* loss, float* dq, float* dp, float* lse,
                            int32_t* argmax, void* workspace, size_t workspace_bytes, void* stream);

/* After the stream has been synchronised by the caller: copies the device error
 * word of `workspace` to the host (a blocking 4-byte copy) and returns GC_OK or
 * GC_ERR_POS_IDX.  workspace == NULL checks the library's own per-device buffer
 * and the static array of gc_loss_and_rep_grad_bf16_static (those that have been used). */
int gc_check_async_error(const void* workspace);

/*
 * Measurement aid for benchmarks (not part of the method; for callers that want per-phase
 * device times without an external profiler).  gc_profile_begin(max_calls) makes
 * every following loss call record HIP events on its stream at the phase
 * boundaries (statistics pass | merge of split statistics and loss | gradient
 * kernel | fixed-order sums of its split partials); gc_profile_end waits for the
 * recorded events, writes the mean milliseconds per call of the four phases and the
 * number of calls seen (each pointer may be NULL), and switches recording off.
 * Host state is process-wide and not thread-safe.  Errors: GC_ERR_SHAPE
 * (max_calls outside [1, 65536]), GC_ERR_UNSUPPORTED (begin twice / end without
 * begin), GC_ERR_HIP.
 */
int gc_profile_begin(int max_calls);
int gc_profile_end(float* ms_stats, float* ms_merge, float* ms_grad, float* ms_reduce, int* calls);

/*
 * NT-Xent over n_views = 2N views (a loss variation in the sense of Step 2's
 * remark; SimCLR is cited in Related Work): z[n_views,d] bf16, rows already
 * L2-normalised; views 2k and 2k+1 are positives of each other; logits
 * <z_i,z_j>/temp with the self-similarity removed; loss = mean over all n_views
 * anchors; dz[n_views,d] float = gradient w.r.t. z (anchor part + target part).
 * workspace: gc_ntxent_workspace_bytes(n_views, d).
 */
size_t gc_ntxent_workspace_bytes(int n_views, int d);
int gc_ntxent_loss_and_grad_bf16(const void* z, int n_views, int d, float temp, float* loss, float* dz,
                                 void* workspace, size_t workspace_bytes, void* stream);

/*
 * Symmetric in-batch-negative loss (anchors against targets and targets against
 * anchors), one of the loss variations Step 2 of Sec. "Gradient Cache Technique"
 * admits: n anchors, n targets, pos_idx a bijection of 0..n-1,
 *   L = 1/2 [ L(F, G, r) + L(G, F, r^-1) ]   with L as in Eq. 1,
 * dq = dL/df(s_i), dp = dL/dg(t_j) (Eq. 5 of one direction + Eq. 6 of the
 * other, halved).  q, p [n,d] bf16, pos_idx [n] int32, loss [1], dq, dp [n,d]
 * float, all device memory, all overwritten.  A pos_idx that is no bijection is
 * reported like a positive out of range (loss = NaN, GC_ERR_POS_IDX from
 * gc_check_async_error(workspace)).
 * workspace: gc_bidirectional_workspace_bytes(n, d).
 */
size_t gc_bidirectional_workspace_bytes(int n, int d);
int gc_bidirectional_loss_and_rep_grad_bf16(const void* q, const void* p, const int32_t* pos_idx, int n, int d,
                                            float scale, float temp, float* loss, float* dq, float* dp,
                                            void* workspace, size_t workspace_bytes, void* stream);

/*
 * Loss with a parameterised distance function (Sec. "Extend to Deep Distance
 * Function"), for the bilinear form Phi_Omega(f, g) = f^T Omega g:
 *   d_ij = f(s_i)^T Omega g(t_j), logits scale * d_ij / temp, loss as Eq. 1.
 * With w_ij = dL/dd_ij (the section's Distance Gradient Cache) the outputs are
 *   u[B,d]      = dL/df(s_i) = sum_j w_ij Omega g(t_j)
 *   v[P,d]      = dL/dg(t_j) = sum_i w_ij Omega^T f(s_i)
 *   domega[d,d] = dL/dOmega  = sum_ij w_ij f(s_i) g(t_j)^T
 * (the section's last three equations); u and v are what Step 3 takes as the
 * Representation Gradient Cache.  w is never stored: it exists tile by tile inside
 * the loss kernels, which run on h_i = Omega^T f(s_i) (kept in bf16) against the
 * targets.  q[B,d], p[P,d], omega[d,d] (row-major) bf16, pos_idx[B] int32; loss[1],
 * u, v, domega float, overwritten; all device memory.  d must be a multiple of 128
 * up to 768 (else GC_ERR_UNSUPPORTED).  Errors as gc_loss_and_rep_grad_ex; the
 * asynchronous pos_idx error is read with gc_check_async_error(workspace).
 * workspace: gc_bilinear_workspace_bytes(B, P, d) (0 for an unsupported shape).
 */
size_t gc_bilinear_workspace_bytes(int B, int P, int d);
/* Where a call leaves its two intermediates inside its workspace (host, pure): byte offsets of H[B,d] (bf16, the
 * stored h_i = Omega^T f(s_i) that the scores were formed from) and of A[B,d] (float, a_i = sum_j w_ij g(t_j), from
 * which u = A Omega^T and dOmega = F^T A follow).  For callers that keep them and for stage-by-stage checks.
 * Errors: GC_ERR_NULL, GC_ERR_SHAPE, GC_ERR_UNSUPPORTED as for the call itself. */
int gc_bilinear_workspace_layout(int B, int P, int d, size_t* off_h, size_t* off_a);
int gc_bilinear_loss_and_grads_bf16(const void* q, const void* p, const int32_t* pos_idx, int B, int P, int d,
                                    const void* omega, float scale, float temp, float* loss, float* u, float* v,
                                    float* domega, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Loss with a deep, non-bilinear distance function (Sec. "Extend to Deep Distance Function", all four equations):
 *   d_ij = Phi_Omega(f(s_i), g(t_j)) = sum_k w_k tanh((A f(s_i))_k + (C g(t_j))_k),   Omega = (A [h,d], C [h,d], w [h]),
 * logits scale * d_ij / temp, loss as Eq. 1.  Phi does not factor over its arguments: each of the B * P distances is
 * evaluated on its own (twice: once for the softmax normaliser, once for the gradients).  With
 * w_ij = dL/dd_ij, the section's Distance Gradient Cache, the outputs are
 *   u[B,d] = sum_j w_ij dd_ij/df(s_i),   v[P,d] = sum_i w_ij dd_ij/dg(t_j)      (the Representation Gradient Cache)
 *   dA[h,d], dC[h,d], dw[h] = sum_ij w_ij dPhi(f(s_i), g(t_j))/dOmega           (the gradient of Omega)
 * w_ij is never stored: it exists for one pair at a time inside the kernel that walks the pairs, and is consumed
 * there for all three sums.  q[B,d], p[P,d], A, C, w bf16; pos_idx[B] int32; loss[1], u, v, dA, dC, dw float,
 * overwritten; all device memory.  d must be a multiple of 128 and h = 128 (else GC_ERR_UNSUPPORTED).  Errors as
 * gc_loss_and_rep_grad_ex; the asynchronous pos_idx error is read with gc_check_async_error(workspace).
 * workspace: gc_deepdist_workspace_bytes(B, P, d, h) (0 for an unsupported shape).
 */
size_t gc_deepdist_workspace_bytes(int B, int P, int d, int h);
int gc_deepdist_loss_and_grads_bf16(const void* q, const void* p, const int32_t* pos_idx, int B, int P, int d,
                                    const void* A, const void* C, const void* w, int h, float scale, float temp,
                                    float* loss, float* u, float* v, float* dA, float* dC, float* dw, void* workspace,
                                    size_t workspace_bytes, void* stream);

/*
 * Stand-in encoder  y = GELU(x W1 + b1) W2 + b2  (exact erf GELU), bf16 storage,
 * fp32 accumulation.  W1[din,dh], b1[dh], W2[dh,dout], b2[dout], all device bf16.
 * din must be a multiple of 64, dh and dout multiples of 128 (else
 * GC_ERR_UNSUPPORTED); the number of rows of a sub-batch is free.
 */
typedef struct {
  const void* W1;
  const void* b1;
  const void* W2;
  const void* b2;
  int din, dh, dout;
} gc_mlp_params;

/* fp32 parameter-gradient accumulators, same shapes as the parameters (device). */
typedef struct {
  float* dW1;
  float* db1;
  float* dW2;
  float* db2;
} gc_mlp_grads;

/* Step 1 for one sub-batch: y[rows,dout] bf16 = encoder(x[rows,din]); no
 * activations are kept.  workspace: gc_mlp_workspace_bytes(rows, w) (fp32
 * activations of the sub-batch and transposed copies of W1, W2, which every
 * call rebuilds: the weights may change between calls). */
size_t gc_mlp_workspace_bytes(int rows, const gc_mlp_params* w);
int gc_mlp_forward_nograd_bf16(const void* x, int rows, const gc_mlp_params* w, void* y, void* workspace,
                               size_t workspace_bytes, void* stream);

/* Step 3 for one sub-batch (the inner sum of Eq. 8 / Eq. 9): re-encodes
 * x_chunk[rows,din] keeping the activations, then back-propagates
 * cached_grad_rows[rows,dout] (float: the sub-batch's rows of dq or dp) and adds
 * the parameter gradients into acc.  workspace: gc_mlp_workspace_bytes(rows, w). */
int gc_chunk_surrogate_backward_bf16(const void* x_chunk, int rows, const gc_mlp_params* w,
                                     const float* cached_grad_rows, const gc_mlp_grads* acc, void* workspace,
                                     size_t workspace_bytes, void* stream);

/*
 * One whole Gradient Cache step on one GPU (Steps 1-3) with the shared stand-in
 * encoder: sub-batches of chunk_q anchors / chunk_p targets in index order (the
 * last one may be short); graph-less forward of every sub-batch, loss and
 * representation-gradient cache, then per-sub-batch surrogate backward.
 *   x_q [B,din], x_p [P,din] bf16; pos_idx [B] int32
 *   loss [1] float (overwritten); grads accumulated (+=): zero them before the call
 *   q_rep [B,dout], p_rep [P,dout] bf16 and dq [B,dout], dp [P,dout] float:
 *     optional outputs (NULL = kept in the workspace only)
 * workspace: gc_step_mlp_workspace_bytes(B, P, chunk_q, chunk_p, w).  It holds the
 *   representations and their gradient cache ((B + P) * dout numbers each), the
 *   loss workspace, three sets of one sub-batch's activations for Step 3, and
 *   the transient activations of Step 1, whose graph-less forward takes up to
 *   2048 rows (whole sub-batches) per launch: rows * dh floats, three times.
 * Everything is enqueued on `stream`; the order in which sub-batches are added
 * to the gradients is the index order, so the result is reproducible bit for
 * bit.  A call that repeats with exactly the same arguments (same buffers) is
 * recorded into a HIP graph the second time and replayed afterwards; the
 * contents of the buffers may change between calls, their addresses and sizes
 * select the recording.
 */
size_t gc_step_mlp_workspace_bytes(int B, int P, int chunk_q, int chunk_p, const gc_mlp_params* w);
int gc_step_mlp_bf16(const void* x_q, int B, const void* x_p, int P, const int32_t* pos_idx, int chunk_q,
                     int chunk_p, const gc_mlp_params* w, float scale, float temp, float* loss,
                     const gc_mlp_grads* grads, void* q_rep, void* p_rep, float* dq, float* dp, void* workspace,
                     size_t workspace_bytes, void* stream);

/*
 * The same step with Step 3 run on groups of accumulate_group (1..8) consecutive sub-batches of one side: the
 * re-encoded activations of a group are alive at once (accumulate_group times the activation memory of a sub-batch:
 * the quantity the sub-batch size exists to bound, hence opt-in), and the fp32 gradient accumulators are read and
 * written once per group instead of once per sub-batch.  The sub-batches of a group are still added in index order
 * and in the same 32-row pieces, so every output has the bits gc_step_mlp_bf16 gives (accumulate_group = 1 is that
 * call).  Grouping needs chunk_q and chunk_p to be multiples of 32; otherwise the call runs ungrouped.
 * workspace: gc_step_mlp_grouped_workspace_bytes(B, P, chunk_q, chunk_p, w, accumulate_group).
 * Errors as gc_step_mlp_bf16; GC_ERR_SHAPE for accumulate_group outside [1, 8].
 */
size_t gc_step_mlp_grouped_workspace_bytes(int B, int P, int chunk_q, int chunk_p, const gc_mlp_params* w,
                                           int accumulate_group);
int gc_step_mlp_grouped_bf16(const void* x_q, int B, const void* x_p, int P, const int32_t* pos_idx, int chunk_q,
                             int chunk_p, int accumulate_group, const gc_mlp_params* w, float scale, float temp,
                             float* loss, const gc_mlp_grads* grads, void* q_rep, void* p_rep, float* dq, float* dp,
                             void* workspace, size_t workspace_bytes, void* stream);

/* Forgets the recordings gc_step_mlp_bf16 keeps for the current device (at most 8 argument sets): call it before
 * freeing buffers that a recorded call named, or to give the graph memory back.  It waits for the device to be
 * idle (the one call besides gc_check_async_error that synchronises), then destroys the recorded graphs and the
 * library's capture stream; later calls record afresh.  A recorded call must always be issued on one stream at a
 * time: replays on two streams share the workspace and race.  Errors: GC_ERR_HIP. */
int gc_step_mlp_release(void);

#ifdef __cplusplus
}
#endif
#endif /* GRADCACHE_H */
