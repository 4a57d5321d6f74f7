/*
 * ll.h - C ABI of the fused logit-lens projection and steering library (MI355X, gfx950).
 *
 * All tensor pointers are DEVICE pointers owned by the caller; they must stay
 * valid until the stream has finished the call's work.  No entry point
 * allocates or frees device memory, and none synchronises the stream unless
 * its comment says so.  `stream` is a hipStream_t passed as void* (NULL = the
 * default stream).  bf16 tensors are raw 16-bit patterns, row-major.
 *
 * Return value: 0 on success, a negative LL_E* code otherwise.  On error no
 * output is defined; nothing is thrown and the process is never aborted.
 */
#ifndef LL_H_
#define LL_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LL_OK           0
#define LL_EINVAL      -1   /* null required pointer, bad size, k out of range, d not a multiple of 8 */
#define LL_EWORKSPACE  -2   /* workspace missing or smaller than ll_workspace_bytes()              */
#define LL_EHIP        -3   /* a HIP call failed; ll_last_hip_error() gives its code                */
#define LL_ESCRATCH    -4   /* ll_project_static: the shape does not fit the library's static buffer  */

#define LL_KMAX         32  /* largest supported top-k */

/* N lens rows (layer x token pairs, row r = l*T + t of the packed trajectories,
 * paper Sec. 3.1 Stage 3), hidden size d, vocabulary size V. */
typedef struct ll_shape {
  int64_t N;
  int32_t d;
  int32_t V;
} ll_shape;

/* Bytes of device workspace ll_project needs for this shape and k.  Pure host
 * arithmetic (no HIP call).  Returns 0 for an invalid shape or k. */
size_t ll_workspace_bytes(const ll_shape* shape, int k);

/*
 * Deferred, batched logit-lens projection (paper Sec. 3.3, Eq. 1 and "Top-k
 * extraction"; Alg. 1, Phase 2), fused so that the [N, V] logits never reach
 * memory:
 *
 *   a[r, :]  = bf16( gamma * hidden[r, :] / sqrt(mean_j hidden[r, j]^2 + eps) )   (final RMSNorm)
 *   z[r, v]  = sum_j a[r, j] * W_U[v, j]                                            (Eq. 1, b = 0)
 *   p[r, :]  = softmax over the whole vocabulary
 *
 * Outputs, per row r:
 *   out_topk_ids [N, k] int32  ids of the k largest logits, descending logit, ascending id on exact ties
 *   out_topk_p   [N, k] fp32   their full-softmax probabilities
 *   out_target_logp [N] fp32   z[r, target_ids[r]] - logsumexp(z[r, :]); NaN if the id is outside [0, V)
 *   out_entropy  [N] fp32      -sum_v p log p, in nats
 *
 *   hidden      bf16 [N, d]
 *   gamma       bf16 [d], or NULL: the rows are already normalised (e.g. the output of
 *               ll_steer_inject) and are used as they are
 *   W_U         bf16 [V, d]
 *   target_ids  int32 [N], or NULL: out_target_logp is not written (and may be NULL)
 *   workspace   device scratch of at least ll_workspace_bytes(shape, k) bytes, 256-byte aligned
 *
 * Requirements: d a positive multiple of 8, V at most 2^31 - 257, 1 <= k <= min(LL_KMAX, V), all
 * tensors 16-byte aligned.  N == 0 is a successful no-op.  Rows are processed in passes of at most 8192 rows
 * so the workspace does not grow with N beyond 4 bytes per row.
 * Arithmetic: bf16 operands, fp32 accumulation and fp32 softmax statistics.  A row of `hidden` that
 * holds NaN or infinity gets NaN statistics and unspecified ids; no other row is affected.
 * Everything is enqueued on `stream`; the call returns without waiting.
 */
int ll_project(const ll_shape* shape, void* workspace, size_t workspace_bytes,
               const void* hidden, const void* gamma, const void* W_U,
               float eps, int k, const int32_t* target_ids,
               int32_t* out_topk_ids, float* out_topk_p,
               float* out_target_logp, float* out_entropy,
               void* stream);

/*
 * ll_project in the paper's own output format.  Same as ll_project, plus:
 *   bias   fp32 [V] or NULL: the b of Eq. 1, added to every logit before the softmax statistics,
 *          the top-k selection and the target gather
 *   flags  LL_FLAG_TOPK_SOFTMAX: out_topk_p holds the softmax over the k selected logits only
 *          (paper Sec. 3.3, "Top-k extraction": a conditional distribution over the candidates),
 *          i.e. p_i / sum_{j in top-k} p_j; entropy and target log-prob stay full-vocabulary.
 *          LL_FLAG_REGISTER_STAGED: run this call on the register-staged kernel, which applies the
 *          RMSNorm scaling inside the A-tile load of the GEMM, even where the default applies (the
 *          direct-to-LDS kernel fed from a normalised bf16 panel written once per row pass; d a
 *          multiple of 64).  Both compute the same quantities from the same bf16 operands (the
 *          normalised row is rounded to bf16 identically); they use different MFMA shapes, so a
 *          logit's fp32 partial sums are added in a different order and results agree to fp32
 *          accumulation rounding.  For tuning and tests; any d that is not a multiple of 64 runs on
 *          this kernel anyway.
 *          Any other bit set is LL_EINVAL.
 */
#define LL_FLAG_TOPK_SOFTMAX    1u
#define LL_FLAG_REGISTER_STAGED 2u
int ll_project_ex(const ll_shape* shape, void* workspace, size_t workspace_bytes,
                  const void* hidden, const void* gamma, const void* W_U, const float* bias,
                  unsigned flags, float eps, int k, const int32_t* target_ids,
                  int32_t* out_topk_ids, float* out_topk_p,
                  float* out_target_logp, float* out_entropy,
                  void* stream);

/*
 * ll_project with per-phase timing, for benchmarks.  Same arguments and results; in addition
 * phase_ms (HOST pointer, 3 floats) receives the GPU time in milliseconds, summed over the row
 * passes, of {normalised panel (RMS statistics where the register-staged kernel runs), fused
 * projection kernel, split merge}, measured with HIP events recorded on `stream` around every
 * launch.  Unlike ll_project this call SYNCHRONISES the stream before it returns; the events
 * are created by a thread's first timed call and kept for its later ones.
 */
int ll_project_timed(const ll_shape* shape, void* workspace, size_t workspace_bytes,
                     const void* hidden, const void* gamma, const void* W_U,
                     float eps, int k, const int32_t* target_ids,
                     int32_t* out_topk_ids, float* out_topk_p,
                     float* out_target_logp, float* out_entropy,
                     void* stream, float* phase_ms);

/*
 * ll_project for callers that cannot allocate device memory or hand over a workspace: code under
 * HIP graph capture, tight serving loops (e.g. the lens of the newest token after every decoding
 * step), harnesses that forbid hipMalloc.  Same arguments, results and kernels as ll_project,
 * minus the workspace: the partial results and the normalised panel live in a device array inside
 * this library, LL_STATIC_SCRATCH_BYTES large, which every GPU the library runs on holds until the
 * process ends.  The call allocates and frees nothing.
 *
 * Rows are processed in passes of ll_project_static_pass_rows(shape, k) rows: 8192 as in
 * ll_project when that plan fits the buffer (then the results are bit-identical to ll_project's),
 * otherwise the largest multiple of 256 that fits (same quantities; the fp32 partial sums of a row
 * are then merged from a different number of vocabulary splits).  LL_ESCRATCH if not even 256 rows
 * fit (d above roughly 100 000).
 *
 * All calls on one GPU share that GPU's buffer: two calls whose kernels may overlap on the same
 * GPU (different streams, different threads) race; calls queued on one stream are safe.  The
 * buffer keeps the last call's contents; the one part that has to start at zero (the top-k bounds
 * the vocabulary splits share) is cleared by a small fill kernel at the start of every call, as
 * in ll_project, never by a memset (the call stays capturable).  The first call on a
 * device looks up the buffer's address (no allocation) and sets a kernel attribute: make it
 * outside stream capture.
 */
#define LL_STATIC_SCRATCH_BYTES (64u << 20)
int ll_project_static(const ll_shape* shape,
                      const void* hidden, const void* gamma, const void* W_U,
                      float eps, int k, const int32_t* target_ids,
                      int32_t* out_topk_ids, float* out_topk_p,
                      float* out_target_logp, float* out_entropy,
                      void* stream);
/* Rows per pass ll_project_static uses for this shape and k (pure host arithmetic); 0 if the
 * shape is invalid or does not fit. */
int64_t ll_project_static_pass_rows(const ll_shape* shape, int k);

/*
 * Steering direction (paper Sec. 3.4, Eq. 2): v = (y+ - y-) / ||y+ - y-||_2 with y+ the mean
 * of the n_target rows of `target` and y- the mean of the n_base rows of `base` (hidden states
 * taken at the label-token position, Sec. 4 steering protocol).  The rows are used as given.
 *
 *   base, target  bf16 [n_base, d], [n_target, d]; n_base, n_target >= 1
 *   normalize     1: Eq. 2; 0: the raw difference of means.  A zero difference gives v = 0.
 *   out_v         fp32 [d]
 *   workspace     optional device scratch (may be NULL): with at least
 *                 ll_steer_workspace_bytes(d) bytes the row reduction is spread over the whole
 *                 GPU; without it a narrower launch is used.  Results are deterministic either
 *                 way (no atomics), but the two paths may differ in the last fp32 bit.
 */
size_t ll_steer_workspace_bytes(int32_t d);
int ll_steer_vector(const void* base, int64_t n_base, const void* target, int64_t n_target,
                    int32_t d, int normalize, float* out_v,
                    void* workspace, size_t workspace_bytes, void* stream);

/*
 * Steering injection after the final norm (paper Sec. 3.4, Eq. 3, applied post-normalisation):
 *
 *   out[r, j] = bf16( gamma[j] * hidden[r, j] / sqrt(mean_j hidden[r, j]^2 + eps) + alpha * v[j] )
 *
 *   shape       N and d are used, V is ignored
 *   hidden      bf16 [N, d];  gamma bf16 [d] (required);  v fp32 [d]
 *   out_hidden  bf16 [N, d]; may be the same buffer as `hidden` (in place), no other overlap
 * The result is what ll_project expects with gamma == NULL.  alpha == 0 gives bf16(RMSNorm(h)).
 */
int ll_steer_inject(const ll_shape* shape, const void* hidden, const void* gamma, float eps,
                    const float* v, float alpha, void* out_hidden, void* stream);

/*
 * Steering inside the model (paper Sec. 3.4, the unnumbered equation h' = h + alpha v after
 * Eq. 2, with the two safeguards of that section's stability paragraph: a per-layer scale and a
 * bound on the size of the shift): the raw activation of a wrapped layer is shifted along v,
 * without any normalisation,
 *
 *   s        = alpha * layer_scale
 *   beta[r]  = sign(s) * min(|s|, clip_ratio * ||hidden[r, :]||_2)     (clip_ratio > 0)
 *   beta[r]  = s                                                       (clip_ratio <= 0: no clipping)
 *   out[r,j] = bf16( hidden[r, j] + beta[r] * v[j] )
 *
 * so that with a unit-norm v the shift never exceeds clip_ratio times the row's own length.
 * The paper names the two safeguards but prints no formula for them: this rule is this
 * library's reading of it.  Same argument conventions as ll_steer_inject (V ignored; out may be
 * `hidden` itself); layer_scale and clip_ratio must be finite.
 */
int ll_steer_inject_raw(const ll_shape* shape, const void* hidden, const float* v, float alpha,
                        float layer_scale, float clip_ratio, void* out_hidden, void* stream);

/*
 * Capture store (paper Sec. 3.1 Stage 2 and the first step of Stage 3; Alg. 1 Phase 1): the
 * wrapped layers' newest activations are appended to per-(layer, type) trajectories that sit in
 * HBM in exactly the row order ll_project reads, store[l, c, t, :] = row ((l*C + c)*T + t), so
 * that "concatenating the slices" costs nothing when decoding starts.
 *
 *   store   bf16 [L, C, T, d]   the trajectories (T = token capacity of the run)
 *   slices  bf16 [L*C, n_tok, d] activations of the n_tok newest tokens for every wrapped layer l
 *           and activation type c, (l, c)-major: n_tok = 1 in a decoding step (the [1, 1, d]
 *           slice per layer and type of the paper), n_tok = prompt length for the prefill
 *   t0      position of the first of these tokens; tokens t0 .. t0 + n_tok - 1 are written
 * LL_EINVAL if t0 < 0, n_tok < 0 or t0 + n_tok > T, d not a multiple of 8, a null or misaligned
 * (16 bytes) pointer.  n_tok == 0 is a successful no-op.  The two buffers must not overlap.
 */
typedef struct ll_capture_shape {
  int32_t L;   /* wrapped layers */
  int32_t C;   /* activation types per layer (attention output, MLP output, block output) */
  int64_t T;   /* tokens per trajectory */
  int32_t d;   /* hidden size */
} ll_capture_shape;
int ll_capture_append(const ll_capture_shape* shape, void* store, const void* slices, int64_t t0, int64_t n_tok,
                      void* stream);

/*
 * Steering sweep: the lens read-out of Eq. 3 (paper Sec. 3.4) for several steering strengths in
 * ONE pass over W_U.  With a[r, :] the normalised row as in ll_project and u = W_U v (fp32),
 *
 *   z_alpha[r, id] = sum_j a[r, j] * W_U[id, j] + alpha * u[id]      ( = W_U (a[r, :] + alpha v) )
 *
 * and for every alpha of the list and every row the call returns the most likely token, its
 * probability, the target token's log-probability and the entropy of softmax(z_alpha[r, :]):
 * the dose-response curve of Sec. 5 for the cost of one projection instead of one per alpha.
 * Unlike ll_steer_inject followed by ll_project, the steered row a + alpha v is never rounded to
 * bf16: the shift alpha * u is added to the fp32 logits.
 *
 *   shape, hidden, gamma (NULL = rows already normalised), W_U, eps: as ll_project
 *   v            fp32 [d], device: the steering direction (e.g. from ll_steer_vector)
 *   alphas       fp32 [n_alpha], HOST memory, read during the call; 1 <= n_alpha <= LL_SWEEP_MAX
 *   target_ids   int32 [N] or NULL (then out_target_logp may be NULL and is not written)
 *   out_top1_ids [n_alpha, N] int32   arg max of z_alpha (smallest id on exact ties)
 *   out_top1_p   [n_alpha, N] fp32    its full-softmax probability
 *   out_target_logp [n_alpha, N] fp32 NaN where the target id is outside [0, V)
 *   out_entropy  [n_alpha, N] fp32    nats
 * Requirements beyond ll_project's: d at most 40960 (the direction v is held in LDS while
 * u = W_U v is formed; LL_EINVAL beyond).  d a multiple of 64 runs on the direct-to-LDS kernel, any
 * other multiple of 8 on the register-staged one.  Workspace: ll_steer_sweep_workspace_bytes(shape,
 * n_alpha).  Same error, ownership, stream and N == 0 conventions as ll_project.
 *
 * ll_steer_sweep_topk: the same with the k most likely tokens per alpha and row instead of one
 * (1 <= k <= LL_SWEEP_KMAX; the paper's figures list k = 3), sorted as in ll_project:
 *   out_topk_ids [n_alpha, N, k] int32,  out_topk_p [n_alpha, N, k] fp32 (full-softmax probabilities)
 * With k == 1 it is ll_steer_sweep.  With k > 1 the lists of five alphas are what fits the
 * register file beside the accumulators, so the call makes ceil(n_alpha / 5) passes over W_U
 * (nine alphas: two passes, against nine for ll_steer_inject + ll_project pairs).  Workspace:
 * ll_steer_sweep_topk_workspace_bytes(shape, n_alpha, k).
 */
#define LL_SWEEP_MAX 9
#define LL_SWEEP_KMAX 4   /* longest top-k list of ll_steer_sweep_topk */
size_t ll_steer_sweep_workspace_bytes(const ll_shape* shape, int n_alpha);
int ll_steer_sweep(const ll_shape* shape, void* workspace, size_t workspace_bytes,
                   const void* hidden, const void* gamma, const void* W_U, float eps,
                   const float* v, const float* alphas, int n_alpha, const int32_t* target_ids,
                   int32_t* out_top1_ids, float* out_top1_p, float* out_target_logp, float* out_entropy,
                   void* stream);
size_t ll_steer_sweep_topk_workspace_bytes(const ll_shape* shape, int n_alpha, int k);
int ll_steer_sweep_topk(const ll_shape* shape, void* workspace, size_t workspace_bytes,
                        const void* hidden, const void* gamma, const void* W_U, float eps,
                        const float* v, const float* alphas, int n_alpha, int k, const int32_t* target_ids,
                        int32_t* out_topk_ids, float* out_topk_p, float* out_target_logp, float* out_entropy,
                        void* stream);

/* Text for an LL_E* code (static storage, never NULL). */
const char* ll_error_string(int code);

/* The hipError_t value of the last failed HIP call in this thread (0 if none). */
int ll_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* LL_H_ */
