/*
 * usl -- training hot path of the uniformly-sparse extreme-classification output layer
 * (every one of m labels has exactly k incoming weights from a layer of width d), as
 * hand-written HIP kernels for gfx950 behind a plain C ABI.
 *
 * Method: Schultheis & Babbar, "Towards Memory-Efficient Training for Extremely Large
 * Output Spaces -- Learning with 500k Labels on a Single Commodity GPU" (arXiv 2306.03725).
 * Sections cited below are the paper's.
 *
 * LAYOUT (all row-major, all DEVICE memory owned by the caller unless marked "host"):
 *   idx    [m][k]  int32    feature that feeds slot t of label j, 0-based, values in [0, d),
 *                           pairwise distinct within a row.  This is the transpose of the
 *                           paper's indices[s][m] (Section 3.2, Figure 1c); k is the paper's s.
 *   W      [m][k]  float32, or bfloat16 when the context was created with USL_BF16
 *   m1, m2 [m][k]  float32  Adam moments
 *   grad_W [m][k]  float32
 *   x      [b][d]  float32 / bfloat16 (same storage type as W)   activations (paper: features)
 *   grad_x [b][d]  float32
 *   out, g [b][m]  float32  scores and upstream gradient (paper: output, backward)
 *   targets        CSR: tgt_off[b+1] int64 (tgt_off[0] = 0), tgt_lab[tgt_off[b]] int32 label ids
 *
 * CALLS are asynchronous: they enqueue kernels on the context's stream and return.  The only
 * calls that wait for the stream are those handed a non-NULL host out-pointer.
 *
 * ERRORS: every call returns a usl_status; nothing aborts or throws across this boundary.
 * Preconditions that can be checked on the host (NULL pointers, batch outside [1, max_b],
 * k > d, fraction outside [0,1], t < 1, ...) are checked before anything is launched, and a
 * failed check launches nothing.  Index CONTENTS are the caller's responsibility on the hot
 * path (usl_validate_indices checks them).  Target label ids must lie in [0, m).
 * usl_last_error returns a context-owned message for the most recent failure.
 *
 * THREADS: a context is not thread-safe; use one context per host thread / stream.
 */
#ifndef USL_H
#define USL_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct usl_ctx usl_ctx; /* opaque: shape, storage type, stream, device scratch */

typedef enum {
    USL_OK = 0,
    USL_EINVAL = 1,       /* NULL pointer or a scalar argument out of range */
    USL_ESHAPE = 2,       /* sizes the library cannot take (k > d, b > max_b, m*k too large...) */
    USL_ENOMEM = 3,       /* host or device allocation failed */
    USL_EHIP = 4,         /* a HIP call failed (message in usl_last_error), or no GPU */
    USL_EUNSUPPORTED = 5, /* a valid request this build has no kernel for */
    USL_ESTALE = 6        /* usl_check: idx was rewritten without usl_invalidate (see there) */
} usl_status;

typedef enum { USL_F32 = 0, USL_BF16 = 1 } usl_dtype; /* storage of x and W; sums are float32 */

/* Create a context for a layer of m labels, input width d, fan-in k, batches of at most
 * max_b instances.  Limits: 1 <= k <= d <= 2^24, 1 <= m, m*k < 2^32, 1 <= max_b <= 65535.
 * Scratch that depends on the batch is sized for max_b when it is first needed, so that a later, larger
 * batch never makes a call reallocate (which would wait for the stream).
 * hip_stream is a hipStream_t (NULL = the null stream).  No device memory is touched until
 * the first call that launches; a context can be created on a host without a GPU. */
usl_status usl_create(usl_ctx** ctx, int64_t m, int32_t d, int32_t k, int32_t max_b,
                      usl_dtype storage, void* hip_stream);
usl_status usl_destroy(usl_ctx* ctx); /* frees the context and its device scratch; NULL is OK */
usl_status usl_set_stream(usl_ctx* ctx, void* hip_stream);
/* The library keeps private views of the connectivity (a column-major copy for usl_backward_input,
 * a per-label visiting order of the slots for the two other products), keyed by the idx pointer and
 * rebuilt after usl_init_indices / usl_redistribute / usl_redistribute_rows.  A caller that rewrites
 * the contents of idx by any other means must call this before the next product call: a stale
 * column-major copy gives wrong input gradients (a stale visiting order only costs speed). */
usl_status usl_invalidate(usl_ctx* ctx);
/* The address alone cannot tell an idx array from another one that an allocator later placed at the same
 * address, or from a checkpoint copied into it.  As a safety net every usl_backward_input on an address it
 * already has lists for re-reads a sample of idx (64 KiB) on the device and compares its fingerprint with the
 * one taken when the lists were built; on a mismatch that call fills grad_x with NaN instead of numbers from
 * stale lists, and the condition stays recorded (usl_backward and usl_train_step, where they take the weight
 * gradient from such lists too: grad_W becomes NaN as well, and usl_train_step leaves W, m1, m2 as they were).  usl_check waits for the stream and returns USL_ESTALE if
 * that happened since the last check (and invalidates the private views), USL_OK otherwise.  A change of a
 * single entry can escape the sample: usl_invalidate remains the contract, this is the net under it. */
usl_status usl_check(usl_ctx* ctx);
const char* usl_last_error(const usl_ctx* ctx); /* never NULL; owned by the context */
const char* usl_version(void);

/* Initial connectivity (Section 4.1: connections drawn uniformly at random, the same number
 * for every label).  Fills idx[m][k] with k distinct columns per row: the refill rule of
 * usl_redistribute applied to rows whose slots are all empty, with epoch = 2^64 - 1. */
usl_status usl_init_indices(usl_ctx* ctx, int32_t* idx, uint64_t seed);

/* Forward product (Section 3.2, Algorithm 1): out[i][j] = sum_t W[j][t] * x[i][idx[j][t]].
 * x: [b][d] storage type; W: [m][k] storage type; out: [b][m] float32, overwritten. */
usl_status usl_forward(usl_ctx* ctx, const void* x, const int32_t* idx, const void* W,
                       float* out, int32_t b);

/* One-vs-all binary cross-entropy summed over all labels (Section 2, sum of a binary loss
 * over labels; BCE is the comparison loss of Section 4.4), on sparse targets:
 *   y[i][j] = 1 iff j is listed for instance i (a set: repeats count once)
 *   loss = scale * sum_ij [ max(z,0) - z*y + log(1 + exp(-|z|)) ],  z = out[i][j]
 *   g[i][j] = scale * (sigmoid(z) - y)
 * g may be the same buffer as out.  loss: one float32 in device memory, overwritten. */
usl_status usl_bce_loss_grad(usl_ctx* ctx, const float* out, const int64_t* tgt_off,
                             const int32_t* tgt_lab, float scale, float* g, float* loss,
                             int32_t b);

/* usl_bce_loss_grad for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): same arguments, same kernels and bit-identical results,
 * but the per-block loss sums live in a static 1 MiB device array of the library instead of scratch that
 * the library allocates, and the call itself allocates and frees nothing (the context's first call on a
 * device, of any kind, reads the device properties and looks the array up).
 * Limit: ceil(m / 4096) * b <= 131072, else USL_ESHAPE and nothing is launched.
 * All contexts on one GPU share that GPU's array: two such calls that overlap in time on one GPU (different
 * streams) race; calls on one stream are ordered and safe.  Every call overwrites the slots it reads. */
usl_status usl_bce_loss_grad_noalloc(usl_ctx* ctx, const float* out, const int64_t* tgt_off,
                                     const int32_t* tgt_lab, float scale, float* g, float* loss,
                                     int32_t b);

/* One-vs-all squared hinge loss, the paper's main loss (Section 3.3), on the same sparse targets:
 *   s[i][j] = +1 iff j is listed for instance i, else -1
 *   loss = scale * sum_ij max(0, 1 - s*z)^2,   g[i][j] = scale * (-2 * s * max(0, 1 - s*z))
 * g is exactly zero wherever s*z >= 1 ("implicit negative mining"): usl_backward_weight and
 * usl_backward_input skip the work of zero entries of g (wavefront- and workgroup-wide in the
 * former, per 32-instance piece of a label's gradient in the latter); results are those of the
 * unskipped sums for finite inputs.  g may be the same buffer as out. */
usl_status usl_sqh_loss_grad(usl_ctx* ctx, const float* out, const int64_t* tgt_off,
                             const int32_t* tgt_lab, float scale, float* g, float* loss,
                             int32_t b);

/* Prediction (Section 2: the k highest-scoring labels are predicted positive).  For every instance
 * i < b, top_lab[i][r] and top_val[i][r] = out[i][top_lab[i][r]], r < kk, list the kk best labels of
 * row i of out[b][m], best first.  Label p ranks before q if out[i][p] > out[i][q], or the two scores
 * compare equal (-0 and +0 do) and p < q.  Scores must not be NaN.  1 <= kk <= min(m, 32).
 * top_lab [b][kk] int32, top_val [b][kk] float32, device memory, overwritten. */
usl_status usl_topk(usl_ctx* ctx, const float* out, int32_t b, int32_t kk, int32_t* top_lab,
                    float* top_val);

/* Prediction from the activations (Section 2: yhat = top_k(W^T psi(x))): usl_forward followed by usl_topk,
 * through scratch memory of the library (the caller never provides a [b][m] array); the scratch is held
 * to 1 GiB, or 64 instances if those take more, and a larger batch goes through it in chunks.
 * Arguments and results as for those two calls. */
usl_status usl_predict(usl_ctx* ctx, const void* x, const int32_t* idx, const void* W, int32_t b,
                       int32_t kk, int32_t* top_lab, float* top_val);

/* Precision at k (Section 2, the equation defining P@k = (1/k) sum_j y_j yhat_j): hits[r], r < kk,
 * is set to the number of instances i < b whose rank-r prediction top_lab[i][r] is one of the
 * instance's targets (a set: repeats count once), so P@k = (hits[0]+...+hits[k-1]) / (k*b) for every
 * k <= kk.  top_lab [b][kk] and hits [kk] (int64) are device memory; 1 <= kk <= 64. */
usl_status usl_precision_hits(usl_ctx* ctx, const int32_t* top_lab, const int64_t* tgt_off,
                              const int32_t* tgt_lab, int32_t b, int32_t kk, int64_t* hits);

/* Gradient of the connection values (Section 3.3, Algorithm 3):
 * grad_W[j][t] = sum_i g[i][j] * x[i][idx[j][t]].  grad_W is overwritten. */
usl_status usl_backward_weight(usl_ctx* ctx, const float* g, const void* x, const int32_t* idx,
                               float* grad_W, int32_t b);

/* Gradient of the input features (Section 3.3, Algorithm 2):
 * grad_x[i][c] = sum over connections (j,t) with idx[j][t] == c of W[j][t] * g[i][j].
 * grad_x is overwritten (not accumulated into).  The order of the additions is not fixed. */
usl_status usl_backward_input(usl_ctx* ctx, const float* g, const int32_t* idx, const void* W,
                              float* grad_x, int32_t b);

/* Both gradients of the backward pass in one call (Section 3.3, Algorithms 2 and 3): grad_W as usl_backward_weight
 * leaves it, grad_x as usl_backward_input does, from the same g [b][m], x [b][d], idx [m][k], W [m][k]; all device
 * pointers, grad_W [m][k] and grad_x [b][d] float32, both overwritten, neither may alias an input.  Where the shape
 * allows, every gathered g[i][j] serves both products (one pass over g instead of two); elsewhere the call is the
 * two separate ones.  Errors as for those: USL_EINVAL for a null pointer or b outside [1, max_b], USL_EHIP if a
 * launch fails.  The order of the additions is not fixed. */
usl_status usl_backward(usl_ctx* ctx, const float* g, const void* x, const int32_t* idx, const void* W,
                        float* grad_W, float* grad_x, int32_t b);

/* The three products restricted to a list of labels (Section 6, outlook: with the uniform format, scoring a
 * subset of labels, e.g. sampled negatives, is a slicing of the [m][k] arrays).  rows[n_rows]: int32
 * label ids in [0, m), device memory, any order, repeats allowed (each occurrence is its own row):
 *   out_rows   [b][n_rows]   out_rows[i][q]   = sum_t W[rows[q]][t] * x[i][idx[rows[q]][t]]
 *   grad_W_rows[n_rows][k]   grad_W_rows[q][t] = sum_i g_rows[i][q] * x[i][idx[rows[q]][t]]
 *   grad_x     [b][d]        grad_x[i][c]     = sum over (q,t) with idx[rows[q]][t] == c of
 *                                               W[rows[q]][t] * g_rows[i][q]       (overwritten)
 * g_rows is [b][n_rows].  1 <= n_rows, n_rows*k < 2^32.  The library copies the named rows of idx / W
 * into scratch on every call; scratch is sized by n_rows, so a run of calls with the same n_rows is
 * the fast case (a change of n_rows reallocates and waits for the stream). */
usl_status usl_forward_rows(usl_ctx* ctx, const void* x, const int32_t* idx, const void* W,
                            const int32_t* rows, int64_t n_rows, float* out_rows, int32_t b);
usl_status usl_backward_weight_rows(usl_ctx* ctx, const float* g_rows, const void* x,
                                    const int32_t* idx, const int32_t* rows, int64_t n_rows,
                                    float* grad_W_rows, int32_t b);
usl_status usl_backward_input_rows(usl_ctx* ctx, const float* g_rows, const int32_t* idx,
                                   const void* W, const int32_t* rows, int64_t n_rows,
                                   float* grad_x, int32_t b);

/* Adam (the optimizer of Section 4.1; update rule of Kingma & Ba, Algorithm 1) on the m*k
 * connection values, t = 1-based step number:
 *   m1 <- beta1*m1 + (1-beta1)*gW;  m2 <- beta2*m2 + (1-beta2)*gW^2
 *   W  <- W - lr * (m1/(1-beta1^t)) / (sqrt(m2/(1-beta2^t)) + eps)
 * With USL_BF16 the new W is rounded to bfloat16 (nearest even); moments stay float32. */
usl_status usl_adam_step(usl_ctx* ctx, void* W, const float* grad_W, float* m1, float* m2,
                         int64_t t, float lr, float beta1, float beta2, float eps);

/* One training step of the layer in one call: usl_forward, the loss (loss_kind 0 = binary
 * cross-entropy, 1 = squared hinge), usl_backward_weight, usl_backward_input and usl_adam_step, in that
 * order (Sections 3.2-3.3, 4.1), with the same arguments and the same results as the separate calls
 * (the loss value up to the order of its additions).  Fused inside: the loss writes the gradient in the
 * two layouts the backward products read, so no separate transposition pass runs.
 *   g      [b][m] float32  work and result: the scores, then the upstream gradient
 *   grad_W [m][k] float32  result: the gradient Adam consumed
 *   grad_x [b][d] float32  result, or NULL to skip the input gradient
 * W, m1, m2 are updated in place; grad_x is computed from W as it was before the update. */
usl_status usl_train_step(usl_ctx* ctx, const void* x, const int32_t* idx, void* W, float* m1, float* m2,
                          const int64_t* tgt_off, const int32_t* tgt_lab, int32_t loss_kind, float scale,
                          int64_t t, float lr, float beta1, float beta2, float eps, float* g,
                          float* grad_W, float* grad_x, float* loss, int32_t b);

/* Connection redistribution (Section 2: the prune / redistribute cycle of SET; Section 3.2:
 * a column's slots never move).  In place:
 *   1. n = floor(fraction * m*k) connections with the smallest magnitude in the whole layer are
 *      removed; the order is (bit pattern of |W|, flat slot number j*k+t), so +0 and -0 tie,
 *      NaN is never removed, and equal magnitudes go in slot order.
 *   2. every removed slot, row by row and in increasing t, takes a new column drawn uniformly
 *      from the features its row is not connected to (columns removed in step 1 are eligible
 *      again): candidate number a = 0,1,2,... is word 0 of Philox-4x32-10 with counter
 *      (j, t, a, epoch mod 2^32) and key (seed mod 2^32, (seed >> 32) xor (epoch >> 32)),
 *      mapped to a column by (word * d) >> 32, and the first candidate that differs from every
 *      occupied slot of the row is taken.
 *   3. a new connection starts with W = +0 and m1 = m2 = 0.
 * The result is a function of (idx, W, fraction, seed, epoch) only.  epoch 2^64-1 is reserved.
 * n_rewired_host: optional host pointer that receives n (known before launch: no wait). */
usl_status usl_redistribute(usl_ctx* ctx, int32_t* idx, void* W, float* m1, float* m2,
                            double fraction, uint64_t seed, uint64_t epoch,
                            int64_t* n_rewired_host);

/* The per-row variant of usl_redistribute (Section 2 does not say whether the prune fraction is taken
 * over the layer or over each unit; this is the second reading): every row loses its per_row
 * connections of smallest magnitude, order (bit pattern of |W|, slot t) -- so NaN goes last -- and the
 * emptied slots are refilled by steps 2 and 3 of usl_redistribute.  0 <= per_row <= k. */
usl_status usl_redistribute_rows(usl_ctx* ctx, int32_t* idx, void* W, float* m1, float* m2,
                                 int32_t per_row, uint64_t seed, uint64_t epoch);

/* Debug check of the uniform-sparsity invariant (Section 3.2): counts rows of idx that hold a
 * value outside [0, d) or the same column twice.  n_bad_host: host pointer; the call waits. */
usl_status usl_validate_indices(usl_ctx* ctx, const int32_t* idx, int64_t* n_bad_host);

/* Raw generator words for conformance tests: out[4*i .. 4*i+3] (device, uint32) receives
 * Philox-4x32-10 of counter ctr[4*i .. 4*i+3] (device) under key (key0, key1), i < n. */
usl_status usl_philox_words(usl_ctx* ctx, const uint32_t* ctr, uint32_t key0, uint32_t key1,
                            uint32_t* out, int64_t n);

#ifdef __cplusplus
}
#endif
#endif /* USL_H */
