// Internal declarations shared by the host layer and the kernel files of libusl.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "../../include/usl.h"

// Largest slice of LDS one workgroup uses to hold activation rows.  gfx950 has 160 KiB per
// compute unit; 128 KiB is one float32 row of 32768 features.
static constexpr int USL_ROW_LDS_BYTES = 128 * 1024;

struct usl_ctx {
    int64_t m;
    int32_t d, k, max_b;
    int storage;  // usl_dtype
    hipStream_t stream;
    int device;        // -1 until the first launch
    int num_cu;
    char err[512];

    // --- device scratch, allocated on first use, freed by usl_destroy ---
    double* bce_partials;     size_t bce_partials_cap;   // per-block loss sums
    uint32_t* sel_hist;       // radix-select histograms + state
    uint8_t* prune_flags;     // [m*k] 1 = slot removed by the current redistribution
    uint32_t* tie_counts;     size_t tie_counts_cap;
    int64_t* counter64;       // small device counter (validate)
    // transposed (column-major) connectivity for backward_input
    uint32_t* csc_ptr;        size_t csc_ptr_cap;     // [nwin*d+1] start of each (window, feature) list
    uint32_t* csc_cursor;     size_t csc_cursor_cap;  // [nwin*d]
    uint32_t* csc_order;      size_t csc_order_cap;   // [3][nwin*d] features of each window by falling list length; rank of each feature; list length by rank
    uint32_t* csc_slot;       // [m*k] flat slot j*k+t, grouped by (label window, feature)
    float* csc_w;             // [m*k] W of that slot (refreshed by every backward_input)
    uint64_t* idx_print;      // [0] fingerprint of idx when the lists were built; word [2] (32 bits): 1 = a later call found idx changed
    const int32_t* idx_to_check;  // idx whose fingerprint the next weight gather compares (NULL right after a build)
    int csc_win_labels;       // labels per window the lists were built with
    const int32_t* csc_built_for;  // idx pointer the lists were built from (NULL = stale)
    // bank-aware order in which a label's slots are visited by the LDS gathers (performance only)
    uint8_t* slot_order;           // [m*k] slot read at step s
    const int32_t* slot_order_for; // idx pointer it was computed from (NULL = stale)
    float* gT;                size_t gT_cap;   // [tiles][m][32] upstream gradient, one 128-byte piece per (tile of 32 instances, label)
    uint8_t* nz_flags;        size_t nz_flags_cap;   // [tiles][m] 1 = that 32-instance piece of gT is not all zero
    // label-subset calls: a child context sized for the subset, and the subset's rows of idx / W
    usl_ctx* sub;
    int32_t* sub_idx;         size_t sub_idx_cap;
    void* sub_W;              size_t sub_W_cap;
    float* predict_out;       size_t predict_out_cap;   // [chunk][m] scores of usl_predict, one chunk of instances at a time
    uint64_t* topk_cand;      size_t topk_cand_cap;  // [b][segments][kk] packed (score, label) keys
    float* gw_part;           size_t gw_part_cap;   // [groups][m*k] partial weight gradients of a split batch
    float* gxT;               size_t gxT_cap;  // [tiles][d][32] input gradient in the same layout
    // per-instance lists of the nonzero entries of g (k_sparse_grad.hip)
    uint32_t* nz_state;       size_t nz_state_cap;   // [0] = 1: gradient is dense, lists abandoned; [16+i] = entries of instance i
    int32_t* nz_lab;          size_t nz_lab_cap;     // [max_b][m/32] label of an entry
    float* nz_val;            size_t nz_val_cap;     // [max_b][m/32] its gradient
    const float* nz_lists_of; // g that has just been looked at (only set inside usl_train_step), else NULL
    bool nz_lists_tried;      // ... and whether lists were built for it (else only the dense kernels run)
    uint32_t* hint_host;      // pinned: [0] serial of the last finished look at a gradient sample, [1] 1 = it was dense
    uint32_t* hint_dev;       // the same words as the device addresses them
    uint32_t hint_seen, probe_serial;
    int sparse_streak;        // looks in a row that found the sample sparse
    // the register-list form of the input gradient (k_backward_input_lds.hip): [0] lists of 68 slots per lane from
    // windows of up to 32768 labels, for usl_backward_input; [1] lists of 36 slots from windows of half that length, for
    // the kernel of usl_train_step that computes the weight gradient from the same gathers
    struct usl_lf {
        uint32_t* count;      size_t count_cap;    // [nwin*d] list lengths
        uint32_t* taken;      size_t taken_cap;    // [nwin*d] positions handed out while filling
        uint32_t* where;      size_t where_cap;    // [nwin*d] where a feature's list starts among its workgroup's entries
        uint16_t* feat;       size_t feat_cap;     // [wg][2][1024] feature of a lane's list
        uint32_t* caps;       size_t caps_cap;     // [wg][16] slots the wavefronts visit
        uint32_t* ov_base;    size_t ov_base_cap;  // [wg+1] start of a workgroup's overflow entries, [wg] their number; the same two for all its entries
        uint32_t* ovr;        size_t ovr_cap;      // [wg][2][1024] a lane's lists' share of the overflow entries held in LDS
        uint16_t* lab;        size_t lab_cap;      // [wg][slots][1024] label within the window
        uint32_t* slot;       size_t slot_cap;     // [wg][slots][1024] flat slot j*k+t (where the weight lives)
        uint32_t* ent;        size_t ent_cap;      // [m*k] flat slots grouped by (workgroup, feature), before the bank-aware order
        uint32_t* ovoff;      size_t ovoff_cap;    // [nwin*d] where a list's overflow starts in its workgroup's
        void* ov;             size_t ov_cap;       // overflow entries
        float* stage;         size_t stage_cap;    // [1] only: the weight gradient in list order, [wg][slots][1024], then one per overflow entry
        uint32_t* pos;        size_t pos_cap;      // [1] only: [m*k] where a slot's weight gradient is in stage
        float* partial;       size_t partial_cap;  // [nwin][rows of a pass][d]
        const int32_t* built_for;                  // idx pointer the lists were built from (NULL = stale)
    } lf[2];
};

#define USL_FAIL(ctx, code, ...)                                   \
    do {                                                           \
        snprintf((ctx)->err, sizeof((ctx)->err), __VA_ARGS__);     \
        return (code);                                             \
    } while (0)

#define USL_HIP(ctx, call)                                                              \
    do {                                                                                \
        hipError_t e_ = (call);                                                         \
        if (e_ != hipSuccess)                                                           \
            USL_FAIL(ctx, USL_EHIP, "%s failed: %s", #call, hipGetErrorString(e_));     \
    } while (0)

#define USL_TRY(expr)                     \
    do {                                  \
        usl_status s_ = (expr);           \
        if (s_ != USL_OK) return s_;      \
    } while (0)

// Makes the device current on first use and reads its compute-unit count.
usl_status usl_prepare_device(usl_ctx* ctx);
// Grows *buf to at least `bytes` (old contents are dropped).
usl_status usl_reserve(usl_ctx* ctx, void** buf, size_t* cap, size_t bytes);
usl_status usl_check_launch(usl_ctx* ctx, const char* what);

usl_status usl_build_slot_order(usl_ctx* ctx, const int32_t* idx);

// Kernel launchers (one per file).  All take validated arguments.
usl_status usl_launch_forward(usl_ctx* ctx, const void* x, const int32_t* idx, const void* W,
                              float* out, int32_t b);
// dense = the caller knows that g holds (almost) no exact zeros: the zero-skipping tests are left out
usl_status usl_launch_backward_weight(usl_ctx* ctx, const float* g, const void* x,
                                      const int32_t* idx, float* grad_W, int32_t b, bool dense = false);
usl_status usl_launch_backward_input(usl_ctx* ctx, const float* g, const int32_t* idx,
                                     const void* W, float* grad_x, int32_t b);
// The products over the nonzero entries of g only (k_sparse_grad.hip).  usl_sparse_compact builds the lists (or
// finds g dense); *gate is a device word, 0 = the lists stand and the sparse kernels do the work, 1 = the dense
// kernels have to.  Dense kernels that are handed the gate leave at once when it reads 0.
bool usl_sparse_supported(const usl_ctx* ctx);
bool usl_sparse_expected(usl_ctx* ctx);
usl_status usl_sparse_compact(usl_ctx* ctx, const float* g, int32_t b, const uint32_t** gate);
usl_status usl_sparse_backward_weight(usl_ctx* ctx, const void* x, const int32_t* idx, float* grad_W, int32_t b);
usl_status usl_sparse_backward_input(usl_ctx* ctx, const int32_t* idx, const void* W, float* grad_x, int32_t b);
// backward_input in pieces, for callers that produce gT / nz_flags / the nonzero count themselves, one group of
// at most usl_bwd_input_group_rows() instances at a time
int usl_bwd_input_group_rows(void);
usl_status usl_bwd_input_prepare(usl_ctx* ctx, const int32_t* idx, int32_t b);
usl_status usl_bwd_input_gather_w(usl_ctx* ctx, const void* W, const uint32_t* gate);
usl_status usl_bwd_input_begin_group(usl_ctx* ctx);
usl_status usl_bwd_input_group(usl_ctx* ctx, float* grad_x_rows, int32_t rows, uint64_t sampled_labels,
                               const uint32_t* gate);
// The same product with the lists of each (label window, 2048 features) held in registers and the rows of g staged
// through LDS (k_backward_input_lds.hip); applies to shapes with about 32 connections per (window, feature).
bool usl_bwi_lds_applies(const usl_ctx* ctx);
usl_status usl_bwi_lds_run(usl_ctx* ctx, const float* g, const int32_t* idx, const void* W, float* grad_x, int32_t b,
                           const uint32_t* gate);
// Both backward products from one pass of gathers through register lists of half the length (k_backward_input_lds.hip):
// grad_W[m][k] and grad_x[b][d] from g[b][m] and x[b][d]; for layers with k / d <= 1/1024, one pass over the batch.
bool usl_both_lds_applies(const usl_ctx* ctx);
usl_status usl_both_lds_run(usl_ctx* ctx, const float* g, const void* x, const int32_t* idx, const void* W, float* grad_x,
                            int32_t b, const uint32_t* gate, const float** stage, const uint32_t** pos, const uint32_t** stale);
// grad_W[f] = stage[pos[f]] (behind a zero gate: nothing, the kernels over the listed nonzeros wrote grad_W)
usl_status usl_launch_unstage(usl_ctx* ctx, const float* stage, const uint32_t* pos, const uint32_t* gate, const uint32_t* stale,
                              float* grad_W);
usl_status usl_launch_adam_staged(usl_ctx* ctx, void* W, const float* stage, const uint32_t* pos, const uint32_t* gate,
                                  const uint32_t* stale, float* grad_W, float* m1, float* m2, float lr, float beta1, float beta2, float eps,
                                  float inv_c1, float inv_c2);
// Records (store = 1) the fingerprint of idx in ctx->idx_print, or compares with the recorded one (store = 0) and
// raises the stale word (32-bit word 4 of idx_print) on a difference.
usl_status usl_idx_fingerprint(usl_ctx* ctx, const int32_t* idx, int store);
static inline uint32_t* usl_nz_cells(usl_ctx* c) { return reinterpret_cast<uint32_t*>(c->counter64) + 4; }
// Loss and gradient in place on zg[b][m], which also leaves the gradient in c->gT (tile-major) with
// its piece flags and sampled nonzero count (usl_bwd_input_prepare must have run); *sampled_labels
// receives the number of labels the count covers.
// One call per group of instances [row0, row0 + rows) (row0 a multiple of 32); the call for the last group also
// sums the loss over the whole batch of b instances.
usl_status usl_launch_loss_tiles(usl_ctx* ctx, int loss_kind, float* zg, const int64_t* tgt_off,
                                 const int32_t* tgt_lab, float scale, float* loss, int32_t b,
                                 uint64_t* sampled_labels, int32_t row0, int32_t rows);
// loss_kind: 0 = binary cross-entropy, 1 = squared hinge
usl_status usl_launch_loss(usl_ctx* ctx, int loss_kind, const float* out, const int64_t* tgt_off,
                           const int32_t* tgt_lab, float scale, float* g, float* loss, int32_t b);
// the same loss through the static scratch array (no allocation); usl_noalloc_setup runs once per device
usl_status usl_noalloc_setup(usl_ctx* ctx);
usl_status usl_launch_loss_noalloc(usl_ctx* ctx, int loss_kind, const float* out, const int64_t* tgt_off,
                                   const int32_t* tgt_lab, float scale, float* g, float* loss, int32_t b);
usl_status usl_launch_adam(usl_ctx* ctx, void* W, const float* grad_W, float* m1, float* m2,
                           float lr, float beta1, float beta2, float eps, float inv_c1,
                           float inv_c2);
usl_status usl_launch_redistribute(usl_ctx* ctx, int32_t* idx, void* W, float* m1, float* m2,
                                   int64_t n, uint64_t seed, uint64_t epoch);
usl_status usl_launch_redistribute_rows(usl_ctx* ctx, int32_t* idx, void* W, float* m1, float* m2,
                                        int32_t per_row, uint64_t seed, uint64_t epoch);
usl_status usl_launch_init_indices(usl_ctx* ctx, int32_t* idx, uint64_t seed);
usl_status usl_launch_topk(usl_ctx* ctx, const float* out, int32_t b, int32_t kk, int32_t* top_lab,
                           float* top_val);
usl_status usl_launch_precision_hits(usl_ctx* ctx, const int32_t* top_lab, const int64_t* tgt_off,
                                     const int32_t* tgt_lab, int32_t b, int32_t kk, int64_t* hits);
int usl_topk_max(void);
// dst_idx[q][:] = idx[rows[q]][:] and (if W) dst_W[q][:] = W[rows[q]][:], q < n; row ids are clamped into [0, m)
usl_status usl_launch_gather_rows(usl_ctx* ctx, const int32_t* idx, const void* W, const int32_t* rows,
                                  int64_t n, int32_t* dst_idx, void* dst_W);  // largest kk usl_launch_topk takes
usl_status usl_launch_validate(usl_ctx* ctx, const int32_t* idx, int64_t* n_bad_host);
usl_status usl_launch_philox(usl_ctx* ctx, const uint32_t* ctr, uint32_t key0, uint32_t key1,
                             uint32_t* out, int64_t n);

// ---- small device helpers -------------------------------------------------------------------
__device__ __forceinline__ float usl_bf16_to_f32(uint16_t v) {
    return __uint_as_float((uint32_t)v << 16);
}
__device__ __forceinline__ uint16_t usl_f32_to_bf16(float f) {  // nearest, ties to even
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x0040u);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
template <typename TS> __device__ __forceinline__ float usl_load_f32(const TS* p, size_t i);
template <> __device__ __forceinline__ float usl_load_f32<float>(const float* p, size_t i) {
    return p[i];
}
template <> __device__ __forceinline__ float usl_load_f32<uint16_t>(const uint16_t* p, size_t i) {
    return usl_bf16_to_f32(p[i]);
}
