// Host layer of libusl: the C ABI, argument checks, context and scratch management.
#include <math.h>
#include <stdlib.h>

#include "usl_internal.h"

extern "C" const char* usl_version(void) { return "usl 0.1 (gfx950)"; }

extern "C" usl_status usl_create(usl_ctx** out, int64_t m, int32_t d, int32_t k, int32_t max_b,
                                 usl_dtype storage, void* hip_stream) {
    if (!out) return USL_EINVAL;
    *out = nullptr;
    if (storage != USL_F32 && storage != USL_BF16) return USL_EINVAL;
    if (m < 1 || d < 1 || k < 1 || max_b < 1) return USL_EINVAL;
    if (k > d || d > (1 << 24) || m > 0x7FFFFFFFll) return USL_ESHAPE;
    if (max_b > 65535) return USL_ESHAPE;   // the instance is a grid dimension of several kernels
    if (m * (int64_t)k >= (int64_t)1 << 32) return USL_ESHAPE;
    usl_ctx* c = (usl_ctx*)calloc(1, sizeof(usl_ctx));
    if (!c) return USL_ENOMEM;
    c->m = m; c->d = d; c->k = k; c->max_b = max_b;
    c->storage = (int)storage;
    c->stream = (hipStream_t)hip_stream;
    c->device = -1;
    c->err[0] = 0;
    *out = c;
    return USL_OK;
}

extern "C" usl_status usl_destroy(usl_ctx* c) {
    if (!c) return USL_OK;
    (void)usl_destroy(c->sub);
    if (c->device >= 0) {
        void* bufs[] = {c->bce_partials, c->sel_hist, c->prune_flags, c->tie_counts, c->counter64,
                        c->csc_ptr, c->csc_cursor, c->csc_order, c->csc_slot, c->csc_w, c->gT, c->gxT, c->nz_flags,
                        c->slot_order, c->topk_cand, c->sub_idx, c->sub_W, c->predict_out, c->gw_part,
                        c->nz_state, c->nz_lab, c->nz_val, c->idx_print};
        (void)hipStreamSynchronize(c->stream);
        for (void* p : bufs)
            if (p) (void)hipFree(p);
        for (auto& L : c->lf) {
            void* lists[] = {L.count, L.taken, L.where, L.feat, L.caps, L.ov_base, L.ovr, L.lab, L.slot, L.ent, L.ovoff,
                             L.ov, L.stage, L.pos, L.partial};
            for (void* p : lists)
                if (p) (void)hipFree(p);
        }
        if (c->hint_host) (void)hipHostFree(c->hint_host);
    }
    free(c);
    return USL_OK;
}

extern "C" usl_status usl_set_stream(usl_ctx* c, void* hip_stream) {
    if (!c) return USL_EINVAL;
    c->stream = (hipStream_t)hip_stream;
    return USL_OK;
}

extern "C" const char* usl_last_error(const usl_ctx* c) { return c ? c->err : "null context"; }

extern "C" usl_status usl_invalidate(usl_ctx* c) {
    if (!c) return USL_EINVAL;
    c->csc_built_for = nullptr;
    c->lf[0].built_for = c->lf[1].built_for = nullptr;
    c->slot_order_for = nullptr;
    return USL_OK;
}

usl_status usl_prepare_device(usl_ctx* c) {
    if (c->device >= 0) return USL_OK;
    int n = 0;
    hipError_t e = hipGetDeviceCount(&n);
    if (e != hipSuccess || n < 1) USL_FAIL(c, USL_EHIP, "no HIP device available");
    int dev = 0;
    USL_HIP(c, hipGetDevice(&dev));
    hipDeviceProp_t p;
    USL_HIP(c, hipGetDeviceProperties(&p, dev));
    if ((size_t)p.sharedMemPerBlock < (size_t)USL_ROW_LDS_BYTES + 1024)
        USL_FAIL(c, USL_EUNSUPPORTED, "device offers %zu bytes of LDS per workgroup, need %d",
                 (size_t)p.sharedMemPerBlock, USL_ROW_LDS_BYTES + 1024);
    c->num_cu = p.multiProcessorCount;
    c->device = dev;
    return usl_noalloc_setup(c);   // where this device holds the static scratch of the no-allocation call
}

usl_status usl_reserve(usl_ctx* c, void** buf, size_t* cap, size_t bytes) {
    if (*buf && *cap >= bytes) return USL_OK;
    if (*buf) {
        USL_HIP(c, hipStreamSynchronize(c->stream));
        USL_HIP(c, hipFree(*buf));
        *buf = nullptr;
        *cap = 0;
    }
    hipError_t e = hipMalloc(buf, bytes);
    if (e != hipSuccess) {
        *buf = nullptr;
        USL_FAIL(c, USL_ENOMEM, "hipMalloc of %zu bytes failed: %s", bytes, hipGetErrorString(e));
    }
    *cap = bytes;
    return USL_OK;
}

usl_status usl_check_launch(usl_ctx* c, const char* what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) USL_FAIL(c, USL_EHIP, "launch of %s failed: %s", what, hipGetErrorString(e));
    return USL_OK;
}

static usl_status check_batch(usl_ctx* c, int32_t b) {
    if (b < 1) USL_FAIL(c, USL_EINVAL, "batch size %d < 1", b);
    if (b > c->max_b) USL_FAIL(c, USL_ESHAPE, "batch size %d exceeds max_b %d", b, c->max_b);
    return USL_OK;
}

#define NEED(ptr)                                                          \
    do {                                                                   \
        if (!(ptr)) USL_FAIL(c, USL_EINVAL, "argument %s is NULL", #ptr);  \
    } while (0)

extern "C" usl_status usl_init_indices(usl_ctx* c, int32_t* idx, uint64_t seed) {
    if (!c) return USL_EINVAL;
    NEED(idx);
    USL_TRY(usl_prepare_device(c));
    c->csc_built_for = nullptr;
    c->lf[0].built_for = c->lf[1].built_for = nullptr;
    c->slot_order_for = nullptr;
    return usl_launch_init_indices(c, idx, seed);
}

extern "C" usl_status usl_forward(usl_ctx* c, const void* x, const int32_t* idx, const void* W,
                                  float* out, int32_t b) {
    if (!c) return USL_EINVAL;
    NEED(x); NEED(idx); NEED(W); NEED(out);
    USL_TRY(check_batch(c, b));
    USL_TRY(usl_prepare_device(c));
    return usl_launch_forward(c, x, idx, W, out, b);
}

extern "C" usl_status usl_bce_loss_grad(usl_ctx* c, const float* out, const int64_t* tgt_off,
                                        const int32_t* tgt_lab, float scale, float* g, float* loss,
                                        int32_t b) {
    if (!c) return USL_EINVAL;
    NEED(out); NEED(tgt_off); NEED(tgt_lab); NEED(g); NEED(loss);
    if (!(scale == scale) || isinf(scale)) USL_FAIL(c, USL_EINVAL, "scale is not finite");
    USL_TRY(check_batch(c, b));
    USL_TRY(usl_prepare_device(c));
    return usl_launch_loss(c, 0, out, tgt_off, tgt_lab, scale, g, loss, b);
}

extern "C" usl_status usl_bce_loss_grad_noalloc(usl_ctx* c, const float* out, const int64_t* tgt_off,
                                                const int32_t* tgt_lab, float scale, float* g, float* loss,
                                                int32_t b) {
    if (!c) return USL_EINVAL;
    NEED(out); NEED(tgt_off); NEED(tgt_lab); NEED(g); NEED(loss);
    if (!(scale == scale) || isinf(scale)) USL_FAIL(c, USL_EINVAL, "scale is not finite");
    USL_TRY(check_batch(c, b));
    USL_TRY(usl_prepare_device(c));
    return usl_launch_loss_noalloc(c, 0, out, tgt_off, tgt_lab, scale, g, loss, b);
}

extern "C" usl_status usl_sqh_loss_grad(usl_ctx* c, const float* out, const int64_t* tgt_off,
                                        const int32_t* tgt_lab, float scale, float* g, float* loss,
                                        int32_t b) {
    if (!c) return USL_EINVAL;
    NEED(out); NEED(tgt_off); NEED(tgt_lab); NEED(g); NEED(loss);
    if (!(scale == scale) || isinf(scale)) USL_FAIL(c, USL_EINVAL, "scale is not finite");
    USL_TRY(check_batch(c, b));
    USL_TRY(usl_prepare_device(c));
    return usl_launch_loss(c, 1, out, tgt_off, tgt_lab, scale, g, loss, b);
}

extern "C" usl_status usl_topk(usl_ctx* c, const float* out, int32_t b, int32_t kk, int32_t* top_lab,
                               float* top_val) {
    if (!c) return USL_EINVAL;
    NEED(out); NEED(top_lab); NEED(top_val);
    USL_TRY(check_batch(c, b));
    if (kk < 1) USL_FAIL(c, USL_EINVAL, "kk = %d, must be at least 1", kk);
    if (kk > c->m || kk > usl_topk_max())
        USL_FAIL(c, USL_ESHAPE, "kk = %d, this build takes at most min(m, %d)", kk, usl_topk_max());
    USL_TRY(usl_prepare_device(c));
    return usl_launch_topk(c, out, b, kk, top_lab, top_val);
}

extern "C" usl_status usl_predict(usl_ctx* c, const void* x, const int32_t* idx, const void* W, int32_t b,
                                  int32_t kk, int32_t* top_lab, float* top_val) {
    if (!c) return USL_EINVAL;
    NEED(x); NEED(idx); NEED(W); NEED(top_lab); NEED(top_val);
    USL_TRY(check_batch(c, b));
    if (kk < 1) USL_FAIL(c, USL_EINVAL, "kk = %d, must be at least 1", kk);
    if (kk > c->m || kk > usl_topk_max())
        USL_FAIL(c, USL_ESHAPE, "kk = %d, this build takes at most min(m, %d)", kk, usl_topk_max());
    USL_TRY(usl_prepare_device(c));
    // the scores live in a scratch array of the library, never in a [b][m] array of the caller; it is capped
    // at 1 GiB (at least 64 instances), so a large batch goes through in chunks: fewer chunks are faster
    // (every forward launch brings idx and W into registers again), 64 instances still amortise that well
    size_t cap_bytes = (size_t)1 << 30;
    if (const char* e = getenv("USL_TUNE_PREDICT_BYTES")) {   // a test aid: a small cap exercises the chunking
        const long long v = atoll(e);
        if (v > 0) cap_bytes = (size_t)v;
    }
    const int64_t cap_rows = (int64_t)(cap_bytes / ((size_t)c->m * 4));
    const int chunk = (int)(b <= 64 || cap_rows >= b ? b : (cap_rows < 64 ? 64 : cap_rows));
    const int mb = c->max_b;   // the scratch takes the chunk of the largest batch, so that no later call has to grow it
    const int chunk_max = (int)(mb <= 64 || cap_rows >= mb ? mb : (cap_rows < 64 ? 64 : cap_rows));
    USL_TRY(usl_reserve(c, (void**)&c->predict_out, &c->predict_out_cap, (size_t)chunk_max * c->m * 4));
    const size_t xrow = (size_t)c->d * (c->storage == USL_F32 ? 4 : 2);
    for (int i0 = 0; i0 < b; i0 += chunk) {
        const int n = b - i0 < chunk ? b - i0 : chunk;
        USL_TRY(usl_launch_forward(c, (const char*)x + (size_t)i0 * xrow, idx, W, c->predict_out, n));
        USL_TRY(usl_launch_topk(c, c->predict_out, n, kk, top_lab + (size_t)i0 * kk, top_val + (size_t)i0 * kk));
    }
    return USL_OK;
}

extern "C" usl_status usl_precision_hits(usl_ctx* c, const int32_t* top_lab, const int64_t* tgt_off,
                                         const int32_t* tgt_lab, int32_t b, int32_t kk, int64_t* hits) {
    if (!c) return USL_EINVAL;
    NEED(top_lab); NEED(tgt_off); NEED(tgt_lab); NEED(hits);
    USL_TRY(check_batch(c, b));
    if (kk < 1) USL_FAIL(c, USL_EINVAL, "kk = %d, must be at least 1", kk);
    if (kk > 64) USL_FAIL(c, USL_ESHAPE, "kk = %d, this build counts at most 64 ranks", kk);
    USL_TRY(usl_prepare_device(c));
    return usl_launch_precision_hits(c, top_lab, tgt_off, tgt_lab, b, kk, hits);
}

extern "C" usl_status usl_backward_weight(usl_ctx* c, const float* g, const void* x,
                                          const int32_t* idx, float* grad_W, int32_t b) {
    if (!c) return USL_EINVAL;
    NEED(g); NEED(x); NEED(idx); NEED(grad_W);
    USL_TRY(check_batch(c, b));
    USL_TRY(usl_prepare_device(c));
    return usl_launch_backward_weight(c, g, x, idx, grad_W, b);
}

extern "C" usl_status usl_backward_input(usl_ctx* c, const float* g, const int32_t* idx,
                                         const void* W, float* grad_x, int32_t b) {
    if (!c) return USL_EINVAL;
    NEED(g); NEED(idx); NEED(W); NEED(grad_x);
    USL_TRY(check_batch(c, b));
    USL_TRY(usl_prepare_device(c));
    return usl_launch_backward_input(c, g, idx, W, grad_x, b);
}

// ---- label-subset calls: the rows named by `rows` are copied out and run through the same kernels
// in a child context whose m is the subset size.

static usl_status subset_context(usl_ctx* c, int64_t n, const int32_t* idx, const void* W,
                                 const int32_t* rows, bool need_W, usl_ctx** child) {
    if (n < 1) USL_FAIL(c, USL_EINVAL, "n_rows = %lld < 1", (long long)n);
    if (n > 0x7FFFFFFFll || n * (int64_t)c->k >= (int64_t)1 << 32)
        USL_FAIL(c, USL_ESHAPE, "n_rows = %lld is too large", (long long)n);
    USL_TRY(usl_prepare_device(c));
    if (c->sub && c->sub->m != n) {   // scratch is sized by m: a new subset size starts afresh
        USL_TRY(usl_destroy(c->sub));
        c->sub = nullptr;
    }
    if (!c->sub) {
        usl_status s = usl_create(&c->sub, n, c->d, c->k, c->max_b, (usl_dtype)c->storage, c->stream);
        if (s != USL_OK) USL_FAIL(c, s, "could not create the context of a %lld-label subset", (long long)n);
    }
    usl_ctx* sub = c->sub;
    sub->stream = c->stream;
    usl_status s = usl_prepare_device(sub);
    if (s != USL_OK) USL_FAIL(c, s, "%s", sub->err);
    sub->csc_built_for = nullptr;
    sub->lf[0].built_for = sub->lf[1].built_for = nullptr;    // same scratch pointer, new contents
    sub->slot_order_for = nullptr;
    const size_t esize = c->storage == USL_F32 ? 4 : 2;
    USL_TRY(usl_reserve(c, (void**)&c->sub_idx, &c->sub_idx_cap, (size_t)n * c->k * 4));
    if (need_W) USL_TRY(usl_reserve(c, &c->sub_W, &c->sub_W_cap, (size_t)n * c->k * esize));
    USL_TRY(usl_launch_gather_rows(c, idx, need_W ? W : nullptr, rows, n, c->sub_idx, need_W ? c->sub_W : nullptr));
    *child = sub;
    return USL_OK;
}

#define SUB_TRY(expr)                                             \
    do {                                                          \
        usl_status s_ = (expr);                                   \
        if (s_ != USL_OK) USL_FAIL(c, s_, "%s", sub->err);        \
    } while (0)

// Both backward products of one g.  The nonzeros of g are listed once where the context expects few (as in
// usl_train_step); the kernels over the lists and the dense ones stand on either side of the gate.
static usl_status backward_both(usl_ctx* c, const float* g, const void* x, const int32_t* idx, const void* W, float* grad_W,
                                float* grad_x, int32_t b, bool lists, bool dense, const uint32_t** gate_out,
                                const float** stage, const uint32_t** pos, const uint32_t** stale) {
    const uint32_t* gate = nullptr;
    if (lists) USL_TRY(usl_sparse_compact(c, g, b, &gate));
    c->nz_lists_of = g;
    c->nz_lists_tried = gate != nullptr;
    usl_status s = USL_OK;
    *stage = nullptr;
    *pos = nullptr;
    if (usl_both_lds_applies(c) && (uintptr_t)g % 16 == 0 && (uintptr_t)grad_x % 16 == 0 && (uintptr_t)x % 16 == 0) {
        // both products from one pass of gathers over the rows of g (k_backward_input_lds.hip); behind the gate like
        // the two dense kernels it stands for.  The weight gradient is left in the order of the lists.
        if (gate) s = usl_sparse_backward_weight(c, x, idx, grad_W, b);
        if (gate && s == USL_OK) s = usl_sparse_backward_input(c, idx, W, grad_x, b);
        if (s == USL_OK) s = usl_both_lds_run(c, g, x, idx, W, grad_x, b, gate, stage, pos, stale);
    } else {
        s = usl_launch_backward_weight(c, g, x, idx, grad_W, b, dense);
        if (s == USL_OK) s = usl_launch_backward_input(c, g, idx, W, grad_x, b);
    }
    c->nz_lists_of = nullptr;
    *gate_out = gate;
    return s;
}

extern "C" usl_status usl_backward(usl_ctx* c, const float* g, const void* x, const int32_t* idx, const void* W,
                                   float* grad_W, float* grad_x, int32_t b) {
    if (!c) return USL_EINVAL;
    NEED(g); NEED(x); NEED(idx); NEED(W); NEED(grad_W); NEED(grad_x);
    USL_TRY(check_batch(c, b));
    USL_TRY(usl_prepare_device(c));
    const uint32_t* gate = nullptr;
    const float* stage = nullptr;
    const uint32_t* pos = nullptr;
    const uint32_t* stale = nullptr;
    USL_TRY(backward_both(c, g, x, idx, W, grad_W, grad_x, b, usl_sparse_supported(c), false, &gate, &stage, &pos, &stale));
    if (stage) USL_TRY(usl_launch_unstage(c, stage, pos, gate, stale, grad_W));
    return USL_OK;
}

extern "C" usl_status usl_forward_rows(usl_ctx* c, const void* x, const int32_t* idx, const void* W,
                                       const int32_t* rows, int64_t n_rows, float* out_rows, int32_t b) {
    if (!c) return USL_EINVAL;
    NEED(x); NEED(idx); NEED(W); NEED(rows); NEED(out_rows);
    USL_TRY(check_batch(c, b));
    usl_ctx* sub = nullptr;
    USL_TRY(subset_context(c, n_rows, idx, W, rows, true, &sub));
    SUB_TRY(usl_launch_forward(sub, x, c->sub_idx, c->sub_W, out_rows, b));
    return USL_OK;
}

extern "C" usl_status usl_backward_weight_rows(usl_ctx* c, const float* g_rows, const void* x,
                                               const int32_t* idx, const int32_t* rows, int64_t n_rows,
                                               float* grad_W_rows, int32_t b) {
    if (!c) return USL_EINVAL;
    NEED(g_rows); NEED(x); NEED(idx); NEED(rows); NEED(grad_W_rows);
    USL_TRY(check_batch(c, b));
    usl_ctx* sub = nullptr;
    USL_TRY(subset_context(c, n_rows, idx, nullptr, rows, false, &sub));
    SUB_TRY(usl_launch_backward_weight(sub, g_rows, x, c->sub_idx, grad_W_rows, b));
    return USL_OK;
}

extern "C" usl_status usl_backward_input_rows(usl_ctx* c, const float* g_rows, const int32_t* idx,
                                              const void* W, const int32_t* rows, int64_t n_rows,
                                              float* grad_x, int32_t b) {
    if (!c) return USL_EINVAL;
    NEED(g_rows); NEED(idx); NEED(W); NEED(rows); NEED(grad_x);
    USL_TRY(check_batch(c, b));
    usl_ctx* sub = nullptr;
    USL_TRY(subset_context(c, n_rows, idx, W, rows, true, &sub));
    SUB_TRY(usl_launch_backward_input(sub, g_rows, c->sub_idx, c->sub_W, grad_x, b));
    return USL_OK;
}

extern "C" usl_status usl_adam_step(usl_ctx* c, void* W, const float* grad_W, float* m1, float* m2,
                                    int64_t t, float lr, float beta1, float beta2, float eps) {
    if (!c) return USL_EINVAL;
    NEED(W); NEED(grad_W); NEED(m1); NEED(m2);
    if (t < 1) USL_FAIL(c, USL_EINVAL, "step number t=%lld < 1", (long long)t);
    if (!(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f))
        USL_FAIL(c, USL_EINVAL, "beta1/beta2 must lie in [0,1)");
    if (!(eps >= 0.f) || !(lr == lr)) USL_FAIL(c, USL_EINVAL, "eps < 0 or lr is NaN");
    USL_TRY(usl_prepare_device(c));
    // bias corrections in double on the host; the kernel multiplies by their reciprocals
    double c1 = 1.0 - pow((double)beta1, (double)t);
    double c2 = 1.0 - pow((double)beta2, (double)t);
    return usl_launch_adam(c, W, grad_W, m1, m2, lr, beta1, beta2, eps, (float)(1.0 / c1),
                           (float)(1.0 / c2));
}

extern "C" usl_status usl_train_step(usl_ctx* c, const void* x, const int32_t* idx, void* W, float* m1,
                                     float* m2, const int64_t* tgt_off, const int32_t* tgt_lab,
                                     int32_t loss_kind, float scale, int64_t t, float lr, float beta1,
                                     float beta2, float eps, float* g, float* grad_W, float* grad_x,
                                     float* loss, int32_t b) {
    if (!c) return USL_EINVAL;
    NEED(x); NEED(idx); NEED(W); NEED(m1); NEED(m2); NEED(tgt_off); NEED(tgt_lab); NEED(g); NEED(grad_W);
    NEED(loss);
    if (loss_kind != 0 && loss_kind != 1) USL_FAIL(c, USL_EINVAL, "loss_kind %d is neither 0 (BCE) nor 1 (squared hinge)", loss_kind);
    if (!(scale == scale) || isinf(scale)) USL_FAIL(c, USL_EINVAL, "scale is not finite");
    if (t < 1) USL_FAIL(c, USL_EINVAL, "step number t = %lld < 1", (long long)t);
    if (!(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f))
        USL_FAIL(c, USL_EINVAL, "beta1, beta2 must lie in [0,1)");
    if (!(eps >= 0.f) || !(lr == lr)) USL_FAIL(c, USL_EINVAL, "eps < 0 or lr is NaN");
    USL_TRY(check_batch(c, b));
    USL_TRY(usl_prepare_device(c));
    USL_TRY(usl_launch_forward(c, x, idx, W, g, b));
    if (grad_x) {
        // The loss writes the gradient in place and, group of 256 instances by group, as the tile-major pieces the
        // input-gradient gathers read; the gathers of a group run before the next group's pieces replace them.
        // Squared hinge: the gradient of a trained layer is almost all zeros (Section 3.3); when the context expects
        // that, its nonzeros are listed once and both backward products try the lists first (k_sparse_grad.hip).
        const int G = usl_bwd_input_group_rows();
        const bool lists = loss_kind == 1 && usl_sparse_supported(c);
        if (usl_bwi_lds_applies(c) || usl_both_lds_applies(c) || (lists && (b > G || usl_sparse_expected(c)))) {
            // squared hinge where a gradient of almost only zeros is expected (or the batch has several groups, and
            // the look at the gradient needs all of it): the loss writes the gradient row-major only, its nonzeros are
            // listed once, and both backward products use the lists (the dense kernels stand by behind the gate)
            USL_TRY(usl_launch_loss(c, loss_kind, g, tgt_off, tgt_lab, scale, g, loss, b));
            // (the same order of calls where the input gradient reads g row-major: its register-list form)
            const uint32_t* gate = nullptr;
            const float* stage = nullptr;
            const uint32_t* pos = nullptr;
            const uint32_t* stale = nullptr;
            USL_TRY(backward_both(c, g, x, idx, W, grad_W, grad_x, b, lists, loss_kind == 0, &gate, &stage, &pos, &stale));
            if (stage) {   // the weight gradient is in the order of the lists: Adam picks it up there and writes grad_W
                const double c1 = 1.0 - pow((double)beta1, (double)t);
                const double c2 = 1.0 - pow((double)beta2, (double)t);
                return usl_launch_adam_staged(c, W, stage, pos, gate, stale, grad_W, m1, m2, lr, beta1, beta2, eps, (float)(1.0 / c1),
                                              (float)(1.0 / c2));
            }
        } else {
            USL_TRY(usl_bwd_input_prepare(c, idx, b));
            const uint32_t* gate = nullptr;
            uint64_t sampled = 0;
            if (!lists) USL_TRY(usl_bwd_input_gather_w(c, W, nullptr));
            for (int i0 = 0; i0 < b; i0 += G) {
                const int rows = b - i0 < G ? b - i0 : G;
                USL_TRY(usl_bwd_input_begin_group(c));
                USL_TRY(usl_launch_loss_tiles(c, loss_kind, g, tgt_off, tgt_lab, scale, loss, b, &sampled, i0, rows));
                if (lists) {                        // one group: its pieces stay valid while g is looked at
                    USL_TRY(usl_sparse_compact(c, g, b, &gate));
                    c->nz_lists_of = g;             // backward-weight below does not look a second time
                    c->nz_lists_tried = gate != nullptr;
                    if (gate) USL_TRY(usl_sparse_backward_input(c, idx, W, grad_x, b));
                    USL_TRY(usl_bwd_input_gather_w(c, W, gate));
                }
                USL_TRY(usl_bwd_input_group(c, grad_x + (size_t)i0 * c->d, rows, sampled, gate));
            }
            const usl_status s = usl_launch_backward_weight(c, g, x, idx, grad_W, b, loss_kind == 0);   // BCE gradients are dense
            c->nz_lists_of = nullptr;
            USL_TRY(s);
        }
    } else {
        USL_TRY(usl_launch_loss(c, loss_kind, g, tgt_off, tgt_lab, scale, g, loss, b));
        USL_TRY(usl_launch_backward_weight(c, g, x, idx, grad_W, b, loss_kind == 0));   // BCE gradients are dense
    }
    const double c1 = 1.0 - pow((double)beta1, (double)t);
    const double c2 = 1.0 - pow((double)beta2, (double)t);
    return usl_launch_adam(c, W, grad_W, m1, m2, lr, beta1, beta2, eps, (float)(1.0 / c1), (float)(1.0 / c2));
}

extern "C" usl_status usl_redistribute(usl_ctx* c, int32_t* idx, void* W, float* m1, float* m2,
                                       double fraction, uint64_t seed, uint64_t epoch,
                                       int64_t* n_rewired_host) {
    if (!c) return USL_EINVAL;
    NEED(idx); NEED(W); NEED(m1); NEED(m2);
    if (!(fraction >= 0.0 && fraction <= 1.0))
        USL_FAIL(c, USL_EINVAL, "fraction %g outside [0,1]", fraction);
    if (epoch == ~(uint64_t)0) USL_FAIL(c, USL_EINVAL, "epoch 2^64-1 is reserved for usl_init_indices");
    int64_t N = c->m * (int64_t)c->k;
    int64_t n = (int64_t)floor(fraction * (double)N);
    if (n > N) n = N;
    if (n_rewired_host) *n_rewired_host = n;
    if (n == 0) return USL_OK;
    USL_TRY(usl_prepare_device(c));
    c->csc_built_for = nullptr;
    c->lf[0].built_for = c->lf[1].built_for = nullptr;
    c->slot_order_for = nullptr;
    return usl_launch_redistribute(c, idx, W, m1, m2, n, seed, epoch);
}

extern "C" usl_status usl_redistribute_rows(usl_ctx* c, int32_t* idx, void* W, float* m1, float* m2,
                                            int32_t per_row, uint64_t seed, uint64_t epoch) {
    if (!c) return USL_EINVAL;
    NEED(idx); NEED(W); NEED(m1); NEED(m2);
    if (per_row < 0 || per_row > c->k) USL_FAIL(c, USL_EINVAL, "per_row %d outside [0, k]", per_row);
    if (epoch == ~(uint64_t)0) USL_FAIL(c, USL_EINVAL, "epoch 2^64-1 is reserved for usl_init_indices");
    if (per_row == 0) return USL_OK;
    USL_TRY(usl_prepare_device(c));
    c->csc_built_for = nullptr;
    c->lf[0].built_for = c->lf[1].built_for = nullptr;
    c->slot_order_for = nullptr;
    return usl_launch_redistribute_rows(c, idx, W, m1, m2, per_row, seed, epoch);
}

extern "C" usl_status usl_check(usl_ctx* c) {
    if (!c) return USL_EINVAL;
    if (c->device < 0) return USL_OK;   // nothing was ever launched
    USL_HIP(c, hipStreamSynchronize(c->stream));
    if (c->idx_print) {
        uint32_t stale = 0;
        USL_HIP(c, hipMemcpy(&stale, reinterpret_cast<uint32_t*>(c->idx_print) + 4, 4, hipMemcpyDeviceToHost));
        if (stale) {
            USL_HIP(c, hipMemset(reinterpret_cast<uint32_t*>(c->idx_print) + 4, 0, 4));
            c->csc_built_for = nullptr;
            c->lf[0].built_for = c->lf[1].built_for = nullptr;
            c->slot_order_for = nullptr;
            USL_FAIL(c, USL_ESTALE, "idx changed without usl_invalidate: a usl_backward_input call since the last "
                                    "check ran on column lists of the old contents and filled grad_x with NaN");
        }
    }
    return USL_OK;
}

extern "C" usl_status usl_validate_indices(usl_ctx* c, const int32_t* idx, int64_t* n_bad_host) {
    if (!c) return USL_EINVAL;
    NEED(idx); NEED(n_bad_host);
    USL_TRY(usl_prepare_device(c));
    return usl_launch_validate(c, idx, n_bad_host);
}

extern "C" usl_status usl_philox_words(usl_ctx* c, const uint32_t* ctr, uint32_t key0,
                                       uint32_t key1, uint32_t* out, int64_t n) {
    if (!c) return USL_EINVAL;
    NEED(ctr); NEED(out);
    if (n < 0) USL_FAIL(c, USL_EINVAL, "n < 0");
    if (n == 0) return USL_OK;
    USL_TRY(usl_prepare_device(c));
    return usl_launch_philox(c, ctr, key0, key1, out, n);
}
