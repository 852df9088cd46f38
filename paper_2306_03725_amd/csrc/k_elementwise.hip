// Sparse-target one-vs-all losses (binary cross-entropy, squared hinge: loss + gradient in one pass
// over the scores) and Adam.
// Both are pure HBM streams: one read and one write of every element, 16 bytes per lane.
#include "usl_internal.h"

namespace {

constexpr int BCE_NT = 256;
constexpr int BCE_PER_THREAD = 16;  // labels per lane, as 4 groups of 4
constexpr int BCE_CHUNK = BCE_NT * BCE_PER_THREAD;
constexpr int BCE_MAX_HITS = 512;

struct Bce1 { float g, l; };
enum { LOSS_BCE = 0, LOSS_SQH = 1 };
// y is 0 or 1.
// BCE:           l = max(z,0) - z*y + log(1 + exp(-|z|));  dl/dz = sigmoid(z) - y
// squared hinge: s = 2y-1, l = max(0, 1 - s*z)^2;          dl/dz = -2*s*max(0, 1 - s*z)  (exact zeros)
template <int LOSS>
__device__ __forceinline__ Bce1 bce_one(float z, float y, float scale) {
    Bce1 o;
    if (LOSS == LOSS_BCE) {
        const float e = __expf(-fabsf(z));
        const float r = __frcp_rn(1.f + e);
        const float sig = z >= 0.f ? r : e * r;
        o.g = scale * (sig - y);
        o.l = fmaxf(z, 0.f) - z * y + __logf(1.f + e);
    } else {
        const float sgn = 2.f * y - 1.f;
        const float margin = fmaxf(0.f, fmaf(-sgn, z, 1.f));
        o.g = scale * (-2.f * sgn * margin);
        o.l = margin * margin;
    }
    return o;
}

// grid (label chunks, b).  The positives of the instance that fall into the block's label range
// are collected in LDS first; nearly always there are none, so the per-element test is free.
template <bool VEC, int LOSS>
__global__ void __launch_bounds__(BCE_NT)
k_bce(const float* out, const int64_t* __restrict__ tgt_off, const int32_t* __restrict__ tgt_lab,
      float scale, float* g, double* __restrict__ partials, int64_t m) {
    __shared__ int32_t hits[BCE_MAX_HITS];
    __shared__ int nh;
    __shared__ double red[BCE_NT / 64];
    const int i = blockIdx.y;
    const int64_t j0 = (int64_t)blockIdx.x * BCE_CHUNK;
    const int64_t j1 = min(m, j0 + BCE_CHUNK);
    if (threadIdx.x == 0) nh = 0;
    __syncthreads();
    const int64_t p0 = tgt_off[i], p1 = tgt_off[i + 1];
    for (int64_t p = p0 + threadIdx.x; p < p1; p += BCE_NT) {
        const int64_t lab = tgt_lab[p];
        if (lab >= j0 && lab < j1) {
            const int pos = atomicAdd(&nh, 1);
            if (pos < BCE_MAX_HITS) hits[pos] = (int32_t)(lab - j0);
        }
    }
    __syncthreads();
    const int nhits = nh;
    const bool overflow = nhits > BCE_MAX_HITS;  // absurdly dense targets: rescan the global list
    const float* zrow = out + (size_t)i * m;
    float* grow = g + (size_t)i * m;
    float lsum = 0.f;
#pragma unroll
    for (int u = 0; u < BCE_PER_THREAD / 4; ++u) {
        const int64_t j = j0 + ((int64_t)u * BCE_NT + threadIdx.x) * 4;
        if (j >= j1) continue;
        const int rel = (int)(j - j0);
        float y[4] = {0.f, 0.f, 0.f, 0.f};
        if (!overflow) {
            for (int h = 0; h < nhits; ++h) {
                const unsigned dlt = (unsigned)(hits[h] - rel);
                if (dlt < 4u) y[dlt] = 1.f;
            }
        } else {
            for (int64_t p = p0; p < p1; ++p) {
                const int64_t dlt = (int64_t)tgt_lab[p] - j;
                if (dlt >= 0 && dlt < 4) y[dlt] = 1.f;
            }
        }
        if (VEC && j + 4 <= j1) {
            const float4 z = *reinterpret_cast<const float4*>(zrow + j);
            const Bce1 a = bce_one<LOSS>(z.x, y[0], scale), b2 = bce_one<LOSS>(z.y, y[1], scale),
                       c = bce_one<LOSS>(z.z, y[2], scale), dd = bce_one<LOSS>(z.w, y[3], scale);
            *reinterpret_cast<float4*>(grow + j) = make_float4(a.g, b2.g, c.g, dd.g);
            lsum += (a.l + b2.l) + (c.l + dd.l);
        } else {
            for (int q = 0; q < 4 && j + q < j1; ++q) {
                const Bce1 a = bce_one<LOSS>(zrow[j + q], y[q], scale);
                grow[j + q] = a.g;
                lsum += a.l;
            }
        }
    }
    double v = (double)lsum;
    for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    if (threadIdx.x == 0) {
        double s = 0.0;
        for (int q = 0; q < BCE_NT / 64; ++q) s += red[q];
        partials[(size_t)blockIdx.y * gridDim.x + blockIdx.x] = s;
    }
}

// One block adds the per-block sums in a fixed order: the loss is reproducible run to run.
__global__ void __launch_bounds__(1024)
k_bce_finish(const double* __restrict__ partials, size_t n, float scale, float* __restrict__ loss) {
    __shared__ double red[16];
    double s = 0.0;
    for (size_t q = threadIdx.x; q < n; q += 1024) s += partials[q];
    for (int o = 32; o > 0; o >>= 1) s += __shfl_down(s, o);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
        for (int q = 0; q < 16; ++q) t += red[q];
        *loss = (float)((double)scale * t);
    }
}

template <typename TS> struct WIo;
template <> struct WIo<float> {
    static __device__ __forceinline__ float get(const float* W, size_t f) { return W[f]; }
    static __device__ __forceinline__ void put(float* W, size_t f, float v) { W[f] = v; }
};
template <> struct WIo<uint16_t> {
    static __device__ __forceinline__ float get(const uint16_t* W, size_t f) { return usl_bf16_to_f32(W[f]); }
    static __device__ __forceinline__ void put(uint16_t* W, size_t f, float v) { W[f] = usl_f32_to_bf16(v); }
};

__device__ __forceinline__ float adam_one(float w, float gw, float& a, float& v, float lr, float b1,
                                          float b2, float eps, float ic1, float ic2) {
    a = fmaf(b1, a, (1.f - b1) * gw);
    v = fmaf(b2, v, (1.f - b2) * gw * gw);
    return w - lr * (a * ic1) / (sqrtf(v * ic2) + eps);
}

template <typename TS>
__global__ void __launch_bounds__(256)
k_adam(TS* __restrict__ W, const float* __restrict__ gW, float* __restrict__ m1,
       float* __restrict__ m2, size_t n, float lr, float b1, float b2, float eps, float ic1,
       float ic2) {
    const size_t stride = (size_t)gridDim.x * 256 * 4;
    for (size_t f = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4; f < n; f += stride) {
        if (f + 4 <= n) {
            const float4 g4 = *reinterpret_cast<const float4*>(gW + f);
            float4 a4 = *reinterpret_cast<const float4*>(m1 + f);
            float4 v4 = *reinterpret_cast<const float4*>(m2 + f);
            float w[4];
            if (sizeof(TS) == 4) {
                const float4 w4 = *reinterpret_cast<const float4*>(W + f);
                w[0] = w4.x; w[1] = w4.y; w[2] = w4.z; w[3] = w4.w;
            } else {
                const uint2 u = *reinterpret_cast<const uint2*>(W + f);
                w[0] = __uint_as_float(u.x << 16); w[1] = __uint_as_float(u.x & 0xFFFF0000u);
                w[2] = __uint_as_float(u.y << 16); w[3] = __uint_as_float(u.y & 0xFFFF0000u);
            }
            w[0] = adam_one(w[0], g4.x, a4.x, v4.x, lr, b1, b2, eps, ic1, ic2);
            w[1] = adam_one(w[1], g4.y, a4.y, v4.y, lr, b1, b2, eps, ic1, ic2);
            w[2] = adam_one(w[2], g4.z, a4.z, v4.z, lr, b1, b2, eps, ic1, ic2);
            w[3] = adam_one(w[3], g4.w, a4.w, v4.w, lr, b1, b2, eps, ic1, ic2);
            *reinterpret_cast<float4*>(m1 + f) = a4;
            *reinterpret_cast<float4*>(m2 + f) = v4;
            if (sizeof(TS) == 4) {
                *reinterpret_cast<float4*>(W + f) = make_float4(w[0], w[1], w[2], w[3]);
            } else {
                uint2 u;
                u.x = (uint32_t)usl_f32_to_bf16(w[0]) | ((uint32_t)usl_f32_to_bf16(w[1]) << 16);
                u.y = (uint32_t)usl_f32_to_bf16(w[2]) | ((uint32_t)usl_f32_to_bf16(w[3]) << 16);
                *reinterpret_cast<uint2*>(W + f) = u;
            }
        } else {
            for (size_t q = f; q < n; ++q) {
                float a = m1[q], v = m2[q];
                const float w = adam_one(WIo<TS>::get(W, q), gW[q], a, v, lr, b1, b2, eps, ic1, ic2);
                m1[q] = a; m2[q] = v;
                WIo<TS>::put(W, q, w);
            }
        }
    }
}

}  // namespace

usl_status usl_launch_loss(usl_ctx* c, int loss_kind, const float* out, const int64_t* tgt_off,
                           const int32_t* tgt_lab, float scale, float* g, float* loss, int32_t b) {
    const int64_t nchunk = (c->m + BCE_CHUNK - 1) / BCE_CHUNK;
    const size_t nblk = (size_t)nchunk * b;
    size_t cap = c->bce_partials_cap;
    USL_TRY(usl_reserve(c, (void**)&c->bce_partials, &cap, nblk * sizeof(double)));
    c->bce_partials_cap = cap;
    const bool vec = (c->m % 4 == 0) && ((uintptr_t)out % 16 == 0) && ((uintptr_t)g % 16 == 0);
    dim3 grid((unsigned)nchunk, (unsigned)b);
#define USL_LOSS(VEC, KIND)                                                                          \
    hipLaunchKernelGGL((k_bce<VEC, KIND>), grid, dim3(BCE_NT), 0, c->stream, out, tgt_off, tgt_lab,  \
                       scale, g, c->bce_partials, c->m)
    if (loss_kind == LOSS_BCE) { if (vec) USL_LOSS(true, LOSS_BCE); else USL_LOSS(false, LOSS_BCE); }
    else                       { if (vec) USL_LOSS(true, LOSS_SQH); else USL_LOSS(false, LOSS_SQH); }
#undef USL_LOSS
    USL_TRY(usl_check_launch(c, "loss"));
    hipLaunchKernelGGL(k_bce_finish, dim3(1), dim3(1024), 0, c->stream, c->bce_partials, nblk, scale, loss);
    return usl_check_launch(c, "loss_finish");
}

usl_status usl_launch_adam(usl_ctx* c, void* W, const float* grad_W, float* m1, float* m2, float lr,
                           float beta1, float beta2, float eps, float inv_c1, float inv_c2) {
    const size_t n = (size_t)c->m * c->k;
    size_t blocks = (n / 4 + 255) / 256;
    const size_t cap = (size_t)c->num_cu * 16;
    if (blocks > cap) blocks = cap;
    if (blocks < 1) blocks = 1;
    const bool aligned = ((uintptr_t)W % 16 == 0) && ((uintptr_t)grad_W % 16 == 0) &&
                         ((uintptr_t)m1 % 16 == 0) && ((uintptr_t)m2 % 16 == 0);
    if (!aligned) USL_FAIL(c, USL_EINVAL, "W, grad_W, m1, m2 must be 16-byte aligned");
    if (c->storage == USL_F32)
        hipLaunchKernelGGL(k_adam<float>, dim3((unsigned)blocks), dim3(256), 0, c->stream, (float*)W,
                           grad_W, m1, m2, n, lr, beta1, beta2, eps, inv_c1, inv_c2);
    else
        hipLaunchKernelGGL(k_adam<uint16_t>, dim3((unsigned)blocks), dim3(256), 0, c->stream,
                           (uint16_t*)W, grad_W, m1, m2, n, lr, beta1, beta2, eps, inv_c1, inv_c2);
    return usl_check_launch(c, "adam");
}

// ---- rows of idx / W picked by a list of label ids (label-subset calls) ----------------------
namespace {
template <typename TS>
__global__ void __launch_bounds__(256)
k_gather_rows(const int32_t* __restrict__ idx, const TS* __restrict__ W, const int32_t* __restrict__ rows,
              int64_t n, int64_t m, int k, int32_t* __restrict__ dst_idx, TS* __restrict__ dst_W) {
    const int64_t total = n * k;
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (int64_t)gridDim.x * 256) {
        const int64_t q = e / k;
        const int t = (int)(e - q * k);
        int64_t j = rows[q];
        j = j < 0 ? 0 : (j >= m ? m - 1 : j);
        dst_idx[e] = idx[j * k + t];
        if (W) dst_W[e] = W[j * k + t];
    }
}
}  // namespace

usl_status usl_launch_gather_rows(usl_ctx* c, const int32_t* idx, const void* W, const int32_t* rows,
                                  int64_t n, int32_t* dst_idx, void* dst_W) {
    int64_t blocks = (n * c->k + 255) / 256;
    if (blocks > (int64_t)c->num_cu * 32) blocks = (int64_t)c->num_cu * 32;
    if (c->storage == USL_F32)
        hipLaunchKernelGGL(k_gather_rows<float>, dim3((unsigned)blocks), dim3(256), 0, c->stream, idx,
                           (const float*)W, rows, n, c->m, c->k, dst_idx, (float*)dst_W);
    else
        hipLaunchKernelGGL(k_gather_rows<uint16_t>, dim3((unsigned)blocks), dim3(256), 0, c->stream, idx,
                           (const uint16_t*)W, rows, n, c->m, c->k, dst_idx, (uint16_t*)dst_W);
    return usl_check_launch(c, "gather_rows");
}
