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

// The same loss, tile by tile, for a caller that wants the gradient twice: in place over the scores
// (row-major, for backward-weight) and as gT[tile][label][32] with the piece flags (for backward-input),
// which saves the separate transposition pass.  grid (blocks of LT_TL labels, tiles of 32 instances).
constexpr int LT_TL = 128;
constexpr int LT_SAMPLE = 16;   // one label block in 16 feeds the nonzero-piece count

template <bool VEC, int LOSS>
__global__ void __launch_bounds__(256)
k_loss_tiles(float* zg, const int64_t* __restrict__ tgt_off, const int32_t* __restrict__ tgt_lab, float scale,
             double* __restrict__ partials, int64_t m, int b, float* __restrict__ gT,
             uint8_t* __restrict__ nzf, uint32_t* __restrict__ nz_cells, int row0) {
    __shared__ float tile[32][LT_TL + 1];
    __shared__ uint32_t ybits[32][LT_TL / 32];
    __shared__ double red[4];
    __shared__ uint32_t block_cells;
    const int tid = threadIdx.x;
    const int i0 = row0 + blockIdx.y * 32;   // gT and the flags are indexed by the tile within the group (blockIdx.y)
    const int64_t j0 = (int64_t)blockIdx.x * LT_TL;
    const int nl = (int)min((int64_t)LT_TL, m - j0);
    if (tid < 32 * (LT_TL / 32)) (&ybits[0][0])[tid] = 0u;
    if (tid == 0) block_cells = 0;
    __syncthreads();
    {   // 8 lanes walk the target list of one instance
        const int ii = tid >> 3, i = i0 + ii;
        if (i < b)
            for (int64_t p = tgt_off[i] + (tid & 7); p < tgt_off[i + 1]; p += 8) {
                const int64_t rel = (int64_t)tgt_lab[p] - j0;
                if (rel >= 0 && rel < nl) atomicOr(&ybits[ii][rel >> 5], 1u << (rel & 31));
            }
    }
    __syncthreads();
    float lsum = 0.f;
    if (VEC) {   // m % 4 == 0 and 16-byte aligned rows: nl is a multiple of 4
        const int c4 = (tid & 31) * 4;
#pragma unroll
        for (int pass = 0; pass < 4; ++pass) {
            const int ii = pass * 8 + (tid >> 5), i = i0 + ii;
            float4 gv = make_float4(0.f, 0.f, 0.f, 0.f);
            if (i < b && c4 < nl) {
                float4* p = reinterpret_cast<float4*>(zg + (size_t)i * m + j0 + c4);
                const float4 z = *p;
                const uint32_t yb = ybits[ii][c4 >> 5] >> (c4 & 31);
                const Bce1 a = bce_one<LOSS>(z.x, (float)(yb & 1u), scale), b2 = bce_one<LOSS>(z.y, (float)((yb >> 1) & 1u), scale),
                           c = bce_one<LOSS>(z.z, (float)((yb >> 2) & 1u), scale), dd = bce_one<LOSS>(z.w, (float)((yb >> 3) & 1u), scale);
                gv = make_float4(a.g, b2.g, c.g, dd.g);
                *p = gv;
                lsum += (a.l + b2.l) + (c.l + dd.l);
            }
            tile[ii][c4] = gv.x; tile[ii][c4 + 1] = gv.y; tile[ii][c4 + 2] = gv.z; tile[ii][c4 + 3] = gv.w;
        }
    } else {
        const int cc = tid & (LT_TL - 1);
#pragma unroll 4
        for (int pass = 0; pass < 16; ++pass) {
            const int ii = pass * 2 + (tid >> 7), i = i0 + ii;
            float gv = 0.f;
            if (i < b && cc < nl) {
                float* p = zg + (size_t)i * m + j0 + cc;
                const Bce1 a = bce_one<LOSS>(*p, (float)((ybits[ii][cc >> 5] >> (cc & 31)) & 1u), scale);
                gv = a.g;
                *p = gv;
                lsum += a.l;
            }
            tile[ii][cc] = gv;
        }
    }
    __syncthreads();
    {   // the tile's pieces are one contiguous run of gT: nl * 32 floats
        float* dst = gT + ((size_t)blockIdx.y * m + j0) * 32;
        for (int e = tid; e < nl * 32; e += 256) dst[e] = tile[e & 31][e >> 5];
        if (tid < nl) {
            bool any = false;
#pragma unroll 8
            for (int ii = 0; ii < 32; ++ii) any |= tile[ii][tid] != 0.f;
            nzf[(size_t)blockIdx.y * m + j0 + tid] = any ? 1 : 0;
            if ((blockIdx.x % LT_SAMPLE) == 0 && any) atomicAdd(&block_cells, 1u);
        }
    }
    double v = (double)lsum;
    for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o);
    if ((tid & 63) == 0) red[tid >> 6] = v;
    __syncthreads();
    if (tid == 0) {
        partials[(size_t)(row0 / 32 + blockIdx.y) * gridDim.x + blockIdx.x] = (red[0] + red[1]) + (red[2] + red[3]);
        if ((blockIdx.x % LT_SAMPLE) == 0 && block_cells) atomicAdd(nz_cells, block_cells);
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

// grad_W[f] = stage[pos[f]]: the weight gradient of k_both_lds brought into the order of the slots (for callers of
// usl_backward; usl_train_step lets Adam do it in passing).  Blocks and XCDs as in k_adam_staged.
__global__ void __launch_bounds__(256)
k_unstage(const float* __restrict__ stage, const uint32_t* __restrict__ pos, const uint32_t* __restrict__ gate,
          const uint32_t* __restrict__ stale, float* __restrict__ gW, size_t n4) {
    if (gate && *gate == 0) return;
    const bool poison = *stale != 0;   // the lists were built from other contents of idx: no number is better than a wrong one
    const size_t per_xcd = (n4 + 7) / 8, first = (size_t)(blockIdx.x & 7) * per_xcd;
    const size_t last = first + per_xcd < n4 ? first + per_xcd : n4;
    const size_t stride = (size_t)(gridDim.x / 8) * 256;
    for (size_t v = first + (size_t)(blockIdx.x >> 3) * 256 + threadIdx.x; v < last; v += stride) {
        const uint4 p4 = reinterpret_cast<const uint4*>(pos)[v];
        const float nan = __uint_as_float(0x7FC00000u);
        reinterpret_cast<float4*>(gW)[v] = poison ? make_float4(nan, nan, nan, nan) : make_float4(stage[p4.x], stage[p4.y], stage[p4.z], stage[p4.w]);
    }
}

// The same update where the weight gradient arrives in the order of the register lists of the input-gradient kernel
// (k_both_lds: stage[pos[f]] is slot f's gradient): picked up here, written to grad_W in passing (whole lines), so
// that the kernel that computed it does not scatter it (4 bytes per line there).  A block works on the f of one
// eighth of the array, the eighth of its XCD (blocks are dealt to the 8 XCDs round robin): the part of stage that
// the slots of a window point into (a few MiB) is then fetched by one L2 only and stays there while they are done.
// gate (may be null): zero means the kernels over the listed nonzero gradients wrote grad_W themselves; read it.
// stale: nonzero means the lists were built from other contents of idx (see usl_check); grad_W then becomes NaN and W,
// m1, m2 stay as they are -- a step from a wrong gradient could not be taken back.
template <typename TS>
__global__ void __launch_bounds__(256)
k_adam_staged(TS* __restrict__ W, const float* __restrict__ stage, const uint32_t* __restrict__ pos,
              const uint32_t* __restrict__ gate, const uint32_t* __restrict__ stale, float* __restrict__ gW,
              float* __restrict__ m1, float* __restrict__ m2, size_t n4, float lr, float b1, float b2, float eps, float ic1,
              float ic2) {
    const bool listed = gate && *gate == 0;
    const bool poison = !listed && *stale != 0;
    const size_t per_xcd = (n4 + 7) / 8, first = (size_t)(blockIdx.x & 7) * per_xcd;
    const size_t last = first + per_xcd < n4 ? first + per_xcd : n4;
    const size_t stride = (size_t)(gridDim.x / 8) * 256;
    for (size_t v = first + (size_t)(blockIdx.x >> 3) * 256 + threadIdx.x; v < last; v += stride) {
        const size_t f = v * 4;
        float4 g4;
        if (listed) {
            g4 = *reinterpret_cast<const float4*>(gW + f);
        } else {
            const uint4 p4 = *reinterpret_cast<const uint4*>(pos + f);
            if (poison) {
                const float nan = __uint_as_float(0x7FC00000u);
                *reinterpret_cast<float4*>(gW + f) = make_float4(nan, nan, nan, nan);
                continue;
            }
            g4 = make_float4(stage[p4.x], stage[p4.y], stage[p4.z], stage[p4.w]);
            *reinterpret_cast<float4*>(gW + f) = g4;
        }
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
    }
}

}  // namespace

// Per-block loss sums of either loss kernel, sized once for max_b instances: a later, larger batch never
// has to grow the buffer (growing frees and allocates, which waits for the stream).
static usl_status usl_reserve_loss_partials(usl_ctx* c) {
    const size_t rows = (size_t)((c->m + BCE_CHUNK - 1) / BCE_CHUNK) * (size_t)c->max_b;
    const size_t tiles = (size_t)((c->m + LT_TL - 1) / LT_TL) * (size_t)((c->max_b + 31) / 32);
    return usl_reserve(c, (void**)&c->bce_partials, &c->bce_partials_cap, (rows > tiles ? rows : tiles) * sizeof(double));
}

usl_status usl_launch_loss(usl_ctx* c, int loss_kind, const float* out, const int64_t* tgt_off,
                           const int32_t* tgt_lab, float scale, float* g, float* loss, int32_t b) {
    const int64_t nchunk = (c->m + BCE_CHUNK - 1) / BCE_CHUNK;
    const size_t nblk = (size_t)nchunk * b;
    USL_TRY(usl_reserve_loss_partials(c));
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

// ---- the loss for callers that cannot allocate: same kernels, per-block sums in a static device array
// (each GPU the library runs on holds its own copy of the array, at its own address, until the process ends)
constexpr size_t NOALLOC_SLOTS = 131072;   // 1 MiB of doubles: one per (block of 4096 labels, instance)
static __device__ __align__(256) double scratch[NOALLOC_SLOTS];
constexpr int NOALLOC_MAX_DEVICES = 64;
static double* scratch_ptr[NOALLOC_MAX_DEVICES];   // device address of `scratch` on each device, set once


// Called once per context when it first touches its device (that device is current): looks up where this
// device holds the array.  In host code the array's name is only a handle for this lookup.
usl_status usl_noalloc_setup(usl_ctx* c) {
    if (c->device < 0 || c->device >= NOALLOC_MAX_DEVICES) return USL_OK;   // the no-alloc call will refuse
    if (scratch_ptr[c->device]) return USL_OK;
    double* p = nullptr;
    USL_HIP(c, hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch)));
    scratch_ptr[c->device] = p;
    return USL_OK;
}

usl_status usl_launch_loss_noalloc(usl_ctx* c, int loss_kind, const float* out, const int64_t* tgt_off,
                                   const int32_t* tgt_lab, float scale, float* g, float* loss, int32_t b) {
    const int64_t nchunk = (c->m + BCE_CHUNK - 1) / BCE_CHUNK;
    const size_t nblk = (size_t)nchunk * b;
    if (nblk > NOALLOC_SLOTS)
        USL_FAIL(c, USL_ESHAPE, "ceil(m / %d) * b = %zu per-block sums exceed the %zu the static scratch holds",
                 BCE_CHUNK, nblk, NOALLOC_SLOTS);
    double* partials = (c->device >= 0 && c->device < NOALLOC_MAX_DEVICES) ? scratch_ptr[c->device] : nullptr;
    if (!partials) USL_FAIL(c, USL_EUNSUPPORTED, "no static scratch on device %d", c->device);
    const bool vec = (c->m % 4 == 0) && ((uintptr_t)out % 16 == 0) && ((uintptr_t)g % 16 == 0);
    dim3 grid((unsigned)nchunk, (unsigned)b);
#define USL_LOSS(VEC, KIND)                                                                          \
    hipLaunchKernelGGL((k_bce<VEC, KIND>), grid, dim3(BCE_NT), 0, c->stream, out, tgt_off, tgt_lab,  \
                       scale, g, partials, c->m)
    if (loss_kind == LOSS_BCE) { if (vec) USL_LOSS(true, LOSS_BCE); else USL_LOSS(false, LOSS_BCE); }
    else                       { if (vec) USL_LOSS(true, LOSS_SQH); else USL_LOSS(false, LOSS_SQH); }
#undef USL_LOSS
    USL_TRY(usl_check_launch(c, "loss (static scratch)"));
    hipLaunchKernelGGL(k_bce_finish, dim3(1), dim3(1024), 0, c->stream, partials, nblk, scale, loss);
    return usl_check_launch(c, "loss_finish (static scratch)");
}

usl_status usl_launch_loss_tiles(usl_ctx* c, int loss_kind, float* zg, const int64_t* tgt_off,
                                 const int32_t* tgt_lab, float scale, float* loss, int32_t b,
                                 uint64_t* sampled_labels, int32_t row0, int32_t rows) {
    const int64_t nlb = (c->m + LT_TL - 1) / LT_TL;
    const int ntile = (rows + 31) / 32;
    USL_TRY(usl_reserve_loss_partials(c));
    const bool vec = (c->m % 4 == 0) && ((uintptr_t)zg % 16 == 0);
    dim3 grid((unsigned)nlb, (unsigned)ntile);
    const int b_end = row0 + rows;   // instances at and past it belong to a later group (or do not exist)
#define USL_LOSS(VEC, KIND)                                                                              \
    hipLaunchKernelGGL((k_loss_tiles<VEC, KIND>), grid, dim3(256), 0, c->stream, zg, tgt_off, tgt_lab,   \
                       scale, c->bce_partials, c->m, b_end, c->gT, c->nz_flags, usl_nz_cells(c), (int)row0)
    if (loss_kind == LOSS_BCE) { if (vec) USL_LOSS(true, LOSS_BCE); else USL_LOSS(false, LOSS_BCE); }
    else                       { if (vec) USL_LOSS(true, LOSS_SQH); else USL_LOSS(false, LOSS_SQH); }
#undef USL_LOSS
    USL_TRY(usl_check_launch(c, "loss (tiles)"));
    *sampled_labels = (uint64_t)((nlb + LT_SAMPLE - 1) / LT_SAMPLE) * LT_TL;
    if (b_end >= b) {   // the last group: every tile of the batch has left its sums
        const size_t nblk = (size_t)nlb * (size_t)((b + 31) / 32);
        hipLaunchKernelGGL(k_bce_finish, dim3(1), dim3(1024), 0, c->stream, c->bce_partials, nblk, scale, loss);
    }
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

usl_status usl_launch_unstage(usl_ctx* c, const float* stage, const uint32_t* pos, const uint32_t* gate, const uint32_t* stale,
                              float* grad_W) {
    const size_t n = (size_t)c->m * c->k;
    if ((uintptr_t)grad_W % 16 || n % 4) USL_FAIL(c, USL_EINVAL, "grad_W must be 16-byte aligned, m * k a multiple of 4");
    const unsigned blocks = (unsigned)(c->num_cu > 0 ? c->num_cu : 8) * 16 / 8 * 8;
    hipLaunchKernelGGL(k_unstage, dim3(blocks), dim3(256), 0, c->stream, stage, pos, gate, stale, grad_W, n / 4);
    return usl_check_launch(c, "weight gradient into slot order");
}

// Adam from a weight gradient in list order (see k_adam_staged); m * k must be a multiple of 4 (the list form's
// shapes are).  grad_W is written (or, behind a zero gate, read).
usl_status usl_launch_adam_staged(usl_ctx* c, void* W, const float* stage, const uint32_t* pos, const uint32_t* gate,
                                  const uint32_t* stale, float* grad_W, float* m1, float* m2, float lr, float beta1, float beta2, float eps,
                                  float inv_c1, float inv_c2) {
    const size_t n = (size_t)c->m * c->k;
    const bool aligned = ((uintptr_t)W % 16 == 0) && ((uintptr_t)grad_W % 16 == 0) &&
                         ((uintptr_t)m1 % 16 == 0) && ((uintptr_t)m2 % 16 == 0);
    if (!aligned || n % 4) USL_FAIL(c, USL_EINVAL, "W, grad_W, m1, m2 must be 16-byte aligned, m * k a multiple of 4");
    const unsigned blocks = (unsigned)(c->num_cu > 0 ? c->num_cu : 8) * 16 / 8 * 8;
    if (c->storage == USL_F32)
        hipLaunchKernelGGL(k_adam_staged<float>, dim3(blocks), dim3(256), 0, c->stream, (float*)W, stage, pos, gate,
                           stale, grad_W, m1, m2, n / 4, lr, beta1, beta2, eps, inv_c1, inv_c2);
    else
        hipLaunchKernelGGL(k_adam_staged<uint16_t>, dim3(blocks), dim3(256), 0, c->stream, (uint16_t*)W, stage, pos, gate,
                           stale, grad_W, m1, m2, n / 4, lr, beta1, beta2, eps, inv_c1, inv_c2);
    return usl_check_launch(c, "adam (staged gradient)");
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
