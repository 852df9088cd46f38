// The two backward products over the nonzero entries of g only (Section 3.3: with the squared hinge loss
// the gradient of every easy negative is exactly zero, "implicit negative mining", and Algorithms 2 and 3
// skip those entries).  The dense kernels walk all b*m*k products and can skip zeros only where a whole
// wavefront group or a whole 32-instance piece is zero; here the work is proportional to the nonzeros:
//   1. k_compact_g reads g once and appends every nonzero (label, value) to a list of its instance;
//      an instance that would exceed its list's capacity (more than 1/32 of the labels) marks the
//      gradient "dense" and the lists are abandoned -- the decision is taken on the device, the host
//      never waits for it;
//   2. if the lists stand: grad_W is cleared and every (entry, slot) adds g * x[i][idx[j][t]] into
//      grad_W[j][t] (float atomics: one 4k-byte row of grad_W per entry, few collisions), and grad_x is
//      built one instance per workgroup in an LDS copy of its row (LDS float atomics are slow, but there
//      are only nnz*k of them) and written out once;
//   3. the dense kernels are launched all the same and leave at their first instruction when the lists
//      stand (and the other way round): `gate` below.
// Results equal the dense sums up to the order of the additions (a skipped term is 0 * finite).
#include <stdlib.h>

#include "usl_internal.h"

namespace {

constexpr int CG_NT = 256, CG_PER = 32, CG_CHUNK = CG_NT * CG_PER;   // labels per block, as 8 x float4 per lane

// A look at a sample of g (four labels in 1024 of every row) before the full pass: a dense gradient, the
// common case after binary cross-entropy, is recognised here and the full pass leaves at its first instruction.
// state[0] = 1 once the gradient counts as dense; state[16 + i] = entries listed for instance i.
__global__ void __launch_bounds__(256)
k_probe_density(const float* __restrict__ g, int64_t m, uint32_t* __restrict__ state,
                uint32_t* __restrict__ hint /* pinned host memory: [0] serial of the last finished look, [1] its verdict */,
                uint32_t serial) {
    __shared__ uint32_t seen, hit;
    if (threadIdx.x == 0) { seen = 0; hit = 0; }
    __syncthreads();
    const float* row = g + (size_t)blockIdx.x * m;
    uint32_t n = 0, nz = 0;
    for (int64_t j = (int64_t)threadIdx.x * 1024; j + 4 <= m; j += 256 * 1024) {   // 4 of every 1024 labels
#pragma unroll
        for (int q = 0; q < 4; ++q) nz += row[j + q] != 0.f ? 1u : 0u;
        n += 4;
    }
    atomicAdd(&seen, n);
    atomicAdd(&hit, nz);
    __syncthreads();
    // the lists hold m/32 entries per instance: a sample twice as dense as that cannot fit
    if (threadIdx.x == 0) {
        if (seen >= 128 && (uint64_t)hit * 16 > seen) atomicOr(&state[0], 1u);
        // what the host reads before its next call: would lists have been worth trying?  (sample at most 1/64 nonzero)
        if ((uint64_t)hit * 64 > seen) atomicOr(&state[2], 1u);
        __threadfence();
        if (atomicAdd(&state[1], 1u) == gridDim.x - 1) {   // the last instance's block
            hint[1] = atomicOr(&state[2], 0u) != 0 ? 1u : 0u;
            __threadfence_system();
            hint[0] = serial;
        }
    }
}

__global__ void __launch_bounds__(CG_NT)
k_compact_g(const float* __restrict__ g, int64_t m, uint32_t cap, uint32_t* __restrict__ state,
            int32_t* __restrict__ nz_lab, float* __restrict__ nz_val) {
    __shared__ uint32_t wave_total[CG_NT / 64];
    __shared__ uint32_t block_base;
    if (*reinterpret_cast<volatile uint32_t*>(state) != 0) return;   // the sample, or an earlier block, found g dense
    const int i = blockIdx.y;
    const int64_t j0 = (int64_t)blockIdx.x * CG_CHUNK;
    const float* row = g + (size_t)i * m;
    const bool vec = (m % 4 == 0) && ((uintptr_t)g % 16 == 0);
    float4 v[CG_PER / 4];
#pragma unroll
    for (int u = 0; u < CG_PER / 4; ++u) {
        const int64_t j = j0 + ((int64_t)u * CG_NT + threadIdx.x) * 4;
        if (vec && j + 4 <= m) {
            v[u] = *reinterpret_cast<const float4*>(row + j);
        } else {
            v[u].x = j < m ? row[j] : 0.f;         v[u].y = j + 1 < m ? row[j + 1] : 0.f;
            v[u].z = j + 2 < m ? row[j + 2] : 0.f; v[u].w = j + 3 < m ? row[j + 3] : 0.f;
        }
    }
    uint32_t cnt = 0;
#pragma unroll
    for (int u = 0; u < CG_PER / 4; ++u)
        cnt += (v[u].x != 0.f ? 1u : 0u) + (v[u].y != 0.f ? 1u : 0u) + (v[u].z != 0.f ? 1u : 0u) + (v[u].w != 0.f ? 1u : 0u);
    // places: prefix over the lanes of a wavefront, then over the wavefronts; one atomic per block reserves them
    uint32_t incl = cnt;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t t = __shfl_up(incl, o);
        if ((int)(threadIdx.x & 63) >= o) incl += t;
    }
    if ((threadIdx.x & 63) == 63) wave_total[threadIdx.x >> 6] = incl;
    __syncthreads();
    uint32_t before = 0, total = 0;
#pragma unroll
    for (int q = 0; q < CG_NT / 64; ++q) {
        const uint32_t t = wave_total[q];
        if (q < (int)(threadIdx.x >> 6)) before += t;
        total += t;
    }
    if (total == 0) return;   // the same for every lane of the block
    if (threadIdx.x == 0) block_base = atomicAdd(&state[16 + i], total);
    __syncthreads();
    const uint32_t base = block_base;
    if (base + total > cap) {
        if (threadIdx.x == 0) atomicOr(&state[0], 1u);
        return;
    }
    uint32_t at = base + before + incl - cnt;
    int32_t* lab = nz_lab + (size_t)i * cap;
    float* val = nz_val + (size_t)i * cap;
#pragma unroll
    for (int u = 0; u < CG_PER / 4; ++u) {
        const int64_t j = j0 + ((int64_t)u * CG_NT + threadIdx.x) * 4;
        if (v[u].x != 0.f) { lab[at] = (int32_t)j; val[at] = v[u].x; ++at; }
        if (v[u].y != 0.f) { lab[at] = (int32_t)(j + 1); val[at] = v[u].y; ++at; }
        if (v[u].z != 0.f) { lab[at] = (int32_t)(j + 2); val[at] = v[u].z; ++at; }
        if (v[u].w != 0.f) { lab[at] = (int32_t)(j + 3); val[at] = v[u].w; ++at; }
    }
}

__global__ void k_zero_state(uint32_t* p, size_t n) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0;
}

// clears p[0..n) when the lists stand (state[0] == 0)
__global__ void k_zero_if_sparse(float* __restrict__ p, size_t n, const uint32_t* __restrict__ state) {
    if (*state != 0) return;
    const size_t stride = (size_t)gridDim.x * blockDim.x * 4;
    for (size_t f = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * 4; f < n; f += stride) {
        if (f + 4 <= n && ((uintptr_t)p % 16 == 0)) *reinterpret_cast<float4*>(p + f) = make_float4(0.f, 0.f, 0.f, 0.f);
        else for (size_t q = f; q < n && q < f + 4; ++q) p[q] = 0.f;
    }
}

// grad_W[j][t] += g * x[i][idx[j][t]] for every listed (i, j, g) and slot t.  grid (blocks, b): the blocks of one
// instance stride over its entries; an item is one (entry, slot) pair, so a row of grad_W gets k neighbouring atomics.
template <typename TS>
__global__ void __launch_bounds__(256)
k_bww_sparse(const TS* __restrict__ x, const int32_t* __restrict__ idx, const uint32_t* __restrict__ state,
             const int32_t* __restrict__ nz_lab, const float* __restrict__ nz_val, uint32_t cap,
             float* __restrict__ grad_W, int d, int k) {
    if (state[0] != 0) return;
    const int i = blockIdx.y;
    const uint64_t items = (uint64_t)state[16 + i] * (uint32_t)k;
    const int32_t* lab = nz_lab + (size_t)i * cap;
    const float* val = nz_val + (size_t)i * cap;
    const TS* row = x + (size_t)i * d;
    for (uint64_t e = (uint64_t)blockIdx.x * 256 + threadIdx.x; e < items; e += (uint64_t)gridDim.x * 256) {
        const uint32_t q = (uint32_t)(e / (uint32_t)k);
        const uint32_t t = (uint32_t)(e - (uint64_t)q * (uint32_t)k);
        const size_t slot = (size_t)lab[q] * k + t;
        const float xv = usl_load_f32<TS>(row, (size_t)idx[slot]);
        if (xv != 0.f) unsafeAtomicAdd(grad_W + slot, val[q] * xv);   // activations after a ReLU are half zeros
    }
}

// grad_x[i][c] = sum over listed (j, g) of instance i and slots t with idx[j][t] == c of W[j][t] * g.
// One workgroup per (instance, slice of at most 32768 columns): the slice lives in LDS, starts at zero, takes
// the additions as LDS atomics and is written out once (the row is overwritten, as the dense path does).
constexpr int XS_NT = 1024, XS_COLS = 32768;
template <typename TS>
__global__ void __launch_bounds__(XS_NT)
k_bwi_sparse(const int32_t* __restrict__ idx, const TS* __restrict__ W, const uint32_t* __restrict__ state,
             const int32_t* __restrict__ nz_lab, const float* __restrict__ nz_val, uint32_t cap,
             float* __restrict__ grad_x, int d, int k) {
    extern __shared__ float acc[];
    if (state[0] != 0) return;
    const int i = blockIdx.y;
    const int c0 = blockIdx.x * XS_COLS;
    const int nc = min(XS_COLS, d - c0);
    for (int c = threadIdx.x; c < nc; c += XS_NT) acc[c] = 0.f;
    __syncthreads();
    const uint64_t items = (uint64_t)state[16 + i] * (uint32_t)k;
    const int32_t* lab = nz_lab + (size_t)i * cap;
    const float* val = nz_val + (size_t)i * cap;
    for (uint64_t e = threadIdx.x; e < items; e += XS_NT) {
        const uint32_t q = (uint32_t)(e / (uint32_t)k);
        const uint32_t t = (uint32_t)(e - (uint64_t)q * (uint32_t)k);
        const size_t slot = (size_t)lab[q] * k + t;
        const uint32_t c = (uint32_t)(idx[slot] - c0);
        if (c < (uint32_t)nc) unsafeAtomicAdd(&acc[c], val[q] * usl_load_f32<TS>(W, slot));
    }
    __syncthreads();
    float* dst = grad_x + (size_t)i * d + c0;
    for (int c = threadIdx.x; c < nc; c += XS_NT) dst[c] = acc[c];
}

}  // namespace

// Labels a list holds at most: an instance with more nonzeros than 1/32 of the labels makes the gradient "dense".
static uint32_t list_capacity(const usl_ctx* c) {
    const int64_t cap = c->m / 32;
    return (uint32_t)(cap < 64 ? 64 : cap);
}

bool usl_sparse_supported(const usl_ctx* c) {
    // lists of max_b * m/32 entries: not worth their memory for tiny layers, and the dense kernels win there anyway
    return c->m >= 65536 && (size_t)c->max_b * list_capacity(c) * 8 <= ((size_t)4 << 30);
}

// Does the context expect a gradient that is almost all zeros?  Reads, without waiting, what the looks of
// earlier calls reported (whichever of them have finished by now).
bool usl_sparse_expected(usl_ctx* c) {
    if (c->hint_host) {
        const volatile uint32_t* h = c->hint_host;
        const uint32_t serial = h[0], dense = h[1];
        if (serial != c->hint_seen) {
            c->hint_seen = serial;
            c->sparse_streak = dense ? 0 : c->sparse_streak + 1;
        }
    }
    bool expected = c->sparse_streak >= 2;
    if (const char* e = getenv("USL_TUNE_SPARSE")) {
        if (!strcmp(e, "always")) expected = true;
        else if (!strcmp(e, "never")) expected = false;
    }
    return expected;
}

// Looks at g[b][m] and, if the context has reason to expect a gradient that is almost all zeros, builds the
// lists of its nonzeros.  Every call enqueues the sample look (a few microseconds), whose verdict reaches the host
// through two pinned words that the NEXT calls read without waiting: after two such looks in a row that found
// the sample sparse the lists are tried, and the first look that finds it dense ends that.  A gradient that turns
// sparse is therefore handled by the dense kernels for two more calls, one that turns dense by the gated dense
// kernels once -- never wrongly, and a steadily dense gradient (binary cross-entropy) pays for the sample only.
// *gate: NULL = only the dense kernels run this time; else the device word that is 0 when the lists stand and 1
// when the dense kernels (which are then enqueued behind the gate) have to do the work.
// USL_TUNE_SPARSE=always / never overrides the expectation (tests, profiling).
usl_status usl_sparse_compact(usl_ctx* c, const float* g, int32_t b, const uint32_t** gate) {
    const uint32_t cap = list_capacity(c);
    *gate = nullptr;
    if (!c->hint_host) {
        USL_HIP(c, hipHostMalloc((void**)&c->hint_host, 64, hipHostMallocMapped));
        c->hint_host[0] = 0; c->hint_host[1] = 1;
        USL_HIP(c, hipHostGetDevicePointer((void**)&c->hint_dev, c->hint_host, 0));
    }
    USL_TRY(usl_reserve(c, (void**)&c->nz_state, &c->nz_state_cap, ((size_t)c->max_b + 16) * 4));
    const bool try_lists = usl_sparse_expected(c);
    hipLaunchKernelGGL(k_zero_state, dim3(1), dim3(256), 0, c->stream, c->nz_state, (size_t)b + 16);
    hipLaunchKernelGGL(k_probe_density, dim3((unsigned)b), dim3(256), 0, c->stream, g, c->m, c->nz_state, c->hint_dev,
                       ++c->probe_serial);
    if (!try_lists) return usl_check_launch(c, "gradient sample");
    USL_TRY(usl_reserve(c, (void**)&c->nz_lab, &c->nz_lab_cap, (size_t)c->max_b * cap * 4));
    USL_TRY(usl_reserve(c, (void**)&c->nz_val, &c->nz_val_cap, (size_t)c->max_b * cap * 4));
    dim3 grid((unsigned)((c->m + CG_CHUNK - 1) / CG_CHUNK), (unsigned)b);
    hipLaunchKernelGGL(k_compact_g, grid, dim3(CG_NT), 0, c->stream, g, c->m, cap, c->nz_state, c->nz_lab, c->nz_val);
    *gate = c->nz_state;
    return usl_check_launch(c, "gradient compaction");
}

usl_status usl_sparse_backward_weight(usl_ctx* c, const void* x, const int32_t* idx, float* grad_W, int32_t b) {
    const uint32_t cap = list_capacity(c);
    const size_t N = (size_t)c->m * c->k;
    hipLaunchKernelGGL(k_zero_if_sparse, dim3(c->num_cu * 8), dim3(256), 0, c->stream, grad_W, N, c->nz_state);
    dim3 grid(64, (unsigned)b);
    if (c->storage == USL_F32)
        hipLaunchKernelGGL(k_bww_sparse<float>, grid, dim3(256), 0, c->stream, (const float*)x, idx, c->nz_state,
                           c->nz_lab, c->nz_val, cap, grad_W, c->d, c->k);
    else
        hipLaunchKernelGGL(k_bww_sparse<uint16_t>, grid, dim3(256), 0, c->stream, (const uint16_t*)x, idx, c->nz_state,
                           c->nz_lab, c->nz_val, cap, grad_W, c->d, c->k);
    return usl_check_launch(c, "backward_weight over the nonzero gradients");
}

usl_status usl_sparse_backward_input(usl_ctx* c, const int32_t* idx, const void* W, float* grad_x, int32_t b) {
    const uint32_t cap = list_capacity(c);
    const size_t lds = (size_t)(c->d < XS_COLS ? c->d : XS_COLS) * 4;
    dim3 grid((unsigned)((c->d + XS_COLS - 1) / XS_COLS), (unsigned)b);
    if (c->storage == USL_F32) {
        USL_HIP(c, hipFuncSetAttribute(reinterpret_cast<const void*>(k_bwi_sparse<float>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        hipLaunchKernelGGL(k_bwi_sparse<float>, grid, dim3(XS_NT), lds, c->stream, idx, (const float*)W, c->nz_state,
                           c->nz_lab, c->nz_val, cap, grad_x, c->d, c->k);
    } else {
        USL_HIP(c, hipFuncSetAttribute(reinterpret_cast<const void*>(k_bwi_sparse<uint16_t>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        hipLaunchKernelGGL(k_bwi_sparse<uint16_t>, grid, dim3(XS_NT), lds, c->stream, idx, (const uint16_t*)W,
                           c->nz_state, c->nz_lab, c->nz_val, cap, grad_x, c->d, c->k);
    }
    return usl_check_launch(c, "backward_input over the nonzero gradients");
}
