// Input gradient (Algorithm 2): grad_x[i][c] = sum over connections (j,t) with idx[j][t]==c of
// W[j][t] * g[i][j].
//
// The paper scatters with one atomic add per (instance, connection).  On gfx950 neither global
// nor LDS float atomics come near the needed rate (b*m*k additions), so the sum is turned into a
// gather: a column-major view of the connectivity (for every feature c the list of its slots) is
// rebuilt whenever idx changes, the upstream gradient is transposed to gT[m][b] so that the b
// values of one label are contiguous, and one wavefront per (feature, tile of 256 instances) adds
// W * gT rows in registers.  No atomics touch grad_x; the only non-determinism is the order of
// the slots inside a column list (filled with an atomic cursor).
#include "usl_internal.h"

namespace {

__global__ void k_zero_u32(uint32_t* p, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t s = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += s) p[i] = 0;
}

__global__ void __launch_bounds__(256)
k_csc_count(const int32_t* __restrict__ idx, size_t N, uint32_t* __restrict__ count) {
    const size_t s = (size_t)gridDim.x * 256;
    for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < N; e += s)
        atomicAdd(&count[idx[e]], 1u);
}

// exclusive scan of count[d] into ptr[d+1]; cursor[c] = ptr[c].  One block.
__global__ void __launch_bounds__(1024)
k_csc_scan(uint32_t* __restrict__ cursor /* in: counts */, uint32_t* __restrict__ ptr, int d) {
    __shared__ uint32_t part[1024];
    const int per = (d + 1023) / 1024;
    const int a = threadIdx.x * per, e = min(d, a + per);
    uint32_t s = 0;
    for (int q = a; q < e; ++q) s += cursor[q];
    part[threadIdx.x] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t run = 0;
        for (int q = 0; q < 1024; ++q) { const uint32_t v = part[q]; part[q] = run; run += v; }
        ptr[d] = run;
    }
    __syncthreads();
    uint32_t run = part[threadIdx.x];
    for (int q = a; q < e; ++q) {
        const uint32_t v = cursor[q];
        ptr[q] = run;
        cursor[q] = run;
        run += v;
    }
}

__global__ void __launch_bounds__(256)
k_csc_fill(const int32_t* __restrict__ idx, size_t N, int k, uint32_t* __restrict__ cursor,
           uint32_t* __restrict__ slot, int32_t* __restrict__ label) {
    const size_t s = (size_t)gridDim.x * 256;
    for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < N; e += s) {
        const uint32_t pos = atomicAdd(&cursor[idx[e]], 1u);
        slot[pos] = (uint32_t)e;
        label[pos] = (int32_t)(e / (size_t)k);
    }
}

// out[c][r] = in[r][c] for r < R, c < C; rows of in / out are ld_in / ld_out elements apart.
__global__ void __launch_bounds__(256)
k_transpose(const float* __restrict__ in, float* __restrict__ out, int64_t R, int64_t C,
            int64_t ld_in, int64_t ld_out) {
    __shared__ float tile[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const int64_t r0 = (int64_t)blockIdx.y * 32, c0 = (int64_t)blockIdx.x * 32;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int64_t r = r0 + ty + 8 * q, cc = c0 + tx;
        if (r < R && cc < C) tile[ty + 8 * q][tx] = in[r * ld_in + cc];
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int64_t cc = c0 + ty + 8 * q, r = r0 + tx;
        if (cc < C && r < R) out[cc * ld_out + r] = tile[tx][ty + 8 * q];
    }
}

// One wavefront per (feature c, tile of 256 instances); lane l owns instances 4l .. 4l+3 of the tile.
template <typename TS>
__global__ void __launch_bounds__(256)
k_bwd_input_gather(const float* __restrict__ gT, const TS* __restrict__ W,
                   const uint32_t* __restrict__ ptr, const uint32_t* __restrict__ slot,
                   const int32_t* __restrict__ label, float* __restrict__ gxT, int d, int bp) {
    const int lane = threadIdx.x & 63;
    const int c = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (c >= d) return;  // whole wavefront leaves together
    const int i0 = blockIdx.y * 256 + lane * 4;
    const bool live = i0 < bp;
    const uint32_t p0 = ptr[c], p1 = ptr[c + 1];
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (uint32_t base = p0; base < p1; base += 64) {
        const int n = (int)min(64u, p1 - base);
        int32_t jv = 0;
        float wv = 0.f;
        if (lane < n) {
            jv = label[base + lane];
            wv = usl_load_f32<TS>(W, (size_t)slot[base + lane]);
        }
        // lanes >= n hold label 0 and weight 0, so the count can be rounded up to the unroll
        // factor: the extra rows are valid memory and contribute nothing
        for (int u0 = 0; u0 < n; u0 += 8) {
            float4 v[8];
            float w[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const int32_t j = __builtin_amdgcn_readlane(jv, u0 + q);
                w[q] = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(wv), u0 + q));
                v[q] = live ? *reinterpret_cast<const float4*>(gT + (size_t)j * bp + i0)
                            : make_float4(0.f, 0.f, 0.f, 0.f);
            }
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                acc.x = fmaf(w[q], v[q].x, acc.x); acc.y = fmaf(w[q], v[q].y, acc.y);
                acc.z = fmaf(w[q], v[q].z, acc.z); acc.w = fmaf(w[q], v[q].w, acc.w);
            }
        }
    }
    if (live) *reinterpret_cast<float4*>(gxT + (size_t)c * bp + i0) = acc;
}

usl_status build_csc(usl_ctx* c, const int32_t* idx) {
    const size_t N = (size_t)c->m * c->k;
    if (!c->csc_ptr) {
        size_t cap = 0;
        USL_TRY(usl_reserve(c, (void**)&c->csc_ptr, &cap, ((size_t)c->d + 1) * 4)); cap = 0;
        USL_TRY(usl_reserve(c, (void**)&c->csc_cursor, &cap, (size_t)c->d * 4)); cap = 0;
        USL_TRY(usl_reserve(c, (void**)&c->csc_slot, &cap, N * 4)); cap = 0;
        USL_TRY(usl_reserve(c, (void**)&c->csc_label, &cap, N * 4));
    }
    size_t blocks = (N + 256 * 8 - 1) / (256 * 8);
    if (blocks > (size_t)c->num_cu * 16) blocks = (size_t)c->num_cu * 16;
    hipLaunchKernelGGL(k_zero_u32, dim3(64), dim3(256), 0, c->stream, c->csc_cursor, (size_t)c->d);
    hipLaunchKernelGGL(k_csc_count, dim3((unsigned)blocks), dim3(256), 0, c->stream, idx, N, c->csc_cursor);
    hipLaunchKernelGGL(k_csc_scan, dim3(1), dim3(1024), 0, c->stream, c->csc_cursor, c->csc_ptr, c->d);
    hipLaunchKernelGGL(k_csc_fill, dim3((unsigned)blocks), dim3(256), 0, c->stream, idx, N, c->k,
                       c->csc_cursor, c->csc_slot, c->csc_label);
    USL_TRY(usl_check_launch(c, "column lists"));
    c->csc_built_for = idx;
    return USL_OK;
}

}  // namespace

usl_status usl_launch_backward_input(usl_ctx* c, const float* g, const int32_t* idx, const void* W,
                                     float* grad_x, int32_t b) {
    if (c->csc_built_for != idx) USL_TRY(build_csc(c, idx));
    const int bp = (b + 3) & ~3;
    USL_TRY(usl_reserve(c, (void**)&c->gT, &c->gT_cap, (size_t)c->m * bp * 4));
    USL_TRY(usl_reserve(c, (void**)&c->gxT, &c->gxT_cap, (size_t)c->d * bp * 4));
    {   // gT[m][bp] = transpose of g[b][m]
        dim3 grid((unsigned)((c->m + 31) / 32), (unsigned)((b + 31) / 32));
        hipLaunchKernelGGL(k_transpose, grid, dim3(256), 0, c->stream, g, c->gT, (int64_t)b, c->m, c->m, (int64_t)bp);
    }
    {
        dim3 grid((unsigned)((c->d + 3) / 4), (unsigned)((bp + 255) / 256));
        if (c->storage == USL_F32)
            hipLaunchKernelGGL(k_bwd_input_gather<float>, grid, dim3(256), 0, c->stream, c->gT,
                               (const float*)W, c->csc_ptr, c->csc_slot, c->csc_label, c->gxT, c->d, bp);
        else
            hipLaunchKernelGGL(k_bwd_input_gather<uint16_t>, grid, dim3(256), 0, c->stream, c->gT,
                               (const uint16_t*)W, c->csc_ptr, c->csc_slot, c->csc_label, c->gxT, c->d, bp);
    }
    {   // grad_x[b][d] = transpose of gxT[d][bp] (first b columns)
        dim3 grid((unsigned)((b + 31) / 32), (unsigned)((c->d + 31) / 32));
        hipLaunchKernelGGL(k_transpose, grid, dim3(256), 0, c->stream, c->gxT, grad_x, (int64_t)c->d,
                           (int64_t)b, (int64_t)bp, (int64_t)c->d);
    }
    return usl_check_launch(c, "backward_input");
}
