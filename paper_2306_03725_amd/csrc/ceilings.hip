// Measurement kernels behind include/usl_ceilings.h: the rates of the chip that bound the layer's
// products.  Everything here is synthetic (hashed addresses, constant data); nothing is shared with
// the training kernels except the instructions they lean on.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/usl_ceilings.h"

namespace {

__device__ __forceinline__ uint32_t mix32(uint32_t x) {
    x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
    return x;
}

// ---- HBM streams: 16 bytes per lane, grid-stride
__global__ void k_stream_copy(const float4* __restrict__ a, float4* __restrict__ b, size_t n) {
    size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
    const size_t s = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += s) b[i] = a[i];
}
__global__ void k_stream_read(const float4* __restrict__ a, float* sink, size_t n) {
    size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
    const size_t s = (size_t)gridDim.x * blockDim.x;
    float acc = 0.f;
    for (; i < n; i += s) { const float4 v = a[i]; acc += (v.x + v.y) + (v.z + v.w); }
    if (acc == 123.456f) sink[0] = acc;
}
__global__ void k_stream_write(float4* __restrict__ b, size_t n) {
    size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
    const size_t s = (size_t)gridDim.x * blockDim.x;
    const float4 v = make_float4(1.f, 2.f, 3.f, 4.f);
    for (; i < n; i += s) b[i] = v;
}

// ---- LDS gathers: one workgroup of 1024 lanes per compute unit, 32 resident addresses per lane,
// WIDTH bytes per read.  PATTERN 0: random addresses.  PATTERN 1: the 32 lanes of a half-wavefront
// read 32 different banks (WIDTH 4: lane l reads bank l of a random row of 32 words; wider reads:
// consecutive lanes read consecutive elements) -- what a perfect bank-aware slot order would reach.
constexpr int LDS_WORDS = 32768;   // 128 KiB, the size of one float32 activation row of 32768 columns
template <int WIDTH, int PATTERN>
__global__ void __launch_bounds__(1024) k_lds_gather(float* sink, int reps) {
    extern __shared__ float lds[];
    for (int i = threadIdx.x; i < LDS_WORDS; i += 1024) lds[i] = (float)(i & 1023) * 1e-3f;
    __syncthreads();
    constexpr int EW = WIDTH / 4;                 // words per element
    constexpr uint32_t NE = LDS_WORDS / EW;       // elements in LDS
    uint32_t at[32];
    uint32_t seed = mix32(blockIdx.x * 1024u + threadIdx.x + 1u);
#pragma unroll
    for (int t = 0; t < 32; ++t) {
        seed = mix32(seed + t);
        uint32_t e = seed % NE;
        if (PATTERN == 1) {
            if (WIDTH == 4) e = (threadIdx.x & 31u) + 32u * (seed % (NE / 32u));
            else e = (threadIdx.x + 64u * (uint32_t)t * 7u) % NE;
        }
        at[t] = e * EW;
    }
    float acc = 0.f;
    for (int r = 0; r < reps; ++r) {
#pragma unroll
        for (int t = 0; t < 32; ++t) {
            if (WIDTH == 4) acc += lds[at[t]];
            else if (WIDTH == 8) { const float2 v = *reinterpret_cast<const float2*>(&lds[at[t]]); acc += v.x + v.y; }
            else { const float4 v = *reinterpret_cast<const float4*>(&lds[at[t]]); acc += (v.x + v.y) + (v.z + v.w); }
        }
#pragma unroll
        for (int t = 0; t < 32; ++t) at[t] = (acc == -1.0f) ? 0u : at[t];   // keeps the reads inside the loop
    }
    if (acc == 123.456f) sink[0] = acc;
}

// ---- L2 -> LDS: every workgroup (one per compute unit) copies the same `rows` rows of 128 KiB with
// global_load_lds_dwordx4, a barrier between rows, as the product kernels stage activation rows.
__global__ void __launch_bounds__(1024) k_row_copy(const uint4* __restrict__ src, float* sink, int rows) {
    extern __shared__ float lds[];
    constexpr int ROW_V = LDS_WORDS / 4;   // 16-byte pieces per row
    uint4* dd = reinterpret_cast<uint4*>(lds);
    const int lane = threadIdx.x & 63;
    float acc = 0.f;
    for (int r = 0; r < rows; ++r) {
        const uint4* s = src + (size_t)r * ROW_V;
        for (int v = (threadIdx.x >> 6) * 64; v < ROW_V; v += 1024)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(s + v + lane),
                                             (__attribute__((address_space(3))) void*)(dd + v), 16, 0, 0);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        acc += lds[(threadIdx.x * 97 + r) & (LDS_WORDS - 1)];
        __syncthreads();
    }
    if (acc == 123.456f) sink[0] = acc;
}

// ---- 128-byte pieces from a region one XCD's L2 holds: workgroups are dealt to the 8 XCDs round robin,
// XCD x gathers from slice x of the array; 8 lanes x 16 bytes read one piece, 8 pieces in flight per lane group.
__global__ void __launch_bounds__(256) k_piece_gather(const float4* __restrict__ region, size_t slice_pieces,
                                                      float* sink, int trips) {
    const float4* base = region + (size_t)(blockIdx.x & 7) * slice_pieces * 8 + (threadIdx.x & 7);
    uint32_t seed = mix32((blockIdx.x * 256u + threadIdx.x) >> 3);
    float acc = 0.f;
    for (int r = 0; r < trips; ++r) {
        float4 v[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            seed = mix32(seed + q + 1);
            v[q] = base[(size_t)(seed % (uint32_t)slice_pieces) * 8];
        }
#pragma unroll
        for (int q = 0; q < 8; ++q) acc += (v[q].x + v[q].y) + (v[q].z + v[q].w);
    }
    if (acc == 123.456f) sink[0] = acc;
}

const char* const NAMES[] = {
    "hbm_read_GBps", "hbm_write_GBps", "hbm_copy_GBps_read_plus_write",
    "lds_gather_b32_random_lanes_per_clk_cu", "lds_gather_b32_conflict_free_lanes_per_clk_cu",
    "lds_gather_b64_random_lanes_per_clk_cu", "lds_gather_b64_conflict_free_lanes_per_clk_cu",
    "lds_gather_b128_random_lanes_per_clk_cu", "lds_gather_b128_conflict_free_lanes_per_clk_cu",
    "l2_to_lds_row_copy_bytes_per_clk_cu", "l2_to_lds_row_copy_aggregate_GBps",
    "l2_piece_gather_3MiB_per_xcd_GBps", "l2_piece_gather_8MiB_per_xcd_GBps",
    "compute_units", "clock_GHz",
};
constexpr int NFIG = (int)(sizeof(NAMES) / sizeof(NAMES[0]));

struct Timer {
    hipEvent_t a, b;
    hipError_t make() { hipError_t e = hipEventCreate(&a); return e != hipSuccess ? e : hipEventCreate(&b); }
    void drop() { (void)hipEventDestroy(a); (void)hipEventDestroy(b); }
};

}  // namespace

extern "C" int usl_ceilings_count(void) { return NFIG; }
extern "C" const char* usl_ceilings_name(int i) { return i >= 0 && i < NFIG ? NAMES[i] : nullptr; }

#define CK(call)                                  \
    do {                                          \
        hipError_t e_ = (call);                   \
        if (e_ != hipSuccess) { rc = (int)e_; goto done; } \
    } while (0)

extern "C" int usl_ceilings_run(double* values, int n) {
    int rc = 0;
    double out[NFIG];
    for (int i = 0; i < NFIG; ++i) out[i] = 0.0;
    Timer t;
    float* sink = nullptr;
    float4 *bufa = nullptr, *bufb = nullptr;
    bool have_timer = false;
    float ms = 0.f;
    int dev = 0, cu = 0;
    double clk = 0.0;
    hipDeviceProp_t p;
    CK(hipGetDevice(&dev));
    CK(hipGetDeviceProperties(&p, dev));
    cu = p.multiProcessorCount;
    clk = (double)p.clockRate * 1e3;
    out[13] = cu;
    out[14] = clk * 1e-9;
    CK(t.make());
    have_timer = true;
    CK(hipMalloc((void**)&sink, 1024));
    {   // HBM streams over 1 GiB
        const size_t bytes = (size_t)1 << 30, nv = bytes / 16;
        CK(hipMalloc((void**)&bufa, bytes));
        CK(hipMalloc((void**)&bufb, bytes));
        CK(hipMemset(bufa, 1, bytes));
        CK(hipMemset(bufb, 0, bytes));
        const int grid = cu * 8, reps = 5;
        hipLaunchKernelGGL(k_stream_read, dim3(grid), dim3(1024), 0, 0, bufa, sink, nv);
        CK(hipEventRecord(t.a, 0));
        for (int r = 0; r < reps; ++r) hipLaunchKernelGGL(k_stream_read, dim3(grid), dim3(1024), 0, 0, bufa, sink, nv);
        CK(hipEventRecord(t.b, 0)); CK(hipEventSynchronize(t.b)); CK(hipEventElapsedTime(&ms, t.a, t.b));
        out[0] = (double)bytes * reps / (ms * 1e-3) / 1e9;
        hipLaunchKernelGGL(k_stream_write, dim3(grid), dim3(1024), 0, 0, bufb, nv);
        CK(hipEventRecord(t.a, 0));
        for (int r = 0; r < reps; ++r) hipLaunchKernelGGL(k_stream_write, dim3(grid), dim3(1024), 0, 0, bufb, nv);
        CK(hipEventRecord(t.b, 0)); CK(hipEventSynchronize(t.b)); CK(hipEventElapsedTime(&ms, t.a, t.b));
        out[1] = (double)bytes * reps / (ms * 1e-3) / 1e9;
        hipLaunchKernelGGL(k_stream_copy, dim3(grid), dim3(1024), 0, 0, bufa, bufb, nv);
        CK(hipEventRecord(t.a, 0));
        for (int r = 0; r < reps; ++r) hipLaunchKernelGGL(k_stream_copy, dim3(grid), dim3(1024), 0, 0, bufa, bufb, nv);
        CK(hipEventRecord(t.b, 0)); CK(hipEventSynchronize(t.b)); CK(hipEventElapsedTime(&ms, t.a, t.b));
        out[2] = 2.0 * (double)bytes * reps / (ms * 1e-3) / 1e9;
        CK(hipGetLastError());
    }
    {   // LDS gathers
        const size_t sh = (size_t)LDS_WORDS * 4;
        const int reps = 1000;
#define USL_LDS_RUN(WIDTH, PATTERN, slot)                                                                        \
        do {                                                                                                     \
            CK(hipFuncSetAttribute(reinterpret_cast<const void*>(k_lds_gather<WIDTH, PATTERN>),                  \
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)sh));                        \
            hipLaunchKernelGGL((k_lds_gather<WIDTH, PATTERN>), dim3(cu), dim3(1024), sh, 0, sink, 10);           \
            CK(hipEventRecord(t.a, 0));                                                                          \
            hipLaunchKernelGGL((k_lds_gather<WIDTH, PATTERN>), dim3(cu), dim3(1024), sh, 0, sink, reps);         \
            CK(hipEventRecord(t.b, 0)); CK(hipEventSynchronize(t.b)); CK(hipEventElapsedTime(&ms, t.a, t.b));    \
            CK(hipGetLastError());                                                                               \
            out[slot] = (double)cu * 1024.0 * 32.0 * reps / (ms * 1e-3) / cu / clk;                              \
        } while (0)
        USL_LDS_RUN(4, 0, 3); USL_LDS_RUN(4, 1, 4);
        USL_LDS_RUN(8, 0, 5); USL_LDS_RUN(8, 1, 6);
        USL_LDS_RUN(16, 0, 7); USL_LDS_RUN(16, 1, 8);
#undef USL_LDS_RUN
    }
    {   // L2 -> LDS row copies: 256 rows of 128 KiB (32 MiB, the activations of one batch)
        const size_t sh = (size_t)LDS_WORDS * 4;
        const int rows = 256;
        CK(hipFuncSetAttribute(reinterpret_cast<const void*>(k_row_copy), hipFuncAttributeMaxDynamicSharedMemorySize, (int)sh));
        hipLaunchKernelGGL(k_row_copy, dim3(cu), dim3(1024), sh, 0, reinterpret_cast<const uint4*>(bufa), sink, rows);
        CK(hipEventRecord(t.a, 0));
        hipLaunchKernelGGL(k_row_copy, dim3(cu), dim3(1024), sh, 0, reinterpret_cast<const uint4*>(bufa), sink, rows);
        CK(hipEventRecord(t.b, 0)); CK(hipEventSynchronize(t.b)); CK(hipEventElapsedTime(&ms, t.a, t.b));
        CK(hipGetLastError());
        const double bytes = (double)rows * sh;
        out[9] = bytes / (ms * 1e-3) / clk;
        out[10] = bytes * cu / (ms * 1e-3) / 1e9;
    }
    for (int which = 0; which < 2; ++which) {   // piece gathers from a slice per XCD
        const size_t slice_bytes = which == 0 ? (size_t)3 << 20 : (size_t)8 << 20;
        const size_t slice_pieces = slice_bytes / 128;
        const int trips = 64, grid = cu * 32;
        hipLaunchKernelGGL(k_piece_gather, dim3(grid), dim3(256), 0, 0, bufa, slice_pieces, sink, trips);
        CK(hipEventRecord(t.a, 0));
        hipLaunchKernelGGL(k_piece_gather, dim3(grid), dim3(256), 0, 0, bufa, slice_pieces, sink, trips);
        CK(hipEventRecord(t.b, 0)); CK(hipEventSynchronize(t.b)); CK(hipEventElapsedTime(&ms, t.a, t.b));
        CK(hipGetLastError());
        out[11 + which] = (double)grid * 32.0 * trips * 8.0 * 128.0 / (ms * 1e-3) / 1e9;
    }
done:
    (void)hipDeviceSynchronize();
    if (bufa) (void)hipFree(bufa);
    if (bufb) (void)hipFree(bufb);
    if (sink) (void)hipFree(sink);
    if (have_timer) t.drop();
    for (int i = 0; i < NFIG && i < n; ++i) values[i] = out[i];
    return rc;
}
