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


// ---- The feature-stationary LDS form of the input gradient (the mirror image of the forward kernel), as a timing
// prototype on synthetic lists: a workgroup owns a window of WL labels and a block of features, keeps the features'
// (label-in-window 16 bit, weight) lists in registers -- two lists of complementary length share the KTOT register
// slots of a lane pair: list A from slot 0 up, list B from slot KTOT-1 down --, walks the batch staging g[i, window]
// through LDS with LDS-DMA, gathers, un-permutes its sums through LDS and leaves one partial sum per window, which a
// second kernel adds up.  BUFS = 1: one row buffer, copy then gathers.  BUFS = 2: two row buffers, the copy of
// instance i+1 (issued from inline assembly, so that the compiler puts no wait in front of the LDS reads) is in
// flight while instance i is gathered.  DISTINCT = 1: every half-wavefront reads 32 different banks at every step (the
// bound a perfect bank-aware order would reach); 0: random labels.  COPY / GATHER switch the two phases off.
typedef const __attribute__((address_space(3))) float lds_f32_t;
template <int N>
__device__ __forceinline__ float lds_gather16(const uint32_t (&pk)[N], int t, uint32_t base) {
    uint32_t a;
    const uint32_t two = 2;
    if (t & 1) asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_1" : "=v"(a) : "s"(two), "v"(pk[t >> 1]));
    else asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_0" : "=v"(a) : "s"(two), "v"(pk[t >> 1]));
    return *reinterpret_cast<lds_f32_t*>(static_cast<uintptr_t>(a + base));
}

template <int KTOT, int PAIRS, int WL, int BUFS, int DISTINCT, int COPY, int GATHER>
__global__ void __launch_bounds__(1024)
k_lds_form(const float* __restrict__ g, int64_t m, int b, int d, int nfb, int nwin, float* __restrict__ partial,
           int acap, int bcap) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    constexpr int NT = 1024, NF = NT * PAIRS * 2;   // features per workgroup
    // all feature blocks of a window on one XCD (workgroups are dealt to the 8 XCDs round robin): its slice of g is
    // fetched from HBM once and served to the others from that XCD's L2
    const int w = (blockIdx.x & 7) + 8 * (blockIdx.x / (8 * nfb)), fb = (blockIdx.x >> 3) % nfb;
    if (w >= nwin) return;
    uint32_t pk[PAIRS][KTOT / 2];
    float wt[PAIRS][KTOT];
    uint32_t seed = mix32(blockIdx.x * 1024u + threadIdx.x + 1u);
#pragma unroll
    for (int p = 0; p < PAIRS; ++p)
#pragma unroll
        for (int t = 0; t < KTOT; ++t) {
            seed = mix32(seed + t);
            uint32_t off = seed % WL;
            if (DISTINCT) off = (threadIdx.x & 31u) + 32u * (seed % (WL / 32));
            if (t & 1) pk[p][t >> 1] |= off << 16; else pk[p][t >> 1] = off;
            wt[p][t] = (float)(seed >> 8) * 1e-8f;
        }
    float* outbuf = reinterpret_cast<float*>(lds_raw + (size_t)BUFS * WL * 4);
    const float* gw = g + (size_t)w * WL;
    const int lane = threadIdx.x & 63;
    auto stage = [&](int i, int buf) {
        const uint4* src = reinterpret_cast<const uint4*>(gw + (size_t)i * m);
        for (int v = (threadIdx.x >> 6) * 64; v < WL / 4; v += NT) {
            const uint32_t la = __builtin_amdgcn_readfirstlane((uint32_t)(buf * WL * 4 + v * 16));
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(la), "v"(src + v + lane) : "memory");
        }
    };
    auto leave = [&](int i) {   // the sums of instance i, un-permuted in LDS, go out as one contiguous run
        float* dst = partial + ((size_t)w * b + i) * d + (size_t)fb * NF;
        const float* ob = outbuf + (BUFS == 2 ? (i & 1) * NF : 0);
        for (int v = threadIdx.x; v < NF / 4; v += NT)
            reinterpret_cast<float4*>(dst)[v] = reinterpret_cast<const float4*>(ob)[v];
    };
    // L2 warm-up of a later row slice, split among the nfb workgroups of the window (they share an XCD): the load is
    // issued from inline assembly and its result never read, so no wait follows it; the register stays reserved
    // until the next vmcnt(0) wait
    uint32_t token = 0;
    auto warm = [&](int i) {
        const int lines = WL * 4 / 128, per = (lines + nfb - 1) / nfb;
        const int line = fb * per + (int)threadIdx.x;
        if ((int)threadIdx.x < per && line < lines) {
            const char* p = reinterpret_cast<const char*>(gw + (size_t)i * m) + (size_t)line * 128;
            asm volatile("global_load_dword %0, %1, off" : "=v"(token) : "v"(p));
        }
    };
    if (BUFS == 2 && COPY) stage(0, 0);
    if (BUFS == 2) { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); __syncthreads(); }
    for (int i = 0; i < b; ++i) {
        if (BUFS == 1) {
            if (COPY) stage(i, 0);
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            asm volatile("" : "+v"(token));
            __syncthreads();
            if (COPY && i + 1 < b) warm(i + 1);
        } else {
            if (COPY && i + 1 < b) stage(i + 1, (i + 1) & 1);
            if (COPY && i + 2 < b) warm(i + 2);
            if (COPY && i > 0) leave(i - 1);
        }
        const uint32_t base = BUFS == 2 ? (uint32_t)(i & 1) * WL * 4 : 0u;
        float* ob = outbuf + (BUFS == 2 ? (i & 1) * NF : 0);
#pragma unroll
        for (int p = 0; p < PAIRS; ++p) {
            float acc_a = 0.f, acc_b = 0.f;
            if (GATHER) {
#pragma unroll
                for (int q = 0; q < KTOT / 4; ++q)
                    if (q * 4 < acap) {
#pragma unroll
                        for (int u = 0; u < 4; ++u) acc_a = fmaf(wt[p][q * 4 + u], lds_gather16(pk[p], q * 4 + u, base), acc_a);
                    }
#pragma unroll
                for (int q = 0; q < KTOT / 4; ++q)
                    if (q * 4 >= KTOT - bcap) {
#pragma unroll
                        for (int u = 0; u < 4; ++u) acc_b = fmaf(wt[p][q * 4 + u], lds_gather16(pk[p], q * 4 + u, base), acc_b);
                    }
            }
            ob[(2 * p) * NT + threadIdx.x] = acc_a;
            ob[(2 * p + 1) * NT + threadIdx.x] = acc_b;
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        asm volatile("" : "+v"(token));
        __syncthreads();
        if (BUFS == 1 && COPY) leave(i);
    }
    if (BUFS == 2 && COPY) leave(b - 1);
}

__global__ void k_add_partials(const float4* __restrict__ partial, int n, size_t n4, float4* __restrict__ out) {
    size_t v = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t step = (size_t)gridDim.x * blockDim.x;
    for (; v < n4; v += step) {
        float4 a = partial[v];
        for (int q = 1; q < n; ++q) {
            const float4 t = partial[(size_t)q * n4 + v];
            a.x += t.x; a.y += t.y; a.z += t.z; a.w += t.w;
        }
        out[v] = a;
    }
}

const char* const NAMES[] = {
    "hbm_read_GBps", "hbm_write_GBps", "hbm_copy_GBps_read_plus_write",
    "lds_gather_b32_random_lanes_per_clk_cu", "lds_gather_b32_conflict_free_lanes_per_clk_cu",
    "lds_gather_b64_random_lanes_per_clk_cu", "lds_gather_b64_conflict_free_lanes_per_clk_cu",
    "lds_gather_b128_random_lanes_per_clk_cu", "lds_gather_b128_conflict_free_lanes_per_clk_cu",
    "l2_to_lds_row_copy_bytes_per_clk_cu", "l2_to_lds_row_copy_aggregate_GBps",
    "l2_piece_gather_3MiB_per_xcd_GBps", "l2_piece_gather_8MiB_per_xcd_GBps",
    "compute_units", "clock_GHz",
    // the LDS form of the input gradient at m = 524288, d = 32768, k = 32, b = 256 (ms per call-equivalent)
    "lds_form_one_buffer_distinct_banks_ms", "lds_form_one_buffer_random_banks_ms", "lds_form_add_16_partials_ms",
    "lds_form_two_buffers_distinct_banks_ms", "lds_form_two_buffers_gathers_only_ms", "lds_form_two_buffers_copies_only_ms",
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
    {   // the LDS form of the input gradient: g = bufa (b x m floats), partial sums = bufb
        const int b = 256, d = 32768;
        const int64_t m = 16 * 32768;
        auto time_form = [&](auto kern, int wl, int nf, int bufs, int acap, int bcap, int slot) -> hipError_t {
            const size_t sh = ((size_t)wl * 4 + (size_t)nf * 4) * bufs;
            const int nwin = (int)(m / wl), nfb = d / nf;
            const int grid = ((nwin + 7) / 8) * 8 * nfb;
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)sh);
            if (e != hipSuccess) return e;
            hipLaunchKernelGGL(kern, dim3(grid), dim3(1024), sh, 0, reinterpret_cast<const float*>(bufa), m, b, d, nfb, nwin,
                               reinterpret_cast<float*>(bufb), acap, bcap);
            if ((e = hipEventRecord(t.a, 0)) != hipSuccess) return e;
            for (int r = 0; r < 3; ++r)
                hipLaunchKernelGGL(kern, dim3(grid), dim3(1024), sh, 0, reinterpret_cast<const float*>(bufa), m, b, d, nfb, nwin,
                                   reinterpret_cast<float*>(bufb), acap, bcap);
            if ((e = hipEventRecord(t.b, 0)) != hipSuccess) return e;
            if ((e = hipEventSynchronize(t.b)) != hipSuccess) return e;
            float t_ms = 0.f;
            if ((e = hipEventElapsedTime(&t_ms, t.a, t.b)) != hipSuccess) return e;
            out[slot] = t_ms / 3;
            return hipGetLastError();
        };
        CK(hipMemset(bufa, 0, (size_t)b * m * 4));
        // one row buffer of 32768 labels, 2048 features per workgroup: lists of 36 + 32 of the 72 slots in use
        CK(time_form(k_lds_form<72, 1, 32768, 1, 1, 1, 1>, 32768, 2048, 1, 36, 32, 15));
        CK(time_form(k_lds_form<72, 1, 32768, 1, 0, 1, 1>, 32768, 2048, 1, 36, 32, 16));
        {
            const size_t n4 = (size_t)b * d / 4;
            float4* sum = reinterpret_cast<float4*>(bufa);   // g is not needed while the partial sums are added
            hipLaunchKernelGGL(k_add_partials, dim3(2048), dim3(256), 0, 0, reinterpret_cast<const float4*>(bufb), 16, n4, sum);
            CK(hipEventRecord(t.a, 0));
            for (int r = 0; r < 3; ++r)
                hipLaunchKernelGGL(k_add_partials, dim3(2048), dim3(256), 0, 0, reinterpret_cast<const float4*>(bufb), 16, n4, sum);
            CK(hipEventRecord(t.b, 0)); CK(hipEventSynchronize(t.b)); CK(hipEventElapsedTime(&ms, t.a, t.b));
            CK(hipGetLastError());
            out[17] = ms / 3;
            CK(hipMemset(bufa, 0, (size_t)b * m * 4));
        }
        // two row buffers of 16384 labels, 4096 features per workgroup (two pairs per lane, 20 + 16 of 36 slots)
        CK(time_form(k_lds_form<36, 2, 16384, 2, 1, 1, 1>, 16384, 4096, 2, 20, 16, 18));
        CK(time_form(k_lds_form<36, 2, 16384, 2, 1, 0, 1>, 16384, 4096, 2, 20, 16, 19));
        CK(time_form(k_lds_form<36, 2, 16384, 2, 1, 1, 0>, 16384, 4096, 2, 20, 16, 20));
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
