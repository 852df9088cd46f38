// Connection redistribution (magnitude prune of the whole layer + random regrow inside each row),
// initial connectivity, the index validator and the raw generator words.
//
// Prune: the n smallest keys (|W| bit pattern, flat slot) are found without sorting: a radix
// select over the magnitude bits (most significant digit first, one histogram pass per digit)
// yields the threshold magnitude T and the number q of slots with magnitude exactly T that still
// have to go; those q are the first in flat order, found with a per-block tie count, a scan of
// the block counts and an in-block rank.  Regrow: a group of lanes owns a row, the lane of slot t
// keeps idx[j][t]; candidates are generated redundantly by the group and tested with a ballot.
#include "usl_internal.h"

namespace {

// ---- Philox-4x32, 10 rounds (Salmon, Moraes, Dror, Shaw, SC'11) --------------------------------
struct U4 { uint32_t x, y, z, w; };
__device__ __forceinline__ U4 philox4x32_10(U4 c, uint32_t k0, uint32_t k1) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hi0 = __umulhi(0xD2511F53u, c.x), lo0 = 0xD2511F53u * c.x;
        const uint32_t hi1 = __umulhi(0xCD9E8D57u, c.z), lo1 = 0xCD9E8D57u * c.z;
        c = U4{hi1 ^ c.y ^ k0, lo1, hi0 ^ c.w ^ k1, lo0};
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return c;
}
// candidate number a for slot t of row j: word 0, mapped to [0, d) by multiply-shift
__device__ __forceinline__ int32_t draw_column(uint32_t k0, uint32_t k1, uint32_t epoch_lo,
                                               uint32_t j, uint32_t t, uint32_t a, uint32_t d) {
    const U4 r = philox4x32_10(U4{j, t, a, epoch_lo}, k0, k1);
    return (int32_t)__umulhi(r.x, d);
}

__global__ void k_philox(const uint32_t* __restrict__ ctr, uint32_t k0, uint32_t k1,
                         uint32_t* __restrict__ out, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const U4 r = philox4x32_10(U4{ctr[4 * i], ctr[4 * i + 1], ctr[4 * i + 2], ctr[4 * i + 3]}, k0, k1);
    out[4 * i] = r.x; out[4 * i + 1] = r.y; out[4 * i + 2] = r.z; out[4 * i + 3] = r.w;
}

// ---- radix select ---------------------------------------------------------------------------
constexpr int SEL_BINS = 2048;
// device state: [0..SEL_BINS) histogram, then: prefix, remaining count, (unused), tie total
enum { ST_PREFIX = SEL_BINS, ST_REMAIN = SEL_BINS + 1, ST_TIES = SEL_BINS + 3, ST_WORDS = SEL_BINS + 4 };

template <typename TS> __device__ __forceinline__ uint32_t mag_key(const TS* W, size_t f);
template <> __device__ __forceinline__ uint32_t mag_key<float>(const float* W, size_t f) {
    return __float_as_uint(W[f]) & 0x7FFFFFFFu;
}
template <> __device__ __forceinline__ uint32_t mag_key<uint16_t>(const uint16_t* W, size_t f) {
    return (uint32_t)W[f] & 0x7FFFu;
}

__global__ void k_sel_init(uint32_t* st, uint32_t n) {
    for (int i = threadIdx.x; i < ST_WORDS; i += blockDim.x) st[i] = 0;
    __syncthreads();
    if (threadIdx.x == 0) st[ST_REMAIN] = n;
}

// histogram of digit (key >> shift) & (2^bits - 1) over the keys whose higher bits equal the prefix
template <typename TS>
__global__ void __launch_bounds__(256)
k_sel_hist(const TS* __restrict__ W, size_t N, uint32_t* st, int shift, int bits, int first) {
    __shared__ uint32_t h[SEL_BINS];
    for (int i = threadIdx.x; i < SEL_BINS; i += 256) h[i] = 0;
    __syncthreads();
    const uint32_t prefix = st[ST_PREFIX];
    const uint32_t mask = (1u << bits) - 1u;
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t f = (size_t)blockIdx.x * 256 + threadIdx.x; f < N; f += stride) {
        const uint32_t key = mag_key<TS>(W, f);
        if (first || (key >> (shift + bits)) == prefix) atomicAdd(&h[(key >> shift) & mask], 1u);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < SEL_BINS; i += 256)
        if (h[i]) atomicAdd(&st[i], h[i]);
}

// picks the digit in which the running count crosses the remaining count; clears the histogram.
// One block of 256 lanes: each sums a run of consecutive bins, a scan over the lanes finds the run that holds
// the crossing, and that lane walks its few bins.
__global__ void __launch_bounds__(256) k_sel_pick(uint32_t* st, int bits) {
    __shared__ uint32_t run_sum[256];
    const int nb = 1 << bits;
    const int per = (nb + 255) / 256;             // at most SEL_BINS / 256
    const int first = (int)threadIdx.x * per;
    uint32_t mine = 0;
    for (int q = 0; q < per; ++q)
        if (first + q < nb) mine += st[first + q];
    run_sum[threadIdx.x] = mine;
    __syncthreads();
    for (int o = 1; o < 256; o <<= 1) {           // inclusive scan
        const uint32_t v = threadIdx.x >= (unsigned)o ? run_sum[threadIdx.x - o] : 0u;
        __syncthreads();
        run_sum[threadIdx.x] += v;
        __syncthreads();
    }
    const uint32_t remain = st[ST_REMAIN], prefix = st[ST_PREFIX];
    const uint32_t before = run_sum[threadIdx.x] - mine;
    const uint32_t total = run_sum[255];
    __syncthreads();
    if (before < remain && before + mine >= remain) {
        uint32_t cum = before;
        int bin = first;
        for (int q = 0; q < per; ++q) {
            const uint32_t hcount = st[first + q];
            if (cum + hcount >= remain) { bin = first + q; break; }
            cum += hcount;
        }
        st[ST_PREFIX] = (prefix << bits) | (uint32_t)bin;
        st[ST_REMAIN] = remain - cum;  // = how many keys equal to the final prefix must go
    } else if (threadIdx.x == 0 && total < remain) {   // cannot happen for a consistent histogram
        st[ST_PREFIX] = (prefix << bits) | (uint32_t)(nb - 1);
        st[ST_REMAIN] = remain - total;
    }
    __syncthreads();
    for (int i = threadIdx.x; i < SEL_BINS; i += blockDim.x) st[i] = 0;
}

constexpr int MARK_NT = 256;
constexpr int MARK_PER = 16;
constexpr int MARK_CHUNK = MARK_NT * MARK_PER;

template <typename TS>
__global__ void __launch_bounds__(MARK_NT)
k_tie_count(const TS* __restrict__ W, size_t N, const uint32_t* __restrict__ st,
            uint32_t* __restrict__ tie_counts) {
    __shared__ uint32_t red[MARK_NT / 64];
    const uint32_t T = st[ST_PREFIX];
    const size_t f0 = (size_t)blockIdx.x * MARK_CHUNK + (size_t)threadIdx.x * MARK_PER;
    uint32_t cnt = 0;
    for (int q = 0; q < MARK_PER; ++q)
        if (f0 + q < N && mag_key<TS>(W, f0 + q) == T) ++cnt;
    for (int o = 32; o > 0; o >>= 1) cnt += __shfl_down(cnt, o);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = cnt;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t s = 0;
        for (int q = 0; q < MARK_NT / 64; ++q) s += red[q];
        tie_counts[blockIdx.x] = s;
    }
}

// exclusive scan of the per-block tie counts, in place (one block)
__global__ void __launch_bounds__(1024) k_tie_scan(uint32_t* tie_counts, size_t nblk) {
    __shared__ uint32_t part[1024];
    const size_t per = (nblk + 1023) / 1024;
    const size_t a = threadIdx.x * per, e = min(nblk, a + per);
    uint32_t s = 0;
    for (size_t q = a; q < e; ++q) s += tie_counts[q];
    part[threadIdx.x] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t run = 0;
        for (int q = 0; q < 1024; ++q) { const uint32_t v = part[q]; part[q] = run; run += v; }
    }
    __syncthreads();
    uint32_t run = part[threadIdx.x];
    for (size_t q = a; q < e; ++q) { const uint32_t v = tie_counts[q]; tie_counts[q] = run; run += v; }
}

// flags every removed slot and resets its value and moments
template <typename TS>
__global__ void __launch_bounds__(MARK_NT)
k_mark(TS* __restrict__ W, float* __restrict__ m1, float* __restrict__ m2, size_t N,
       const uint32_t* __restrict__ st, const uint32_t* __restrict__ tie_off,
       uint8_t* __restrict__ flags) {
    __shared__ uint32_t scan[MARK_NT];
    const uint32_t T = st[ST_PREFIX], q_take = st[ST_REMAIN];
    const size_t f0 = (size_t)blockIdx.x * MARK_CHUNK + (size_t)threadIdx.x * MARK_PER;
    uint32_t keys[MARK_PER];
    uint32_t mine = 0;
#pragma unroll
    for (int q = 0; q < MARK_PER; ++q) {
        keys[q] = f0 + q < N ? mag_key<TS>(W, f0 + q) : 0xFFFFFFFFu;
        mine += keys[q] == T;
    }
    scan[threadIdx.x] = mine;
    __syncthreads();
    for (int o = 1; o < MARK_NT; o <<= 1) {  // inclusive scan of the per-lane tie counts
        const uint32_t v = threadIdx.x >= (unsigned)o ? scan[threadIdx.x - o] : 0u;
        __syncthreads();
        scan[threadIdx.x] += v;
        __syncthreads();
    }
    uint32_t rank = tie_off[blockIdx.x] + scan[threadIdx.x] - mine;
#pragma unroll
    for (int q = 0; q < MARK_PER; ++q) {
        if (f0 + q >= N) break;
        bool gone = keys[q] < T;
        if (keys[q] == T) { gone = rank < q_take; ++rank; }
        flags[f0 + q] = gone ? 1 : 0;
        if (gone) {
            W[f0 + q] = (TS)0;
            m1[f0 + q] = 0.f;
            m2[f0 + q] = 0.f;
        }
    }
}

// Per-row variant of the prune: GS lanes own one row (as in k_regrow); lane t ranks its own magnitude among the
// row's by (key, slot) with GS shuffles and gives up its slot if fewer than per_row rank below it.
template <int GS, typename TS>
__global__ void __launch_bounds__(256)
k_mark_rows(TS* __restrict__ W, float* __restrict__ m1, float* __restrict__ m2, int64_t m, int k, int per_row,
            uint8_t* __restrict__ flags) {
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t row = gid / GS;
    const int t = (int)(gid % GS);
    const int lane = threadIdx.x & 63;
    const int gbase = lane & ~(GS - 1);
    const bool active = row < m && t < k;
    const size_t f = (size_t)row * k + t;
    const uint32_t key = active ? mag_key<TS>(W, f) : 0xFFFFFFFFu;   // idle lanes rank last
    int rank = 0;
#pragma unroll
    for (int u = 0; u < GS; ++u) {
        const uint32_t other = (uint32_t)__shfl((int)key, gbase + u);
        rank += (other < key || (other == key && u < t)) ? 1 : 0;
    }
    if (active) {
        const bool gone = rank < per_row;
        flags[f] = gone ? 1 : 0;
        if (gone) { W[f] = (TS)0; m1[f] = 0.f; m2[f] = 0.f; }
    }
}

// any k: one thread per row; the flags of the whole row are settled before the first value is reset
template <typename TS>
__global__ void __launch_bounds__(256)
k_mark_rows_serial(TS* __restrict__ W, float* __restrict__ m1, float* __restrict__ m2, int64_t m, int k,
                   int per_row, uint8_t* __restrict__ flags) {
    const int64_t row = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (row >= m) return;
    const size_t f0 = (size_t)row * k;
    for (int t = 0; t < k; ++t) {
        const uint32_t key = mag_key<TS>(W, f0 + t);
        int rank = 0;
        for (int u = 0; u < k; ++u) {
            const uint32_t other = mag_key<TS>(W, f0 + u);
            rank += (other < key || (other == key && u < t)) ? 1 : 0;
        }
        flags[f0 + t] = rank < per_row ? 1 : 0;
    }
    for (int t = 0; t < k; ++t)
        if (flags[f0 + t]) { W[f0 + t] = (TS)0; m1[f0 + t] = 0.f; m2[f0 + t] = 0.f; }
}

// ---- regrow ---------------------------------------------------------------------------------
// GS lanes own one row (GS = power of two >= k, <= 64); lane t of the group holds slot t.
// flags == nullptr means every slot is empty (initial connectivity).
template <int GS>
__global__ void __launch_bounds__(256)
k_regrow(int32_t* __restrict__ idx, const uint8_t* __restrict__ flags, int64_t m, uint32_t d, int k,
         uint32_t k0, uint32_t k1, uint32_t epoch_lo) {
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t row = gid / GS;
    const int t = (int)(gid % GS);
    const int lane = threadIdx.x & 63;
    const int gshift = lane & ~(GS - 1);
    const uint64_t gmask = GS == 64 ? ~0ull : ((1ull << GS) - 1ull);
    const bool active = row < m && t < k;
    const size_t f = (size_t)row * k + t;
    bool empty = active && (flags ? flags[f] != 0 : true);
    bool occupied = active && !empty;
    int32_t mine = occupied ? idx[f] : -1;
    const bool was_empty = empty;
    uint64_t todo = (__ballot(empty) >> gshift) & gmask;  // empty slots of my row, bit = slot
    uint32_t attempt = 0;
    while (__any(todo != 0)) {
        const int ts = todo ? __ffsll((unsigned long long)todo) - 1 : 0;
        const int32_t c = todo ? draw_column(k0, k1, epoch_lo, (uint32_t)row, (uint32_t)ts, attempt, d) : -2;
        const uint64_t clash = (__ballot(todo != 0 && occupied && mine == c) >> gshift) & gmask;
        if (todo) {
            if (clash == 0) {
                if (t == ts) { mine = c; occupied = true; }
                todo &= todo - 1;
                attempt = 0;
            } else {
                ++attempt;
            }
        }
    }
    if (was_empty) idx[f] = mine;
}

// any k: one thread per row, row kept in global memory
__global__ void __launch_bounds__(256)
k_regrow_serial(int32_t* __restrict__ idx, uint8_t* __restrict__ flags_rw, int64_t m, uint32_t d, int k,
                uint32_t k0, uint32_t k1, uint32_t epoch_lo) {
    const int64_t row = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (row >= m) return;
    int32_t* r = idx + row * k;
    uint8_t* e = flags_rw + row * k;  // 1 = empty; cleared as slots are filled
    for (int t = 0; t < k; ++t) {
        if (!e[t]) continue;
        for (uint32_t a = 0;; ++a) {
            const int32_t c = draw_column(k0, k1, epoch_lo, (uint32_t)row, (uint32_t)t, a, d);
            bool clash = false;
            for (int u = 0; u < k && !clash; ++u) clash = !e[u] && r[u] == c;
            if (!clash) { r[t] = c; e[t] = 0; break; }
        }
    }
}

__global__ void k_fill_u8(uint8_t* p, size_t n, uint8_t v) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t s = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += s) p[i] = v;
}

__global__ void __launch_bounds__(256)
k_validate(const int32_t* __restrict__ idx, int64_t m, int32_t d, int k, unsigned long long* bad) {
    const int64_t row = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (row >= m) return;
    const int32_t* r = idx + row * k;
    bool b = false;
    for (int t = 0; t < k && !b; ++t) {
        const int32_t c = r[t];
        if (c < 0 || c >= d) { b = true; break; }
        for (int u = 0; u < t; ++u)
            if (r[u] == c) { b = true; break; }
    }
    if (b) atomicAdd(bad, 1ull);
}

usl_status regrow(usl_ctx* c, int32_t* idx, uint8_t* flags, bool all_empty, uint64_t seed,
                  uint64_t epoch) {
    const uint32_t k0 = (uint32_t)seed;
    const uint32_t k1 = (uint32_t)(seed >> 32) ^ (uint32_t)(epoch >> 32);
    const uint32_t elo = (uint32_t)epoch;
    const int k = c->k;
    if (k > 64) {
        const size_t N = (size_t)c->m * k;
        if (all_empty)
            hipLaunchKernelGGL(k_fill_u8, dim3(c->num_cu * 4), dim3(256), 0, c->stream, flags, N, (uint8_t)1);
        hipLaunchKernelGGL(k_regrow_serial, dim3((unsigned)((c->m + 255) / 256)), dim3(256), 0, c->stream,
                           idx, flags, c->m, (uint32_t)c->d, k, k0, k1, elo);
        return usl_check_launch(c, "regrow (serial)");
    }
    int gs = 1;
    while (gs < k) gs <<= 1;
    const uint8_t* fl = all_empty ? nullptr : flags;
    const int64_t lanes = c->m * gs;
    const unsigned grid = (unsigned)((lanes + 255) / 256);
#define USL_RG(GS)                                                                             \
    hipLaunchKernelGGL(k_regrow<GS>, dim3(grid), dim3(256), 0, c->stream, idx, fl, c->m,       \
                       (uint32_t)c->d, k, k0, k1, elo)
    switch (gs) {
        case 1: USL_RG(1); break;
        case 2: USL_RG(2); break;
        case 4: USL_RG(4); break;
        case 8: USL_RG(8); break;
        case 16: USL_RG(16); break;
        case 32: USL_RG(32); break;
        default: USL_RG(64); break;
    }
#undef USL_RG
    return usl_check_launch(c, "regrow");
}

usl_status ensure_flags(usl_ctx* c) {
    if (c->prune_flags) return USL_OK;
    size_t cap = 0;
    return usl_reserve(c, (void**)&c->prune_flags, &cap, (size_t)c->m * c->k);
}

template <typename TS>
usl_status redistribute_t(usl_ctx* c, int32_t* idx, TS* W, float* m1, float* m2, int64_t n,
                          uint64_t seed, uint64_t epoch) {
    const size_t N = (size_t)c->m * c->k;
    if (!c->sel_hist) {
        size_t cap = 0;
        USL_TRY(usl_reserve(c, (void**)&c->sel_hist, &cap, ST_WORDS * sizeof(uint32_t)));
    }
    USL_TRY(ensure_flags(c));
    const size_t nmark = (N + MARK_CHUNK - 1) / MARK_CHUNK;
    size_t cap = c->tie_counts_cap;
    USL_TRY(usl_reserve(c, (void**)&c->tie_counts, &cap, nmark * sizeof(uint32_t)));
    c->tie_counts_cap = cap;
    uint32_t* st = c->sel_hist;
    hipLaunchKernelGGL(k_sel_init, dim3(1), dim3(256), 0, c->stream, st, (uint32_t)n);
    // digits, most significant first: 31 magnitude bits of a float, 15 of a bfloat16
    const int f32_bits[3] = {11, 10, 10}, bf_bits[2] = {8, 7};
    const int npass = sizeof(TS) == 4 ? 3 : 2;
    const int* bits = sizeof(TS) == 4 ? f32_bits : bf_bits;
    int shift = sizeof(TS) == 4 ? 31 : 15;
    size_t hblocks = (N + 256 * 16 - 1) / (256 * 16);
    if (hblocks > (size_t)c->num_cu * 8) hblocks = (size_t)c->num_cu * 8;
    for (int p = 0; p < npass; ++p) {
        shift -= bits[p];
        hipLaunchKernelGGL(k_sel_hist<TS>, dim3((unsigned)hblocks), dim3(256), 0, c->stream, W, N, st,
                           shift, bits[p], p == 0 ? 1 : 0);
        hipLaunchKernelGGL(k_sel_pick, dim3(1), dim3(256), 0, c->stream, st, bits[p]);
    }
    hipLaunchKernelGGL(k_tie_count<TS>, dim3((unsigned)nmark), dim3(MARK_NT), 0, c->stream, W, N, st,
                       c->tie_counts);
    hipLaunchKernelGGL(k_tie_scan, dim3(1), dim3(1024), 0, c->stream, c->tie_counts, nmark);
    hipLaunchKernelGGL(k_mark<TS>, dim3((unsigned)nmark), dim3(MARK_NT), 0, c->stream, W, m1, m2, N, st,
                       c->tie_counts, c->prune_flags);
    USL_TRY(usl_check_launch(c, "prune"));
    return regrow(c, idx, c->prune_flags, false, seed, epoch);
}

template <typename TS>
usl_status redistribute_rows_t(usl_ctx* c, int32_t* idx, TS* W, float* m1, float* m2, int per_row,
                               uint64_t seed, uint64_t epoch) {
    USL_TRY(ensure_flags(c));
    const int k = c->k;
    if (k > 64) {
        hipLaunchKernelGGL(k_mark_rows_serial<TS>, dim3((unsigned)((c->m + 255) / 256)), dim3(256), 0, c->stream,
                           W, m1, m2, c->m, k, per_row, c->prune_flags);
    } else {
        int gs = 1;
        while (gs < k) gs <<= 1;
        const unsigned grid = (unsigned)((c->m * gs + 255) / 256);
#define USL_MR(GS)                                                                                       \
    hipLaunchKernelGGL((k_mark_rows<GS, TS>), dim3(grid), dim3(256), 0, c->stream, W, m1, m2, c->m, k,   \
                       per_row, c->prune_flags)
        switch (gs) {
            case 1: USL_MR(1); break;
            case 2: USL_MR(2); break;
            case 4: USL_MR(4); break;
            case 8: USL_MR(8); break;
            case 16: USL_MR(16); break;
            case 32: USL_MR(32); break;
            default: USL_MR(64); break;
        }
#undef USL_MR
    }
    USL_TRY(usl_check_launch(c, "prune (per row)"));
    return regrow(c, idx, c->prune_flags, false, seed, epoch);
}

}  // namespace

usl_status usl_launch_redistribute(usl_ctx* c, int32_t* idx, void* W, float* m1, float* m2,
                                   int64_t n, uint64_t seed, uint64_t epoch) {
    return c->storage == USL_F32
               ? redistribute_t<float>(c, idx, (float*)W, m1, m2, n, seed, epoch)
               : redistribute_t<uint16_t>(c, idx, (uint16_t*)W, m1, m2, n, seed, epoch);
}

usl_status usl_launch_redistribute_rows(usl_ctx* c, int32_t* idx, void* W, float* m1, float* m2,
                                        int32_t per_row, uint64_t seed, uint64_t epoch) {
    return c->storage == USL_F32
               ? redistribute_rows_t<float>(c, idx, (float*)W, m1, m2, per_row, seed, epoch)
               : redistribute_rows_t<uint16_t>(c, idx, (uint16_t*)W, m1, m2, per_row, seed, epoch);
}

usl_status usl_launch_init_indices(usl_ctx* c, int32_t* idx, uint64_t seed) {
    if (c->k > 64) USL_TRY(ensure_flags(c));
    return regrow(c, idx, c->prune_flags, true, seed, ~(uint64_t)0);
}

usl_status usl_launch_validate(usl_ctx* c, const int32_t* idx, int64_t* n_bad_host) {
    if (!c->counter64) {
        size_t cap = 0;
        USL_TRY(usl_reserve(c, (void**)&c->counter64, &cap, 64));
    }
    hipLaunchKernelGGL(k_fill_u8, dim3(1), dim3(64), 0, c->stream, (uint8_t*)c->counter64, (size_t)8, (uint8_t)0);
    hipLaunchKernelGGL(k_validate, dim3((unsigned)((c->m + 255) / 256)), dim3(256), 0, c->stream, idx,
                       c->m, c->d, c->k, (unsigned long long*)c->counter64);
    USL_TRY(usl_check_launch(c, "validate"));
    int64_t v = 0;
    USL_HIP(c, hipMemcpyAsync(&v, c->counter64, 8, hipMemcpyDeviceToHost, c->stream));
    USL_HIP(c, hipStreamSynchronize(c->stream));
    *n_bad_host = v;
    return USL_OK;
}

usl_status usl_launch_philox(usl_ctx* c, const uint32_t* ctr, uint32_t key0, uint32_t key1,
                             uint32_t* out, int64_t n) {
    hipLaunchKernelGGL(k_philox, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, c->stream, ctr, key0,
                       key1, out, n);
    return usl_check_launch(c, "philox");
}
