// Input gradient (Algorithm 2): grad_x[i][c] = sum over connections (j,t) with idx[j][t]==c of
// W[j][t] * g[i][j].
//
// The paper scatters with one atomic add per (instance, connection).  On gfx950 neither global nor
// LDS float atomics come near the needed rate (b*m*k additions), so the sum is turned into a gather
// over a private column-major view of the connectivity, rebuilt whenever idx changes.
//
// Memory plan.  g is re-laid as gT[tile][m][32]: the batch is cut into tiles of 32 instances and every
// (tile, label) owns one contiguous 128-byte piece (one cache line).  The naive gather (one wavefront per
// feature reading all of a label's values) re-reads every label k times from HBM / Infinity Cache
// (m*k*b*4 bytes: 16 GB at m=500k, k=32, b=256).  Instead:
//   * the tile index is the fastest grid dimension, so that with round-robin dispatch of workgroups to
//     the 8 XCDs all work on tile t lands on XCD t mod 8 and shares one L2;
//   * the labels are cut into windows whose tile-slice of gT fits that L2; the kernel is launched
//     once per window and handles the connections of every feature that fall into the window, so
//     each 128-byte piece is fetched once and then served k times from L2;
//   * the column lists are therefore grouped by (window, feature), and inside a window ordered by
//     falling length; partial sums are added into gxT[tile][d][32] by the later windows (plain
//     read-modify-write: launches are ordered).
// A list entry is the flat slot number j*k+t of a connection: the label is slot / k, and the same
// number tells the per-call weight gather where W[j][t] lives.
// Eight lanes (8 x float4 = 32 instances) form a group that walks one feature's list; a wavefront
// reads eight 128-byte pieces per load instruction.  No atomics touch grad_x; the only
// non-determinism is the order of the slots inside one (window, feature) list.
#include <math.h>
#include <stdlib.h>

#include "usl_internal.h"

namespace {

__global__ void k_zero_u32(uint32_t* p, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t s = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += s) p[i] = 0;
}

// Fingerprint of idx: a sum of mixed 16-byte groups at up to 4096 evenly spaced places (64 KiB read by one
// workgroup, every load in flight at once: a few microseconds).  store = 1 records it when the column lists
// are built; store = 0 compares on a later call and raises print[2] (as a 32-bit word) when the contents are
// no longer those the lists were built from: a new tensor at a recycled address, a checkpoint copied in, ...
// A single edited entry can slip through the sample; wholesale replacement cannot.
__device__ __forceinline__ void idx_fingerprint_block(const uint32_t* __restrict__ idx, size_t n_words,
                                                      uint64_t* __restrict__ print, int store) {   // 1024 lanes
    __shared__ uint64_t red[16];
    const size_t groups = n_words / 4;
    const size_t samples = groups < 4096 ? groups : 4096;
    const size_t stride = samples ? groups / samples : 1;   // >= 1
    uint4 v[4];
    size_t at[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const size_t s = (size_t)q * 1024 + threadIdx.x;
        at[q] = s < samples ? s * stride : 0;
        v[q] = s < samples ? reinterpret_cast<const uint4*>(idx)[at[q]] : make_uint4(0, 0, 0, 0);
    }
    uint64_t h = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        if ((size_t)q * 1024 + threadIdx.x >= samples) continue;
        uint64_t a = ((uint64_t)v[q].x << 32 | v[q].y) ^ (at[q] * 0x9E3779B97F4A7C15ull);
        uint64_t b2 = ((uint64_t)v[q].z << 32 | v[q].w) + (at[q] << 7);
        a ^= a >> 31; a *= 0xD6E8FEB86659FD93ull; a ^= a >> 29;
        b2 ^= b2 >> 33; b2 *= 0xC2B2AE3D27D4EB4Full; b2 ^= b2 >> 30;
        h += a + (b2 << 1 | b2 >> 63);
    }
    for (size_t w = groups * 4 + threadIdx.x; w < n_words; w += 1024) h += (uint64_t)idx[w] * 0xFF51AFD7ED558CCDull;   // ragged tail
    for (int o = 32; o > 0; o >>= 1) h += __shfl_down(h, o);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = h;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint64_t t = 0;
        for (int q = 0; q < 16; ++q) t += red[q];
        if (store) { print[0] = t; }
        else if (print[0] != t) reinterpret_cast<uint32_t*>(print)[4] = 1u;
    }
}
__global__ void __launch_bounds__(1024)
k_idx_fingerprint(const uint32_t* __restrict__ idx, size_t n_words, uint64_t* __restrict__ print, int store) {
    idx_fingerprint_block(idx, n_words, print, store);
}

// Lists are grouped by (label window, feature).  A workgroup takes one of `splits` equal shares of
// a window's slots (contiguous in idx) and a chunk of up to 32768 features, and counts its share in
// an LDS histogram; global memory sees one coalesced atomic per (workgroup, feature), not one per slot.
constexpr int CSC_NT = 1024, CSC_CHUNK = 32768;

__device__ __forceinline__ void csc_share(int64_t m, int k, int win_labels, int splits, size_t* e0, size_t* e1) {
    const int w = blockIdx.x / splits, s = blockIdx.x % splits;
    const size_t w0 = (size_t)w * win_labels * k;
    const size_t w1 = (size_t)min((int64_t)(w + 1) * win_labels, m) * k;
    const size_t per = (w1 - w0 + splits - 1) / splits;
    *e0 = min(w0 + per * s, w1);
    *e1 = min(*e0 + per, w1);
}

__device__ __forceinline__ void csc_histogram(const int32_t* __restrict__ idx, size_t e0, size_t e1, int c0, int nc,
                                              uint32_t* hist) {
    for (int q = threadIdx.x; q < nc; q += CSC_NT) hist[q] = 0;
    __syncthreads();
    for (size_t e = e0 + threadIdx.x; e < e1; e += CSC_NT) {
        const uint32_t c = (uint32_t)(idx[e] - c0);
        if (c < (uint32_t)nc) atomicAdd(&hist[c], 1u);
    }
    __syncthreads();
}

// count (zeroed by the caller) += this workgroup's histogram
__global__ void __launch_bounds__(CSC_NT)
k_csc_count(const int32_t* __restrict__ idx, int64_t m, int k, int d, int win_labels, int splits,
            uint32_t* __restrict__ count) {
    extern __shared__ uint32_t hist[];
    const int c0 = blockIdx.y * CSC_CHUNK, nc = min(CSC_CHUNK, d - c0);
    size_t e0, e1;
    csc_share(m, k, win_labels, splits, &e0, &e1);
    csc_histogram(idx, e0, e1, c0, nc, hist);
    uint32_t* dst = count + (size_t)(blockIdx.x / splits) * d + c0;
    for (int q = threadIdx.x; q < nc; q += CSC_NT)
        if (hist[q]) atomicAdd(&dst[q], hist[q]);
}

// Exclusive scan of count[n] into ptr[n+1] (and cursor[c] = ptr[c]) in three launches: per-chunk
// sums, a one-block scan of those, and a per-chunk rescan with the chunk's offset.
constexpr int SCAN_NT = 1024, SCAN_PER = 8, SCAN_CHUNK = SCAN_NT * SCAN_PER;

__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t* sh, uint32_t* total) {
    // sh: SCAN_NT words.  Returns the sum of v over lower thread ids; *total = sum over the block.
    sh[threadIdx.x] = v;
    __syncthreads();
    for (int o = 1; o < SCAN_NT; o <<= 1) {
        const uint32_t t = threadIdx.x >= (unsigned)o ? sh[threadIdx.x - o] : 0u;
        __syncthreads();
        sh[threadIdx.x] += t;
        __syncthreads();
    }
    *total = sh[SCAN_NT - 1];
    return sh[threadIdx.x] - v;
}

__global__ void __launch_bounds__(SCAN_NT)
k_scan_sums(const uint32_t* __restrict__ count, size_t n, uint32_t* __restrict__ sums) {
    __shared__ uint32_t sh[SCAN_NT];
    const size_t f0 = (size_t)blockIdx.x * SCAN_CHUNK + (size_t)threadIdx.x * SCAN_PER;
    uint32_t s = 0;
    for (int q = 0; q < SCAN_PER; ++q)
        if (f0 + q < n) s += count[f0 + q];
    uint32_t total;
    block_exclusive_scan(s, sh, &total);
    if (threadIdx.x == 0) sums[blockIdx.x] = total;
}

__global__ void __launch_bounds__(SCAN_NT)
k_scan_top(uint32_t* __restrict__ sums, size_t nchunks, uint32_t* __restrict__ ptr_end) {
    __shared__ uint32_t sh[SCAN_NT];
    const size_t per = (nchunks + SCAN_NT - 1) / SCAN_NT;
    const size_t a = min(nchunks, threadIdx.x * per), e = min(nchunks, a + per);
    uint32_t s = 0;
    for (size_t q = a; q < e; ++q) s += sums[q];
    uint32_t total;
    uint32_t run = block_exclusive_scan(s, sh, &total);
    for (size_t q = a; q < e; ++q) { const uint32_t v = sums[q]; sums[q] = run; run += v; }
    if (threadIdx.x == 0) *ptr_end = total;
}

__global__ void __launch_bounds__(SCAN_NT)
k_scan_apply(uint32_t* __restrict__ cursor /* in: counts */, const uint32_t* __restrict__ sums,
             size_t n, uint32_t* __restrict__ ptr) {
    __shared__ uint32_t sh[SCAN_NT];
    const size_t f0 = (size_t)blockIdx.x * SCAN_CHUNK + (size_t)threadIdx.x * SCAN_PER;
    uint32_t v[SCAN_PER];
    uint32_t s = 0;
#pragma unroll
    for (int q = 0; q < SCAN_PER; ++q) { v[q] = f0 + q < n ? cursor[f0 + q] : 0u; s += v[q]; }
    uint32_t total;
    uint32_t run = sums[blockIdx.x] + block_exclusive_scan(s, sh, &total);
#pragma unroll
    for (int q = 0; q < SCAN_PER; ++q) {
        if (f0 + q < n) { ptr[f0 + q] = run; cursor[f0 + q] = run; }
        run += v[q];
    }
}

// Same decomposition.  The workgroup counts its share again, reserves that many places in every
// list with one atomic on `taken` (zeroed by the caller), and hands the places out from LDS cursors.
// The order of a list's entries is therefore not fixed; the sums that walk it do not fix theirs either.
__global__ void __launch_bounds__(CSC_NT)
k_csc_fill(const int32_t* __restrict__ idx, int64_t m, int k, int d, int win_labels, int splits,
           const uint32_t* __restrict__ ptr /* by rank */, const uint32_t* __restrict__ rank_of,
           uint32_t* __restrict__ taken, uint32_t* __restrict__ slot) {
    extern __shared__ uint32_t cur[];
    const int c0 = blockIdx.y * CSC_CHUNK, nc = min(CSC_CHUNK, d - c0);
    size_t e0, e1;
    csc_share(m, k, win_labels, splits, &e0, &e1);
    csc_histogram(idx, e0, e1, c0, nc, cur);
    const size_t bin0 = (size_t)(blockIdx.x / splits) * d + c0;
    for (int q = threadIdx.x; q < nc; q += CSC_NT) {
        const uint32_t n = cur[q];
        if (n) cur[q] = ptr[bin0 - c0 + rank_of[bin0 + q]] + atomicAdd(&taken[bin0 + q], n);
    }
    __syncthreads();
    for (size_t e = e0 + threadIdx.x; e < e1; e += CSC_NT) {
        const uint32_t c = (uint32_t)(idx[e] - c0);
        if (c < (uint32_t)nc) {
            const uint32_t pos = atomicAdd(&cur[c], 1u);
            slot[pos] = (uint32_t)e;
        }
    }
}

// Features of one window in the order of falling list length (one workgroup per window).  A wavefront
// of the gather kernel walks 8 lists in lockstep and pays for the longest of them; with this order the 8
// are of (nearly) one length.  The lists themselves are laid out in this order too, so neighbours in the
// kernel are neighbours in memory.  order[rank] = feature, rank_of[feature] = rank, by_rank[rank] = its
// list length.  Lists of 1023 entries or more share the first bucket.
__global__ void __launch_bounds__(1024)
k_csc_order(const uint32_t* __restrict__ count, int d, uint32_t* __restrict__ order,
            uint32_t* __restrict__ rank_of, uint32_t* __restrict__ by_rank) {
    __shared__ uint32_t start[1024];
    const size_t w0 = (size_t)blockIdx.x * d;
    start[threadIdx.x] = 0;
    __syncthreads();
    for (int c = threadIdx.x; c < d; c += 1024) atomicAdd(&start[min(count[w0 + c], 1023u)], 1u);
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t run = 0;
        for (int q = 1023; q >= 0; --q) { const uint32_t n = start[q]; start[q] = run; run += n; }
    }
    __syncthreads();
    for (int c = threadIdx.x; c < d; c += 1024) {
        const uint32_t n = count[w0 + c];
        const uint32_t r = atomicAdd(&start[min(n, 1023u)], 1u);
        order[w0 + r] = (uint32_t)c;
        rank_of[w0 + c] = r;
        by_rank[w0 + r] = n;
    }
}

// Weights in list order, as float32 (refreshed on every call: W changes with every Adam step).  The lists of
// one label window draw on a contiguous slice of W (window labels * k values); workgroups are dealt round-robin to the 8 XCDs,
// so window = f(blockIdx % 8) keeps a slice in one XCD's L2 while its bpw workgroups pick it apart.
// bpw workgroups share a window: 32, or 128 when there are so few windows that 32 would leave most of
// the chip idle and every lane a long chain of dependent loads.
constexpr int GW_NT = 1024;
template <typename TS>
__global__ void __launch_bounds__(GW_NT)
k_gather_w(const TS* __restrict__ W, const uint32_t* __restrict__ slot, const uint32_t* __restrict__ ptr,
           int d, int nwin, float* __restrict__ wl, int bpw, const uint32_t* __restrict__ gate,
           const uint32_t* __restrict__ idx_check /* or NULL */, size_t n_words, uint64_t* __restrict__ print) {
    if (gate && *gate == 0) return;   // the sparse kernels do this call's work
    // the first workgroup also checks that idx still holds what the lists were built from (see idx_fingerprint_block)
    if (idx_check && blockIdx.x == 0) idx_fingerprint_block(idx_check, n_words, print, 0);
    int w, local;
    if (nwin >= 8) {
        const int xcd = blockIdx.x & 7;
        local = blockIdx.x >> 3;
        w = (local / bpw) * 8 + xcd;
        if (w >= nwin) return;
    } else {   // fewer windows than XCDs (W is small then): every window is spread over the whole chip
        w = (int)(blockIdx.x % (unsigned)nwin);
        local = (int)(blockIdx.x / (unsigned)nwin);
    }
    const uint32_t p0 = ptr[(size_t)w * d], p1 = ptr[(size_t)(w + 1) * d];
    const uint32_t STEP = (uint32_t)bpw * GW_NT;
    uint32_t p = p0 + (local % bpw) * GW_NT + threadIdx.x;
    for (; p + 3 * STEP < p1; p += 4 * STEP) {
        uint32_t e[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) e[q] = slot[p + q * STEP];
        float v[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) v[q] = usl_load_f32<TS>(W, (size_t)e[q]);
#pragma unroll
        for (int q = 0; q < 4; ++q) wl[p + q * STEP] = v[q];
    }
    for (; p < p1; p += STEP) wl[p] = usl_load_f32<TS>(W, (size_t)slot[p]);
}

// grad_x[i][c] = gxT[i/32][c][i%32] for i < b.  blockIdx.y = tile, blockIdx.x = block of 32 features.
__global__ void __launch_bounds__(256)
k_untile(const float* __restrict__ gxT, float* __restrict__ grad_x, int64_t b, int64_t d,
         const uint32_t* __restrict__ gate, const uint32_t* __restrict__ stale) {
    __shared__ float tile[32][33];
    if (gate && *gate == 0) return;
    const bool poison = *stale != 0;   // the lists were built from other contents of idx: no number is better than a wrong one
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const int64_t i0 = (int64_t)blockIdx.y * 32, c0 = (int64_t)blockIdx.x * 32;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int64_t c = c0 + ty + 8 * q;
        if (c < d) tile[ty + 8 * q][tx] = gxT[((size_t)blockIdx.y * d + c) * 32 + tx];
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int64_t i = i0 + ty + 8 * q, c = c0 + tx;
        if (i < b && c < d) grad_x[i * d + c] = poison ? __uint_as_float(0x7FC00000u) : tile[tx][ty + 8 * q];
    }
}

// gT[i/32][j][i%32] = g[i][j] (one contiguous 128-byte piece per label and tile of 32 instances: with rows of
// b values a tile's pieces would sit a fixed distance apart and crowd into a fraction of the L2's sets and
// channels), and for every label j and tile of 32 instances a byte that tells whether any of
// the 32 values is non-zero, plus the number of such (label, tile) cells in a 1/64 sample of the labels.  A squared-hinge gradient
// is zero for every easy negative (Section 3.3), and the gather below skips those pieces.
// blockIdx.y is the tile, so the 32 instances of a block are exactly one tile.
__global__ void __launch_bounds__(256)
k_transpose_g(const float* __restrict__ g, float* __restrict__ gT, int64_t b, int64_t m,
              uint8_t* __restrict__ nzf, uint32_t* __restrict__ nz_cells, const uint32_t* __restrict__ gate) {
    __shared__ float tile[32][33];
    if (gate && *gate == 0) return;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const int64_t r0 = (int64_t)blockIdx.y * 32, c0 = (int64_t)blockIdx.x * 32;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int64_t r = r0 + ty + 8 * q, cc = c0 + tx;
        tile[ty + 8 * q][tx] = (r < b && cc < m) ? g[r * m + cc] : 0.f;
    }
    __syncthreads();
    __shared__ uint32_t block_cells;
    if (threadIdx.x == 0) block_cells = 0;
    uint32_t cells = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int64_t cc = c0 + ty + 8 * q, r = r0 + tx;   // label cc, instance r
        const float v = tile[tx][ty + 8 * q];
        if (cc < m) gT[((size_t)blockIdx.y * m + cc) * 32 + tx] = v;   // instances past b hold zeros
        const unsigned long long bal = __ballot(v != 0.f);
        const bool any = ((bal >> (threadIdx.x & 32)) & 0xFFFFFFFFull) != 0;   // my half-wavefront = one label
        if (tx == 0 && cc < m) {
            nzf[(size_t)blockIdx.y * m + cc] = any ? 1 : 0;
            cells += any ? 1u : 0u;
        }
    }
    // the count only steers a heuristic: one block of labels in 64 is sampled, one atomic per block
    if ((blockIdx.x & 63) == 0) {
        if (cells) atomicAdd(&block_cells, cells);
        __syncthreads();
        if (threadIdx.x == 0 && block_cells) atomicAdd(nz_cells, block_cells);
    }
}

// One launch per label window: launch boundaries are what keeps all workgroups of an XCD inside the
// same window (a single persistent sweep, with or without a soft pacing counter, drifted apart and
// lost the L2 reuse -- measured slower).  blockIdx.x = tile of 32 instances within the launch's 8 (fastest, so that a
// tile stays on one XCD), blockIdx.y = block of 32 features; lanes 8g..8g+7 of a wavefront walk the
// list of one feature, lane l of the group owns instances 4l..4l+3 of the tile.
// SPLIT = 8 (few features, long lists: small d) gives a feature a whole wavefront: each of its 8 lane
// groups walks a contiguous eighth of the list and the eight sums are added by lane shuffles, so a launch
// has 8 times the workgroups and an eighth of the dependent trips.
template <int SPLIT>
__global__ void __launch_bounds__(256)
k_bwd_input_window(const float* __restrict__ gT, const float* __restrict__ wl,
                   const uint32_t* __restrict__ ptr /* this window's d+1 offsets, by rank */,
                   const uint32_t* __restrict__ order /* this window's features by falling list length */,
                   const uint32_t* __restrict__ slot, int k, int kshift /* log2 k, or -1 */,
                   float* __restrict__ gxT, int d, int tile0,
                   int accumulate, const uint8_t* __restrict__ nzf /* this tile row is nzf + tile*m */,
                   int64_t m, const uint32_t* __restrict__ nz_cells, uint32_t sparse_below,
                   const uint32_t* __restrict__ gate) {
    if (gate && *gate == 0) return;
    const int rank = SPLIT == 1 ? blockIdx.y * 32 + (threadIdx.x >> 3) : blockIdx.y * 4 + (threadIdx.x >> 6);
    if (rank >= d) return;   // SPLIT = 8: the whole wavefront leaves
    const int c = (int)order[rank];
    auto label_of = [&](uint32_t e) -> int32_t { return (int32_t)(kshift >= 0 ? e >> kshift : e / (uint32_t)k); };
    uint32_t p = ptr[rank];
    uint32_t p1 = ptr[rank + 1];
    if (SPLIT > 1) {   // this lane group's share: a multiple of 8 entries, the last share takes the rest
        const uint32_t per = ((p1 - p + SPLIT * 8 - 1) / (SPLIT * 8)) * 8;
        const uint32_t sg = (threadIdx.x >> 3) & (SPLIT - 1);
        p = min(p1, p + sg * per);
        p1 = min(p1, p + per);
    }
    const int tile = tile0 + (int)blockIdx.x;
    const float* col = gT + (size_t)tile * m * 32 + (threadIdx.x & 7) * 4;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    // Mostly-zero gradient (decided on the device from the cell count, the same for every lane):
    // look the piece up in the flag table first and fetch only pieces that hold something.
    if (*nz_cells < sparse_below) {
        const uint8_t* fl = nzf + (size_t)tile * m;
        const int sub = threadIdx.x & 7, gl = (threadIdx.x & 63) & ~7;
        for (; p < p1; p += 8) {   // lane s of the group looks entry s up; the group then visits the live ones
            const uint32_t pp = min(p + sub, p1 - 1);
            const int32_t jm = label_of(slot[pp]);
            const float wm = wl[pp];
            const bool live = p + sub < p1 && fl[jm] != 0;
            uint32_t todo = (uint32_t)(__ballot(live) >> gl) & 0xFFu;
            while (todo) {
                const int q = __ffs(todo) - 1;
                todo &= todo - 1;
                const int32_t j = __shfl(jm, gl + q);
                const float w = __shfl(wm, gl + q);
                const float4 v = *reinterpret_cast<const float4*>(col + (size_t)j * 32);
                acc.x = fmaf(w, v.x, acc.x); acc.y = fmaf(w, v.y, acc.y);
                acc.z = fmaf(w, v.z, acc.z); acc.w = fmaf(w, v.w, acc.w);
            }
        }
    }
    // Lists are short (window labels * k / d entries: 24 at Large), so the walk is a chain of
    // dependent load latencies, not a stream, and the memory pipeline spends as long on a one-word
    // load as on a 16-byte one.  U entries go per trip: lane s of the group fetches the (label, weight)
    // of entry s with one load each and the group passes them round by lane shuffles; the tail is
    // masked rather than walked one by one; the next trip's pairs are requested while this trip's
    // pieces are in flight.
    constexpr int U = 8;
    if (p < p1) {
        const int sub = threadIdx.x & 7, gl = (threadIdx.x & 63) & ~7;
        // The (slot, weight) pairs are requested two trips ahead, into two register sets used in turn: they
        // stream from HBM, and one trip is less than that round trip.
        auto fetch = [&](uint32_t at, uint32_t& raw, float& wv) {
            const uint32_t pp = min(at + sub, p1 - 1);
            raw = slot[pp];
            wv = at + sub < p1 ? wl[pp] : 0.f;   // a masked entry adds 0*0, whatever the repeated piece holds
        };
        uint32_t rawA, rawB = 0;
        float wA, wB = 0.f;
        fetch(p, rawA, wA);
        if (p + U < p1) fetch(p + U, rawB, wB);
        auto trip = [&](uint32_t& raw, float& wv) -> bool {
            const int32_t jm = label_of(raw);
            const float wm = wv;
            int32_t j[U];
#pragma unroll
            for (int q = 0; q < U; ++q) j[q] = __shfl(jm, gl + q);
            float4 v[U];
#pragma unroll
            for (int q = 0; q < U / 2; ++q) v[q] = *reinterpret_cast<const float4*>(col + (size_t)j[q] * 32);
            // the second half of a trip is not even requested when the list ends before it (lists of one
            // wavefront are of nearly one length, so the instruction is then skipped by the whole wavefront)
            if (p + U / 2 < p1) {
#pragma unroll
                for (int q = U / 2; q < U; ++q) v[q] = *reinterpret_cast<const float4*>(col + (size_t)j[q] * 32);
            } else {
#pragma unroll
                for (int q = U / 2; q < U; ++q) v[q] = make_float4(0.f, 0.f, 0.f, 0.f);
            }
            float w[U];
#pragma unroll
            for (int q = 0; q < U; ++q) w[q] = __shfl(wm, gl + q);
            if (p + 2 * U < p1) fetch(p + 2 * U, raw, wv);
#pragma unroll
            for (int q = 0; q < U; ++q) {
                const float4 vv = p + q < p1 ? v[q] : make_float4(0.f, 0.f, 0.f, 0.f);
                acc.x = fmaf(w[q], vv.x, acc.x); acc.y = fmaf(w[q], vv.y, acc.y);
                acc.z = fmaf(w[q], vv.z, acc.z); acc.w = fmaf(w[q], vv.w, acc.w);
            }
            p += U;
            return p >= p1;
        };
        while (true) {
            if (trip(rawA, wA)) break;
            if (trip(rawB, wB)) break;
        }
    }
    if (SPLIT > 1) {
#pragma unroll
        for (int o = 8; o < 8 * SPLIT; o <<= 1) {
            acc.x += __shfl_xor(acc.x, o); acc.y += __shfl_xor(acc.y, o);
            acc.z += __shfl_xor(acc.z, o); acc.w += __shfl_xor(acc.w, o);
        }
        if (((threadIdx.x >> 3) & (SPLIT - 1)) != 0) return;
    }
    float4* dst = reinterpret_cast<float4*>(gxT + ((size_t)tile * d + c) * 32 + (threadIdx.x & 7) * 4);
    if (accumulate) {
        const float4 o = *dst;
        acc.x += o.x; acc.y += o.y; acc.z += o.z; acc.w += o.w;
    }
    *dst = acc;
}

int window_labels(const usl_ctx* c) {
    // A window's 128-byte-per-label slice of gT (3 MiB at 24576 labels) should sit in one XCD's 4 MiB L2 with room for
    // the list entries that stream past it (window * k * 8 bytes per tile), while every window costs a round trip of
    // the partial sums (d * 256 bytes per tile).  Measured best: 24576 at k = 32, d = 32768 (among 8192 ... 32768),
    // 16384 at k = 64, d = 32768, 32768 at k = 32, d = 65536 -- the rule below meets all three.
    double w = 24576.0 * sqrt(((double)c->d / 32768.0) * (32.0 / (double)c->k));
    int win = (int)((w + 2048.0) / 4096.0) * 4096;
    win = win < 16384 ? 16384 : win > 49152 ? 49152 : win;
    const char* e = getenv("USL_TUNE_WIN");
    if (e && atoi(e) > 0) win = atoi(e);
    return win;
}

usl_status build_csc(usl_ctx* c, const int32_t* idx) {
    const size_t N = (size_t)c->m * c->k;
    const int wl = window_labels(c);
    const size_t nwin = ((size_t)c->m + wl - 1) / wl;
    const size_t nbins = nwin * (size_t)c->d;
    if (nbins + 1 > (size_t)0xFFFFFFF0u) USL_FAIL(c, USL_ESHAPE, "too many (window, feature) lists");
    if (!c->csc_ptr || c->csc_win_labels != wl) {
        size_t cap = c->csc_ptr_cap;
        USL_TRY(usl_reserve(c, (void**)&c->csc_ptr, &cap, (nbins + 1) * 4));
        c->csc_ptr_cap = cap; cap = c->csc_cursor_cap;
        USL_TRY(usl_reserve(c, (void**)&c->csc_cursor, &cap, nbins * 4));
        c->csc_cursor_cap = cap;
        if (!c->csc_slot) {
            cap = 0; USL_TRY(usl_reserve(c, (void**)&c->csc_slot, &cap, N * 4));
            cap = 0; USL_TRY(usl_reserve(c, (void**)&c->csc_w, &cap, N * 4));
        }
        c->csc_win_labels = wl;
    }
    const unsigned cchunks = (unsigned)((c->d + CSC_CHUNK - 1) / CSC_CHUNK);
    // a workgroup fills a compute unit (1024 lanes, up to 128 KiB of LDS): as many shares as give one full round
    int splits = (int)((size_t)c->num_cu / (nwin * cchunks));
    splits = splits < 1 ? 1 : splits > 16 ? 16 : splits;
    const dim3 cgrid((unsigned)(nwin * splits), cchunks);
    const size_t clds = (size_t)(c->d < CSC_CHUNK ? c->d : CSC_CHUNK) * 4;
    USL_HIP(c, hipFuncSetAttribute(reinterpret_cast<const void*>(k_csc_count),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)clds));
    USL_HIP(c, hipFuncSetAttribute(reinterpret_cast<const void*>(k_csc_fill),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)clds));
    hipLaunchKernelGGL(k_zero_u32, dim3(c->num_cu), dim3(256), 0, c->stream, c->csc_cursor, nbins);
    hipLaunchKernelGGL(k_csc_count, cgrid, dim3(CSC_NT), clds, c->stream, idx, c->m, c->k, c->d, wl,
                       splits, c->csc_cursor);
    const size_t nchunks = (nbins + SCAN_CHUNK - 1) / SCAN_CHUNK;
    {
        size_t cap = c->tie_counts_cap;  // the redistribution's block-count buffer doubles as scan scratch
        USL_TRY(usl_reserve(c, (void**)&c->tie_counts, &cap, nchunks * 4));
        c->tie_counts_cap = cap;
    }
    USL_TRY(usl_reserve(c, (void**)&c->csc_order, &c->csc_order_cap, 3 * nbins * 4));
    uint32_t* rank_of = c->csc_order + nbins;
    uint32_t* by_rank = c->csc_order + 2 * nbins;
    hipLaunchKernelGGL(k_csc_order, dim3((unsigned)nwin), dim3(1024), 0, c->stream, c->csc_cursor, c->d,
                       c->csc_order, rank_of, by_rank);
    hipLaunchKernelGGL(k_scan_sums, dim3((unsigned)nchunks), dim3(SCAN_NT), 0, c->stream, by_rank,
                       nbins, c->tie_counts);
    hipLaunchKernelGGL(k_scan_top, dim3(1), dim3(SCAN_NT), 0, c->stream, c->tie_counts, nchunks,
                       c->csc_ptr + nbins);
    hipLaunchKernelGGL(k_scan_apply, dim3((unsigned)nchunks), dim3(SCAN_NT), 0, c->stream, by_rank,
                       c->tie_counts, nbins, c->csc_ptr);
    hipLaunchKernelGGL(k_zero_u32, dim3(c->num_cu), dim3(256), 0, c->stream, c->csc_cursor, nbins);
    hipLaunchKernelGGL(k_csc_fill, cgrid, dim3(CSC_NT), clds, c->stream, idx, c->m, c->k, c->d, wl,
                       splits, c->csc_ptr, rank_of, c->csc_cursor, c->csc_slot);
    USL_TRY(usl_idx_fingerprint(c, idx, 1));
    USL_TRY(usl_check_launch(c, "column lists"));
    c->csc_built_for = idx;
    c->lf[0].built_for = c->lf[1].built_for = nullptr;   // one fingerprint: it belongs to the lists built last
    return USL_OK;
}

}  // namespace

usl_status usl_idx_fingerprint(usl_ctx* c, const int32_t* idx, int store) {
    if (!c->idx_print) {
        size_t cap = 0;
        USL_TRY(usl_reserve(c, (void**)&c->idx_print, &cap, 64));
        hipLaunchKernelGGL(k_zero_u32, dim3(1), dim3(64), 0, c->stream, reinterpret_cast<uint32_t*>(c->idx_print), (size_t)16);
    }
    hipLaunchKernelGGL(k_idx_fingerprint, dim3(1), dim3(1024), 0, c->stream, reinterpret_cast<const uint32_t*>(idx),
                       (size_t)c->m * c->k, c->idx_print, store);
    return USL_OK;
}

// The batch goes through the gathers in groups of 256 instances (8 tiles, one per XCD): gT, its piece flags and
// gxT are sized for one group, whatever the batch (at m = 3 million and b = 1024 that is 3 GB instead of 12).
int usl_bwd_input_group_rows(void) { return 256; }

// Lists for this idx, and the scratch of one group of instances.
usl_status usl_bwd_input_prepare(usl_ctx* c, const int32_t* idx, int32_t b) {
    (void)b;
    if (c->csc_built_for != idx || c->csc_win_labels != window_labels(c)) {
        USL_TRY(build_csc(c, idx));
        c->idx_to_check = nullptr;
    } else {   // same address as when the lists were built: the weight gather checks that the contents are the same
        c->idx_to_check = idx;
    }
    const int rows = c->max_b < usl_bwd_input_group_rows() ? c->max_b : usl_bwd_input_group_rows();
    const int ntile = (rows + 31) / 32;   // sized once, for the largest group any batch up to max_b brings
    USL_TRY(usl_reserve(c, (void**)&c->gT, &c->gT_cap, (size_t)ntile * c->m * 32 * 4));
    USL_TRY(usl_reserve(c, (void**)&c->gxT, &c->gxT_cap, (size_t)ntile * c->d * 32 * 4));
    USL_TRY(usl_reserve(c, (void**)&c->nz_flags, &c->nz_flags_cap, (size_t)ntile * c->m));
    if (!c->counter64) {
        size_t cap = 0;
        USL_TRY(usl_reserve(c, (void**)&c->counter64, &cap, 64));
    }
    return USL_OK;
}

// Weights in list order, once per call (every group of instances uses them).
usl_status usl_bwd_input_gather_w(usl_ctx* c, const void* W, const uint32_t* gate) {
    const int wl = c->csc_win_labels;
    const int nwin = (int)((c->m + wl - 1) / wl);
    const int bpw = nwin >= 8 ? 32 : 128;
    const unsigned blocks = (unsigned)(nwin >= 8 ? (nwin + 7) / 8 * 8 : nwin) * bpw;
    if (c->storage == USL_F32)
        hipLaunchKernelGGL(k_gather_w<float>, dim3(blocks), dim3(GW_NT), 0, c->stream, (const float*)W,
                           c->csc_slot, c->csc_ptr, c->d, nwin, c->csc_w, bpw, gate,
                           reinterpret_cast<const uint32_t*>(c->idx_to_check), (size_t)c->m * c->k, c->idx_print);
    else
        hipLaunchKernelGGL(k_gather_w<uint16_t>, dim3(blocks), dim3(GW_NT), 0, c->stream, (const uint16_t*)W,
                           c->csc_slot, c->csc_ptr, c->d, nwin, c->csc_w, bpw, gate,
                           reinterpret_cast<const uint32_t*>(c->idx_to_check), (size_t)c->m * c->k, c->idx_print);
    return usl_check_launch(c, "backward_input weights");
}

// Clears the count of nonzero pieces before a group's gT is produced.
usl_status usl_bwd_input_begin_group(usl_ctx* c) {
    hipLaunchKernelGGL(k_zero_u32, dim3(1), dim3(64), 0, c->stream, usl_nz_cells(c), (size_t)1);
    return usl_check_launch(c, "backward_input scratch");
}

// The gathers of one group of rows instances, once its gT, piece flags and sampled count of nonzero pieces are in
// place; grad_x_rows = the group's rows of grad_x.  sampled_labels = how many labels the count covers (per tile).
usl_status usl_bwd_input_group(usl_ctx* c, float* grad_x_rows, int32_t rows, uint64_t sampled_labels,
                               const uint32_t* gate) {
    const int wl = c->csc_win_labels;
    const int nwin = (int)((c->m + wl - 1) / wl);
    const int ntile = (rows + 31) / 32;   // at most 8: one per XCD, so that an XCD's L2 holds one window slice
    int kshift = -1;
    for (int q = 0; q < 31; ++q)
        if ((1 << q) == c->k) kshift = q;
    // the flag lookup costs a dependent load per connection: worth it when under half the pieces are live
    const uint64_t cells = (uint64_t)ntile * (sampled_labels < (uint64_t)c->m ? sampled_labels : (uint64_t)c->m);
    const uint32_t sparse_below = (uint32_t)(cells / 2 > 0xFFFFFFFFull ? 0xFFFFFFFFull : cells / 2);
    // too few (tile, 32 features) workgroups to fill the chip: a wavefront per feature instead
    bool split = (int64_t)ntile * ((c->d + 31) / 32) < 2 * (int64_t)c->num_cu;
    if ((c->d + 3) / 4 > 65535) split = false;   // the grid's second dimension
    dim3 grid((unsigned)ntile, (unsigned)(split ? (c->d + 3) / 4 : (c->d + 31) / 32));
    for (int w = 0; w < nwin; ++w) {
        if (split)
            hipLaunchKernelGGL(k_bwd_input_window<8>, grid, dim3(256), 0, c->stream, c->gT, c->csc_w,
                               c->csc_ptr + (size_t)w * c->d, c->csc_order + (size_t)w * c->d, c->csc_slot,
                               c->k, kshift, c->gxT, c->d, 0,
                               w > 0 ? 1 : 0, c->nz_flags, c->m, usl_nz_cells(c), sparse_below, gate);
        else
            hipLaunchKernelGGL(k_bwd_input_window<1>, grid, dim3(256), 0, c->stream, c->gT, c->csc_w,
                               c->csc_ptr + (size_t)w * c->d, c->csc_order + (size_t)w * c->d, c->csc_slot,
                               c->k, kshift, c->gxT, c->d, 0,
                               w > 0 ? 1 : 0, c->nz_flags, c->m, usl_nz_cells(c), sparse_below, gate);
    }
    {
        dim3 grid2((unsigned)((c->d + 31) / 32), (unsigned)ntile);
        hipLaunchKernelGGL(k_untile, grid2, dim3(256), 0, c->stream, c->gxT, grad_x_rows, (int64_t)rows, (int64_t)c->d, gate,
                           reinterpret_cast<const uint32_t*>(c->idx_print) + 4);
    }
    return usl_check_launch(c, "backward_input");
}

usl_status usl_launch_backward_input(usl_ctx* c, const float* g, const int32_t* idx, const void* W,
                                     float* grad_x, int32_t b) {
    // the register-list form copies rows of g and writes grad_x 16 bytes at a time
    const bool lds_form = usl_bwi_lds_applies(c) && (uintptr_t)g % 16 == 0 && (uintptr_t)grad_x % 16 == 0;
    if (!lds_form) USL_TRY(usl_bwd_input_prepare(c, idx, b));
    // a gradient that is almost all zeros goes through per-instance lists of its nonzeros instead; which of the
    // two paths does the work is decided on the device (gate), both are enqueued
    const uint32_t* gate = nullptr;
    if (usl_sparse_supported(c)) {
        if (c->nz_lists_of == g) gate = c->nz_lists_tried ? c->nz_state : nullptr;   // usl_train_step has looked already
        else USL_TRY(usl_sparse_compact(c, g, b, &gate));
        if (gate) USL_TRY(usl_sparse_backward_input(c, idx, W, grad_x, b));
    }
    if (lds_form) return usl_bwi_lds_run(c, g, idx, W, grad_x, b, gate);
    USL_TRY(usl_bwd_input_gather_w(c, W, gate));
    const int G = usl_bwd_input_group_rows();
    for (int i0 = 0; i0 < b; i0 += G) {
        const int rows = b - i0 < G ? b - i0 : G;
        USL_TRY(usl_bwd_input_begin_group(c));
        {   // gT = the group's rows of g transposed tile by tile, with the zero flags of every (label, tile) piece
            dim3 grid((unsigned)((c->m + 31) / 32), (unsigned)((rows + 31) / 32));
            hipLaunchKernelGGL(k_transpose_g, grid, dim3(256), 0, c->stream, g + (size_t)i0 * c->m, c->gT, (int64_t)rows,
                               c->m, c->nz_flags, usl_nz_cells(c), gate);
        }
        USL_TRY(usl_bwd_input_group(c, grad_x + (size_t)i0 * c->d, rows, (uint64_t)(((c->m + 31) / 32 + 63) / 64) * 32, gate));
    }
    return USL_OK;
}
