// Input gradient (Algorithm 2) in its feature-stationary LDS form: the mirror image of the forward kernel.
//
//   grad_x[i][c] = sum over connections (j,t) with idx[j][t]==c of W[j][t] * g[i][j]
//
// A workgroup owns a window of wl labels and a block of NF features.  Every lane keeps the list of one pair of
// features -- (label-in-window, 16 bit) and weight of every connection that leads from the window into the feature
// -- in registers for the workgroup's whole life, walks the batch staging g[i][window] (wl floats) through LDS with
// LDS-DMA, and gathers: the same ds_read_b32 stream as the forward kernel, reading g row-major (no transposed copy
// of the gradient, no zero flags).  The sums of a window go to partial[window][i][c]; a second kernel adds the
// windows up.
//
// Lists of one (window, feature) have Poisson-distributed lengths (mean wl*k/d, at most 32: the windows are sized
// for that), registers are allocated for a fixed number of slots.  Per (window, feature block) the features are
// therefore ranked by list length and paired longest with shortest: lane l holds list A = rank l from slot 0 upwards
// and list B = rank NF-1-l from slot KTOT-1 downwards; a wavefront (64 neighbouring ranks: nearly equal lengths)
// visits slots [0, acap) for its A lists and [KTOT-bcap, KTOT) for its B lists, acap + bcap <= KTOT chosen per
// wavefront so that as little as possible is left over.  Entries that do not fit (a few dozen per workgroup for
// uniform connectivity: the very longest lists; anything for a caller's skewed idx) go to an overflow list of the
// workgroup, kept list by list: its first 1024 entries sit in LDS with their weights and the list's own lane adds
// them after its registers; what is beyond that is added with LDS atomics from memory: slow, rare, and what keeps
// the form valid for any connectivity.  Within a lane's allowance the entries are put in a bank-aware order
// (k_lf_schedule), the empty places of shorter lists included.
//
// Registers: 34 for the packed labels and 68 for the weights of the 68 slots leave 26 of a lane's 128 (1024 lanes
// per compute unit) for everything else; the gathers are therefore written out in assembly, four in flight.
#include <stdlib.h>

#include "usl_internal.h"

namespace {

constexpr int WL = 32768;      // most labels a window has: one float32 row of 128 KiB in LDS.  A layer's windows are of equal
                               // size wl <= WL (a multiple of 4): no short last window whose workgroups idle
constexpr int NF = 2048;       // features per workgroup (two per lane)
constexpr int NT = 1024;
constexpr int KT_BWI = 68;     // list slots per lane, shared by its two lists (with the rest of the kernel: the 128 registers a lane has)
constexpr int KT_BOTH = 36;    // ... in the kernel that also keeps a weight-gradient sum per slot (windows of half the length)
constexpr uint32_t PAD_SLOT = 0xFFFFFFFFu;
// LDS of the gather kernel: the row slice, NF floats through which the sums are un-permuted, NT words (the features of
// every lane), NT entries of 8 bytes (the nearest part of the overflow list), 2 * NT words (each lane's share of it) and
// 32 words of zeros, one per bank: what the empty places of a list read (weight 0 times a real gradient would turn an
// infinity in g into NaNs in features that have nothing to do with it).  ZERO_LABEL + b is the "label" whose address is
// zero word b; it fits the 16 bits of a packed label.
constexpr size_t LDS_BYTES = (size_t)32768 * 4 + (size_t)2048 * 4 + (size_t)1024 * 4 + (size_t)1024 * 8 + (size_t)1024 * 8 + 128;
constexpr uint32_t ZERO_LABEL = (uint32_t)((LDS_BYTES - 128) / 4);
static_assert(ZERO_LABEL % 32 == 0 && ZERO_LABEL + 31 < 65536 && LDS_BYTES <= 160 * 1024, "zero words: bank b, 16-bit label, inside LDS");
// LDS of the kernel for both backward products, which stages two rows of g at a time: two row buffers RS2 bytes apart
// (so that one address and the 16-bit offset field of a ds_read reach both), each ending in 32 zero words (ZERO_LABEL2
// is their "label": a window has at most that many labels), 2 * NF floats for the sums of the two instances, NT words
// (features), NEAR2 overflow entries of 8 bytes, 2 * NT words (each lane's share of them), NEAR2 floats (their
// weight-gradient sums).
constexpr int RS2 = 64000;
constexpr uint32_t ZERO_LABEL2 = (RS2 - 128) / 4;
constexpr int NEAR2 = 512;
constexpr size_t LDS2_BYTES = (size_t)2 * RS2 + (size_t)2 * 2048 * 4 + (size_t)1024 * 4 + (size_t)NEAR2 * 8 + (size_t)2 * 1024 * 4 + (size_t)NEAR2 * 4;
static_assert(ZERO_LABEL2 % 32 == 0 && RS2 < 65536 && RS2 % 16 == 0 && LDS2_BYTES <= 160 * 1024, "two row buffers within one ds_read offset, inside LDS");
template <int KT> struct ListLayout;   // what depends on which kernel the lists are for
template <> struct ListLayout<68> { static constexpr uint32_t zero_label = ZERO_LABEL; static constexpr uint32_t near = 1024; };
template <> struct ListLayout<36> { static constexpr uint32_t zero_label = ZERO_LABEL2; static constexpr uint32_t near = NEAR2; };
constexpr int CHUNK = 32768;   // features per LDS histogram

__global__ void k_fill_u32(uint32_t* p, size_t n, uint32_t v) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}

// The slots of one window's labels, cut into `splits` contiguous shares.
__device__ __forceinline__ void share_of(int64_t m, int k, int wl, int splits, size_t* e0, size_t* e1) {
    const int w = blockIdx.x / splits, s = blockIdx.x % splits;
    const size_t w0 = (size_t)w * wl * k;
    const size_t w1 = (size_t)min((int64_t)(w + 1) * wl, m) * k;
    const size_t per = (w1 - w0 + splits - 1) / splits;
    *e0 = min(w0 + per * s, w1);
    *e1 = min(*e0 + per, w1);
}

// count[w][c] += connections of this workgroup's share that lead into feature c (LDS histogram, then one global
// atomic per feature that occurs).  grid (nwin * splits, feature chunks).
__global__ void __launch_bounds__(NT)
k_lf_count(const int32_t* __restrict__ idx, int64_t m, int k, int d, int wl, int splits, uint32_t* __restrict__ count) {
    extern __shared__ uint32_t hist[];
    const int c0 = blockIdx.y * CHUNK, nc = min(CHUNK, d - c0);
    size_t e0, e1;
    share_of(m, k, wl, splits, &e0, &e1);
    for (int q = threadIdx.x; q < nc; q += NT) hist[q] = 0;
    __syncthreads();
    for (size_t e = e0 + threadIdx.x; e < e1; e += NT) {
        const uint32_t c = (uint32_t)(idx[e] - c0);
        if (c < (uint32_t)nc) atomicAdd(&hist[c], 1u);
    }
    __syncthreads();
    uint32_t* dst = count + (size_t)(blockIdx.x / splits) * d + c0;
    for (int q = threadIdx.x; q < nc; q += NT)
        if (hist[q]) atomicAdd(&dst[q], hist[q]);
}

// One workgroup per (window, feature block): ranks the block's NF features by list length, pairs them, fixes the
// slot ranges of every wavefront and counts what will not fit.
//   feat[wg][z][lane] = feature (within the block) whose list lane holds in zone z
//   caps[wg][wave]    = acap | bcap << 8
//   where[w][c]       = where the list of feature c starts among the workgroup's entries (k_lf_fill puts them there)
//   n_ent[wg]         = entries of the workgroup
//   ov_off[w][c]      = where what does not fit of that list starts in the workgroup's overflow list
//   n_ov[wg]          = entries beyond the allowances
//   ovr[wg][z][lane]  = start | n << 16: the part of that list's overflow among the first NT (NEAR2) entries (those the
//                       gather kernel keeps in LDS and the list's own lane adds up)
template <int KTOT>
__global__ void __launch_bounds__(NT)
k_lf_plan(const uint32_t* __restrict__ count, int d, int nfb, uint32_t* __restrict__ where, uint32_t* __restrict__ ov_off,
          uint16_t* __restrict__ feat, uint32_t* __restrict__ caps, uint32_t* __restrict__ n_ent,
          uint32_t* __restrict__ n_ov, uint32_t* __restrict__ ovr) {
    __shared__ uint32_t start[256];
    __shared__ uint32_t scan[NT];
    __shared__ uint16_t len_of[2][NT];
    __shared__ uint32_t cap_of[NT / 64];
    const int wg = blockIdx.x, w = wg / nfb, fb = wg % nfb;
    const uint32_t* cnt = count + (size_t)w * d + (size_t)fb * NF;
    if (threadIdx.x < 256) start[threadIdx.x] = 0;
    __syncthreads();
    uint32_t n[2];
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        n[q] = cnt[threadIdx.x + q * NT];
        atomicAdd(&start[min(n[q], 255u)], 1u);
    }
    __syncthreads();
    if (threadIdx.x == 0) {   // ranks of the buckets, longest lists first
        uint32_t run = 0;
        for (int q = 255; q >= 0; --q) { const uint32_t t = start[q]; start[q] = run; run += t; }
    }
    __syncthreads();
    uint32_t lane_of[2], zone_of[2];
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        const uint32_t r = atomicAdd(&start[min(n[q], 255u)], 1u);   // rank (order among equal lengths is arbitrary)
        zone_of[q] = r < (uint32_t)NT ? 0u : 1u;
        lane_of[q] = r < (uint32_t)NT ? r : (uint32_t)(NF - 1) - r;
        len_of[zone_of[q]][lane_of[q]] = (uint16_t)min(n[q], 65535u);
        feat[((size_t)wg * 2 + zone_of[q]) * NT + lane_of[q]] = (uint16_t)(threadIdx.x + q * NT);
    }
    __syncthreads();
    {   // the wavefront's two slot allowances (multiples of 4, KTOT together): those that leave the least outside
        // the registers, counting the longest leftover of a single lane (its lane walks that alone) 16-fold
        const uint32_t la = len_of[0][threadIdx.x], lb = len_of[1][threadIdx.x];
        uint32_t best = 0xFFFFFFFFu;
        for (uint32_t ca = 0; ca <= (uint32_t)KTOT; ca += 4) {
            const uint32_t cb = (uint32_t)KTOT - ca;
            uint32_t tot = (la > ca ? la - ca : 0u) + (lb > cb ? lb - cb : 0u);
            uint32_t mx = max(la > ca ? la - ca : 0u, lb > cb ? lb - cb : 0u);
            for (int o = 32; o > 0; o >>= 1) {
                tot += __shfl_xor(tot, o);
                mx = max(mx, (uint32_t)__shfl_xor(mx, o));
            }
            const uint32_t cost = min(tot + 16u * mx, 0xFFFFFFu);
            best = min(best, cost << 8 | ca);
        }
        // no more than the longest list needs (slots a wavefront visits are time)
        uint32_t amax = la, bmax = lb;
        for (int o = 32; o > 0; o >>= 1) {
            amax = max(amax, (uint32_t)__shfl_xor(amax, o));
            bmax = max(bmax, (uint32_t)__shfl_xor(bmax, o));
        }
        const uint32_t acap = min(best & 0xFFu, (amax + 3u) & ~3u);
        const uint32_t bcap = min((uint32_t)KTOT - (best & 0xFFu), (bmax + 3u) & ~3u);
        if ((threadIdx.x & 63) == 0) {
            cap_of[threadIdx.x >> 6] = acap | (bcap << 8);
            caps[(size_t)wg * (NT / 64) + (threadIdx.x >> 6)] = acap | (bcap << 8);
        }
    }
    __syncthreads();
    uint32_t ov[2];
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        const uint32_t cw = cap_of[lane_of[q] >> 6];
        const uint32_t cap = zone_of[q] == 0 ? (cw & 0xFFu) : (cw >> 8);
        ov[q] = n[q] > cap ? n[q] - cap : 0u;
        ov[q] = (ov[q] + 1u) & ~1u;   // an even number of places: the list's lane walks them two at a time
    }
    auto block_scan = [&](uint32_t mine) -> uint32_t {   // inclusive, over the lanes of the workgroup
        __syncthreads();
        scan[threadIdx.x] = mine;
        __syncthreads();
        for (int o = 1; o < NT; o <<= 1) {
            const uint32_t t = threadIdx.x >= (unsigned)o ? scan[threadIdx.x - o] : 0u;
            __syncthreads();
            scan[threadIdx.x] += t;
            __syncthreads();
        }
        return scan[threadIdx.x];
    };
    const size_t bin = (size_t)w * d + (size_t)fb * NF + threadIdx.x;
    {
        const uint32_t incl = block_scan(n[0] + n[1]);
        where[bin] = incl - n[0] - n[1];
        where[bin + NT] = incl - n[1];
        if (threadIdx.x == NT - 1) n_ent[wg] = incl;
    }
    {
        const uint32_t incl = block_scan(ov[0] + ov[1]);
        uint32_t at = incl - ov[0] - ov[1];
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            ov_off[bin + q * NT] = at;
            const uint32_t first = min(at, ListLayout<KTOT>::near);
            ovr[((size_t)wg * 2 + zone_of[q]) * NT + lane_of[q]] = first | (min(ov[q], ListLayout<KTOT>::near - first) << 16);
            at += ov[q];
        }
        if (threadIdx.x == NT - 1) n_ov[wg] = incl;
    }
}

// ov_base[wg] = sum of ov_count over the workgroups before wg; ov_base[nwg] = all of them (one block).
__global__ void __launch_bounds__(1024)
k_lf_scan(const uint32_t* __restrict__ ov_count, int nwg, uint32_t* __restrict__ ov_base) {
    __shared__ uint32_t part[1024];
    const int per = (nwg + 1023) / 1024;
    const int a = min(nwg, (int)threadIdx.x * per), e = min(nwg, a + per);
    uint32_t s = 0;
    for (int q = a; q < e; ++q) s += ov_count[q];
    part[threadIdx.x] = s;
    __syncthreads();
    for (int o = 1; o < 1024; o <<= 1) {
        const uint32_t t = threadIdx.x >= (unsigned)o ? part[threadIdx.x - o] : 0u;
        __syncthreads();
        part[threadIdx.x] += t;
        __syncthreads();
    }
    uint32_t run = part[threadIdx.x] - s;
    for (int q = a; q < e; ++q) { ov_base[q] = run; run += ov_count[q]; }
    if (threadIdx.x == 1023) ov_base[nwg] = part[1023];
}

// Groups the connections by (workgroup of the gather kernel, feature): ent[ent_base[wg] + where[w][c] + p] = flat
// slot j*k+t of the p-th connection from window w into feature c (p by a cursor: the order inside a list is not
// fixed).  Same decomposition as k_lf_count: a share's positions in every list are reserved with one global atomic
// per feature, then handed out from LDS cursors.
struct OvEntry { uint16_t feature; uint16_t label; uint32_t slot; };
__global__ void __launch_bounds__(NT)
k_lf_fill(const int32_t* __restrict__ idx, int64_t m, int k, int d, int wl, int nfb, int splits, const uint32_t* __restrict__ where,
          uint32_t* __restrict__ taken, const uint32_t* __restrict__ ent_base, uint32_t* __restrict__ ent) {
    extern __shared__ uint32_t cur[];
    const int c0 = blockIdx.y * CHUNK, nc = min(CHUNK, d - c0);
    const int w = blockIdx.x / splits;
    size_t e0, e1;
    share_of(m, k, wl, splits, &e0, &e1);
    for (int q = threadIdx.x; q < nc; q += NT) cur[q] = 0;
    __syncthreads();
    for (size_t e = e0 + threadIdx.x; e < e1; e += NT) {
        const uint32_t c = (uint32_t)(idx[e] - c0);
        if (c < (uint32_t)nc) atomicAdd(&cur[c], 1u);
    }
    __syncthreads();
    const size_t bin0 = (size_t)w * d + c0;
    for (int q = threadIdx.x; q < nc; q += NT) {   // from here cur[q] = where this share's part of the list starts
        const uint32_t n = cur[q];
        if (n) cur[q] = atomicAdd(&taken[bin0 + q], n) + where[bin0 + q] + ent_base[(size_t)w * nfb + (c0 + q) / NF];
    }
    __syncthreads();
    for (size_t e = e0 + threadIdx.x; e < e1; e += NT) {
        const uint32_t c = (uint32_t)(idx[e] - c0);
        if (c < (uint32_t)nc) ent[atomicAdd(&cur[c], 1u)] = (uint32_t)e;
    }
}

// Where the kernel for both products leaves the weight gradient of every connection (pos[flat slot], a place in an
// array of m * k floats): the connections of a (window, feature block) workgroup together (from ent_base[wg], as in
// ent), and within it in the order of their flat slots, up to the order inside a run of SEG slots.  The Adam kernel,
// which goes through the slots in order, then reads 16 or so neighbouring places from each of the window's nfb
// workgroups per wavefront -- whole lines; in the order of the lists it would fetch a line per value.
// Three kernels: the counts of every run per feature block, their running sums, the places.
constexpr int SEG = 256;   // slots of a run: one wavefront, four per lane
__device__ __forceinline__ bool seg_of_wave(int64_t m, int k, int wl, int nseg, int64_t total, int* w, int* seg, size_t* s0, size_t* s1) {
    const int64_t gs = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (gs >= total) return false;
    *w = (int)(gs / nseg); *seg = (int)(gs % nseg);
    const size_t w0 = (size_t)*w * wl * k, w1 = (size_t)min((int64_t)(*w + 1) * wl, m) * k;
    *s0 = min(w0 + (size_t)*seg * SEG, w1);
    *s1 = min(*s0 + SEG, w1);
    return true;
}
__global__ void __launch_bounds__(256)
k_lf_seg_count(const int32_t* __restrict__ idx, int64_t m, int k, int wl, int nfb, int nseg, int64_t total, uint32_t* __restrict__ segcnt) {
    __shared__ uint32_t h[4][32];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    if (lane < 32) h[wave][lane] = 0;
    __syncthreads();
    int w, seg; size_t s0, s1;
    const bool on = seg_of_wave(m, k, wl, nseg, total, &w, &seg, &s0, &s1);
    if (on)
        for (size_t e = s0 + lane; e < s1; e += 64) atomicAdd(&h[wave][min((uint32_t)idx[e] / NF, 31u)], 1u);
    __syncthreads();
    if (on && lane < nfb) segcnt[((size_t)w * nfb + lane) * nseg + seg] = h[wave][lane];
}
// segcnt[wg][seg] -> ent_base[wg] + the counts of the runs before seg (in place).  One block per workgroup wg.
__global__ void __launch_bounds__(256)
k_lf_seg_scan(uint32_t* __restrict__ segcnt, int nseg, const uint32_t* __restrict__ ent_base) {
    __shared__ uint32_t part[256];
    uint32_t* c = segcnt + (size_t)blockIdx.x * nseg;
    uint32_t carry = ent_base[blockIdx.x];
    for (int q0 = 0; q0 < nseg; q0 += 256) {
        const int q = q0 + (int)threadIdx.x;
        const uint32_t mine = q < nseg ? c[q] : 0u;
        part[threadIdx.x] = mine;
        __syncthreads();
        for (int o = 1; o < 256; o <<= 1) {
            const uint32_t t = threadIdx.x >= (unsigned)o ? part[threadIdx.x - o] : 0u;
            __syncthreads();
            part[threadIdx.x] += t;
            __syncthreads();
        }
        if (q < nseg) c[q] = carry + part[threadIdx.x] - mine;
        carry += part[255];
        __syncthreads();
    }
}
__global__ void __launch_bounds__(256)
k_lf_seg_place(const int32_t* __restrict__ idx, int64_t m, int k, int wl, int nfb, int nseg, int64_t total,
               const uint32_t* __restrict__ segbase, uint32_t* __restrict__ pos) {
    __shared__ uint32_t h[4][32];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    int w, seg; size_t s0, s1;
    const bool on = seg_of_wave(m, k, wl, nseg, total, &w, &seg, &s0, &s1);
    if (on && lane < nfb) h[wave][lane] = segbase[((size_t)w * nfb + lane) * nseg + seg];
    __syncthreads();
    if (on)
        for (size_t e = s0 + lane; e < s1; e += 64) pos[e] = atomicAdd(&h[wave][min((uint32_t)idx[e] / NF, 31u)], 1u);
}

// Bank-aware order of the entries in every lane's lists.  At step t of the gathers the 32 lanes of a half-wavefront
// read slot t of their own lists; the sum does not depend on the order of a list, so each list is permuted so that
// the 32 addresses of a step fall into different LDS banks as far as possible (a step costs as many LDS cycles as its
// fullest bank has lanes).  The order is built step by step as a sequence of matchings between the 32 lanes and the
// 32 banks over the entries not placed yet -- a few rounds of proposals, then augmenting paths from the banks still
// free, then lanes whose banks are all taken double up on the least loaded one --, the same construction as for the
// slots of a label in the forward product, with one addition: a list shorter than the wavefront's allowance has
// empty places, which may go to any step and read any bank.  A lane that finds no bank among its entries spends an
// empty place (it then reads the zero word of a free bank, see ZERO_LABEL) while it has one.
// One half-wavefront per (workgroup of the gather kernel, zone, 32 lanes); lane i is list i and also bank i.
// Reads the lists as k_lf_fill grouped them (ent), writes them ordered into the places the gather kernel loads its
// registers from (lab / slot: [workgroup][slot][lane]) and what exceeds the allowance into the overflow list.  Any
// outcome is a valid order: it changes speed, never results.  rounds = 0: the lists stay in the order of ent.
// pos (if given, see k_lf_seg_place): every entry's place among its workgroup's weight gradients goes along, into rk
// (beside lab / slot) or ovrk (beside ov); an empty place gets PAD_SLOT.
constexpr int SG = 8;   // half-wavefronts per workgroup
template <int KTOT>
__global__ void __launch_bounds__(SG * 32)
k_lf_schedule(const uint32_t* __restrict__ ent, const uint32_t* __restrict__ ent_base, const uint32_t* __restrict__ where,
              const uint32_t* __restrict__ count, const uint16_t* __restrict__ feat, const uint32_t* __restrict__ caps,
              const uint32_t* __restrict__ ov_base, const uint32_t* __restrict__ ov_off, int k, int d, int wl, int nfb,
              int rounds, uint16_t* __restrict__ lab, uint32_t* __restrict__ slot, OvEntry* __restrict__ ov,
              const uint32_t* __restrict__ pos, uint32_t* __restrict__ rk, uint32_t* __restrict__ ovrk) {
    __shared__ uint8_t slots[SG][32][KTOT + 4];   // my entries sorted by bank
    __shared__ uint8_t left_in[SG][32][36];       // entries of mine not placed yet, per bank
    __shared__ uint8_t end_of[SG][32][36];        // where bank b's entries end in the sorted list
    __shared__ int deg0[SG][32];
    __shared__ int win[SG][32];
    const int gl = threadIdx.x >> 5, lane = threadIdx.x & 31;
    const int hs = threadIdx.x & 32;              // where my group's 32 bits sit in a wavefront ballot
    const size_t gid = (size_t)blockIdx.x * SG + gl;
    const size_t wg = gid >> 6;
    const int zone = (int)(gid >> 5) & 1, half = (int)gid & 31;   // the two halves of a wavefront are neighbours: same allowance
    const uint32_t cw = caps[wg * (NT / 64) + (half >> 1)];
    const int cap = zone ? (int)(cw >> 8) : (int)(cw & 0xFFu);
    const int w = (int)(wg / nfb), fb = (int)(wg % nfb);
    auto at = [&](int p) -> size_t { return (wg * KTOT + (zone ? KTOT - 1 - p : p)) * NT + half * 32 + lane; };
    // my list: feature, length, where its entries are; label of an entry = its flat slot / k, counted from the window's first
    const uint32_t f = feat[(wg * 2 + zone) * NT + half * 32 + lane];
    const size_t bin = (size_t)w * d + (size_t)fb * NF + f;
    const uint32_t len = count[bin];
    const uint32_t* my = ent + ent_base[wg] + where[bin];
    auto label_of = [&](uint32_t e) -> uint32_t { return e / (uint32_t)k - (uint32_t)w * (uint32_t)wl; };
    const int n = (int)min(len, (uint32_t)cap);     // entries that get a register slot
    for (uint32_t p = (uint32_t)cap; p < len; ++p) {   // the others: to the list's part of the overflow list
        OvEntry o;
        o.feature = (uint16_t)f; o.label = (uint16_t)label_of(my[p]); o.slot = my[p];
        ov[(size_t)ov_base[wg] + ov_off[bin] + (p - (uint32_t)cap)] = o;
        if (pos) ovrk[(size_t)ov_base[wg] + ov_off[bin] + (p - (uint32_t)cap)] = pos[my[p]] - ent_base[wg];
    }
    if (len > (uint32_t)cap && ((len - (uint32_t)cap) & 1u)) {   // an odd number: one empty place behind them
        OvEntry o;
        o.feature = (uint16_t)f; o.label = (uint16_t)ListLayout<KTOT>::zero_label; o.slot = PAD_SLOT;
        ov[(size_t)ov_base[wg] + ov_off[bin] + (len - (uint32_t)cap)] = o;
        if (pos) ovrk[(size_t)ov_base[wg] + ov_off[bin] + (len - (uint32_t)cap)] = PAD_SLOT;
    }
    if (rounds <= 0) {
        for (int s = 0; s < cap; ++s) {
            lab[at(s)] = s < n ? (uint16_t)label_of(my[s]) : (uint16_t)ListLayout<KTOT>::zero_label;
            slot[at(s)] = s < n ? my[s] : PAD_SLOT;
            if (pos) rk[at(s)] = s < n ? pos[my[s]] - ent_base[wg] : PAD_SLOT;
        }
        return;   // the whole wavefront: rounds is the same for all
    }
    deg0[gl][lane] = 0;
    for (int b = 0; b < 32; ++b) left_in[gl][lane][b] = 0;
    __syncthreads();
    uint8_t* mine = slots[gl][lane];
    uint8_t* cnt = left_in[gl][lane];
    uint8_t* ends = end_of[gl][lane];
    for (int p = 0; p < n; ++p) {
        const int b = (int)(label_of(my[p]) & 31u);
        ++cnt[b];
        atomicAdd(&deg0[gl][b], 1);
    }
    int wild = cap - n;            // empty places left
    uint32_t avail = 0;            // banks my unplaced entries read
    {   // counting sort of my entries by bank (their banks are read a second time: no room to keep them)
        int run = 0;
        for (int b = 0; b < 32; ++b) { run += cnt[b]; ends[b] = (uint8_t)run; if (cnt[b]) avail |= 1u << b; }
        for (int p = n - 1; p >= 0; --p) { const int b = (int)(label_of(my[p]) & 31u); ends[b] = (uint8_t)(ends[b] - 1); mine[ends[b]] = (uint8_t)p; }
        for (int b = 0; b < 32; ++b) ends[b] = (uint8_t)(ends[b] + cnt[b]);   // back from starts to ends
    }
    __syncthreads();
    auto gballot = [&](bool p) -> uint32_t { return (uint32_t)(__ballot(p) >> hs); };
    volatile int* gwin = win[gl];
    int mydeg = deg0[gl][lane];    // bank role: entries of the group that read bank `lane` and are not placed yet
    for (int s = 0; s < cap; ++s) {
        int mb = -1;               // list role: my bank at this step
        int ml = -1;               // bank role: the list that reads me at this step
        for (int r = 0; r < rounds; ++r) {
            const uint32_t freeb = gballot(ml < 0);
            gwin[lane] = 255;
            int prop = -1;
            const uint32_t cand = mb < 0 ? (avail & freeb) : 0u;
            if (cand) {            // first candidate bank at or after a lane- and round-dependent start
                const int sh = (lane + 7 * r) & 31;
                const uint32_t rc = (cand >> sh) | (cand << ((32 - sh) & 31));
                prop = (__ffs(rc) - 1 + sh) & 31;
                atomicMin(&win[gl][prop], lane);
            }
            const int wnr = gwin[lane];
            if (ml < 0 && wnr < 32) ml = wnr;
            if (prop >= 0 && gwin[prop] == lane) mb = prop;
        }
        // augmenting paths from the banks still free
        uint32_t todo = gballot(ml < 0 && mydeg > 0);
        while (__any(todo != 0)) {
            const bool act = todo != 0;
            const int b0 = act ? __ffs(todo) - 1 : 0;
            todo &= todo - 1;
            uint32_t front = act ? (1u << b0) : 0u, seen = 0;
            int par = -1, found = -1;
            bool searching = act;
            while (__any(searching)) {
                const bool reach = searching && !((seen >> lane) & 1u) && (avail & front) != 0;
                if (reach) par = __ffs(avail & front) - 1;
                const uint32_t fresh = gballot(reach);
                const uint32_t fresh_free = gballot(reach && mb < 0);
                const uint32_t next = gballot(ml >= 0 && ((fresh >> (ml & 31)) & 1u));
                seen |= fresh;
                if (searching) {
                    if (fresh_free) { found = __ffs(fresh_free) - 1; searching = false; }
                    else if (next == 0) searching = false;
                    else front = next;
                }
            }
            int cur = found;       // walk back: every list on the path takes the bank it was reached through
            while (__any(cur >= 0)) {
                const bool a = cur >= 0;
                const int cl = a ? cur : 0;
                const int b = __shfl(par, cl, 32) & 31;
                const int prev = __shfl(ml, b, 32);
                if (a) {
                    if (lane == cl) mb = b;
                    if (lane == b) ml = cl;
                    cur = b == b0 ? -1 : prev;
                }
            }
        }
        // lists without a bank: an empty place if one is left, on a bank nobody reads (there are as many free banks as
        // lists without one)
        int wb = -1;
        {
            const bool spend = mb < 0 && wild > 0;
            const uint32_t spenders = gballot(spend);
            uint32_t fb = gballot(ml < 0);
            if (spend) {
                for (int q = __popc(spenders & ((1u << lane) - 1u)); q > 0; --q) fb &= fb - 1;
                wb = __ffs(fb) - 1;
                --wild;
            }
        }
        // the others double up: least loaded reachable bank, then the fullest
        int myload = ml >= 0 ? 1 : 0;
        uint32_t left = gballot(mb < 0 && wb < 0);
        while (__any(left != 0)) {
            const bool a = left != 0;
            const int l = a ? __ffs(left) - 1 : 0;
            left &= left - 1;
            const uint32_t av = (uint32_t)__shfl((int)avail, l, 32);
            int key = (a && ((av >> lane) & 1u)) ? (((255 - myload) << 17) | (mydeg << 5) | lane) : -1;
#pragma unroll
            for (int o = 16; o > 0; o >>= 1) key = max(key, __shfl_xor(key, o, 32));
            if (a && key >= 0) {
                const int bb = key & 31;
                if (lane == l) mb = bb;
                if (lane == bb) ++myload;
            }
        }
        if (wb >= 0) {             // an empty place: the zero word of the free bank, no weight
            lab[at(s)] = (uint16_t)(ListLayout<KTOT>::zero_label + (uint32_t)wb);
            slot[at(s)] = PAD_SLOT;
            if (pos) rk[at(s)] = PAD_SLOT;
        } else {                   // my next unplaced entry in that bank
            const int pick = mine[ends[mb] - cnt[mb]];
            if (--cnt[mb] == 0) avail &= ~(1u << mb);
            lab[at(s)] = (uint16_t)label_of(my[pick]);
            slot[at(s)] = my[pick];
            if (pos) rk[at(s)] = pos[my[pick]] - ent_base[wg];
        }
        mydeg -= myload;
    }
}

typedef const __attribute__((address_space(3))) float lds_f32_t;
// acc += sum of w[u] * row[label u] over the four labels packed in p0, p1 (16 bits each).  One instruction per
// address (the 16-bit half is selected and scaled to a byte offset in one go; the row starts at LDS address 0: the
// kernel has no static LDS, and the launcher checks that), the four reads in flight together, each multiply-add as
// soon as its value is there.  Written out because the compiler, short of registers in this kernel, issues one read
// at a time and waits for it.
__device__ __forceinline__ void gather4(float& acc, uint32_t p0, uint32_t p1, float w0, float w1, float w2, float w3) {
    uint32_t a0, a1, a2, a3;
    const uint32_t two = 2;
    asm volatile(
        "v_lshlrev_b32_sdwa %1, %5, %6 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_0\n\t"
        "v_lshlrev_b32_sdwa %2, %5, %6 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_1\n\t"
        "v_lshlrev_b32_sdwa %3, %5, %7 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_0\n\t"
        "v_lshlrev_b32_sdwa %4, %5, %7 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_1\n\t"
        "ds_read_b32 %1, %1\n\t"
        "ds_read_b32 %2, %2\n\t"
        "ds_read_b32 %3, %3\n\t"
        "ds_read_b32 %4, %4\n\t"
        "s_waitcnt lgkmcnt(3)\n\t"
        "v_fmac_f32 %0, %8, %1\n\t"
        "s_waitcnt lgkmcnt(2)\n\t"
        "v_fmac_f32 %0, %9, %2\n\t"
        "s_waitcnt lgkmcnt(1)\n\t"
        "v_fmac_f32 %0, %10, %3\n\t"
        "s_waitcnt lgkmcnt(0)\n\t"
        "v_fmac_f32 %0, %11, %4"
        : "+v"(acc), "=&v"(a0), "=&v"(a1), "=&v"(a2), "=&v"(a3)
        : "s"(two), "v"(p0), "v"(p1), "v"(w0), "v"(w1), "v"(w2), "v"(w3)
        : "memory");
}

// The gathers.  grid: ceil(nwin / 8) * 8 * nfb workgroups; all feature blocks of a window run on one XCD (workgroups
// are dealt to the 8 XCDs round robin), so its slice of g is fetched from HBM once and served from that XCD's L2.
// LDS: see LDS_BYTES.
template <typename TS>
__global__ void __launch_bounds__(NT)
k_bwi_lds(const float* __restrict__ g, const TS* __restrict__ W, int64_t m, int k, int rows, int d, int wl, int nfb, int nwin,
          const uint16_t* __restrict__ lab, const uint32_t* __restrict__ slot, const uint16_t* __restrict__ feat,
          const uint32_t* __restrict__ caps, const uint32_t* __restrict__ ov_base, const OvEntry* __restrict__ ov,
          const uint32_t* __restrict__ ovr, float* __restrict__ partial, const uint32_t* __restrict__ gate) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    if (gate && *gate == 0) return;   // the kernels over the nonzero gradients do this call's work
    const int w = (blockIdx.x & 7) + 8 * (blockIdx.x / (8 * nfb)), fb = (blockIdx.x >> 3) % nfb;
    if (w >= nwin) return;
    const size_t wg = (size_t)w * nfb + fb;
    const uint32_t cw = caps[wg * (NT / 64) + (threadIdx.x >> 6)];
    const int acap = __builtin_amdgcn_readfirstlane((int)(cw & 0xFFu)), bcap = __builtin_amdgcn_readfirstlane((int)(cw >> 8));
    uint32_t pk[KT_BWI / 2];
    float wt[KT_BWI];
    const uint32_t last_slot = (uint32_t)(m * k - 1);
#pragma unroll
    for (int q = 0; q < KT_BWI / 4; ++q) {
        const bool used = q * 4 < acap || q * 4 >= KT_BWI - bcap;   // the same for the whole wavefront
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int t = q * 4 + u;
            uint32_t l16 = 0;
            float wv = 0.f;
            if (used) {
                const size_t at = (wg * KT_BWI + t) * NT + threadIdx.x;
                l16 = lab[at];
                const uint32_t s = slot[at];
                wv = usl_load_f32<TS>(W, (size_t)min(s, last_slot));   // an empty place reads some weight and drops it
                wv = s != PAD_SLOT ? wv : 0.f;
            }
            if (t & 1) pk[t >> 1] |= l16 << 16; else pk[t >> 1] = l16;
            wt[t] = wv;
        }
    }
    const uint32_t ov0 = ov_base[wg], ov_n = ov_base[wg + 1] - ov0;
    float* row = reinterpret_cast<float*>(lds_raw);
    float* outbuf = row + WL;
    // which features the lane's two sums belong to: kept in LDS, not in registers (the lists need those)
    uint32_t* feat_of = reinterpret_cast<uint32_t*>(outbuf + NF);
    feat_of[threadIdx.x] = (uint32_t)feat[(wg * 2 + 0) * NT + threadIdx.x] | (uint32_t)feat[(wg * 2 + 1) * NT + threadIdx.x] << 16;
    // the first NT entries that did not fit the registers, with their weights: {feature | label << 16, weight}
    uint2* ov_near = reinterpret_cast<uint2*>(feat_of + NT);
    if (threadIdx.x < ov_n) {
        const OvEntry o = ov[(size_t)ov0 + threadIdx.x];
        ov_near[threadIdx.x] = make_uint2((uint32_t)o.label * 4u,   // an empty place: the zero word, no weight
                                          o.slot == PAD_SLOT ? 0u : __float_as_uint(usl_load_f32<TS>(W, (size_t)o.slot)));
    } else {
        ov_near[threadIdx.x] = make_uint2(ZERO_LABEL * 4u, 0u);
    }
    // ... and which of them belong to the lane's two lists (start | n << 16)
    uint32_t* ovr_a = reinterpret_cast<uint32_t*>(ov_near + NT);
    uint32_t* ovr_b = ovr_a + NT;
    ovr_a[threadIdx.x] = ovr[(wg * 2 + 0) * NT + threadIdx.x];
    ovr_b[threadIdx.x] = ovr[(wg * 2 + 1) * NT + threadIdx.x];
    if (threadIdx.x < 32) reinterpret_cast<uint32_t*>(lds_raw)[ZERO_LABEL + threadIdx.x] = 0u;
    const int nl = (int)min((int64_t)wl, m - (int64_t)w * wl);   // labels of this window (the last one may be short)
    const int nv = nl / 4, full = nv & ~63;                      // 16-byte pieces of a row slice; those in whole 1 KiB runs
    const int lines = (nl * 4 + 127) / 128, per = (lines + nfb - 1) / nfb;   // 128-byte lines; this workgroup's share of the warm-up
    const bool warms = (int)threadIdx.x < per && fb * per + (int)threadIdx.x < lines;
    // the rest of a list (r = start | n << 16 in ov_near, n even), two entries in flight at a time
    auto more = [&](float& acc, uint32_t r) {
        for (uint32_t q = r & 0xFFFFu, e = q + (r >> 16); q < e; q += 2) {
            const uint2 o0 = ov_near[q], o1 = ov_near[q + 1];
            const float v0 = *reinterpret_cast<lds_f32_t*>(static_cast<uintptr_t>(o0.x));
            const float v1 = *reinterpret_cast<lds_f32_t*>(static_cast<uintptr_t>(o1.x));
            acc = fmaf(__uint_as_float(o0.y), v0, acc);
            acc = fmaf(__uint_as_float(o1.y), v1, acc);
        }
    };
    // Receives the L2 warm-up loads, which are issued from inline assembly: the compiler then puts no wait behind them
    // (behind a load it knows of whose value is never used, or a volatile one, it waits on the spot: a trip to memory
    // at the start of this wavefront's gathers, 0.14 ms per call at m = 500k).  The register must not be touched until
    // the vmcnt(0) wait at the top of the next pass; the build checks that in the compiler's listing (build.py).
    uint32_t token = 0;
    for (int i = 0; i < rows; ++i) {
        const char* grow = reinterpret_cast<const char*>(g + (size_t)w * wl + (size_t)i * m);   // uniform
        {   // the row slice: whole 1 KiB pieces by LDS-DMA, the ragged end through registers
            for (int v = (threadIdx.x >> 6) * 64; v < full; v += NT)
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(grow + ((uint32_t)v * 16u + (threadIdx.x & 63u) * 16u)),
                                                 (__attribute__((address_space(3))) void*)(lds_raw + (size_t)v * 16), 16, 0, 0);
            for (int v = full + threadIdx.x; v < nv; v += NT)
                reinterpret_cast<uint4*>(lds_raw)[v] = reinterpret_cast<const uint4*>(grow)[v];
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            asm volatile("" : "+v"(token));
        }
        __syncthreads();
        if (i + 1 < rows && warms)   // the window's workgroups share the warm-up of the next row slice, one load per 128-byte line
            asm volatile("global_load_dword %0, %1, %2" : "=v"(token) : "v"((uint32_t)(fb * per + (int)threadIdx.x) * 128u), "s"(grow + (size_t)m * 4));
        float acc_a = 0.f, acc_b = 0.f;
        // compared afresh in every pass (one scalar compare per group): kept across the loop, the 34 outcomes would
        // each take a pair of scalar registers, more than there are
        int ac = acap, bc = bcap;
        asm volatile("" : "+s"(ac), "+s"(bc));
#pragma unroll
        for (int q = 0; q < KT_BWI / 4; ++q) {
            if (q * 4 < ac) {
                gather4(acc_a, pk[q * 2], pk[q * 2 + 1], wt[q * 4], wt[q * 4 + 1], wt[q * 4 + 2], wt[q * 4 + 3]);
            }
        }
#pragma unroll
        for (int q = 0; q < KT_BWI / 4; ++q) {
            if (q * 4 >= KT_BWI - bc) {
                gather4(acc_b, pk[q * 2], pk[q * 2 + 1], wt[q * 4], wt[q * 4 + 1], wt[q * 4 + 2], wt[q * 4 + 3]);
            }
        }
        if (ov_n) {   // the same for the whole workgroup: the few lanes whose lists did not fit go on through LDS
            more(acc_a, ovr_a[threadIdx.x]);
            more(acc_b, ovr_b[threadIdx.x]);
        }
        {
            const uint32_t f = feat_of[threadIdx.x];
            outbuf[f & 0xFFFFu] = acc_a;
            outbuf[f >> 16] = acc_b;
        }
        if (ov_n > (uint32_t)NT) {   // only a skewed connectivity gets here: what LDS does not hold, by atomics
            __syncthreads();
            for (uint32_t q = NT + threadIdx.x; q < ov_n; q += NT) {
                const OvEntry o = ov[(size_t)ov0 + q];
                if (o.slot != PAD_SLOT) unsafeAtomicAdd(&outbuf[o.feature], usl_load_f32<TS>(W, (size_t)o.slot) * row[o.label]);
            }
        }
        __syncthreads();
        {   // the block's NF sums leave as one contiguous run
            float* dst = partial + ((size_t)w * rows + i) * d + (size_t)fb * NF;
            for (int v = threadIdx.x; v < NF / 4; v += NT)
                reinterpret_cast<float4*>(dst)[v] = reinterpret_cast<const float4*>(outbuf)[v];
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    asm volatile("" : "+v"(token));
}

// ---------------------------------------------------------------------------------------------------------------
// Both backward products from one pass of gathers (usl_train_step).  Every gathered g[i][j] serves twice: times the
// connection's weight it goes into the feature's sum (Algorithm 2), times the feature's activation x[i][c] into a sum
// that the lane keeps per slot over the whole batch (Algorithm 3) and stores at the end -- every slot of the layer
// belongs to exactly one list of one workgroup, so every weight gradient is written once, without atomics.  The third
// register per slot halves the slots (KT_BOTH = 36) and with them the windows; the row buffer then has room for the
// slices of two instances, RS2 bytes apart, and a pass of the loop does two instances: one address, two reads (the
// second through the instruction's offset field), four multiply-adds.  A pass is then long enough again for the
// warm-up of the next rows to arrive in time (with one instance per pass of half the length it was not: the kernel
// took 1.46 ms at m = 500k).
// The sums of overflow entries live in LDS (ov_sum) or, beyond the NEAR2 that LDS holds, in memory (ovgw).
__device__ __forceinline__ void gather4_two(float& acc0, float& acc1, float& s0, float& s1, float& s2, float& s3,
                                            uint32_t p0, uint32_t p1, float w0, float w1, float w2, float w3, float x0, float x1) {
    uint32_t a0, a1, a2, a3, b0, b1, b2, b3;
    const uint32_t two = 2;
    asm volatile(
        "v_lshlrev_b32_sdwa %6, %14, %15 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_0\n\t"
        "v_lshlrev_b32_sdwa %7, %14, %15 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_1\n\t"
        "v_lshlrev_b32_sdwa %8, %14, %16 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_0\n\t"
        "v_lshlrev_b32_sdwa %9, %14, %16 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_1\n\t"
        "ds_read_b32 %10, %6 offset:64000\n\t"
        "ds_read_b32 %6, %6\n\t"
        "ds_read_b32 %11, %7 offset:64000\n\t"
        "ds_read_b32 %7, %7\n\t"
        "ds_read_b32 %12, %8 offset:64000\n\t"
        "ds_read_b32 %8, %8\n\t"
        "ds_read_b32 %13, %9 offset:64000\n\t"
        "ds_read_b32 %9, %9\n\t"
        "s_waitcnt lgkmcnt(6)\n\t"
        "v_fmac_f32 %0, %17, %6\n\t"
        "v_fmac_f32 %1, %17, %10\n\t"
        "v_fmac_f32 %2, %21, %6\n\t"
        "v_fmac_f32 %2, %22, %10\n\t"
        "s_waitcnt lgkmcnt(4)\n\t"
        "v_fmac_f32 %0, %18, %7\n\t"
        "v_fmac_f32 %1, %18, %11\n\t"
        "v_fmac_f32 %3, %21, %7\n\t"
        "v_fmac_f32 %3, %22, %11\n\t"
        "s_waitcnt lgkmcnt(2)\n\t"
        "v_fmac_f32 %0, %19, %8\n\t"
        "v_fmac_f32 %1, %19, %12\n\t"
        "v_fmac_f32 %4, %21, %8\n\t"
        "v_fmac_f32 %4, %22, %12\n\t"
        "s_waitcnt lgkmcnt(0)\n\t"
        "v_fmac_f32 %0, %20, %9\n\t"
        "v_fmac_f32 %1, %20, %13\n\t"
        "v_fmac_f32 %5, %21, %9\n\t"
        "v_fmac_f32 %5, %22, %13"
        : "+v"(acc0), "+v"(acc1), "+v"(s0), "+v"(s1), "+v"(s2), "+v"(s3),
          "=&v"(a0), "=&v"(a1), "=&v"(a2), "=&v"(a3), "=&v"(b0), "=&v"(b1), "=&v"(b2), "=&v"(b3)
        : "s"(two), "v"(p0), "v"(p1), "v"(w0), "v"(w1), "v"(w2), "v"(w3), "v"(x0), "v"(x1)
        : "memory");
}
static_assert(RS2 == 64000, "the offset of the second row buffer is written into gather4_two");

template <typename TS>
__global__ void __launch_bounds__(NT)
k_both_lds(const float* __restrict__ g, const TS* __restrict__ W, const TS* __restrict__ x, int64_t m, int k, int rows, int d,
           int wl, int nfb, int nwin, const uint16_t* __restrict__ lab, const uint32_t* __restrict__ slot,
           const uint16_t* __restrict__ feat, const uint32_t* __restrict__ caps, const uint32_t* __restrict__ ov_base,
           const OvEntry* __restrict__ ov, const uint32_t* __restrict__ ovr, float* __restrict__ partial,
           const uint32_t* __restrict__ rk, const uint32_t* __restrict__ ovrk, const uint32_t* __restrict__ ent_base,
           float* __restrict__ stage, float* __restrict__ ovgw, const uint32_t* __restrict__ gate, int accumulate) {
    constexpr int KT = KT_BOTH;
    extern __shared__ __align__(16) unsigned char lds_raw[];
    if (gate && *gate == 0) return;   // the kernels over the nonzero gradients do this call's work
    const int w = (blockIdx.x & 7) + 8 * (blockIdx.x / (8 * nfb)), fb = (blockIdx.x >> 3) % nfb;
    if (w >= nwin) return;
    const size_t wg = (size_t)w * nfb + fb;
    const uint32_t cw = caps[wg * (NT / 64) + (threadIdx.x >> 6)];
    const int acap = __builtin_amdgcn_readfirstlane((int)(cw & 0xFFu)), bcap = __builtin_amdgcn_readfirstlane((int)(cw >> 8));
    uint32_t pk[KT / 2];
    float wt[KT], gw[KT];
    const uint32_t last_slot = (uint32_t)(m * k - 1);
#pragma unroll
    for (int q = 0; q < KT / 4; ++q) {
        const bool used = q * 4 < acap || q * 4 >= KT - bcap;   // the same for the whole wavefront
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int t = q * 4 + u;
            uint32_t l16 = 0;
            float wv = 0.f;
            if (used) {
                const size_t at = (wg * KT + t) * NT + threadIdx.x;
                l16 = lab[at];
                const uint32_t s = slot[at];
                wv = usl_load_f32<TS>(W, (size_t)min(s, last_slot));   // an empty place reads some weight and drops it
                wv = s != PAD_SLOT ? wv : 0.f;
            }
            if (t & 1) pk[t >> 1] |= l16 << 16; else pk[t >> 1] = l16;
            wt[t] = wv;
            gw[t] = 0.f;
        }
    }
    const uint32_t ov0 = ov_base[wg], ov_n = ov_base[wg + 1] - ov0;
    float* row = reinterpret_cast<float*>(lds_raw);                       // row[label], row[RS2 / 4 + label]
    float* outbuf = reinterpret_cast<float*>(lds_raw + 2 * RS2);          // [2][NF]
    uint32_t* feat_of = reinterpret_cast<uint32_t*>(outbuf + 2 * NF);     // [NT]
    uint2* ov_near = reinterpret_cast<uint2*>(feat_of + NT);              // [NEAR2] {address of the label in row 0, weight}
    uint32_t* ovr_a = reinterpret_cast<uint32_t*>(ov_near + NEAR2);       // [NT] start | n << 16
    uint32_t* ovr_b = ovr_a + NT;
    float* ov_sum = reinterpret_cast<float*>(ovr_b + NT);                 // [NEAR2]
    feat_of[threadIdx.x] = (uint32_t)feat[(wg * 2 + 0) * NT + threadIdx.x] | (uint32_t)feat[(wg * 2 + 1) * NT + threadIdx.x] << 16;
    if (threadIdx.x < NEAR2) {
        uint2 e = make_uint2(ZERO_LABEL2 * 4u, 0u);
        if (threadIdx.x < ov_n) {
            const OvEntry o = ov[(size_t)ov0 + threadIdx.x];
            e = make_uint2((uint32_t)o.label * 4u, o.slot == PAD_SLOT ? 0u : __float_as_uint(usl_load_f32<TS>(W, (size_t)o.slot)));
        }
        ov_near[threadIdx.x] = e;
        ov_sum[threadIdx.x] = 0.f;
    }
    ovr_a[threadIdx.x] = ovr[(wg * 2 + 0) * NT + threadIdx.x];
    ovr_b[threadIdx.x] = ovr[(wg * 2 + 1) * NT + threadIdx.x];
    if (threadIdx.x < 64)   // the zero words behind both row buffers
        reinterpret_cast<uint32_t*>(lds_raw)[ZERO_LABEL2 + (threadIdx.x >> 5) * (RS2 / 4) + (threadIdx.x & 31)] = 0u;
    for (uint32_t q = NEAR2 + threadIdx.x; q < ov_n; q += NT) ovgw[(size_t)ov0 + q] = 0.f;   // entry q is lane q % NT's
    const int nl = (int)min((int64_t)wl, m - (int64_t)w * wl);   // labels of this window (the last one may be short)
    const int nv = nl / 4;                                       // 16-byte pieces of a row slice
    const int lines = (nl * 4 + 127) / 128, per = (lines + nfb - 1) / nfb;   // 128-byte lines; this workgroup's share of the warm-up
    constexpr int XL = NF * (int)sizeof(TS) / 128;   // 128-byte lines of a feature block's activations
    // the rest of a list (r = start | n << 16 in ov_near, n even), two entries in flight at a time
    auto more = [&](float& acc0, float& acc1, uint32_t r, float x0, float x1) {
        for (uint32_t q = r & 0xFFFFu, e = q + (r >> 16); q < e; q += 2) {
            const uint2 o0 = ov_near[q], o1 = ov_near[q + 1];
            const float u0 = *reinterpret_cast<lds_f32_t*>(static_cast<uintptr_t>(o0.x));
            const float u1 = *reinterpret_cast<lds_f32_t*>(static_cast<uintptr_t>(o0.x + RS2));
            const float v0 = *reinterpret_cast<lds_f32_t*>(static_cast<uintptr_t>(o1.x));
            const float v1 = *reinterpret_cast<lds_f32_t*>(static_cast<uintptr_t>(o1.x + RS2));
            acc0 = fmaf(__uint_as_float(o0.y), u0, acc0);
            acc1 = fmaf(__uint_as_float(o0.y), u1, acc1);
            acc0 = fmaf(__uint_as_float(o1.y), v0, acc0);
            acc1 = fmaf(__uint_as_float(o1.y), v1, acc1);
            ov_sum[q] = fmaf(x1, u1, fmaf(x0, u0, ov_sum[q]));           // the entries of a list are its lane's alone
            ov_sum[q + 1] = fmaf(x1, v1, fmaf(x0, v0, ov_sum[q + 1]));
        }
    };
    // the activations of the lane's two features for the two instances of a pass
    float xa0 = 0.f, xb0 = 0.f, xa1 = 0.f, xb1 = 0.f;
    // receives the L2 warm-up loads (issued from inline assembly, see k_bwi_lds; the build checks this kernel too)
    uint32_t token = 0;
    for (int i = 0; i < rows; i += 2) {
        const bool pair = i + 1 < rows;
        const char* grow = reinterpret_cast<const char*>(g + (size_t)w * wl + (size_t)i * m);   // uniform
        const TS* xrow = x + (size_t)i * d + (size_t)fb * NF;
        // The lane's number, taken afresh in each part of a pass: whatever is computed from it (addresses in LDS, offsets
        // of copies) is then computed there, in a few instructions, and not kept in a register of its own across the
        // gathers -- there are none to spare, and a value that is spilled comes back through a load whose wait also
        // waits for the warm-up loads.
        uint32_t tid = threadIdx.x;
        asm volatile("" : "+v"(tid));
        {   // the block's activations of the two instances: 1 KiB pieces by LDS-DMA into the place of the sums (free
            // until the gathers are done); read from memory by feature they cost as much as the slices of g.
            // Wavefront v overwrites bytes [1024 v, 1024 v + 1024) of that place: the piece that it alone read when the
            // sums of the pass before left (no barrier since then), so nobody else's sums are lost.
            static_assert(2 * NF / 4 == NT, "a lane copies out one float4 of the sums: wavefront v the v-th KiB");
            constexpr int PR = NF * (int)sizeof(TS) / 1024;
            const int wv = (int)(tid >> 6);
            if (wv < (pair ? 2 : 1) * PR)
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(reinterpret_cast<const char*>(xrow + (size_t)(wv / PR) * d) + ((uint32_t)(wv % PR) * 1024u + (tid & 63u) * 16u)),
                                                 (__attribute__((address_space(3))) void*)(reinterpret_cast<unsigned char*>(outbuf) + (size_t)(wv / PR) * NF * sizeof(TS) + (size_t)(wv % PR) * 1024), 16, 0, 0);
        }
        {   // the two row slices by LDS-DMA, 1 KiB per wavefront and instruction; in the last piece only the lanes that
            // still have 16 bytes of the slice take part (a lane's data lands at its own place whoever else is masked).
            // Through registers, the ragged end cost a round trip to L2 per slice, one after the other.
            for (int v = (int)(tid >> 6) * 64; v < nv; v += NT) {
                if (v + (int)(tid & 63u) < nv) {
                    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(grow + ((uint32_t)v * 16u + (tid & 63u) * 16u)),
                                                     (__attribute__((address_space(3))) void*)(lds_raw + (size_t)v * 16), 16, 0, 0);
                    if (pair)
                        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(grow + (size_t)m * 4 + ((uint32_t)v * 16u + (tid & 63u) * 16u)),
                                                         (__attribute__((address_space(3))) void*)(lds_raw + RS2 + (size_t)v * 16), 16, 0, 0);
                }
            }
            if (!pair)   // an odd batch: the last pass has one instance, the second buffer reads as zeros
                for (int v = (int)tid; v < nv; v += NT) reinterpret_cast<uint4*>(lds_raw + RS2)[v] = make_uint4(0u, 0u, 0u, 0u);
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            asm volatile("" : "+v"(token));
        }
        __syncthreads();
        tid = threadIdx.x;
        asm volatile("" : "+v"(tid));
        {
            const uint32_t f = feat_of[tid];
            const TS* xbuf = reinterpret_cast<const TS*>(outbuf);
            xa0 = usl_load_f32<TS>(xbuf, (size_t)(f & 0xFFFFu));
            xb0 = usl_load_f32<TS>(xbuf, (size_t)(f >> 16));
            xa1 = pair ? usl_load_f32<TS>(xbuf, (size_t)NF + (f & 0xFFFFu)) : 0.f;
            xb1 = pair ? usl_load_f32<TS>(xbuf, (size_t)NF + (f >> 16)) : 0.f;
        }
        if (i + 2 < rows) {   // one load per 128-byte line of what the next pass reads: the window's workgroups share
            // the lines of its two slices of g, then come the block's own lines of the two rows of x
            for (int j = (int)tid; j < 2 * per + 2 * XL; j += NT) {   // (no divisions: every lane comes through here)
                const bool of_g = j < 2 * per;
                const int jj = of_g ? j : j - 2 * per, half = of_g ? per : XL;
                const int r = jj >= half ? 1 : 0, c = (of_g ? fb * per : 0) + jj - r * half;
                const char* line = (of_g ? grow + (size_t)m * 4 * (2 + r) : reinterpret_cast<const char*>(xrow + (size_t)(2 + r) * d)) + (size_t)c * 128;
                if (i + 2 + r < rows && (!of_g || c < lines))
                    asm volatile("global_load_dword %0, %1, off" : "+v"(token) : "v"(line));
            }
        }
        float acc_a0 = 0.f, acc_a1 = 0.f, acc_b0 = 0.f, acc_b1 = 0.f;
        int ac = acap, bc = bcap;   // compared afresh in every pass, see k_bwi_lds
        asm volatile("" : "+s"(ac), "+s"(bc));
#pragma unroll
        for (int q = 0; q < KT / 4; ++q) {
            if (q * 4 < ac)
                gather4_two(acc_a0, acc_a1, gw[q * 4], gw[q * 4 + 1], gw[q * 4 + 2], gw[q * 4 + 3], pk[q * 2], pk[q * 2 + 1],
                            wt[q * 4], wt[q * 4 + 1], wt[q * 4 + 2], wt[q * 4 + 3], xa0, xa1);
        }
#pragma unroll
        for (int q = 0; q < KT / 4; ++q) {
            if (q * 4 >= KT - bc)
                gather4_two(acc_b0, acc_b1, gw[q * 4], gw[q * 4 + 1], gw[q * 4 + 2], gw[q * 4 + 3], pk[q * 2], pk[q * 2 + 1],
                            wt[q * 4], wt[q * 4 + 1], wt[q * 4 + 2], wt[q * 4 + 3], xb0, xb1);
        }
        tid = threadIdx.x;
        asm volatile("" : "+v"(tid));
        if (ov_n) {   // the same for the whole workgroup: the few lanes whose lists did not fit go on through LDS
            more(acc_a0, acc_a1, ovr_a[tid], xa0, xa1);
            more(acc_b0, acc_b1, ovr_b[tid], xb0, xb1);
        }
        __syncthreads();   // every lane has taken its activations from the place of the sums
        {
            const uint32_t f = feat_of[tid];
            outbuf[f & 0xFFFFu] = acc_a0;
            outbuf[NF + (f & 0xFFFFu)] = acc_a1;
            outbuf[f >> 16] = acc_b0;
            outbuf[NF + (f >> 16)] = acc_b1;
        }
        if (ov_n > (uint32_t)NEAR2) {   // only a skewed connectivity gets here: what LDS does not hold, by atomics
            __syncthreads();
            const TS* xr = xrow;
            for (uint32_t q = NEAR2 + tid; q < ov_n; q += NT) {
                const OvEntry o = ov[(size_t)ov0 + q];
                if (o.slot == PAD_SLOT) continue;
                const float wv = usl_load_f32<TS>(W, (size_t)o.slot), u0 = row[o.label], u1 = row[RS2 / 4 + o.label];
                unsafeAtomicAdd(&outbuf[o.feature], wv * u0);
                unsafeAtomicAdd(&outbuf[NF + o.feature], wv * u1);
                float t = fmaf(usl_load_f32<TS>(xr, (size_t)o.feature), u0, ovgw[(size_t)ov0 + q]);
                if (pair) t = fmaf(usl_load_f32<TS>(xr + d, (size_t)o.feature), u1, t);
                ovgw[(size_t)ov0 + q] = t;
            }
        }
        __syncthreads();
        {   // the block's sums of the two instances leave as two contiguous runs
            float* dst = partial + ((size_t)w * rows + i) * d + (size_t)fb * NF;
            for (int v = (int)tid; v < (pair ? 2 : 1) * (NF / 4); v += NT)
                reinterpret_cast<float4*>(dst + (size_t)(v / (NF / 4)) * d)[v % (NF / 4)] = reinterpret_cast<const float4*>(outbuf)[v];
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    asm volatile("" : "+v"(token));
    // Every slot's sum leaves for its place in stage (rk, ovrk: the workgroup's connections in the order of their
    // flat slots, see k_lf_seg_place), through LDS, which is free now: whole lines.  Written to grad_W[slot] from here
    // they would be 4 bytes each into lines that 16 workgroups share (0.29 ms at m = 500k, a fifth of this kernel); the
    // Adam kernel picks them up through pos instead, and finds neighbours there.  As many places at a time as LDS
    // holds below ov_sum (all of them, unless the connectivity is skewed).
    constexpr uint32_t CH = (uint32_t)((LDS2_BYTES - (size_t)NEAR2 * 4) / 4);
    float* perm = reinterpret_cast<float*>(lds_raw);
    const uint32_t e0 = ent_base[wg], n_ent = ent_base[wg + 1] - e0;
    for (uint32_t c0 = 0; c0 < n_ent; c0 += CH) {
        __syncthreads();   // the last pass's reads of LDS, the owners' last additions to ov_sum; the copy before
#pragma unroll
        for (int q = 0; q < KT / 4; ++q) {
            if (q * 4 < acap || q * 4 >= KT - bcap) {
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const uint32_t r = rk[(wg * KT + q * 4 + u) * NT + threadIdx.x] - c0;   // an empty place: far beyond
                    if (r < CH) perm[r] = gw[q * 4 + u];
                }
            }
        }
        for (uint32_t q = threadIdx.x; q < ov_n; q += NT) {
            const uint32_t r = ovrk[(size_t)ov0 + q] - c0;
            if (r < CH) perm[r] = q < (uint32_t)NEAR2 ? ov_sum[q] : ovgw[(size_t)ov0 + q];
        }
        __syncthreads();
        for (uint32_t r = threadIdx.x; r < min(CH, n_ent - c0); r += NT)   // a later pass over the batch adds to the earlier ones
            stage[(size_t)e0 + c0 + r] = accumulate ? stage[(size_t)e0 + c0 + r] + perm[r] : perm[r];
    }
}

// grad_x[i][c] = sum over the windows of partial[w][i][c].  BOTH only names the kernel after the one whose sums it
// adds (twice the windows there), so that a profile tells the two apart.
template <bool BOTH>
__global__ void __launch_bounds__(256)
k_lf_reduce(const float4* __restrict__ partial, int nwin, size_t n4, float4* __restrict__ out,
            const uint32_t* __restrict__ gate, const uint32_t* __restrict__ stale) {
    if (gate && *gate == 0) return;
    const bool poison = *stale != 0;   // the lists were built from other contents of idx: no number is better than a wrong one
    size_t v = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t step = (size_t)gridDim.x * blockDim.x;
    for (; v < n4; v += step) {
        float4 a = partial[v];
        for (int q = 1; q < nwin; ++q) {
            const float4 t = partial[(size_t)q * n4 + v];
            a.x += t.x; a.y += t.y; a.z += t.z; a.w += t.w;
        }
        if (poison) a.x = a.y = a.z = a.w = __uint_as_float(0x7FC00000u);
        out[v] = a;
    }
}

}  // namespace

// Windows: as many labels as send about 32 connections into a feature (the registers of a lane hold two such lists;
// 16 connections for the lists of the kernel that keeps a weight-gradient sum per slot as well), at most WL (the LDS
// row; ZERO_LABEL2 there, two rows), a multiple of 4 (16-byte copies); a layer's windows are of equal size.
static int lf_window_cap(const usl_ctx* c, int set) {
    const int64_t by_lists = (int64_t)(set ? 16 : 32) * c->d / c->k, most = set ? (int64_t)ZERO_LABEL2 : (int64_t)WL;
    return (int)((by_lists < most ? by_lists : most) / 4 * 4);
}
static int lf_windows(const usl_ctx* c, int set) {
    const int cap = lf_window_cap(c, set);
    int64_t nwin = (c->m + cap - 1) / cap;
    // (window, feature block) workgroups run in rounds of one per compute unit: a last round that is not full takes as
    // long as a full one, so the windows are made a little shorter until the rounds are full (up to a quarter more
    // windows: more than that and the extra partial sums cost what the shorter lists save)
    const int64_t nfb = c->d / NF, cu = c->num_cu > 0 ? c->num_cu : 1;
    const int64_t rounds = (nwin * nfb + cu - 1) / cu;
    const int64_t full = rounds * cu / nfb;
    if (full > nwin && full * 4 <= nwin * 5) nwin = full;
    return (int)nwin;
}
static int lf_window_labels(const usl_ctx* c, int set) {
    const int64_t nwin = lf_windows(c, set);
    return (int)(((c->m + nwin - 1) / nwin + 3) / 4 * 4);
}

// The most that the partial sums of a pass over the batch may take: 16 GiB on a device with 128 GiB or more (every
// pass loads lists and weights anew: at m = 3M, d = 65536, b = 1024 the two products take 74 ms with passes of 4 GiB,
// 62 ms with passes of 16 GiB, 65 ms with one pass of 48 GiB), else 4 GiB.  USL_TUNE_LF_GIB overrides.
static size_t lf_partial_bytes() {
    if (const char* e = getenv("USL_TUNE_LF_GIB")) return (size_t)(atoi(e) > 0 ? atoi(e) : 1) << 30;
    static size_t cached = 0;
    if (!cached) {
        size_t free_b = 0, total_b = 0;
        cached = (hipMemGetInfo(&free_b, &total_b) == hipSuccess && total_b >= ((size_t)128 << 30)) ? (size_t)16 << 30 : (size_t)4 << 30;
    }
    return cached;
}

// runs of SEG slots in a window of the lists for both products
static int lf_runs(const usl_ctx* c) { return (int)(((int64_t)lf_window_labels(c, 1) * c->k + SEG - 1) / SEG); }

static bool lf_shape_ok(const usl_ctx* c, int set) {
    const int64_t lists = (int64_t)(set ? 16 : 32) * c->d / c->k;   // labels that send that many connections into a feature
    return c->d % NF == 0 && c->d <= 65536 && c->m % 4 == 0 && lists >= 2048 && lists <= WL &&
           c->m * (int64_t)c->k < (int64_t)PAD_SLOT;
}

// Is this layer one for the LDS form?  Lists of about 32 entries per (window, feature) from windows of 16384 to
// 32768 labels (k / d between 1/1024 and 1/512: longer windows do not fit LDS, with shorter ones the partial sums of
// the many windows outweigh the gain), whole feature blocks, 16-byte aligned rows of g, and enough (window, feature
// block) workgroups to fill the chip.  USL_TUNE_BWI=lds forces it where the shape allows at all, =l2 forbids it.
bool usl_bwi_lds_applies(const usl_ctx* c) {
    if (!lf_shape_ok(c, 0)) return false;
    if (const char* e = getenv("USL_TUNE_BWI")) {
        if (!strcmp(e, "lds")) return true;
        if (!strcmp(e, "l2")) return false;
    }
    return (int64_t)32 * c->d / c->k >= 16384 && (int64_t)lf_windows(c, 0) * (c->d / NF) * 4 >= (int64_t)c->num_cu * 3;
}

// ... and one for the kernel that computes both backward products from one pass of gathers?  The same with lists of
// 16 entries or fewer from windows of 8192 to 15968 labels (k / d of 1/512 or less: twice the windows, twice the
// partial sums).
// USL_TUNE_BOTH=on forces it where the shape allows at all, =off forbids it.
static bool lf_a_pass_fits(const usl_ctx* c);
bool usl_both_lds_applies(const usl_ctx* c) {
    if (!lf_shape_ok(c, 1) || !lf_a_pass_fits(c)) return false;
    if (const char* e = getenv("USL_TUNE_BOTH")) {
        if (!strcmp(e, "on")) return true;
        if (!strcmp(e, "off")) return false;
    }
    return (int64_t)16 * c->d / c->k >= 8192 && (int64_t)lf_windows(c, 1) * (c->d / NF) * 4 >= (int64_t)c->num_cu * 3;
}

// The partial sums of a pass of 64 instances (the fewest a pass takes) must fit the allowance.
static bool lf_a_pass_fits(const usl_ctx* c) {
    return (size_t)lf_windows(c, 1) * 64 * (size_t)c->d * 4 <= lf_partial_bytes();
}

template <int KT>
static usl_status lf_build_t(usl_ctx* c, const int32_t* idx, int set) {
    auto& L = c->lf[set];
    const size_t N = (size_t)c->m * c->k;
    const int nwin = lf_windows(c, set), wl = lf_window_labels(c, set), nfb = c->d / NF, nwg = nwin * nfb;
    const size_t nbins = (size_t)nwin * c->d;
    USL_TRY(usl_reserve(c, (void**)&L.count, &L.count_cap, nbins * 4));
    USL_TRY(usl_reserve(c, (void**)&L.taken, &L.taken_cap, nbins * 4));
    USL_TRY(usl_reserve(c, (void**)&L.where, &L.where_cap, nbins * 4));
    USL_TRY(usl_reserve(c, (void**)&L.feat, &L.feat_cap, (size_t)nwg * 2 * NT * 2));
    USL_TRY(usl_reserve(c, (void**)&L.caps, &L.caps_cap, (size_t)nwg * (NT / 64) * 4));
    USL_TRY(usl_reserve(c, (void**)&L.ov_base, &L.ov_base_cap, ((size_t)nwg * 4 + 2) * 4));
    USL_TRY(usl_reserve(c, (void**)&L.ovr, &L.ovr_cap, (size_t)nwg * 2 * NT * 4));
    USL_TRY(usl_reserve(c, (void**)&L.lab, &L.lab_cap, (size_t)nwg * KT * NT * 2));
    USL_TRY(usl_reserve(c, (void**)&L.slot, &L.slot_cap, (size_t)nwg * KT * NT * 4));
    USL_TRY(usl_reserve(c, (void**)&L.ent, &L.ent_cap, N * 4));
    USL_TRY(usl_reserve(c, (void**)&L.ovoff, &L.ovoff_cap, nbins * 4));
    USL_TRY(usl_reserve(c, (void**)&L.ov, &L.ov_cap, (N + nbins) * sizeof(OvEntry)));   // worst case, + an empty place per list
    if (set == 1) {
        // stage [N], the sums of the overflow entries beyond LDS [N + nbins]; pos [N], rk [nwg][KT][NT], ovrk [N + nbins],
        // the counts of the runs [nwg][nseg]
        USL_TRY(usl_reserve(c, (void**)&L.stage, &L.stage_cap, (N + N + nbins) * 4));
        USL_TRY(usl_reserve(c, (void**)&L.pos, &L.pos_cap, (N + (size_t)nwg * KT * NT + N + nbins + (size_t)nwg * lf_runs(c)) * 4));
    }
    int rounds = 3;                // of proposals per step of the bank-aware order; 0 = lists stay as filled
    if (const char* e = getenv("USL_TUNE_ROUNDS")) rounds = atoi(e);
    uint32_t* ov_base = L.ov_base;                   // [nwg + 1]
    uint32_t* n_ov = ov_base + nwg + 1;              // [nwg]
    uint32_t* ent_base = n_ov + nwg;                 // [nwg + 1]
    uint32_t* n_ent = ent_base + nwg + 1;            // [nwg]
    const unsigned chunks = (unsigned)((c->d + CHUNK - 1) / CHUNK);
    int splits = (int)((size_t)c->num_cu / ((size_t)nwin * chunks));
    splits = splits < 1 ? 1 : splits > 16 ? 16 : splits;
    const dim3 grid((unsigned)(nwin * splits), chunks);
    const size_t lds = (size_t)(c->d < CHUNK ? c->d : CHUNK) * 4;
    USL_HIP(c, hipFuncSetAttribute(reinterpret_cast<const void*>(k_lf_count), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    USL_HIP(c, hipFuncSetAttribute(reinterpret_cast<const void*>(k_lf_fill), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    const dim3 fillg(c->num_cu * 4), fillb(256);
    hipLaunchKernelGGL(k_fill_u32, fillg, fillb, 0, c->stream, L.count, nbins, 0u);
    hipLaunchKernelGGL(k_fill_u32, fillg, fillb, 0, c->stream, L.taken, nbins, 0u);
    hipLaunchKernelGGL(k_lf_count, grid, dim3(NT), lds, c->stream, idx, c->m, c->k, c->d, wl, splits, L.count);
    hipLaunchKernelGGL(k_lf_plan<KT>, dim3((unsigned)nwg), dim3(NT), 0, c->stream, L.count, c->d, nfb, L.where, L.ovoff,
                       L.feat, L.caps, n_ent, n_ov, L.ovr);
    hipLaunchKernelGGL(k_lf_scan, dim3(1), dim3(1024), 0, c->stream, n_ov, nwg, ov_base);
    hipLaunchKernelGGL(k_lf_scan, dim3(1), dim3(1024), 0, c->stream, n_ent, nwg, ent_base);
    hipLaunchKernelGGL(k_lf_fill, grid, dim3(NT), lds, c->stream, idx, c->m, c->k, c->d, wl, nfb, splits, L.where, L.taken,
                       ent_base, L.ent);
    if (set == 1) {   // where the weight gradients go (before the order of the lists, which hands the places on)
        const int nseg = lf_runs(c);
        const int64_t total = (int64_t)nwin * nseg;
        uint32_t* segcnt = L.pos + N + (size_t)nwg * KT * NT + N + nbins;
        const dim3 sg((unsigned)((total + 3) / 4));
        hipLaunchKernelGGL(k_lf_seg_count, sg, dim3(256), 0, c->stream, idx, c->m, c->k, wl, nfb, nseg, total, segcnt);
        hipLaunchKernelGGL(k_lf_seg_scan, dim3((unsigned)nwg), dim3(256), 0, c->stream, segcnt, nseg, ent_base);
        hipLaunchKernelGGL(k_lf_seg_place, sg, dim3(256), 0, c->stream, idx, c->m, c->k, wl, nfb, nseg, total, segcnt, L.pos);
    }
    hipLaunchKernelGGL(k_lf_schedule<KT>, dim3((unsigned)(nwg * 64 / SG)), dim3(SG * 32), 0, c->stream, L.ent, ent_base,
                       L.where, L.count, L.feat, L.caps, ov_base, L.ovoff, c->k, c->d, wl, nfb, rounds,
                       L.lab, L.slot, reinterpret_cast<OvEntry*>(L.ov), set == 1 ? L.pos : nullptr,
                       set == 1 ? L.pos + N : nullptr, set == 1 ? L.pos + N + (size_t)nwg * KT * NT : nullptr);
    USL_TRY(usl_idx_fingerprint(c, idx, 1));
    USL_TRY(usl_check_launch(c, "register lists of the input gradient"));
    // one fingerprint: it belongs to the lists built last
    c->csc_built_for = nullptr;
    c->lf[0].built_for = c->lf[1].built_for = nullptr;
    L.built_for = idx;
    return USL_OK;
}

// One or both backward products through the register lists (set 0: grad_x only; set 1: grad_x and grad_W).
template <int KT, bool BOTH>
static usl_status lf_run_t(usl_ctx* c, int set, const float* g, const void* x, const int32_t* idx, const void* W,
                           float* grad_x, int32_t b, const uint32_t* gate) {
    auto& L = c->lf[set];
    // same address as when the lists were built: check that the contents are the same (else grad_x becomes NaN and
    // usl_check reports it)
    if (L.built_for != idx) USL_TRY(lf_build_t<KT>(c, idx, set));
    else USL_TRY(usl_idx_fingerprint(c, idx, 0));
    const uint32_t* stale = reinterpret_cast<const uint32_t*>(c->idx_print) + 4;
    const int nwin = lf_windows(c, set), wl = lf_window_labels(c, set), nfb = c->d / NF;
    // instances per pass: every pass loads the lists and the weights anew, and its partial sums are nwin * G * d
    // floats; as many as the allowance for partial sums admits, sized once for max_b.  The weight gradient is a sum over the
    // whole batch, kept in registers during a pass: a later pass adds its sums to what the earlier ones left.
    int G = (int)(lf_partial_bytes() / ((size_t)nwin * c->d * 4));
    if (const char* e = getenv("USL_TUNE_BWI_ROWS")) G = atoi(e) < G ? atoi(e) : G;   // tests: several passes on a small layer
    G = G < 64 ? 64 : G;
    G = G > c->max_b ? c->max_b : G;
    if (BOTH && G > 1) G &= ~1;   // two instances per pass of the loop: an even number, so that only the last pass over the batch has an odd one left
    USL_TRY(usl_reserve(c, (void**)&L.partial, &L.partial_cap, (size_t)nwin * G * c->d * 4));
    const size_t lds = BOTH ? LDS2_BYTES : LDS_BYTES, N = (size_t)c->m * c->k;
    const unsigned grid = (unsigned)(((nwin + 7) / 8) * 8 * nfb);
    static bool checked[2] = {false, false};
    for (int i0 = 0; i0 < b; i0 += G) {
        const int rows = b - i0 < G ? b - i0 : G;
#define USL_LDS_FORM(TS, WHICH, KERNEL, ...)                                                                             \
        do {                                                                                                             \
            if (!checked[WHICH]) {                                                                                       \
                hipFuncAttributes fa;                                                                                    \
                USL_HIP(c, hipFuncGetAttributes(&fa, reinterpret_cast<const void*>(KERNEL<TS>)));                        \
                if (fa.sharedSizeBytes != 0)                                                                             \
                    USL_FAIL(c, USL_EUNSUPPORTED, "backward_input (LDS form): the kernel has static LDS, its row buffer " \
                                                  "does not start at LDS address 0");                                    \
                USL_HIP(c, hipFuncSetAttribute(reinterpret_cast<const void*>(KERNEL<TS>),                                \
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));                   \
                checked[WHICH] = true;                                                                                   \
            }                                                                                                            \
            hipLaunchKernelGGL(KERNEL<TS>, dim3(grid), dim3(NT), lds, c->stream, g + (size_t)i0 * c->m, (const TS*)W,    \
                               __VA_ARGS__);                                                                             \
        } while (0)
        if (BOTH) {
            if (c->storage == USL_F32)
                USL_LDS_FORM(float, 0, k_both_lds, (const float*)x + (size_t)i0 * c->d, c->m, c->k, rows, c->d, wl, nfb, nwin, L.lab,
                             L.slot, L.feat, L.caps, L.ov_base, reinterpret_cast<const OvEntry*>(L.ov), L.ovr, L.partial, L.pos + N,
                             L.pos + N + (size_t)nwin * nfb * KT * NT, L.ov_base + 2 * ((size_t)nwin * nfb) + 1, L.stage,
                             L.stage + N, gate, i0 > 0 ? 1 : 0);
            else
                USL_LDS_FORM(uint16_t, 1, k_both_lds, (const uint16_t*)x + (size_t)i0 * c->d, c->m, c->k, rows, c->d, wl, nfb, nwin,
                             L.lab, L.slot, L.feat, L.caps, L.ov_base, reinterpret_cast<const OvEntry*>(L.ov), L.ovr, L.partial,
                             L.pos + N, L.pos + N + (size_t)nwin * nfb * KT * NT, L.ov_base + 2 * ((size_t)nwin * nfb) + 1,
                             L.stage, L.stage + N, gate, i0 > 0 ? 1 : 0);
        } else {
            if (c->storage == USL_F32)
                USL_LDS_FORM(float, 0, k_bwi_lds, c->m, c->k, rows, c->d, wl, nfb, nwin, L.lab, L.slot, L.feat, L.caps, L.ov_base,
                             reinterpret_cast<const OvEntry*>(L.ov), L.ovr, L.partial, gate);
            else
                USL_LDS_FORM(uint16_t, 1, k_bwi_lds, c->m, c->k, rows, c->d, wl, nfb, nwin, L.lab, L.slot, L.feat, L.caps, L.ov_base,
                             reinterpret_cast<const OvEntry*>(L.ov), L.ovr, L.partial, gate);
        }
#undef USL_LDS_FORM
        const size_t n4 = (size_t)rows * c->d / 4;
        hipLaunchKernelGGL(k_lf_reduce<BOTH>, dim3(c->num_cu * 8), dim3(256), 0, c->stream,
                           reinterpret_cast<const float4*>(L.partial), nwin, n4,
                           reinterpret_cast<float4*>(grad_x + (size_t)i0 * c->d), gate, stale);
    }
    return usl_check_launch(c, BOTH ? "backward products (LDS form)" : "backward_input (LDS form)");
}

// grad_x[b][d] from g[b][m] (row-major).  gate as for the other dense kernels.
usl_status usl_bwi_lds_run(usl_ctx* c, const float* g, const int32_t* idx, const void* W, float* grad_x, int32_t b,
                           const uint32_t* gate) {
    return lf_run_t<KT_BWI, false>(c, 0, g, nullptr, idx, W, grad_x, b, gate);
}

// grad_x[b][d] and the weight gradient from g[b][m] and x[b][d].  The weight gradient is left in the order of the lists:
// slot f's is (*stage)[(*pos)[f]] (usl_launch_adam_staged takes it from there); both arrays belong to the context and
// hold until the next call or a change of idx.  A stale idx (see usl_check) poisons grad_x here; *stale is the device
// word that says so, for whoever picks up the weight gradient.
usl_status usl_both_lds_run(usl_ctx* c, const float* g, const void* x, const int32_t* idx, const void* W, float* grad_x,
                            int32_t b, const uint32_t* gate, const float** stage, const uint32_t** pos, const uint32_t** stale) {
    USL_TRY((lf_run_t<KT_BOTH, true>(c, 1, g, x, idx, W, grad_x, b, gate)));
    *stage = c->lf[1].stage;
    *pos = c->lf[1].pos;
    *stale = reinterpret_cast<const uint32_t*>(c->idx_print) + 4;
    return USL_OK;
}
