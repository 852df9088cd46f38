// Bank-aware slot order for the LDS gathers of forward / backward-weight.
//
// In those kernels the 32 lanes of a half-wavefront own 32 consecutive labels and, at step s, all
// read slot order[s] of their own label from the activation row in LDS.  With the slots in their
// natural order the 32 addresses are random and collide in the 32 LDS banks (a step then costs as
// many cycles as the fullest bank, 3.5 on average).  The sum over a label's slots may be taken in
// any order, so each label gets a private permutation of its slots, chosen so that the lanes of a
// half-wavefront hit different banks at the same step as far as possible.
//
// A step costs as many LDS cycles as its fullest bank holds lanes, so what counts is the number of steps with
// a collision, not the number of collisions: banks that the group's 32*k slots over-subscribe must collide
// somewhere, and the aim is to gather those collisions in few steps.  The order is therefore built step by
// step as a sequence of bipartite matchings between the 32 labels and the 32 banks (over the slots not used
// yet): a few rounds of proposals match most labels, augmenting paths (breadth-first, one per bank still
// free) complete the matching, and the labels that cannot be matched -- their banks are all taken -- double
// up on the least loaded bank they can reach.  One half-wavefront works on one group: lane i is label i and
// also bank i, all state is in registers and moves by ballots and shuffles; only a label's own bank list and
// the proposal slots live in LDS.  The result is a deterministic function of idx.  Any outcome is a valid
// permutation: it changes speed, never results.  (A local search on the sum of squared bank counts, used
// before, spread the unavoidable collisions over all steps: 2.0 cycles per step against 1.5 now.)
#include <stdlib.h>

#include "usl_internal.h"

namespace {

constexpr int SCHED_GROUPS = 8;   // groups of 32 labels per workgroup of 256 lanes

template <int K>
__global__ void __launch_bounds__(SCHED_GROUPS * 32)
k_schedule(const int32_t* __restrict__ idx, int64_t m, int shift, int rounds, uint8_t* __restrict__ perm) {
    constexpr int G = SCHED_GROUPS;
    // per label (rows padded by 4 bytes: lanes of a group then hit different LDS banks)
    __shared__ uint8_t slots[G][32][K + 4];   // first the bank of every slot, then my slots sorted by bank
    __shared__ uint8_t ord[G][32][K + 4];     // slot read at step s
    __shared__ uint8_t left_in[G][32][36];    // unused slots of mine per bank
    __shared__ uint8_t end_of[G][32][36];     // where bank b's slots end in the sorted list
    __shared__ int deg0[G][32];
    __shared__ int win[G][32];
    const int gl = threadIdx.x >> 5, lane = threadIdx.x & 31;
    const int hs = threadIdx.x & 32;        // where my group's 32 bits sit in a wavefront ballot
    const int64_t j = ((int64_t)blockIdx.x * G + gl) * 32 + lane;
    const bool valid = j < m;
    deg0[gl][lane] = 0;
    for (int b = 0; b < 32; ++b) left_in[gl][lane][b] = 0;
    __syncthreads();
    uint8_t* mine = slots[gl][lane];
    uint8_t* cnt = left_in[gl][lane];
    uint8_t* ends = end_of[gl][lane];
    for (int t = 0; t < K; ++t) {
        const int b = valid ? ((idx[j * K + t] >> shift) & 31) : ((lane + t) & 31);
        mine[t] = (uint8_t)b;
        ++cnt[b];
        atomicAdd(&deg0[gl][b], 1);
    }
    uint32_t avail = 0;           // banks my unused slots read
    {   // counting sort of my slots by bank, in place through ord (free until the first step)
        int run = 0;
        for (int b = 0; b < 32; ++b) { run += cnt[b]; ends[b] = (uint8_t)run; if (cnt[b]) avail |= 1u << b; }
        uint8_t* tmp = ord[gl][lane];
        for (int t = 0; t < K; ++t) tmp[t] = mine[t];
        for (int t = K - 1; t >= 0; --t) { const int b = tmp[t]; ends[b] = (uint8_t)(ends[b] - 1); mine[ends[b]] = (uint8_t)t; }
        for (int b = 0; b < 32; ++b) ends[b] = (uint8_t)(ends[b] + cnt[b]);   // back from starts to ends
    }
    __syncthreads();
    auto gballot = [&](bool p) -> uint32_t { return (uint32_t)(__ballot(p) >> hs); };
    volatile int* gwin = win[gl];
    // bank role
    int mydeg = deg0[gl][lane];   // slots of the group that read bank `lane` and are not used yet
    for (int s = 0; s < K; ++s) {
        int mb = -1;              // label role: my bank at this step
        int ml = -1;              // bank role: the label that reads me at this step
        for (int r = 0; r < rounds; ++r) {
            const uint32_t freeb = gballot(ml < 0);
            gwin[lane] = 255;
            int prop = -1;
            const uint32_t cand = mb < 0 ? (avail & freeb) : 0u;
            if (cand) {           // first candidate bank at or after a lane- and round-dependent start
                const int sh = (lane + 7 * r) & 31;
                const uint32_t rc = (cand >> sh) | (cand << ((32 - sh) & 31));
                prop = (__ffs(rc) - 1 + sh) & 31;
                atomicMin(&win[gl][prop], lane);
            }
            const int w = gwin[lane];
            if (ml < 0 && w < 32) ml = w;
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
            int cur = found;      // walk back: every label on the path takes the bank it was reached through
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
        // labels without a bank of their own double up: least loaded reachable bank, then the fullest
        int myload = ml >= 0 ? 1 : 0;
        uint32_t left = gballot(mb < 0);
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
        // my next unused slot in that bank (slots of a bank are used in rising slot number)
        const int pick = mine[ends[mb] - cnt[mb]];
        if (--cnt[mb] == 0) avail &= ~(1u << mb);
        ord[gl][lane][s] = (uint8_t)pick;
        mydeg -= myload;
    }
    if (valid)
        for (int s = 0; s < K; ++s) perm[j * K + s] = ord[gl][lane][s];
}

// slots in stored order (tuning aid: what the gathers cost without a bank-aware order)
__global__ void k_identity_order(int64_t m, int k, uint8_t* __restrict__ perm) {
    const int64_t N = m * k;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < N; e += (int64_t)gridDim.x * blockDim.x)
        perm[e] = (uint8_t)(e % k);
}

}  // namespace

// Fills ctx->slot_order for the connectivity in idx (fast-path shapes only: k in {8,16,32,64}).
usl_status usl_build_slot_order(usl_ctx* c, const int32_t* idx) {
    const size_t N = (size_t)c->m * c->k;
    if (!c->slot_order) {
        size_t cap = 0;
        USL_TRY(usl_reserve(c, (void**)&c->slot_order, &cap, N));
    }
    const int shift = c->storage == USL_F32 ? 0 : 1;  // two bfloat16 columns share a bank word
    int rounds = 3;
    if (const char* e = getenv("USL_TUNE_ROUNDS")) rounds = atoi(e);   // 0 = slots in stored order
    const int64_t groups = (c->m + 31) / 32;
    const unsigned grid = (unsigned)((groups + SCHED_GROUPS - 1) / SCHED_GROUPS);
    if (rounds <= 0) {
        hipLaunchKernelGGL(k_identity_order, dim3(c->num_cu * 4), dim3(256), 0, c->stream, c->m, c->k, c->slot_order);
    } else {
#define USL_SCHED(K) \
    hipLaunchKernelGGL((k_schedule<K>), dim3(grid), dim3(SCHED_GROUPS * 32), 0, c->stream, idx, c->m, shift, rounds, \
                       c->slot_order)
        switch (c->k) {
            case 8: USL_SCHED(8); break;
            case 16: USL_SCHED(16); break;
            case 32: USL_SCHED(32); break;
            case 64: USL_SCHED(64); break;
            default: USL_FAIL(c, USL_EUNSUPPORTED, "no slot order for k=%d", c->k);
        }
#undef USL_SCHED
    }
    USL_TRY(usl_check_launch(c, "slot order"));
    c->slot_order_for = idx;
    return USL_OK;
}
