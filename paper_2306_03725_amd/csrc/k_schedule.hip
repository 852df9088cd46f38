// Bank-aware slot order for the LDS gathers of forward / backward-weight.
//
// In those kernels the 32 lanes of a half-wavefront own 32 consecutive labels and, at step s, all
// read slot order[s] of their own label from the activation row in LDS.  With the slots in their
// natural order the 32 addresses are random and collide in the 32 LDS banks (a step then costs as
// many cycles as the fullest bank, 3.5 on average).  The sum over a label's slots may be taken in
// any order, so each label gets a private permutation of its slots, chosen so that the lanes of a
// half-wavefront hit different banks at the same step as far as possible.
//
// The permutation is found by a local search that every group of 32 labels runs on its own: cnt[s][b]
// counts the lanes that read bank b at step s; a lane looks for its most crowded step and for the
// partner step whose exchange lowers the sum of squared counts most.  Half of the lanes move per
// sweep (alternating parity), all reads of a sweep happen before its writes, so the result is a
// deterministic function of idx.  Any outcome is a valid permutation: it changes speed, never results.
#include "usl_internal.h"

namespace {

template <int K, int GROUPS>
__global__ void __launch_bounds__(GROUPS * 32)
k_schedule(const int32_t* __restrict__ idx, int64_t m, int shift, int sweeps,
           uint8_t* __restrict__ perm) {
    __shared__ int cnt[GROUPS][K][32];
    __shared__ uint8_t bnk[GROUPS][32][K];   // bank read at step s (current order)
    __shared__ uint8_t ord[GROUPS][32][K];   // slot read at step s
    const int gl = threadIdx.x >> 5, lane = threadIdx.x & 31;
    const int64_t j = ((int64_t)blockIdx.x * GROUPS + gl) * 32 + lane;
    const bool valid = j < m;
    for (int q = lane; q < K * 32; q += 32) (&cnt[gl][0][0])[q] = 0;
    __syncthreads();
    for (int s = 0; s < K; ++s) {
        const int b = valid ? ((idx[j * K + s] >> shift) & 31) : ((lane + s) & 31);
        bnk[gl][lane][s] = (uint8_t)b;
        ord[gl][lane][s] = (uint8_t)s;
        atomicAdd(&cnt[gl][s][b], 1);
    }
    __syncthreads();
    for (int sw = 0; sw < sweeps; ++sw) {
        int worst = -1, wc = 1;
        for (int s = 0; s < K; ++s) {
            const int c = cnt[gl][s][bnk[gl][lane][s]];
            if (c > wc) { wc = c; worst = s; }
        }
        int best = -1, b1 = 0, b2best = 0;
        if (((lane + sw) & 1) && worst >= 0) {
            b1 = bnk[gl][lane][worst];
            int bd = -2;  // accept only exchanges that lower the sum of squares
            for (int s2 = 0; s2 < K; ++s2) {
                const int b2 = bnk[gl][lane][s2];
                if (s2 == worst || b2 == b1) continue;
                const int dlt = cnt[gl][worst][b2] - wc + cnt[gl][s2][b1] - cnt[gl][s2][b2];
                if (dlt < bd) { bd = dlt; best = s2; b2best = b2; }
            }
        }
        __syncthreads();
        if (best >= 0) {
            atomicSub(&cnt[gl][worst][b1], 1); atomicAdd(&cnt[gl][worst][b2best], 1);
            atomicSub(&cnt[gl][best][b2best], 1); atomicAdd(&cnt[gl][best][b1], 1);
            bnk[gl][lane][worst] = (uint8_t)b2best; bnk[gl][lane][best] = (uint8_t)b1;
            const uint8_t o = ord[gl][lane][worst];
            ord[gl][lane][worst] = ord[gl][lane][best];
            ord[gl][lane][best] = o;
        }
        __syncthreads();
    }
    if (valid)
        for (int s = 0; s < K; ++s) perm[j * K + s] = ord[gl][lane][s];
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
    const int sweeps = 16;
    const int64_t groups = (c->m + 31) / 32;
#define USL_SCHED(K, G)                                                                          \
    hipLaunchKernelGGL((k_schedule<K, G>), dim3((unsigned)((groups + G - 1) / G)), dim3(G * 32), 0, \
                       c->stream, idx, c->m, shift, sweeps, c->slot_order)
    switch (c->k) {
        case 8: USL_SCHED(8, 8); break;
        case 16: USL_SCHED(16, 8); break;
        case 32: USL_SCHED(32, 8); break;
        case 64: USL_SCHED(64, 4); break;
        default: USL_FAIL(c, USL_EUNSUPPORTED, "no slot order for k=%d", c->k);
    }
#undef USL_SCHED
    USL_TRY(usl_check_launch(c, "slot order"));
    c->slot_order_for = idx;
    return USL_OK;
}
