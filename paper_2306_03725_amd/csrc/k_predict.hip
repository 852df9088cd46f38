// Prediction (Section 2): the kk highest-scoring labels of every instance, and the hit counts that
// precision-at-k is made of.
//
// A (score, label) pair is packed into one 64-bit key whose unsigned order is the ranking: the upper
// word is the score's bit pattern made monotone (negative values complemented, the sign bit set on the
// rest; -0 folded onto +0 first), the lower word is ~label, so equal scores rank the smaller label
// higher and no two keys of a row are equal.  Key 0 never occurs for a real pair and means "nothing".
#include "usl_internal.h"

namespace {

constexpr int TK_NT = 256;             // lanes per workgroup
constexpr int TK_EPT = 64;             // scores a lane holds in registers
constexpr int TK_SEG = TK_NT * TK_EPT; // labels per workgroup
constexpr int TK_MAX = 32;             // largest kk

__device__ __forceinline__ uint64_t score_key(float z, uint32_t label) {
    uint32_t u = __float_as_uint(z);
    if (u == 0x80000000u) u = 0u;
    u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
    return ((uint64_t)u << 32) | (uint64_t)(uint32_t)~label;
}

// Largest v of the workgroup, returned to every lane.  Two barriers: red may be reused right away.
__device__ __forceinline__ uint64_t block_max(uint64_t v, uint64_t* red) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const uint64_t t = __shfl_xor((unsigned long long)v, o);
        v = t > v ? t : v;
    }
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    uint64_t r = red[0];
#pragma unroll
    for (int w = 1; w < TK_NT / 64; ++w) r = red[w] > r ? red[w] : r;
    return r;
}

// The kk best keys of one segment of TK_SEG labels of one row, best first, into cand[row][segment][kk]
// (0 where the segment has fewer than kk labels).
//   1. every lane loads its 64 scores (all loads in flight at once) and finds its own best key;
//   2. tau = the kk-th best of the 256 lane maxima: at least kk keys of the segment are >= tau, and
//      every key >= tau belongs to one of the kk lanes whose maximum is >= tau, so at most kk*64 keys pass;
//   3. those keys are collected in LDS and the best kk are peeled off one by one ("largest key below the
//      previous winner": keys are distinct, so nothing has to be removed).
// VEC: rows are 16-byte aligned and m % 4 == 0, so a lane reads 16 groups of 4 consecutive labels.
template <bool VEC>
__global__ void __launch_bounds__(TK_NT)
k_topk_segments(const float* __restrict__ out, int64_t m, int kk, int nseg, uint64_t* __restrict__ cand) {
    __shared__ uint64_t red[TK_NT / 64];
    __shared__ uint64_t list[TK_MAX * TK_EPT];
    __shared__ uint32_t count;
    const int64_t seg0 = (int64_t)blockIdx.x * TK_SEG;
    const float* row = out + (int64_t)blockIdx.y * m + seg0;
    const int lim = (int)min((int64_t)TK_SEG, m - seg0);   // labels of this segment that exist
    const int tid = (int)threadIdx.x;
    // label of register e of this lane, counted from the segment's first (32-bit arithmetic throughout)
    auto local_of = [&](int e) -> int {
        return VEC ? ((e >> 2) * TK_NT + tid) * 4 + (e & 3) : e * TK_NT + tid;
    };
    float v[TK_EPT];
    if (VEC) {
#pragma unroll
        for (int e = 0; e < TK_EPT; e += 4) {
            const int j = local_of(e);
            const float4 q = j < lim ? *reinterpret_cast<const float4*>(row + j) : make_float4(0.f, 0.f, 0.f, 0.f);
            v[e] = q.x; v[e + 1] = q.y; v[e + 2] = q.z; v[e + 3] = q.w;
        }
    } else {
#pragma unroll
        for (int e = 0; e < TK_EPT; ++e) {
            const int j = local_of(e);
            v[e] = j < lim ? row[j] : 0.f;
        }
    }
    // the lane's best score; labels grow with e, so the first of equal scores is the smaller label
    float top = 0.f;
    int top_j = -1;
#pragma unroll
    for (int e = 0; e < TK_EPT; ++e) {
        const int j = local_of(e);
        const bool better = j < lim && (top_j < 0 || v[e] > top);
        top = better ? v[e] : top;
        top_j = better ? j : top_j;
    }
    const uint64_t mine = top_j >= 0 ? score_key(top, (uint32_t)(seg0 + top_j)) : 0ull;
    uint64_t tau = ~0ull;
    for (int r = 0; r < kk && tau != 0; ++r) tau = block_max(mine < tau ? mine : 0ull, red);
    if (threadIdx.x == 0) count = 0;
    __syncthreads();
    // keys are built only for scores that reach tau's score (a cheap float test first)
    const uint32_t tu = (uint32_t)(tau >> 32);
    const float tau_score = tau == 0 ? -INFINITY : __uint_as_float((tu & 0x80000000u) ? (tu & 0x7FFFFFFFu) : ~tu);
#pragma unroll
    for (int e = 0; e < TK_EPT; ++e) {
        const int j = local_of(e);
        if (j < lim && v[e] >= tau_score) {
            const uint64_t key = score_key(v[e], (uint32_t)(seg0 + j));
            if (key >= tau) list[atomicAdd(&count, 1u)] = key;
        }
    }
    __syncthreads();
    const uint32_t n = count;
    uint64_t* dst = cand + ((size_t)blockIdx.y * nseg + blockIdx.x) * kk;
    uint64_t prev = ~0ull;
    for (int r = 0; r < kk; ++r) {
        uint64_t best = 0;
        for (uint32_t q = threadIdx.x; q < n; q += TK_NT) {
            const uint64_t key = list[q];
            if (key < prev && key > best) best = key;
        }
        prev = block_max(best, red);
        if (threadIdx.x == 0) dst[r] = prev;
    }
}

// One workgroup per row: the best kk of the row's nseg*kk candidate keys, unpacked.  The score is read
// back from out so that it keeps its own bits (a -0 stays -0).
__global__ void __launch_bounds__(TK_NT)
k_topk_merge(const uint64_t* __restrict__ cand, int n, int kk, const float* __restrict__ out, int64_t m,
             int32_t* __restrict__ top_lab, float* __restrict__ top_val) {
    __shared__ uint64_t red[TK_NT / 64];
    const uint64_t* c = cand + (size_t)blockIdx.x * n;
    uint64_t prev = ~0ull;
    for (int r = 0; r < kk; ++r) {
        uint64_t best = 0;
        for (int q = threadIdx.x; q < n; q += TK_NT) {
            const uint64_t key = c[q];
            if (key < prev && key > best) best = key;
        }
        prev = block_max(best, red);
        if (threadIdx.x == 0) {
            const uint32_t label = ~(uint32_t)prev;
            top_lab[(size_t)blockIdx.x * kk + r] = (int32_t)label;
            top_val[(size_t)blockIdx.x * kk + r] = out[(int64_t)blockIdx.x * m + label];
        }
    }
}

__global__ void k_zero_hits(unsigned long long* hits, int kk) {
    if ((int)threadIdx.x < kk) hits[threadIdx.x] = 0ull;
}

// hits[r] += 1 for every instance whose rank-r prediction is one of its targets
__global__ void __launch_bounds__(256)
k_precision_hits(const int32_t* __restrict__ top_lab, const int64_t* __restrict__ tgt_off,
                 const int32_t* __restrict__ tgt_lab, int b, int kk, unsigned long long* __restrict__ hits) {
    const int q = blockIdx.x * 256 + threadIdx.x;
    if (q >= b * kk) return;
    const int i = q / kk, r = q % kk;
    const int32_t label = top_lab[q];
    bool hit = false;
    for (int64_t p = tgt_off[i]; p < tgt_off[i + 1]; ++p) hit |= tgt_lab[p] == label;
    if (hit) atomicAdd(&hits[r], 1ull);
}

}  // namespace

int usl_topk_max(void) { return TK_MAX; }

usl_status usl_launch_topk(usl_ctx* c, const float* out, int32_t b, int32_t kk, int32_t* top_lab,
                           float* top_val) {
    const int nseg = (int)((c->m + TK_SEG - 1) / TK_SEG);
    // sized once for the largest batch and the largest kk, so that no later call has to grow it (growing waits for the stream)
    USL_TRY(usl_reserve(c, (void**)&c->topk_cand, &c->topk_cand_cap, (size_t)c->max_b * nseg * TK_MAX * 8));
    if (c->m % 4 == 0 && (uintptr_t)out % 16 == 0)
        hipLaunchKernelGGL(k_topk_segments<true>, dim3((unsigned)nseg, (unsigned)b), dim3(TK_NT), 0, c->stream, out,
                           c->m, (int)kk, nseg, c->topk_cand);
    else
        hipLaunchKernelGGL(k_topk_segments<false>, dim3((unsigned)nseg, (unsigned)b), dim3(TK_NT), 0, c->stream, out,
                           c->m, (int)kk, nseg, c->topk_cand);
    hipLaunchKernelGGL(k_topk_merge, dim3((unsigned)b), dim3(TK_NT), 0, c->stream, c->topk_cand, nseg * kk,
                       (int)kk, out, c->m, top_lab, top_val);
    return usl_check_launch(c, "topk");
}

usl_status usl_launch_precision_hits(usl_ctx* c, const int32_t* top_lab, const int64_t* tgt_off,
                                     const int32_t* tgt_lab, int32_t b, int32_t kk, int64_t* hits) {
    hipLaunchKernelGGL(k_zero_hits, dim3(1), dim3(64), 0, c->stream, (unsigned long long*)hits, (int)kk);
    hipLaunchKernelGGL(k_precision_hits, dim3((unsigned)((b * kk + 255) / 256)), dim3(256), 0, c->stream,
                       top_lab, tgt_off, tgt_lab, (int)b, (int)kk, (unsigned long long*)hits);
    return usl_check_launch(c, "precision_hits");
}
