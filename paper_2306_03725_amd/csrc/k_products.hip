// Forward product (Algorithm 1) and weight gradient (Algorithm 3) of the uniformly-sparse layer.
//
// Both walk the same gather: for a pair (instance i, label j) the k values x[i][idx[j][t]].
// Design for gfx950: a workgroup owns a block of labels and keeps their k indices (packed two
// per register) and k weights -- or k gradient accumulators -- in VGPRs for its whole life.
// It then walks over the instances; each activation row (or a tile of rows when d is small,
// or a slice of the row when it exceeds the LDS budget) is copied once into LDS with coalesced
// 16-byte loads, and every gather is an LDS read.  idx and W therefore leave HBM once per
// workgroup, x is re-read once per label block (it stays in L2 / Infinity Cache), and out /
// grad_W are written with coalesced stores.
#include "k_products_common.h"

using namespace usl_products;

namespace {

// Warms the L2 of this workgroup's XCD with a slice of the next activation row.  All workgroups
// walk the batch in step, so without this every row is first touched by all of them at once and
// the whole chip waits out an HBM round trip per row.  Workgroups are dealt to the 8 XCDs round
// robin; those of one XCD share the row between them, one load per 128-byte line.
// `share` = workgroups of one XCD that are resident together (the grid may hold several rounds of them):
// those, consecutive in blockIdx, split the row between them.
template <typename TS>
__device__ __forceinline__ void prefetch_row_slice(const TS* __restrict__ row, int n, int share,
                                                   int tid = (int)threadIdx.x) {
    const int lines = (int)(((size_t)n * sizeof(TS) + 127) / 128);
    const int nsl = max(1, min((int)(gridDim.x >> 3), share));
    const int sl = (int)(blockIdx.x >> 3) % nsl;
    const int per = (lines + nsl - 1) / nsl;
    const int line = sl * per + tid;
    if (tid < per && line < lines)
        (void)*reinterpret_cast<const volatile uint32_t*>(reinterpret_cast<const char*>(row) + (size_t)line * 128);
}

struct TileGeom {
    int rows_per_tile;  // activation rows staged together (1 when the row is sliced)
    int part_cols;      // columns per slice
    int nparts;         // slices per row
    int inst_per_group; // instances handled by one blockIdx.y
    int vec_ok;         // 16-byte copies allowed
    int flag_offset;    // byte offset in LDS of the per-wavefront flags of backward_weight
    int buf_stride;     // elements between the two row buffers of MODE 3 (0 = one buffer)
    int share;          // workgroups resident together on one XCD (they split the warm-up of a row)
};

// ---------------------------------------------------------------------------- forward
// MODE 0: a whole activation row fits LDS, one row per stage.
// MODE 1: the row is cut into slices of part_cols columns; gathers outside the slice are masked.
// MODE 2: small rows, rows_per_tile of them per stage (used with one label per lane).
// MODE 3: two rows fit LDS: the next row is copied in while this one is gathered (one barrier per instance).
template <int K, int LPT, int NT, typename TS, int MODE>
__global__ void __launch_bounds__(NT)
k_forward(const TS* __restrict__ x, const int32_t* __restrict__ idx, const TS* __restrict__ W,
          float* __restrict__ out, int64_t m, int d, int b, TileGeom tg,
          const uint8_t* __restrict__ perm) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    TS* lds = reinterpret_cast<TS*>(lds_raw);
    if ((MODE == 0 || MODE == 1) && sizeof(TS) == 4 && !lds_starts_at_zero(lds_raw)) return;   // see gather_row0
    // sliced float32 rows are exactly two halves of 32768 columns (the fast path stops at d = 65536)
    constexpr bool HALVES = MODE == 1 && sizeof(TS) == 4 && USL_ROW_LDS_BYTES == 131072;
    const int64_t j0 = (int64_t)blockIdx.x * (NT * LPT);
    uint32_t pk[LPT][K / 2];
    float w[LPT][K];
#pragma unroll
    for (int l = 0; l < LPT; ++l) {
        const int64_t row0 = j0 + (int64_t)l * NT;
        SlotOrder<K> so;
        so.load(perm, row0 + threadIdx.x, row0 + threadIdx.x < m);
        fetch_idx_packed<K, NT>(idx, row0, m, reinterpret_cast<uint32_t*>(lds_raw), so, pk[l]);
        fetch_w<K, NT>(W, row0, m, reinterpret_cast<uint32_t*>(lds_raw), so, w[l]);
    }
    const int64_t jme = j0 + threadIdx.x;
    // 32 words of zeros (one per bank) behind the slice buffer, for the masked gathers of MODE 1
    const uint32_t zcol = (uint32_t)tg.part_cols;   // every masked lane reads the same word: one broadcast, one bank
    if (MODE == 1) {
        __syncthreads();
        if (threadIdx.x < 32)
            reinterpret_cast<uint32_t*>(lds_raw)[(size_t)tg.part_cols * sizeof(TS) / 4 + threadIdx.x] = 0u;
    }
  // label of slot l is jme + l*NT
    const int i_begin = blockIdx.y * tg.inst_per_group;
    const int i_end = min(b, i_begin + tg.inst_per_group);
    if (MODE == 3) {
        // two bfloat16 rows fit only if the row has at most 32768 columns: a column's byte offset then fits
        // the 16 bits of a packed index, and the gathers save the scaling (they are bound by vector
        // instructions, not by LDS, on bfloat16 rows)
        constexpr bool SCALED = sizeof(TS) == 2;
        if (SCALED) {
#pragma unroll
            for (int l = 0; l < LPT; ++l)
#pragma unroll
                for (int q = 0; q < K / 2; ++q) pk[l][q] <<= 1;
        }
        // bfloat16: the weights go back to pairs (they are exact bfloat16 values), two gathered activations are
        // joined into one register, and one dot-product instruction does both multiply-adds in float32
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
        uint32_t wp[SCALED ? LPT : 1][SCALED ? K / 2 : 1];
        if (SCALED) {
#pragma unroll
            for (int l = 0; l < LPT; ++l)
#pragma unroll
                for (int q = 0; q < K / 2; ++q)
                    wp[l][q] = (__float_as_uint(w[l][2 * q]) >> 16) | (__float_as_uint(w[l][2 * q + 1]) & 0xFFFF0000u);
        }
        float prev[LPT];
        __syncthreads();   // the transposition buffer is free
        if (i_begin < i_end) stage<TS, NT>(x + (size_t)i_begin * d, lds, d, tg.vec_ok);
        __syncthreads();
#pragma unroll 1
        for (int i = i_begin; i < i_end; ++i) {
            const TS* cur = lds + (size_t)((i - i_begin) & 1) * tg.buf_stride;
            // the other buffer was last read one instance ago, before the barrier that ended it
            if (i + 1 < i_end)
                stage<TS, NT, false>(x + (size_t)(i + 1) * d, lds + (size_t)((i + 1 - i_begin) & 1) * tg.buf_stride, d,
                                     tg.vec_ok);
            if (i + 2 < i_end) prefetch_row_slice<TS>(x + (size_t)(i + 2) * d, d, tg.share);
#pragma unroll
            for (int l = 0; l < LPT; ++l) {
                if (i > i_begin && jme + (int64_t)l * NT < m)   // spread over the gathers, as in the loop below
                    out[(size_t)(i - 1) * m + jme + (int64_t)l * NT] = prev[l];
                float acc = 0.f;
                keep_packed(pk[l]);
                if (SCALED) {
                    const char* base = reinterpret_cast<const char*>(cur);
#pragma unroll
                    for (int q = 0; q < K / 2; ++q) {
                        const uint32_t lo = *reinterpret_cast<const uint16_t*>(base + (pk[l][q] & 0xFFFFu));
                        const uint32_t hi = *reinterpret_cast<const uint16_t*>(base + (pk[l][q] >> 16));
                        const uint32_t pair = lo | (hi << 16);
                        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pair),
                                                              __builtin_bit_cast(bf16x2, wp[SCALED ? l : 0][SCALED ? q : 0]), acc, false);
                        if ((q & 3) == 3) __builtin_amdgcn_sched_barrier(0);
                    }
                } else {
#pragma unroll
                    for (int t = 0; t < K; ++t) {
                        acc = fmaf(w[l][t], lds_val(cur, col_of<K>(pk[l], t)), acc);
                        if ((t & 7) == 7) __builtin_amdgcn_sched_barrier(0);
                    }
                }
                asm volatile("" : "+v"(acc));
                prev[l] = acc;
            }
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the next row has landed
            __syncthreads();
        }
        if (i_end > i_begin) {
#pragma unroll
            for (int l = 0; l < LPT; ++l)
                if (jme + (int64_t)l * NT < m) out[(size_t)(i_end - 1) * m + jme + (int64_t)l * NT] = prev[l];
        }
    } else if (MODE == 2) {
        for (int it = i_begin; it < i_end; it += tg.rows_per_tile) {
            const int rows = min(tg.rows_per_tile, i_end - it);
            __syncthreads();
            stage<TS, NT>(x + (size_t)it * d, lds, rows * d, tg.vec_ok);
            __syncthreads();
#pragma unroll 1
            for (int r = 0; r < rows; ++r) {
                const TS* row = lds + (size_t)r * d;
#pragma unroll
                for (int l = 0; l < LPT; ++l) {
                    float acc = 0.f;
                    keep_packed(pk[l]);
#pragma unroll
                    for (int t = 0; t < K; ++t)
                        acc = fmaf(w[l][t], lds_val(row, col_of<K>(pk[l], t)), acc);
                    if (jme + (int64_t)l * NT < m) out[(size_t)(it + r) * m + jme + (int64_t)l * NT] = acc;
                }
            }
        }
    } else {
        // The scores of an instance are written while the next instance's row is being gathered: a
        // store issued right before the next staging would make its vmcnt(0) wait for the store too.
        float prev[LPT];
#pragma unroll 1
        for (int i = i_begin; i < i_end; ++i) {
            float acc[LPT];
#pragma unroll
            for (int l = 0; l < LPT; ++l) acc[l] = 0.f;
            const int nparts = MODE == 1 ? tg.nparts : 1;
#pragma unroll 1
            for (int part = 0; part < nparts; ++part) {
                const int c0 = part * tg.part_cols;
                const uint32_t cols = (uint32_t)min(tg.part_cols, d - c0);
                __syncthreads();
                stage<TS, NT>(x + (size_t)i * d + c0, lds, (int)cols, tg.vec_ok);
                __syncthreads();
                if (part == nparts - 1 && i + 1 < i_end) prefetch_row_slice<TS>(x + (size_t)(i + 1) * d, d, tg.share);
                if (HALVES && part > 0) {
#pragma unroll
                    for (int l = 0; l < LPT; ++l) flip_half(pk[l]);
                }
#pragma unroll
                for (int l = 0; l < LPT; ++l) {
                    // one score of the previous instance leaves between two labels' gathers: four stores
                    // in a row would hold the wavefront at the memory pipeline before it starts to gather
                    if (part == 0 && i > i_begin && jme + (int64_t)l * NT < m)
                        out[(size_t)(i - 1) * m + jme + (int64_t)l * NT] = prev[l];
                    keep_packed(pk[l]);
#pragma unroll
                    for (int t = 0; t < K; ++t) {
                        float xv;
                        if (MODE == 0 && sizeof(TS) == 4) {
                            xv = gather_row0<K>(pk[l], t);
                        } else if (MODE == 0) {
                            xv = lds_val(lds, col_of<K>(pk[l], t));
                        } else if (HALVES) {
                            xv = gather_half<K>(pk[l], t, zcol * 4u);
                        } else {
                            // sliced rows: a slot outside the slice reads a word of zeros behind it
                            // (no branch, so the gathers stay pipelined)
                            const uint32_t c = col_of<K>(pk[l], t) - (uint32_t)c0;
                            xv = lds_val(lds, c < cols ? c : zcol);
                        }
                        acc[l] = fmaf(w[l][t], xv, acc[l]);
                        // a few gathers in flight at a time: their results would otherwise
                        // crowd out the resident indices and weights
                        if ((t & 7) == 7) {
                            if (MODE == 0 && sizeof(TS) == 4) {
                                __builtin_amdgcn_sched_group_barrier(0x002, 8, 0);
                                __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
                                __builtin_amdgcn_sched_group_barrier(0x002, 8, 0);
                            } else if (HALVES) {   // two instructions per address here
                                __builtin_amdgcn_sched_group_barrier(0x002, 16, 0);
                                __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
                                __builtin_amdgcn_sched_group_barrier(0x002, 8, 0);
                            }
                            __builtin_amdgcn_sched_barrier(0);
                        }
                    }
                    // finish the sum here; left alone the compiler sinks the multiply-adds into
                    // the guarded store and keeps every gathered value alive until then
                    asm volatile("" : "+v"(acc[l]));
                }
                if (HALVES && part > 0) {
#pragma unroll
                    for (int l = 0; l < LPT; ++l) flip_half(pk[l]);
                }
            }
#pragma unroll
            for (int l = 0; l < LPT; ++l) prev[l] = acc[l];
        }
        if (i_end > i_begin) {
#pragma unroll
            for (int l = 0; l < LPT; ++l)
                if (jme + (int64_t)l * NT < m) out[(size_t)(i_end - 1) * m + jme + (int64_t)l * NT] = prev[l];
        }
    }
}

// any k, any d: one thread per label, idx / W re-read from global memory for every instance
template <int NT, typename TS>
__global__ void __launch_bounds__(NT)
k_forward_generic(const TS* __restrict__ x, const int32_t* __restrict__ idx,
                  const TS* __restrict__ W, float* __restrict__ out, int64_t m, int d, int k, int b,
                  TileGeom tg) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    TS* lds = reinterpret_cast<TS*>(lds_raw);
    const int64_t j = (int64_t)blockIdx.x * NT + threadIdx.x;
    const int64_t jj = j < m ? j : m - 1;
    const int i_begin = blockIdx.y * tg.inst_per_group;
    const int i_end = min(b, i_begin + tg.inst_per_group);
    for (int i = i_begin; i < i_end; ++i) {
        float acc = 0.f;
        for (int part = 0; part < tg.nparts; ++part) {
            const int c0 = part * tg.part_cols;
            const uint32_t cols = (uint32_t)min(tg.part_cols, d - c0);
            __syncthreads();
            stage<TS, NT>(x + (size_t)i * d + c0, lds, (int)cols, tg.vec_ok);
            __syncthreads();
            for (int t = 0; t < k; ++t) {
                const uint32_t c = (uint32_t)idx[jj * k + t] - (uint32_t)c0;
                if (c < cols) acc = fmaf(usl_load_f32<TS>(W, (size_t)(jj * k + t)), lds_val(lds, c), acc);
            }
        }
        if (j < m) out[(size_t)i * m + j] = acc;
    }
}

// OR of four consecutive flag words (16-byte aligned) with one LDS read.
__device__ __forceinline__ uint32_t or4(const uint32_t* p) {
    const uint4 v = *reinterpret_cast<const uint4*>(p);
    return (v.x | v.y) | (v.z | v.w);
}

// ---------------------------------------------------------------------------- weight gradient
// SKIP = false leaves the zero-skipping out (callers that know the gradient is dense, e.g. after BCE).
template <int K, int LPT, int NT, typename TS, int MODE, bool ATOMIC, bool SKIP>
__global__ void __launch_bounds__(NT)
k_backward_weight(const float* __restrict__ g, const TS* __restrict__ x,
                  const int32_t* __restrict__ idx, float* __restrict__ grad_W, int64_t m, int d,
                  int b, TileGeom tg, const uint8_t* __restrict__ perm, int64_t part_stride,
                  const uint32_t* __restrict__ gate) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    TS* lds = reinterpret_cast<TS*>(lds_raw);
    if (gate && *gate == 0) return;   // the gradient is almost all zeros: the kernels over its nonzeros do the work
    if ((MODE == 0 || MODE == 1) && sizeof(TS) == 4 && !lds_starts_at_zero(lds_raw)) return;   // see gather_row0
    // sliced float32 rows are exactly two halves of 32768 columns (the fast path stops at d = 65536)
    constexpr bool HALVES = MODE == 1 && sizeof(TS) == 4 && USL_ROW_LDS_BYTES == 131072;
    const int64_t j0 = (int64_t)blockIdx.x * (NT * LPT);
    uint32_t pk[LPT][K / 2];
    float acc[LPT][K];
#pragma unroll
    for (int l = 0; l < LPT; ++l) {
        const int64_t row0 = j0 + (int64_t)l * NT;
        SlotOrder<K> so;
        so.load(perm, row0 + threadIdx.x, row0 + threadIdx.x < m);
        fetch_idx_packed<K, NT>(idx, row0, m, reinterpret_cast<uint32_t*>(lds_raw), so, pk[l]);
#pragma unroll
        for (int t = 0; t < K; ++t) acc[l][t] = 0.f;
    }
    const int64_t jme = j0 + threadIdx.x;
    // 32 words of zeros (one per bank) behind the slice buffer, for the masked gathers of MODE 1
    const uint32_t zcol = (uint32_t)tg.part_cols;   // every masked lane reads the same word: one broadcast, one bank
    if (MODE == 1) {
        __syncthreads();
        if (threadIdx.x < 32)
            reinterpret_cast<uint32_t*>(lds_raw)[(size_t)tg.part_cols * sizeof(TS) / 4 + threadIdx.x] = 0u;
    }

    const int i_begin = blockIdx.y * tg.inst_per_group;
    const int i_end = min(b, i_begin + tg.inst_per_group);
    if (MODE == 3) {
        constexpr bool SCALED = sizeof(TS) == 2;   // byte offsets in the packed indices, as in the forward kernel
        if (SCALED) {
#pragma unroll
            for (int l = 0; l < LPT; ++l)
#pragma unroll
                for (int q = 0; q < K / 2; ++q) pk[l][q] <<= 1;
        }
        // as in the single-buffer loop below, an instance (a label group) whose gradients are all zero skips
        // its gathers; the row copy is not skipped, it runs one instance ahead
        uint32_t* live_flags = reinterpret_cast<uint32_t*>(lds_raw + tg.flag_offset);
        float gnext[LPT];
        bool any_next = false;
#pragma unroll
        for (int l = 0; l < LPT; ++l) {
            const int64_t j = jme + (int64_t)l * NT;
            gnext[l] = (j < m && i_begin < i_end) ? g[(size_t)i_begin * m + j] : 0.f;
            any_next = any_next || gnext[l] != 0.f;
        }
        __syncthreads();   // the transposition buffer is free
        if (i_begin < i_end) stage<TS, NT>(x + (size_t)i_begin * d, lds, d, tg.vec_ok);
        {
            const bool wave_any = __any(any_next);
            if ((threadIdx.x & 63) == 0) live_flags[threadIdx.x >> 6] = wave_any ? 1u : 0u;
        }
        __syncthreads();
#pragma unroll 1
        for (int i = i_begin; i < i_end; ++i) {
            const TS* cur = lds + (size_t)((i - i_begin) & 1) * tg.buf_stride;
            if (i + 1 < i_end)
                stage<TS, NT, false>(x + (size_t)(i + 1) * d, lds + (size_t)((i + 1 - i_begin) & 1) * tg.buf_stride, d,
                                     tg.vec_ok);
            float gv[LPT];
#pragma unroll
            for (int l = 0; l < LPT; ++l) gv[l] = gnext[l];
#pragma unroll
            for (int l = 0; l < LPT; ++l) {
                const int64_t j = jme + (int64_t)l * NT;
                gnext[l] = (j < m && i + 1 < i_end) ? g[(size_t)(i + 1) * m + j] : 0.f;
            }
            if (i + 2 < i_end) prefetch_row_slice<TS>(x + (size_t)(i + 2) * d, d, tg.share);
            const uint32_t* wf = live_flags + ((i - i_begin) & 1) * (NT / 64);
            uint32_t live = 0;
#pragma unroll
            for (int q = 0; q < NT / 256; ++q) live |= or4(wf + 4 * q);
            if (live) {
#pragma unroll
                for (int l = 0; l < LPT; ++l) {
                    if (!__any(gv[l] != 0.f)) continue;
                    keep_packed(pk[l]);
#pragma unroll
                    for (int t = 0; t < K; ++t) {
                        acc[l][t] = fmaf(gv[l], SCALED ? lds_at(cur, col_of<K>(pk[l], t)) : lds_val(cur, col_of<K>(pk[l], t)), acc[l][t]);
                        if ((t & 7) == 7) __builtin_amdgcn_sched_barrier(0);
                    }
                }
            }
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the next row and the next gradients have landed
            {
                bool any = false;
#pragma unroll
                for (int l = 0; l < LPT; ++l) any = any || gnext[l] != 0.f;
                const bool wave_any = __any(any);
                if ((threadIdx.x & 63) == 0)
                    live_flags[((i + 1 - i_begin) & 1) * (NT / 64) + (threadIdx.x >> 6)] = wave_any ? 1u : 0u;
            }
            __syncthreads();
        }
    } else if (MODE == 2) {
        for (int it = i_begin; it < i_end; it += tg.rows_per_tile) {
            const int rows = min(tg.rows_per_tile, i_end - it);
            __syncthreads();
            stage<TS, NT>(x + (size_t)it * d, lds, rows * d, tg.vec_ok);
            __syncthreads();
#pragma unroll 1
            for (int r = 0; r < rows; ++r) {
                const TS* row = lds + (size_t)r * d;
#pragma unroll
                for (int l = 0; l < LPT; ++l) {
                    const int64_t j = jme + (int64_t)l * NT;
                    const float gv = j < m ? g[(size_t)(it + r) * m + j] : 0.f;
                    if (!__any(gv != 0.f)) continue;
                    keep_packed(pk[l]);
#pragma unroll
                    for (int t = 0; t < K; ++t)
                        acc[l][t] = fmaf(gv, lds_val(row, col_of<K>(pk[l], t)), acc[l][t]);
                }
            }
        }
    } else {
        // Zero entries of g contribute nothing (Algorithm 3 skips them): a label whose gradient is
        // zero in all 64 lanes of the wavefront skips its gathers, and an instance whose gradient is
        // zero for every label of the workgroup is not even staged.  The gradient of the next
        // instance is fetched one instance ahead so that this test costs no memory round trip.
        uint32_t* live_flags = reinterpret_cast<uint32_t*>(lds_raw + tg.flag_offset);
        float gnext[LPT];
#pragma unroll
        for (int l = 0; l < LPT; ++l) {
            const int64_t j = jme + (int64_t)l * NT;
            gnext[l] = (j < m && i_begin < i_end) ? g[(size_t)i_begin * m + j] : 0.f;
        }
        // with a short row the flag words lie inside the buffer the indices were transposed through:
        // every wavefront must have picked up its indices before the first flag is written
        __syncthreads();
        // labels of this workgroup that exist; the gradient loads address them with 32-bit offsets
        const int nlab = (int)min((int64_t)NT * LPT, m - j0);
#pragma unroll 1
        for (int i = i_begin; i < i_end; ++i) {
            // the lane number is taken afresh every instance: addresses derived from it (row copy,
            // warm-up, gradient loads) are then rebuilt with a few instructions each time round
            // instead of living in a dozen registers across the gathers, which need them more
            int tid = (int)threadIdx.x;
            asm volatile("" : "+v"(tid));
            float gv[LPT];
            bool any = false;
#pragma unroll
            for (int l = 0; l < LPT; ++l) { gv[l] = gnext[l]; any = any || gv[l] != 0.f; }
            // workgroup-wide OR through one word per wavefront behind the row buffer (two sets,
            // alternating, so the next instance's writers cannot overtake this instance's readers);
            // the barrier is the one that frees the row buffer anyway
            uint32_t live = 1;
            if (SKIP) {
                uint32_t* wf = live_flags + (i & 1) * (NT / 64);
                const bool wave_any = __any(any);
                if ((tid & 63) == 0) wf[tid >> 6] = wave_any ? 1u : 0u;
                __syncthreads();
                live = 0;
#pragma unroll
                for (int q = 0; q < NT / 256; ++q) live |= or4(wf + 4 * q);
            } else {
                __syncthreads();
            }
            // The next instance's gradients are requested after the row copy, not before it: they come
            // from HBM, and the copy's wait for its own loads would wait for them as well.
            auto load_next = [&]() {
                const float* gr = g + (size_t)(i + 1) * m + j0;
#pragma unroll
                for (int l = 0; l < LPT; ++l) {
                    const int jl = tid + l * NT;
                    gnext[l] = (jl < nlab && i + 1 < i_end) ? gr[jl] : 0.f;
                }
            };
            const int nparts = MODE == 1 ? tg.nparts : 1;
#pragma unroll 1
            for (int part = 0; part < nparts; ++part) {
                const int c0 = part * tg.part_cols;
                const uint32_t cols = (uint32_t)min(tg.part_cols, d - c0);
                if (live) {   // the same for every lane of the workgroup
                    if (part > 0) __syncthreads();
                    stage<TS, NT>(x + (size_t)i * d + c0, lds, (int)cols, tg.vec_ok, tid);
                    __syncthreads();
                    if (part == nparts - 1 && i + 1 < i_end) prefetch_row_slice<TS>(x + (size_t)(i + 1) * d, d, tg.share, tid);
                }
                if (part == 0) load_next();
                if (!live) break;
                if (HALVES && part > 0) {
#pragma unroll
                    for (int l = 0; l < LPT; ++l) flip_half(pk[l]);
                }
#pragma unroll
                for (int l = 0; l < LPT; ++l) {
                    if (SKIP && !__any(gv[l] != 0.f)) continue;
                    keep_packed(pk[l]);
#pragma unroll
                    for (int t = 0; t < K; ++t) {
                        float xv;
                        if (MODE == 0 && sizeof(TS) == 4) {
                            xv = gather_row0<K>(pk[l], t);
                        } else if (MODE == 0) {
                            xv = lds_val(lds, col_of<K>(pk[l], t));
                        } else if (HALVES) {
                            xv = gather_half<K>(pk[l], t, zcol * 4u);
                        } else {
                            const uint32_t c = col_of<K>(pk[l], t) - (uint32_t)c0;
                            xv = lds_val(lds, c < cols ? c : zcol);
                        }
                        acc[l][t] = fmaf(gv[l], xv, acc[l][t]);
                        if ((t & 7) == 7) {
                            if (MODE == 0 && sizeof(TS) == 4) {   // 8 addresses, 8 reads, 8 multiply-adds
                                __builtin_amdgcn_sched_group_barrier(0x002, 8, 0);
                                __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
                                __builtin_amdgcn_sched_group_barrier(0x002, 8, 0);
                            } else if (HALVES) {
                                __builtin_amdgcn_sched_group_barrier(0x002, 16, 0);
                                __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
                                __builtin_amdgcn_sched_group_barrier(0x002, 8, 0);
                            }
                            __builtin_amdgcn_sched_barrier(0);
                        }
                    }
                }
                if (HALVES && part > 0) {
#pragma unroll
                    for (int l = 0; l < LPT; ++l) flip_half(pk[l]);
                }
            }
        }
    }
    uint32_t* tr = reinterpret_cast<uint32_t*>(lds_raw);
#pragma unroll
    for (int l = 0; l < LPT; ++l) {
        const int64_t row0 = j0 + (int64_t)l * NT;
        SlotOrder<K> so;
        so.load(perm, row0 + threadIdx.x, row0 + threadIdx.x < m);
        __syncthreads();
#pragma unroll
        for (int t = 0; t < K; ++t) tr[threadIdx.x * (K + 1) + so.at(t)] = __float_as_uint(acc[l][t]);
        __syncthreads();
        // batch split over blockIdx.y: every group writes its own partial array (part_stride
        // elements apart, summed afterwards in a fixed order), or adds atomically into the one array
        if (ATOMIC && part_stride == 0)
            lds_to_rows<K, NT, true>(tr, grad_W, j0 + (int64_t)l * NT, m);
        else
            lds_to_rows<K, NT, false>(tr, grad_W + (size_t)blockIdx.y * (size_t)part_stride, j0 + (int64_t)l * NT, m);
    }
}

// any k, any d: one thread per connection
template <int NT, typename TS, bool ATOMIC>
__global__ void __launch_bounds__(NT)
k_backward_weight_generic(const float* __restrict__ g, const TS* __restrict__ x,
                          const int32_t* __restrict__ idx, float* __restrict__ grad_W, int64_t m,
                          int d, int k, int b, TileGeom tg) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    TS* lds = reinterpret_cast<TS*>(lds_raw);
    const int64_t N = m * k;
    const int64_t e = (int64_t)blockIdx.x * NT + threadIdx.x;
    const int64_t ee = e < N ? e : N - 1;
    const int64_t j = ee / k;
    const uint32_t col = (uint32_t)idx[ee];
    const int i_begin = blockIdx.y * tg.inst_per_group;
    const int i_end = min(b, i_begin + tg.inst_per_group);
    float acc = 0.f;
    for (int i = i_begin; i < i_end; ++i) {
        const float gv = g[(size_t)i * m + j];
        for (int part = 0; part < tg.nparts; ++part) {
            const int c0 = part * tg.part_cols;
            const uint32_t cols = (uint32_t)min(tg.part_cols, d - c0);
            __syncthreads();
            stage<TS, NT>(x + (size_t)i * d + c0, lds, (int)cols, tg.vec_ok);
            __syncthreads();
            const uint32_t c = col - (uint32_t)c0;
            if (c < cols) acc = fmaf(gv, lds_val(lds, c), acc);
        }
    }
    if (e < N) {
        if (ATOMIC) unsafeAtomicAdd(grad_W + e, acc);
        else grad_W[e] = acc;
    }
}

// out[e] = part[0][e] + part[1][e] + ... (n % 4 == 0, 16-byte aligned): the partial weight gradients of
// a split batch, added in a fixed order.
__global__ void k_sum_parts(const float* __restrict__ part, int groups, size_t n, float* __restrict__ out) {
    size_t v = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t step = (size_t)gridDim.x * blockDim.x, nv = n / 4;
    for (; v < nv; v += step) {
        float4 a = reinterpret_cast<const float4*>(part)[v];
        for (int q = 1; q < groups; ++q) {
            const float4 t = reinterpret_cast<const float4*>(part + (size_t)q * n)[v];
            a.x += t.x; a.y += t.y; a.z += t.z; a.w += t.w;
        }
        reinterpret_cast<float4*>(out)[v] = a;
    }
}

__global__ void k_fill_zero(float* __restrict__ p, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t s = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += s) p[i] = 0.f;
}

// Picks how rows are tiled / sliced through LDS and how instances are spread over blockIdx.y.
TileGeom plan(const usl_ctx* c, int esize, int b, int64_t nblk, const void* x, size_t* lds_bytes,
              int* groups, bool multi_row = false) {
    TileGeom tg;
    const size_t row_bytes = (size_t)c->d * esize;
    tg.vec_ok = (row_bytes % 16 == 0) && (((uintptr_t)x) % 16 == 0);
    if (row_bytes <= (size_t)USL_ROW_LDS_BYTES) {
        tg.nparts = 1;
        tg.part_cols = c->d;
        // small rows: several per tile, but keep the tile at 32 KiB so more than one workgroup
        // fits a compute unit
        int rpt = multi_row ? (int)((size_t)32768 / row_bytes) : 1;
        tg.rows_per_tile = rpt < 1 ? 1 : rpt;
    } else {
        tg.part_cols = USL_ROW_LDS_BYTES / esize;
        tg.nparts = (c->d + tg.part_cols - 1) / tg.part_cols;
        tg.rows_per_tile = 1;
    }
    // enough workgroups to fill the chip: split the batch when there are few label blocks
    const int64_t want = (int64_t)c->num_cu * (row_bytes > 40960 ? 1 : 2);
    int G = 1;
    if (nblk * 4 < want * 3) {
        G = (int)((want + nblk - 1) / nblk);
        if (G > b) G = b;
    }
    tg.inst_per_group = (b + G - 1) / G;
    if (tg.rows_per_tile > tg.inst_per_group) tg.rows_per_tile = tg.inst_per_group;
    G = (b + tg.inst_per_group - 1) / tg.inst_per_group;
    *groups = G;
    *lds_bytes = tg.nparts == 1 ? (size_t)tg.rows_per_tile * row_bytes
                                : (size_t)tg.part_cols * esize + 128;   // + the zero words
    *lds_bytes = (*lds_bytes + 15) & ~(size_t)15;
    tg.buf_stride = 0;
    tg.share = 1;
    // bfloat16 rows in two buffers are gathered through byte offsets held in 16 bits: at most 32768 columns
    const bool offsets_fit = esize == 4 || c->d <= 32768;
    if (!multi_row && tg.nparts == 1 && offsets_fit && 2 * *lds_bytes + 256 <= (size_t)USL_ROW_LDS_BYTES + 8192) {
        tg.buf_stride = (int)(*lds_bytes / esize);   // a second row buffer: copy and gathers overlap
        *lds_bytes *= 2;
    }
    tg.flag_offset = (int)*lds_bytes;
    *lds_bytes += 256;                                                   // + per-wavefront flags
    return tg;
}

inline size_t max_sz(size_t a, size_t b) { return a > b ? a : b; }

// Workgroups of nt lanes and lds bytes that one XCD (an eighth of the compute units) holds at a time:
// per compute unit 160 KB of LDS and 2048 lanes.
inline int resident_per_xcd(const usl_ctx* c, size_t lds, int nt) {
    size_t per_cu = (size_t)(160 * 1024) / (lds ? lds : 1);
    if (per_cu > (size_t)(2048 / nt)) per_cu = (size_t)(2048 / nt);
    if (per_cu < 1) per_cu = 1;
    const int cus = c->num_cu / 8 > 0 ? c->num_cu / 8 : 1;
    return (int)per_cu * cus;
}

template <typename KERNEL>
usl_status allow_lds(usl_ctx* c, KERNEL kern, size_t bytes) {
    if (bytes > 65536)
        USL_HIP(c, hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
    return USL_OK;
}

// The float32 whole-row and half-row gathers use the column's byte offset as the LDS address: the
// kernel's dynamic LDS must start at address 0, which holds exactly when the kernel has no static LDS.
// That is a property of the compiled kernel, so it is checked here, once per kernel, before the launch:
// a kernel that lost it is refused with an error instead of leaving its output unwritten.
template <typename KERNEL>
usl_status require_lds_at_zero(usl_ctx* c, KERNEL kern, const char* what) {
    hipFuncAttributes fa;
    USL_HIP(c, hipFuncGetAttributes(&fa, reinterpret_cast<const void*>(kern)));
    if (fa.sharedSizeBytes != 0)
        USL_FAIL(c, USL_EUNSUPPORTED, "%s: the kernel has %zu bytes of static LDS, its row buffer does not start at LDS address 0",
                 what, (size_t)fa.sharedSizeBytes);
    return USL_OK;
}

template <int K, int LPT, int NT, typename TS>
usl_status run_forward(usl_ctx* c, const void* x, const int32_t* idx, const void* W, float* out,
                       int b) {
    const int64_t nblk = (c->m + (int64_t)NT * LPT - 1) / ((int64_t)NT * LPT);
    size_t lds;
    int G;
    TileGeom tg = plan(c, (int)sizeof(TS), b, nblk, x, &lds, &G, LPT == 1);
    lds = max_sz(lds, (size_t)NT * (K + 1) * 4);  // row tile, or the idx / W transposition buffer
    tg.share = resident_per_xcd(c, lds, NT);
    if (c->slot_order_for != idx) USL_TRY(usl_build_slot_order(c, idx));
    const uint8_t* perm = c->slot_order;
    dim3 grid((unsigned)nblk, (unsigned)G);
#define USL_FW(MODE)                                                                        \
    do {                                                                                    \
        USL_TRY(allow_lds(c, k_forward<K, LPT, NT, TS, MODE>, lds));                        \
        if (((MODE) == 0 || (MODE) == 1) && sizeof(TS) == 4) {                              \
            static bool checked = false;                                                    \
            if (!checked) USL_TRY(require_lds_at_zero(c, k_forward<K, LPT, NT, TS, MODE>, "forward")); \
            checked = true;                                                                 \
        }                                                                                   \
        hipLaunchKernelGGL((k_forward<K, LPT, NT, TS, MODE>), grid, dim3(NT), lds, c->stream, \
                           (const TS*)x, idx, (const TS*)W, out, c->m, c->d, b, tg, perm);  \
    } while (0)
    if (tg.nparts > 1) USL_FW(1);
    else if (LPT == 1 && tg.rows_per_tile > 1) USL_FW(LPT == 1 ? 2 : 0);
    else if (tg.buf_stride) USL_FW(LPT == 1 ? 0 : 3);
    else USL_FW(0);
#undef USL_FW
    return usl_check_launch(c, "forward");
}

template <typename TS>
usl_status run_forward_generic(usl_ctx* c, const void* x, const int32_t* idx, const void* W,
                               float* out, int b) {
    constexpr int NT = 256;
    const int64_t nblk = (c->m + NT - 1) / NT;
    size_t lds;
    int G;
    TileGeom tg = plan(c, (int)sizeof(TS), b, nblk, x, &lds, &G);
    if (tg.nparts == 1) { lds = (size_t)c->d * sizeof(TS); tg.rows_per_tile = 1; }
    USL_TRY(allow_lds(c, k_forward_generic<NT, TS>, lds));
    hipLaunchKernelGGL((k_forward_generic<NT, TS>), dim3((unsigned)nblk, (unsigned)G), dim3(NT), lds,
                       c->stream, (const TS*)x, idx, (const TS*)W, out, c->m, c->d, c->k, b, tg);
    return usl_check_launch(c, "forward (generic)");
}

template <int K, int LPT, int NT, typename TS>
usl_status run_backward_weight(usl_ctx* c, const float* g, const void* x, const int32_t* idx,
                               float* grad_W, int b, bool dense) {
    const int64_t nblk = (c->m + (int64_t)NT * LPT - 1) / ((int64_t)NT * LPT);
    size_t lds;
    int G;
    TileGeom tg = plan(c, (int)sizeof(TS), b, nblk, x, &lds, &G, LPT == 1);
    lds = max_sz(lds, (size_t)NT * (K + 1) * 4);
    tg.share = resident_per_xcd(c, lds, NT);
    if (c->slot_order_for != idx) USL_TRY(usl_build_slot_order(c, idx));
    const uint8_t* perm = c->slot_order;
    dim3 grid((unsigned)nblk, (unsigned)G);
    // a split batch leaves G partial gradients: in scratch, summed afterwards in a fixed order (no
    // atomics, reproducible), unless that scratch would be out of proportion
    const size_t N = (size_t)c->m * c->k;
    int64_t part_stride = 0;
    float* dst = grad_W;
    // one group of instances per label block (the large layers): a gradient that may be almost all zeros is first
    // tried through the lists of its nonzeros; the device decides which path does the work
    const uint32_t* gate = nullptr;
    if (!dense && G == 1 && usl_sparse_supported(c)) {
        if (c->nz_lists_of == g) gate = c->nz_lists_tried ? c->nz_state : nullptr;
        else USL_TRY(usl_sparse_compact(c, g, b, &gate));
        if (gate) USL_TRY(usl_sparse_backward_weight(c, x, idx, grad_W, b));
    }
    if (G > 1 && (size_t)G * N * 4 <= ((size_t)1 << 29) && N % 4 == 0 && (uintptr_t)grad_W % 16 == 0) {
        size_t lds_max;
        int Gmax = G;   // groups a batch of max_b instances would be split into: sized once, never grown by a later call
        (void)plan(c, (int)sizeof(TS), c->max_b, nblk, x, &lds_max, &Gmax, LPT == 1);
        if ((size_t)Gmax * N * 4 > ((size_t)1 << 29) || Gmax < G) Gmax = G;
        USL_TRY(usl_reserve(c, (void**)&c->gw_part, &c->gw_part_cap, (size_t)Gmax * N * 4));
        part_stride = (int64_t)N;
        dst = c->gw_part;
    } else if (G > 1) {
        hipLaunchKernelGGL(k_fill_zero, dim3(c->num_cu * 4), dim3(256), 0, c->stream, grad_W, N);
    }
#define USL_BW(MODE, AT)                                                                                \
    do {                                                                                                \
        constexpr bool DENSE_OK = (MODE) == 0;   /* the variant without the tests exists for whole rows only */ \
        if (((MODE) == 0 || (MODE) == 1) && sizeof(TS) == 4) {                                          \
            static bool checked = false;                                                                \
            if (!checked) {                                                                             \
                USL_TRY(require_lds_at_zero(c, k_backward_weight<K, LPT, NT, TS, MODE, AT, true>, "backward_weight")); \
                if (DENSE_OK) USL_TRY(require_lds_at_zero(c, k_backward_weight<K, LPT, NT, TS, MODE, AT, !DENSE_OK>, "backward_weight")); \
            }                                                                                           \
            checked = true;                                                                             \
        }                                                                                               \
        if (dense && DENSE_OK) {                                                                        \
            USL_TRY(allow_lds(c, k_backward_weight<K, LPT, NT, TS, MODE, AT, !DENSE_OK>, lds));         \
            hipLaunchKernelGGL((k_backward_weight<K, LPT, NT, TS, MODE, AT, !DENSE_OK>), grid, dim3(NT), lds, \
                               c->stream, g, (const TS*)x, idx, dst, c->m, c->d, b, tg, perm, part_stride, gate); \
        } else {                                                                                        \
            USL_TRY(allow_lds(c, k_backward_weight<K, LPT, NT, TS, MODE, AT, true>, lds));              \
            hipLaunchKernelGGL((k_backward_weight<K, LPT, NT, TS, MODE, AT, true>), grid, dim3(NT), lds, \
                               c->stream, g, (const TS*)x, idx, dst, c->m, c->d, b, tg, perm, part_stride, gate); \
        }                                                                                               \
    } while (0)
    const int mode = tg.nparts > 1 ? 1 : ((LPT == 1 && tg.rows_per_tile > 1) ? 2 : (tg.buf_stride && LPT > 1 ? 3 : 0));
    if (mode == 1) { if (G > 1) USL_BW(1, true); else USL_BW(1, false); }
    else if (mode == 3) { if (G > 1) USL_BW(LPT == 1 ? 0 : 3, true); else USL_BW(LPT == 1 ? 0 : 3, false); }
    else if (mode == 2) { if (G > 1) USL_BW(LPT == 1 ? 2 : 0, true); else USL_BW(LPT == 1 ? 2 : 0, false); }
    else { if (G > 1) USL_BW(0, true); else USL_BW(0, false); }
#undef USL_BW
    if (part_stride) {
        USL_TRY(usl_check_launch(c, "backward_weight"));
        const size_t blocks = (N / 4 + 255) / 256;
        hipLaunchKernelGGL(k_sum_parts, dim3((unsigned)(blocks < (size_t)c->num_cu * 8 ? blocks : (size_t)c->num_cu * 8)),
                           dim3(256), 0, c->stream, c->gw_part, G, N, grad_W);
    }
    return usl_check_launch(c, "backward_weight");
}

template <typename TS>
usl_status run_backward_weight_generic(usl_ctx* c, const float* g, const void* x,
                                       const int32_t* idx, float* grad_W, int b) {
    constexpr int NT = 256;
    const int64_t N = c->m * (int64_t)c->k;
    const int64_t nblk = (N + NT - 1) / NT;
    size_t lds;
    int G;
    TileGeom tg = plan(c, (int)sizeof(TS), b, nblk, x, &lds, &G);
    if (tg.nparts == 1) { lds = (size_t)c->d * sizeof(TS); tg.rows_per_tile = 1; }
    dim3 grid((unsigned)nblk, (unsigned)G);
    if (G > 1) {
        hipLaunchKernelGGL(k_fill_zero, dim3(c->num_cu * 4), dim3(256), 0, c->stream, grad_W, (size_t)N);
        USL_TRY(allow_lds(c, k_backward_weight_generic<NT, TS, true>, lds));
        hipLaunchKernelGGL((k_backward_weight_generic<NT, TS, true>), grid, dim3(NT), lds, c->stream,
                           g, (const TS*)x, idx, grad_W, c->m, c->d, c->k, b, tg);
    } else {
        USL_TRY(allow_lds(c, k_backward_weight_generic<NT, TS, false>, lds));
        hipLaunchKernelGGL((k_backward_weight_generic<NT, TS, false>), grid, dim3(NT), lds, c->stream,
                           g, (const TS*)x, idx, grad_W, c->m, c->d, c->k, b, tg);
    }
    return usl_check_launch(c, "backward_weight (generic)");
}

// The register-resident kernels need k in {8,16,32,64}, indices that fit 16 bits, and 16-byte
// aligned idx / W rows (guaranteed by k % 8 == 0 for allocations aligned to 16 bytes).
bool fast_path_ok(const usl_ctx* c, const void* idx, const void* W) {
    return c->d <= 65536 && (c->k == 8 || c->k == 16 || c->k == 32 || c->k == 64) &&
           ((uintptr_t)idx % 16 == 0) && (W == nullptr || (uintptr_t)W % 16 == 0);
}

template <typename TS>
usl_status forward_t(usl_ctx* c, const void* x, const int32_t* idx, const void* W, float* out, int b) {
    if (!fast_path_ok(c, idx, W)) return run_forward_generic<TS>(c, x, idx, W, out, b);
    const bool big = c->m >= (int64_t)c->num_cu * 1024;
    switch (c->k) {
        case 8:  return big ? run_forward<8, 8, 512, TS>(c, x, idx, W, out, b) : run_forward<8, 1, 256, TS>(c, x, idx, W, out, b);
        case 16: return big ? run_forward<16, 8, 512, TS>(c, x, idx, W, out, b) : run_forward<16, 1, 256, TS>(c, x, idx, W, out, b);
        case 32:
            // float32: 1024 lanes with two labels each keep twice the wavefronts of 512 x 4 on a
            // compute unit that the row buffer limits to one workgroup, within the 128 registers
            // such a workgroup leaves each lane; the bfloat16 variant would spill there.
            if (!big) return run_forward<32, 1, 256, TS>(c, x, idx, W, out, b);
            if constexpr (sizeof(TS) == 4) return run_forward<32, 2, 1024, TS>(c, x, idx, W, out, b);
            else return run_forward<32, 4, 512, TS>(c, x, idx, W, out, b);
        default: return big ? run_forward<64, 2, 512, TS>(c, x, idx, W, out, b) : run_forward<64, 1, 256, TS>(c, x, idx, W, out, b);
    }
}

template <typename TS>
usl_status backward_weight_t(usl_ctx* c, const float* g, const void* x, const int32_t* idx, bool dense,
                             float* grad_W, int b) {
    if (!fast_path_ok(c, idx, nullptr) || (uintptr_t)grad_W % 16 != 0)
        return run_backward_weight_generic<TS>(c, g, x, idx, grad_W, b);
    const bool big = c->m >= (int64_t)c->num_cu * 1024;
    switch (c->k) {
        case 8:  return big ? run_backward_weight<8, 8, 512, TS>(c, g, x, idx, grad_W, b, dense) : run_backward_weight<8, 1, 256, TS>(c, g, x, idx, grad_W, b, dense);
        case 16: return big ? run_backward_weight<16, 8, 512, TS>(c, g, x, idx, grad_W, b, dense) : run_backward_weight<16, 1, 256, TS>(c, g, x, idx, grad_W, b, dense);
        case 32:
            if (!big) return run_backward_weight<32, 1, 256, TS>(c, g, x, idx, grad_W, b, dense);
            // 1024 lanes pay only for float32 rows that take the whole buffer (one workgroup per compute
            // unit, one row at a time): measured 3 % there, nothing or a loss for sliced or paired rows
            if constexpr (sizeof(TS) == 4) {
                const size_t row_bytes = (size_t)c->d * 4;
                if (row_bytes <= (size_t)USL_ROW_LDS_BYTES && 2 * row_bytes + 256 > (size_t)USL_ROW_LDS_BYTES + 8192)
                    return run_backward_weight<32, 2, 1024, TS>(c, g, x, idx, grad_W, b, dense);
            }
            return run_backward_weight<32, 4, 512, TS>(c, g, x, idx, grad_W, b, dense);
        default: return big ? run_backward_weight<64, 2, 512, TS>(c, g, x, idx, grad_W, b, dense) : run_backward_weight<64, 1, 256, TS>(c, g, x, idx, grad_W, b, dense);
    }
}

}  // namespace

usl_status usl_launch_forward(usl_ctx* c, const void* x, const int32_t* idx, const void* W,
                              float* out, int32_t b) {
    return c->storage == USL_F32 ? forward_t<float>(c, x, idx, W, out, b)
                                 : forward_t<uint16_t>(c, x, idx, W, out, b);
}

usl_status usl_launch_backward_weight(usl_ctx* c, const float* g, const void* x,
                                      const int32_t* idx, float* grad_W, int32_t b, bool dense) {
    return c->storage == USL_F32 ? backward_weight_t<float>(c, g, x, idx, dense, grad_W, b)
                                 : backward_weight_t<uint16_t>(c, g, x, idx, dense, grad_W, b);
}
