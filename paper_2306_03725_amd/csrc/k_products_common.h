// Device helpers shared by the forward / backward-weight kernels: LDS staging of activation rows,
// coalesced movement of idx / W / grad_W rows through an LDS transposition buffer, and the private
// slot order of a label.
#pragma once
#include "usl_internal.h"

namespace usl_products {

// Copies n elements from global memory into LDS.  With 16-byte alignment the bulk goes through
// global_load_lds_dwordx4: each wavefront moves 1 KiB per instruction straight into LDS (the LDS
// address is wave-uniform, the hardware adds lane*16), no VGPRs are used and all of a lane's loads
// are in flight together.  The caller's barrier follows the vmcnt wait.
// WAIT = false leaves the copies in flight: the caller waits (vmcnt) before its barrier.
template <typename TS, int NT, bool WAIT = true>
__device__ __forceinline__ void stage(const TS* __restrict__ src, TS* __restrict__ lds, int n,
                                      bool vec_ok, int tid = (int)threadIdx.x) {
    if (vec_ok) {
        const uint4* s = reinterpret_cast<const uint4*>(src);
        uint4* dd = reinterpret_cast<uint4*>(lds);
        const int nv = (int)((size_t)n * sizeof(TS) / 16);
        const int full = nv & ~63;
        const int lane = tid & 63;
        for (int v = (tid >> 6) * 64; v < full; v += NT)
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void*)(s + v + lane),
                (__attribute__((address_space(3))) void*)(dd + v), 16, 0, 0);
        for (int v = full + tid; v < nv; v += NT) dd[v] = s[v];
        if (WAIT) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    } else {
        for (int c = tid; c < n; c += NT) lds[c] = src[c];
    }
}

// The same with the byte offset of the element instead of its column (indices scaled once, outside the loop).
__device__ __forceinline__ float lds_at(const float* row, uint32_t byte_off) {
    return *reinterpret_cast<const float*>(reinterpret_cast<const char*>(row) + byte_off);
}
__device__ __forceinline__ float lds_at(const uint16_t* row, uint32_t byte_off) {
    return usl_bf16_to_f32(*reinterpret_cast<const uint16_t*>(reinterpret_cast<const char*>(row) + byte_off));
}
__device__ __forceinline__ float lds_val(const float* row, uint32_t c) { return row[c]; }
__device__ __forceinline__ float lds_val(const uint16_t* row, uint32_t c) {
    return usl_bf16_to_f32(row[c]);
}

// Rows [row0, row0+NT) of a row-major [m][KW] matrix of 32-bit words (KW % 4 == 0, base 16-byte
// aligned) are copied into LDS with coalesced 16-byte loads, one padding word per row, so that
// afterwards lane r can read "its" row word by word without bank conflicts (stride KW+1).
template <int KW, int NT>
__device__ __forceinline__ void rows_to_lds(const uint32_t* __restrict__ src, int64_t row0,
                                            int64_t m, uint32_t* __restrict__ lds) {
    int64_t nvalid = m - row0;
    nvalid = nvalid < 0 ? 0 : (nvalid > NT ? NT : nvalid);
    const int nv = (int)(nvalid * KW / 4);
    const uint4* s = reinterpret_cast<const uint4*>(src + row0 * KW);
    for (int v = threadIdx.x; v < nv; v += NT) {
        const uint4 q = s[v];
        const int f = v * 4, r = f / KW, t = f % KW;
        uint32_t* p = lds + r * (KW + 1) + t;
        p[0] = q.x; p[1] = q.y; p[2] = q.z; p[3] = q.w;
    }
}
// The reverse: every lane has put its KW words at lds[lane*(KW+1) ..]; rows leave with coalesced
// 16-byte stores, or float atomic adds when several workgroups share the destination.
template <int KW, int NT, bool ATOMIC>
__device__ __forceinline__ void lds_to_rows(const uint32_t* __restrict__ lds, float* __restrict__ dst,
                                            int64_t row0, int64_t m) {
    int64_t nvalid = m - row0;
    nvalid = nvalid < 0 ? 0 : (nvalid > NT ? NT : nvalid);
    const int nv = (int)(nvalid * KW / 4);
    float* base = dst + row0 * KW;
    for (int v = threadIdx.x; v < nv; v += NT) {
        const int f = v * 4, r = f / KW, t = f % KW;
        const uint32_t* p = lds + r * (KW + 1) + t;
        const float4 q = make_float4(__uint_as_float(p[0]), __uint_as_float(p[1]),
                                     __uint_as_float(p[2]), __uint_as_float(p[3]));
        if (ATOMIC) {
            unsafeAtomicAdd(base + f, q.x); unsafeAtomicAdd(base + f + 1, q.y);
            unsafeAtomicAdd(base + f + 2, q.z); unsafeAtomicAdd(base + f + 3, q.w);
        } else {
            reinterpret_cast<float4*>(base)[v] = q;
        }
    }
}

// Private slot order of one label: K bytes (slot visited at step s), held as K/4 words while the
// registers are being filled.  A null table means natural order.
template <int K>
struct SlotOrder {
    uint32_t w[K / 4];
    bool on;
    __device__ __forceinline__ void load(const uint8_t* __restrict__ perm, int64_t j, bool valid) {
        on = perm != nullptr;
        if (on) {
            const uint32_t* p = reinterpret_cast<const uint32_t*>(perm + j * K);
#pragma unroll
            for (int q = 0; q < K / 4; ++q) w[q] = valid ? p[q] : (0x03020100u + 0x04040404u * q);
        }
    }
    __device__ __forceinline__ int at(int s) const {
        return on ? (int)((w[s >> 2] >> (8 * (s & 3))) & 0xFFu) : s;
    }
};

// Brings the k indices of NT consecutive labels into registers, two 16-bit indices per register,
// in the label's private slot order.
template <int K, int NT>
__device__ __forceinline__ void fetch_idx_packed(const int32_t* __restrict__ idx, int64_t row0,
                                                 int64_t m, uint32_t* lds, const SlotOrder<K>& so,
                                                 uint32_t (&pk)[K / 2]) {
    __syncthreads();
    rows_to_lds<K, NT>(reinterpret_cast<const uint32_t*>(idx), row0, m, lds);
    __syncthreads();
    const bool valid = row0 + threadIdx.x < m;
    const uint32_t* p = lds + threadIdx.x * (K + 1);
#pragma unroll
    for (int q = 0; q < K / 2; ++q)
        pk[q] = valid ? (p[so.at(2 * q)] | (p[so.at(2 * q + 1)] << 16)) : 0u;
}
template <int K>
__device__ __forceinline__ uint32_t col_of(const uint32_t (&pk)[K / 2], int t) {
    return (t & 1) ? (pk[t >> 1] >> 16) : (pk[t >> 1] & 0xFFFFu);
}

// Byte offset (column * 4) of slot t in a float32 row.  The 16-bit half of the packed word is
// selected and shifted by one instruction (sub-dword operand select) where mask-and-shift takes two.
template <int K>
__device__ __forceinline__ uint32_t byte_off4(const uint32_t (&pk)[K / 2], int t) {
    uint32_t a;
    const uint32_t two = 2;
    if (t & 1)
        asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_1"
            : "=v"(a) : "s"(two), "v"(pk[t >> 1]));
    else
        asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_0"
            : "=v"(a) : "s"(two), "v"(pk[t >> 1]));
    return a;
}
// Slot t of the float32 row that starts at the very beginning of the workgroup's LDS: the byte offset
// is the LDS address itself, so no base is added (one vector instruction per gather instead of two).
// Kernels that use it have no static LDS, which puts their dynamic LDS at address 0; they check that
// once (lds_starts_at_zero) before relying on it.
typedef const __attribute__((address_space(3))) float lds_f32_t;
template <int K>
__device__ __forceinline__ float gather_row0(const uint32_t (&pk)[K / 2], int t) {
    return *reinterpret_cast<lds_f32_t*>(static_cast<uintptr_t>(byte_off4<K>(pk, t)));
}
// A float32 row cut into two halves of 32768 columns (the LDS budget): slot t of the half that is staged,
// or, for a slot of the other half, the lane's word of zeros behind the buffer (zbyte >= 131072 is its LDS
// address).  While the upper half is staged the packed indices have bit 15 flipped, so "in this half" is
// "column < 32768" both times and the choice is one unsigned minimum.
template <int K>
__device__ __forceinline__ float gather_half(const uint32_t (&pk)[K / 2], int t, uint32_t zbyte) {
    const uint32_t off = byte_off4<K>(pk, t);
    return *reinterpret_cast<lds_f32_t*>(static_cast<uintptr_t>(off < zbyte ? off : zbyte));
}
template <int N>
__device__ __forceinline__ void flip_half(uint32_t (&pk)[N]) {
#pragma unroll
    for (int q = 0; q < N; ++q) pk[q] ^= 0x80008000u;
}
__device__ __forceinline__ bool lds_starts_at_zero(const void* dyn_lds) {
    return (uint32_t)(uintptr_t)((const __attribute__((address_space(3))) void*)dyn_lds) == 0u;
}

template <int K, int NT>
__device__ __forceinline__ void fetch_w(const float* __restrict__ W, int64_t row0, int64_t m,
                                        uint32_t* lds, const SlotOrder<K>& so, float (&w)[K]) {
    __syncthreads();
    rows_to_lds<K, NT>(reinterpret_cast<const uint32_t*>(W), row0, m, lds);
    __syncthreads();
    const bool valid = row0 + threadIdx.x < m;
    const uint32_t* p = lds + threadIdx.x * (K + 1);
#pragma unroll
    for (int t = 0; t < K; ++t) w[t] = valid ? __uint_as_float(p[so.at(t)]) : 0.f;
}
// bfloat16 rows are widened to float32 words on their way into the transposition buffer, so the
// per-lane part is the same as for float32.
template <int K, int NT>
__device__ __forceinline__ void fetch_w(const uint16_t* __restrict__ W, int64_t row0, int64_t m,
                                        uint32_t* lds, const SlotOrder<K>& so, float (&w)[K]) {
    __syncthreads();
    {
        int64_t nvalid = m - row0;
        nvalid = nvalid < 0 ? 0 : (nvalid > NT ? NT : nvalid);
        const int nv = (int)(nvalid * K / 8);
        const uint4* s = reinterpret_cast<const uint4*>(W + row0 * K);
        for (int v = threadIdx.x; v < nv; v += NT) {
            const uint4 q = s[v];
            const int f = v * 8, r = f / K, t = f % K;
            uint32_t* p = lds + r * (K + 1) + t;
            p[0] = q.x << 16; p[1] = q.x & 0xFFFF0000u; p[2] = q.y << 16; p[3] = q.y & 0xFFFF0000u;
            p[4] = q.z << 16; p[5] = q.z & 0xFFFF0000u; p[6] = q.w << 16; p[7] = q.w & 0xFFFF0000u;
        }
    }
    __syncthreads();
    const bool valid = row0 + threadIdx.x < m;
    const uint32_t* p = lds + threadIdx.x * (K + 1);
#pragma unroll
    for (int t = 0; t < K; ++t) w[t] = valid ? __uint_as_float(p[so.at(t)]) : 0.f;
}

// Stops the compiler from hoisting the unpacked indices out of the instance loop: unpacking is two
// cheap VALU operations per gather, holding all k unpacked indices would double the register need.
template <int N>
__device__ __forceinline__ void keep_packed(uint32_t (&pk)[N]) {
#pragma unroll
    for (int q = 0; q < N; ++q) asm volatile("" : "+v"(pk[q]));
}

}  // namespace usl_products
