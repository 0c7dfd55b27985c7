// Shared device helpers for the gfx950 kernels: storage types, bf16 conversion,
// wave-level reductions.  Wavefronts are 64 lanes wide throughout.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>
#include <utility>

namespace dyn {

typedef uint16_t bf16_t;   // raw bfloat16 storage word

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float bf2f(bf16_t v) { return __uint_as_float(static_cast<uint32_t>(v) << 16); }

// Round to nearest, ties to even.  NaN keeps a quiet payload.
__device__ __forceinline__ bf16_t f2bf(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<bf16_t>((u >> 16) | 0x40);
    u += 0x7fffu + ((u >> 16) & 1u);
    return static_cast<bf16_t>(u >> 16);
}

template <typename T> __device__ __forceinline__ float to_f32(T v);
template <> __device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f32<bf16_t>(bf16_t v) { return bf2f(v); }

template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return f2bf(v); }

// Butterfly reductions over the 64 lanes of a wave; every lane ends with the result and
// the combination order is fixed by the lane ids.
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}

// LDS operand reads as inline assembly, with their waits placed by hand (wait_lgkmcnt).  The compiler's own
// wait insertion waits for every outstanding LDS read before each block of MFMAs, which serialises
// reads and matrix products; reads it does not see it does not wait for.  The price: the compiler
// believes a result is in its registers as soon as the read has been issued, so nothing but
// instructions placed after the matching wait (and a scheduling barrier, where the consumer is not
// assembly itself) may touch them.  LDS operations return in issue order, so "at most N outstanding"
// means everything but the N most recent has arrived; LDS operations the compiler issues in between
// can only make such a wait stricter, never laxer.
template <int OFFSET>
__device__ __forceinline__ bf16x8 lds_read16(unsigned addr) {        // 16 bytes per lane at LDS byte address addr + OFFSET
    static_assert(OFFSET >= 0 && OFFSET < 65536, "ds_read offset field");
    bf16x8 v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFFSET) : "memory");
    return v;
}
template <int OFFSET>
__device__ __forceinline__ u32x2 lds_read8(unsigned addr) {          // 8 bytes per lane
    static_assert(OFFSET >= 0 && OFFSET < 65536, "ds_read offset field");
    u32x2 v;
    asm volatile("ds_read_b64 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFFSET) : "memory");
    return v;
}
template <int N>
__device__ __forceinline__ void wait_lgkmcnt() {                   // s_waitcnt lgkmcnt(N) only (vmcnt 63, expcnt 7 = no wait)
    static_assert(N >= 0 && N <= 15, "lgkmcnt is a 4-bit counter");
    __builtin_amdgcn_s_waitcnt(0xc07f | (N << 8));
}

// f(integral_constant<int, I0>), ..., f(integral_constant<int, I1 - 1>): a loop whose index is a compile-time
// constant in the body (immediate offsets of the assembly above, register-array indices).
template <int I0, int I1, class F>
__device__ __forceinline__ void static_for(F &&f) {
    if constexpr (I0 < I1) {
        f(std::integral_constant<int, I0>());
        static_for<I0 + 1, I1>(f);
    }
}

// Split-KV chunk size (cached positions per work item) of a query block of a multi-token
// sequence, from `reach` = the largest key count a token of its aligned position block can
// attend.  1024 positions, doubled until the block has at most 8 chunks, up to 8192: behind a
// long cached prefix fixed 1024-position chunks leave one fp32 partial set per 1024 keys and
// token for the merge to read back.  A function of the block's positions alone, so a token's
// chunks - and the order its partials are merged in - do not depend on the batch around it.
__host__ __device__ inline int prefill_chunk_positions(int reach) {
    int ct = 1024;
    while (reach > 8 * ct && ct < 8192) ct *= 2;
    return ct;
}
constexpr int kPrefillChunkPagesMax = 8192 / 16;     // in 16-position pages

}  // namespace dyn
