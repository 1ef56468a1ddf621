// Shared device helpers of the linear-angular attention kernels (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>
#include <utility>

namespace castling {

typedef uint16_t bf16_t;  // raw bfloat16 bits

constexpr float kInvPi = 0.31830988618379067154f;

__device__ __forceinline__ float bf16_to_f32(bf16_t b)
{
    return __uint_as_float(static_cast<uint32_t>(b) << 16);
}

// round to nearest even; NaN stays NaN
__device__ __forceinline__ bf16_t f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<bf16_t>((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return static_cast<bf16_t>(u >> 16);
}

// 16-byte global access of the I/O type, widened to fp32 in registers.
template <typename T>
struct IO;

template <>
struct IO<float> {
    static constexpr int VEC = 4;
    // 16 raw bytes -> VEC values in fp32
    __device__ static __forceinline__ void widen16(const uint4& r, float (&x)[4])
    {
        x[0] = __uint_as_float(r.x); x[1] = __uint_as_float(r.y);
        x[2] = __uint_as_float(r.z); x[3] = __uint_as_float(r.w);
    }
    __device__ static __forceinline__ void load16(const float* p, float (&x)[4])
    {
        widen16(*reinterpret_cast<const uint4*>(p), x);
    }
    __device__ static __forceinline__ float to_f32(float a) { return a; }
    __device__ static __forceinline__ float from_f32(float a) { return a; }
};

template <>
struct IO<bf16_t> {
    static constexpr int VEC = 8;
    __device__ static __forceinline__ void widen16(const uint4& r, float (&x)[8])
    {
        const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            x[2 * i] = __uint_as_float(w[i] << 16);
            x[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
    __device__ static __forceinline__ void load16(const bf16_t* p, float (&x)[8])
    {
        widen16(*reinterpret_cast<const uint4*>(p), x);
    }
    __device__ static __forceinline__ float to_f32(bf16_t a) { return bf16_to_f32(a); }
    __device__ static __forceinline__ bf16_t from_f32(float a) { return f32_to_bf16(a); }
};

typedef _Float16 f16_t;

template <>
struct IO<f16_t> {
    static constexpr int VEC = 8;
    __device__ static __forceinline__ void widen16(const uint4& r, float (&x)[8])
    {
        typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_t;
        const f16x8_t h = __builtin_bit_cast(f16x8_t, r);
#pragma unroll
        for (int i = 0; i < 8; ++i) x[i] = static_cast<float>(h[i]);
    }
    __device__ static __forceinline__ void load16(const f16_t* p, float (&x)[8])
    {
        widen16(*reinterpret_cast<const uint4*>(p), x);
    }
    __device__ static __forceinline__ float to_f32(f16_t a) { return static_cast<float>(a); }
    // round to nearest even; values beyond the fp16 range become infinity
    __device__ static __forceinline__ f16_t from_f32(float a) { return static_cast<f16_t>(a); }
};

// Sum over groups of LANES consecutive lanes (LANES a power of two <= 64).
template <int LANES>
__device__ __forceinline__ float group_sum(float x)
{
#pragma unroll
    for (int m = LANES / 2; m >= 1; m >>= 1) x += __shfl_xor(x, m, 64);
    return x;
}

// Element strides of a [B][heads][N][d] tensor view; the d axis is contiguous.
struct TensorStrides {
    long long b, h, n;
};

// element offset of token 0 of unit = b * heads + h
__device__ __forceinline__ long long unit_offset(int unit, int heads, const TensorStrides& s)
{
    return (unit / heads) * s.b + (unit % heads) * s.h;
}

// Floats per unit of the internal state: S = K_hat^T V (D x D, row-major), then
// the K_hat column sum (D), then the V column sum (D).  N is known to the host.
template <int D>
struct StateLayout {
    static constexpr int S = 0;
    static constexpr int KSUM = D * D;
    static constexpr int VSUM = D * D + D;
    static constexpr int SIZE = D * D + 2 * D;
};

// store(i, load(i)) for i = tid, tid + NTHR, ... < N by the NTHR threads of a block, with the loads
// of up to MAXB items in flight per thread before the first store (a plain loop of this kind
// is compiled to one load, one wait, one store per iteration: a chain of memory latencies).
template <int N, typename V, int NTHR = 256, int MAXB = 16, typename LoadFn, typename StoreFn>
__device__ __forceinline__ void block_stage(int tid, LoadFn&& load, StoreFn&& store)
{
    constexpr int IT = (N + NTHR - 1) / NTHR;
    constexpr int B = IT < MAXB ? IT : MAXB;
#pragma unroll 1
    for (int b0 = 0; b0 < IT; b0 += B) {
        V r[B];
#pragma unroll
        for (int k = 0; k < B; ++k) {
            const int i = tid + NTHR * (b0 + k);
            r[k] = i < N ? load(i) : V{};
        }
#pragma unroll
        for (int k = 0; k < B; ++k) {
            const int i = tid + NTHR * (b0 + k);
            if (i < N) store(i, r[k]);
        }
    }
}

// Sum of `n` partials that lie `stride` floats apart, in index order, with the loads
// of sixteen partials in flight at a time (the order of the additions is fixed).
__device__ __forceinline__ float sum_partials(const float* p, int n, size_t stride)
{
    float s = 0.f;
    int sp = 0;
    for (; sp + 16 <= n; sp += 16) {
        float t[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) t[u] = p[(sp + u) * stride];
#pragma unroll
        for (int u = 0; u < 16; ++u) s += t[u];
    }
    float t[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) t[u] = (sp + u < n) ? p[(sp + u) * stride] : 0.f;
#pragma unroll
    for (int u = 0; u < 16; ++u)
        if (sp + u < n) s += t[u];
    return s;
}

// The value in a vector register the compiler knows nothing about.  Packed 16-bit operands
// must not be folded into an instruction's inline constants: the encoding of "1.0" there is
// not the bit pattern this code means.
__device__ __forceinline__ uint32_t opaque_u32(uint32_t x)
{
    asm volatile("" : "+v"(x));
    return x;
}

template <int N, typename F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>)
{
    (f(std::integral_constant<int, I>{}), ...);
}
// f(integral_constant<int, 0>), ..., f(integral_constant<int, N - 1>), fully unrolled
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f)
{
    static_for_impl<N>(f, std::make_integer_sequence<int, N>{});
}

// Global loads whose completion this code tracks itself.  The compiler's own wait
// insertion has to assume the worst across the software pipeline's loop (it waits for
// every load in flight, which serialises the prefetch); these loads are invisible to
// it and are followed, before the first use of their registers, by wait_async_loads
// with the number of younger loads that may still be in flight.  Loads complete in
// issue order, and any further memory operation issued in between only makes the
// wait stricter, never too weak.
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;

// base: wave-uniform pointer (scalar registers), offset: per-lane byte offset
__device__ __forceinline__ void async_load16(u32x4_t& dst, const void* base, uint32_t offset)
{
    asm volatile("global_load_dwordx4 %0, %1, %2" : "=v"(dst) : "v"(offset), "s"(base) : "memory");
}
// same, for data that is read exactly once: non-temporal, so that it does not push
// re-used lines (the V halo columns) out of the L2
__device__ __forceinline__ void async_load16_stream(u32x4_t& dst, const void* base, uint32_t offset)
{
    asm volatile("global_load_dwordx4 %0, %1, %2 nt" : "=v"(dst) : "v"(offset), "s"(base) : "memory");
}
template <int YOUNGER>
__device__ __forceinline__ void wait_async_loads(u32x4_t& a, u32x4_t& b, u32x4_t& c)
{
    static_assert(YOUNGER >= 0 && YOUNGER < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%3)" : "+v"(a), "+v"(b), "+v"(c) : "n"(YOUNGER) : "memory");
}
template <int YOUNGER>
__device__ __forceinline__ void wait_async_loads(u32x4_t& a, u32x4_t& b, u32x4_t& c, u32x4_t& d)
{
    static_assert(YOUNGER >= 0 && YOUNGER < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%4)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d) : "n"(YOUNGER) : "memory");
}
template <int YOUNGER>
__device__ __forceinline__ void wait_async_loads(u32x4_t& a)
{
    static_assert(YOUNGER >= 0 && YOUNGER < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%1)" : "+v"(a) : "n"(YOUNGER) : "memory");
}
template <int YOUNGER>
__device__ __forceinline__ void wait_async_loads(u32x4_t& a, u32x4_t& b)
{
    static_assert(YOUNGER >= 0 && YOUNGER < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%2)" : "+v"(a), "+v"(b) : "n"(YOUNGER) : "memory");
}

}  // namespace castling
