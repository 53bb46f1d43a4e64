// Device-side storage types and small helpers shared by the HIP kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace bapipe {

// bfloat16 storage: the upper 16 bits of an IEEE fp32, rounded to nearest even.
struct bf16_t {
    uint16_t v;
};

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16_t x) { return __uint_as_float(((uint32_t)x.v) << 16); }

__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);   // quiet NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

template <class T> __device__ __forceinline__ T from_f32(float f);
template <> __device__ __forceinline__ float from_f32<float>(float f) { return f; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float f)
{
    bf16_t r;
    r.v = f32_to_bf16_bits(f);
    return r;
}

// value as it will read back from storage of type T
template <class T> __device__ __forceinline__ float round_to(float f) { return to_f32(from_f32<T>(f)); }

// Aligned vector of V storage elements: one 16-byte access for V*sizeof(T) == 16.
template <class T, int V> struct alignas(sizeof(T) * V) vec_t {
    T e[V];
};

// Epilogue shared by every kernel that writes an activation gradient:
//   v      : fp32 contribution of this layer to the gradient of tensor t
//   old    : value already stored for t (only read when accum)
//   gate   : forward value that decides the fused-ReLU mask of t's producer (only if masked)
// The contribution is rounded to storage first, added to the stored value (rounded again)
// and zeroed where the gate is not positive.
template <class T>
__device__ __forceinline__ T grad_out(float v, bool accum, T old, bool masked, T gate)
{
    float r = round_to<T>(v);
    if (accum) r = round_to<T>(r + to_f32(old));
    if (masked && !(to_f32(gate) > 0.0f)) r = 0.0f;
    return from_f32<T>(r);
}

// grad_out() on two bf16 values packed in a 32-bit word whose contribution `v` is already rounded
// to bf16.  Without accumulation the result is v where the gate is positive and +0 elsewhere; a
// positive finite bf16 is exactly a positive 16-bit integer, so the gate is an integer compare.
__device__ __forceinline__ uint32_t grad_epilogue_pair(uint32_t v, uint32_t old, uint32_t gate, bool accum, bool masked)
{
    if (!accum) {
        if (!masked) return v;
        const uint32_t m = ((int32_t)(gate << 16) > 0 ? 0x0000FFFFu : 0u) | ((int32_t)(gate & 0xFFFF0000u) > 0 ? 0xFFFF0000u : 0u);
        return v & m;
    }
    uint32_t packed = 0;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        bf16_t a, o, g;
        a.v = (uint16_t)(v >> (16 * h));
        o.v = (uint16_t)(old >> (16 * h));
        g.v = (uint16_t)(gate >> (16 * h));
        packed |= (uint32_t)grad_out<bf16_t>(to_f32(a), true, o, masked, g).v << (16 * h);
    }
    return packed;
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

}  // namespace bapipe
