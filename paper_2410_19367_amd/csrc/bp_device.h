// Device-side helpers shared by the gfx950 kernels: bf16 <-> fp32, 8-element (16-byte for bf16)
// vector loads/stores that widen to fp32, and 64-lane wave reductions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace bp {

typedef __bf16 bf16_t;

template <typename T> __device__ __forceinline__ float to_float(T v);
template <> __device__ __forceinline__ float to_float<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_float<bf16_t>(bf16_t v) { return (float)v; }

template <typename T> __device__ __forceinline__ T from_float(float v);
template <> __device__ __forceinline__ float from_float<float>(float v) { return v; }
// round to nearest even (the compiler emits the hardware conversion on gfx950)
template <> __device__ __forceinline__ bf16_t from_float<bf16_t>(float v) { return (bf16_t)v; }

__device__ __forceinline__ float bf16_bits_to_float(uint32_t bits16) {
    return __uint_as_float(bits16 << 16);
}

// 8 consecutive elements -> fp32.  Pointers must be 16-byte aligned (bf16) / 16-byte (fp32).
__device__ __forceinline__ void load8(const bf16_t* p, float (&v)[8]) {
    const uint4 r = *reinterpret_cast<const uint4*>(p);
    v[0] = __uint_as_float(r.x << 16); v[1] = __uint_as_float(r.x & 0xffff0000u);
    v[2] = __uint_as_float(r.y << 16); v[3] = __uint_as_float(r.y & 0xffff0000u);
    v[4] = __uint_as_float(r.z << 16); v[5] = __uint_as_float(r.z & 0xffff0000u);
    v[6] = __uint_as_float(r.w << 16); v[7] = __uint_as_float(r.w & 0xffff0000u);
}
__device__ __forceinline__ void load8(const float* p, float (&v)[8]) {
    const float4 a = reinterpret_cast<const float4*>(p)[0];
    const float4 b = reinterpret_cast<const float4*>(p)[1];
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
    v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    typedef bf16_t bf16x2 __attribute__((ext_vector_type(2)));
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    f32x2 f = {lo, hi};
    bf16x2 b = __builtin_convertvector(f, bf16x2);
    return __builtin_bit_cast(uint32_t, b);
}

__device__ __forceinline__ void store8(bf16_t* p, const float (&v)[8]) {
    uint4 r;
    r.x = pack_bf16x2(v[0], v[1]);
    r.y = pack_bf16x2(v[2], v[3]);
    r.z = pack_bf16x2(v[4], v[5]);
    r.w = pack_bf16x2(v[6], v[7]);
    *reinterpret_cast<uint4*>(p) = r;
}
__device__ __forceinline__ void store8(float* p, const float (&v)[8]) {
    reinterpret_cast<float4*>(p)[0] = make_float4(v[0], v[1], v[2], v[3]);
    reinterpret_cast<float4*>(p)[1] = make_float4(v[4], v[5], v[6], v[7]);
}

// Reductions over the two 32-lane halves of a wave (lane l and lane l ^ 32) with one
// v_permlane32_swap instead of a round trip through the LDS permute unit: swapping a register with
// itself yields the lower half's values on all lanes in one result and the upper half's in the other.
__device__ __forceinline__ float halves_max(float v) {
    typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
    const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float halves_sum(float v) {
    typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
    const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// ---- GELU, tanh form (the approximation GPT-2 / Megatron use):
//   g(x) = x/2 (1 + tanh(w)),  w = sqrt(2/pi) (x + 0.044715 x^3),  and  (1 + tanh(w))/2 = sigmoid(2w).
// Written with the bare exp2 / reciprocal instructions: s = 1 / (1 + 2^(-2 w log2 e)) has the exact
// limits 0 and 1 for large |x| (2^(+big) = inf, 1/inf = 0), so no range checks are needed.
__device__ __forceinline__ float gelu_sigmoid(float x) {
    const float x2 = x * x;
    const float w2 = x * (-2.302208198f - 0.1029432397f * x2);    // -2 log2(e) sqrt(2/pi) (x + 0.044715 x^3)
    return __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(w2));
}
__device__ __forceinline__ float gelu_value(float x) { return x * gelu_sigmoid(x); }
// g'(x) = s + x s (1 - s) 2 w'(x),  2 w'(x) = 2 sqrt(2/pi) (1 + 3 * 0.044715 x^2)
__device__ __forceinline__ float gelu_slope(float x) {
    const float s = gelu_sigmoid(x);
    const float dw2 = 1.5957691216f + 0.2140644488f * x * x;
    return s + x * s * (1.f - s) * dw2;
}

}  // namespace bp
