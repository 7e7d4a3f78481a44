// Storage types of the activation and delta tensors: fp32, or bf16 with fp32 arithmetic
// (every kernel converts on load and rounds to nearest-even on store; sums, softmax, loss
// and parameter gradients are always fp32 or wider).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mpcnn {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 bf16;
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));

// four consecutive elements (the address must be a multiple of four elements)
__device__ __forceinline__ v4f load4(const float* p) { return *reinterpret_cast<const v4f*>(p); }
__device__ __forceinline__ v4f load4(const bf16* p)
{
    return __builtin_convertvector(*reinterpret_cast<const bf16x4*>(p), v4f);
}
__device__ __forceinline__ void store4(float* p, v4f v) { *reinterpret_cast<v4f*>(p) = v; }
__device__ __forceinline__ void store4(bf16* p, v4f v)
{
    *reinterpret_cast<bf16x4*>(p) = __builtin_convertvector(v, bf16x4);
}
// The same four elements through a buffer descriptor: byte offset = per-lane part + scalar part (no address
// arithmetic on the vector ALU; out-of-range reads return zeros)
template <typename T>
__device__ __forceinline__ v4f buffer_load4(__amdgpu_buffer_rsrc_t rsrc, unsigned lane_bytes, unsigned scalar_bytes)
{
    typedef unsigned v4u __attribute__((ext_vector_type(4)));
    typedef unsigned v2u __attribute__((ext_vector_type(2)));
    if constexpr (sizeof(T) == 4) {
        return __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)lane_bytes, (int)scalar_bytes, 0));
    } else {
        const v2u r = __builtin_amdgcn_raw_buffer_load_b64(rsrc, (int)lane_bytes, (int)scalar_bytes, 0);
        return __builtin_convertvector(__builtin_bit_cast(bf16x4, r), v4f);
    }
}
__device__ __forceinline__ float load1(const float* p) { return *p; }
__device__ __forceinline__ float load1(const bf16* p) { return (float)*p; }
__device__ __forceinline__ void store1(float* p, float v) { *p = v; }
__device__ __forceinline__ void store1(bf16* p, float v) { *p = (bf16)v; }

// The squashing function of C and hidden FC layers (Background, layer C: tanh or logistic) and its
// derivative written in terms of its output.  Both functions are one formula with three constants
// picked by the (launch-uniform) flag, so that no branch or select stands between the values:
//   y = A / (exp2(c x) + 1) + B     tanh: c = 2 log2 e, A = -2, B = 1   (tanh x = 1 - 2 / (e^(2x) + 1))
//                                   logistic: c = -log2 e, A = 1, B = 0 (1 / (1 + e^(-x)))
// with the hardware exp2 and reciprocal: absolute error about 1e-7; saturates correctly
// (exp -> inf gives B, exp -> 0 gives A + B).
//   dy/dx = l0 + y (l1 - y)         tanh: 1 - y^2;  logistic: y (1 - y)
__device__ __forceinline__ float squash(float x, int logistic)
{
    const float c = logistic ? -1.4426950408889634f : 2.885390081777927f;
    const float A = logistic ? 1.f : -2.f, B = logistic ? 0.f : 1.f;
    return fmaf(A, __builtin_amdgcn_rcpf(__builtin_amdgcn_exp2f(c * x) + 1.f), B);
}
__device__ __forceinline__ float squash_slope(float y, int logistic)
{
    const float l0 = logistic ? 0.f : 1.f, l1 = logistic ? 1.f : 0.f;
    return fmaf(y, fmaf(y, -1.f, l1), l0);
}

}  // namespace mpcnn
