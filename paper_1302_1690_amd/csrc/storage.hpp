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
__device__ __forceinline__ float load1(const float* p) { return *p; }
__device__ __forceinline__ float load1(const bf16* p) { return (float)*p; }
__device__ __forceinline__ void store1(float* p, float v) { *p = v; }
__device__ __forceinline__ void store1(bf16* p, float v) { *p = (bf16)v; }

// tanh(x) = 1 - 2 / (exp(2x) + 1) with the hardware exp2 and reciprocal: absolute error
// about 1e-7; saturates correctly (exp -> inf gives 1, exp -> 0 gives -1).
__device__ __forceinline__ float fast_tanh(float x)
{
    const float e = __builtin_amdgcn_exp2f(2.885390081777927f * x);   // e^(2x) = 2^(2x log2 e)
    return fmaf(-2.f, __builtin_amdgcn_rcpf(e + 1.f), 1.f);
}

// logistic function 1 / (1 + exp(-x)), same hardware functions (exp -> inf gives 0, exp -> 0 gives 1)
__device__ __forceinline__ float fast_logistic(float x)
{
    const float e = __builtin_amdgcn_exp2f(-1.4426950408889634f * x);
    return __builtin_amdgcn_rcpf(e + 1.f);
}
// The squashing function of C and hidden FC layers (Background, layer C: tanh or logistic) and
// its derivative written in terms of its output.
__device__ __forceinline__ float squash(float x, int logistic) { return logistic ? fast_logistic(x) : fast_tanh(x); }
__device__ __forceinline__ float squash_slope(float y, int logistic) { return logistic ? y * (1.f - y) : 1.f - y * y; }

}  // namespace mpcnn
