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

}  // namespace mpcnn
