// Host-side launch functions of the matrix-core kernel families.  Each family's template
// instances are compiled in a translation unit of its own (launch_*.hip), so that the library
// builds in parallel; mpcnn.hip picks the instance through these plain functions.
#pragma once
#include <hip/hip_runtime.h>

#include "kernels_mfma.hpp"
#include "kernels_wgrad.hpp"

namespace mpcnn {

// Forward / data gradient (kernels_mfma.hpp).  W = channel tile side (16 or 32), OT = channel
// tiles per workgroup, PT = position tiles, NW = waves (conv_mfma_kernel), MP > 0 selects
// conv_ts_kernel with MP position tiles per wave.  False if no instance is built for the tuple.
bool launch_conv_f32(const ConvArgs& a, int W, int OT, int PT, int NW, int MP, dim3 grid, size_t lds, hipStream_t st);
bool launch_conv_b16(const ConvArgs& a, int W, int OT, int PT, int NW, int MP, dim3 grid, size_t lds, hipStream_t st);
// bf16 storage on the bf16 matrix instruction: conv_ts_kernel<OT, PT, MP, bf16, true>
bool launch_conv_bm(const ConvArgs& a, int OT, int PT, int NW, int MP, dim3 grid, size_t lds, hipStream_t st);

// Weight gradient (kernels_wgrad.hpp, kernels_wgrad_bf16.hpp); a.mw selects the instance.
bool launch_wgrad_f32(const WgradArgs& a, int hl, dim3 grid, size_t lds, hipStream_t st);
bool launch_wgrad_b16(const WgradArgs& a, int hl, dim3 grid, size_t lds, hipStream_t st);
bool launch_wgrad_bm(const WgradArgs& a, int nch, dim3 grid, size_t lds, hipStream_t st);
bool launch_wgrad_tr(const WgradArgs& a, int nch, dim3 grid, size_t lds, hipStream_t st);   // kernels_wgrad_tr.hpp

// Kernels that may ask for more than 64 KiB of dynamic LDS must say so once per device.
hipError_t conv_attrs_f32();
hipError_t conv_attrs_b16();
hipError_t wgrad_attrs_f32();
hipError_t wgrad_attrs_b16();

}  // namespace mpcnn
