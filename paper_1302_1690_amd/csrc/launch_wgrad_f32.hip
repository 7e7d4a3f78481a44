// Instances of the matrix-core weight-gradient kernel for fp32 storage.
#include "launchers.hpp"

namespace mpcnn {
namespace {
typedef float T;
#define WGRAD_MW(X) X(1) X(2) X(3) X(4) X(5) X(6) X(7) X(8) X(9) X(10) X(11)
}  // namespace

bool launch_wgrad_f32(const WgradArgs& a, int hl, dim3 grid, size_t lds, hipStream_t st)
{
#define CASE(m) case m:                                                                             \
        if (hl > kWgStageH) wgrad_mfma_kernel<m, 2 * kWgStageH, T><<<grid, 512, lds, st>>>(a);      \
        else wgrad_mfma_kernel<m, kWgStageH, T><<<grid, 512, lds, st>>>(a);                         \
        return true;
    switch (a.mw) {
    WGRAD_MW(CASE)
    }
#undef CASE
    return false;
}

hipError_t wgrad_attrs_f32()
{
    hipError_t e = hipSuccess;
#define ATTR(...)                                                                            \
    if (e == hipSuccess)                                                                     \
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&__VA_ARGS__),                 \
                                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024)
#define WG(m) ATTR(wgrad_mfma_kernel<m, kWgStageH, T>); ATTR(wgrad_mfma_kernel<m, 2 * kWgStageH, T>);
    WGRAD_MW(WG)
#undef WG
#undef ATTR
    return e;
}

}  // namespace mpcnn
