// Instances of the matrix-core weight-gradient kernels for bf16 storage.
#include "launchers.hpp"
#include "kernels_wgrad_bf16.hpp"
#include "kernels_wgrad_tr.hpp"

namespace mpcnn {
namespace {
typedef bf16 T;
#define WGRAD_MW(X) X(1) X(2) X(3) X(4) X(5) X(6) X(7) X(8) X(9) X(10) X(11)
}  // namespace

bool launch_wgrad_b16(const WgradArgs& a, int hl, dim3 grid, size_t lds, hipStream_t st)
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

bool launch_wgrad_bm(const WgradArgs& a, int nch, dim3 grid, size_t lds, hipStream_t st)
{
#define CASE(m, c) case 4 * m + c - 5: wgrad_bm_kernel<m, c><<<grid, 512, lds, st>>>(a); return true;
#define ROW(m) CASE(m, 1) CASE(m, 2) CASE(m, 3) CASE(m, 4)
    if (nch < 1 || nch > 4 || a.mw < 1 || a.mw > kWgBmMaxTiles) return false;
    switch (4 * a.mw + nch - 5) {
    ROW(1) ROW(2) ROW(3) ROW(4) ROW(5)
    }
#undef ROW
#undef CASE
    return false;
}

bool launch_wgrad_tr(const WgradArgs& a, int nch, dim3 grid, size_t lds, hipStream_t st)
{
#define CASE(m, c) case 4 * m + c - 5: wgrad_tr_kernel<m, c><<<grid, 512, lds, st>>>(a); return true;
#define ROW(m) CASE(m, 1) CASE(m, 2) CASE(m, 3) CASE(m, 4)
    if (nch < 1 || nch > 4 || a.mw < 1 || a.mw > kWgTrMaxTiles) return false;
    switch (4 * a.mw + nch - 5) {
    ROW(1) ROW(2) ROW(3) ROW(4) ROW(5)
    }
#undef ROW
#undef CASE
    return false;
}

hipError_t wgrad_attrs_b16()
{
    hipError_t e = hipSuccess;
#define ATTR(...)                                                                            \
    if (e == hipSuccess)                                                                     \
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&__VA_ARGS__),                 \
                                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024)
#define WG(m) ATTR(wgrad_mfma_kernel<m, kWgStageH, T>); ATTR(wgrad_mfma_kernel<m, 2 * kWgStageH, T>);
    WGRAD_MW(WG)
#undef WG
#define ROW(m) ATTR(wgrad_bm_kernel<m, 1>); ATTR(wgrad_bm_kernel<m, 2>); ATTR(wgrad_bm_kernel<m, 3>); ATTR(wgrad_bm_kernel<m, 4>); \
               ATTR(wgrad_tr_kernel<m, 1>); ATTR(wgrad_tr_kernel<m, 2>); ATTR(wgrad_tr_kernel<m, 3>); ATTR(wgrad_tr_kernel<m, 4>);
    ROW(1) ROW(2) ROW(3) ROW(4) ROW(5)
#undef ROW
#undef ATTR
    return e;
}

}  // namespace mpcnn
