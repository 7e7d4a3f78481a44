// Instances of the matrix-core convolution kernels for fp32 storage.
#include "launchers.hpp"

namespace mpcnn {
namespace {
typedef float T;
// (OT, PT, MP) instances of conv_ts_kernel: OT*PT/MP is 4 or 8 waves
#define CONV_TS_INSTANCES(X) \
    X(4, 2, 1) X(4, 2, 2) X(4, 4, 2) X(2, 2, 1) X(2, 4, 1) X(2, 4, 2) X(2, 8, 2) X(1, 4, 1) X(1, 8, 1) X(1, 8, 2) X(4, 4, 4) X(4, 8, 4) X(2, 8, 4) X(1, 16, 4)
// ... and its 16-wide form (layers with 16 outputs or fewer): (PT, MP), PT/MP is 4 or 8 waves
#define CONV_TS16_INSTANCES(X) X(4, 1) X(8, 1) X(8, 2) X(16, 2) X(16, 4)
// (W, OT, PT) instances of conv_mfma_kernel, each with 4 and 8 waves
#define CONV_MFMA_INSTANCES(X) \
    X(16, 1, 4) X(16, 2, 4) X(16, 4, 4) X(16, 1, 8) X(16, 2, 8) X(32, 1, 2) X(32, 2, 2) X(32, 4, 2) X(32, 1, 4) X(32, 2, 4)
}  // namespace

bool launch_conv_f32(const ConvArgs& a, int W, int OT, int PT, int NW, int MP, dim3 grid, size_t lds, hipStream_t st)
{
    if (MP > 0 && W == 16) {
        if (OT != 1) return false;
#define CASE(p, m)                                                                    \
        if (PT == p && MP == m) {                                                     \
            conv_ts_kernel<1, p, m, T, 16><<<grid, 64 * p / m, lds, st>>>(a);         \
            return true;                                                              \
        }
        CONV_TS16_INSTANCES(CASE)
#undef CASE
        return false;
    }
    if (MP > 0) {
        if (W != 32) return false;
#define CASE(o, p, m)                                                                 \
        if (OT == o && PT == p && MP == m) {                                          \
            conv_ts_kernel<o, p, m, T><<<grid, 64 * o * p / m, lds, st>>>(a);         \
            return true;                                                              \
        }
        CONV_TS_INSTANCES(CASE)
#undef CASE
        return false;
    }
#define CASE(w, o, p)                                                                 \
    if (W == w && OT == o && PT == p) {                                               \
        if (NW == 8) conv_mfma_kernel<w, o, p, 8, T><<<grid, 512, lds, st>>>(a);      \
        else conv_mfma_kernel<w, o, p, 4, T><<<grid, 256, lds, st>>>(a);              \
        return true;                                                                  \
    }
    CONV_MFMA_INSTANCES(CASE)
#undef CASE
    return false;
}

hipError_t conv_attrs_f32()
{
    hipError_t e = hipSuccess;
#define ATTR(...)                                                                            \
    if (e == hipSuccess)                                                                     \
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&__VA_ARGS__),                 \
                                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024)
#define TS_ATTR(o, p, m) ATTR(conv_ts_kernel<o, p, m, T>);
    CONV_TS_INSTANCES(TS_ATTR)
#undef TS_ATTR
#define TS16_ATTR(p, m) ATTR(conv_ts_kernel<1, p, m, T, 16>);
    CONV_TS16_INSTANCES(TS16_ATTR)
#undef TS16_ATTR
#define MF_ATTR(w, o, p) ATTR(conv_mfma_kernel<w, o, p, 4, T>); ATTR(conv_mfma_kernel<w, o, p, 8, T>);
    CONV_MFMA_INSTANCES(MF_ATTR)
#undef MF_ATTR
#undef ATTR
    return e;
}

}  // namespace mpcnn
