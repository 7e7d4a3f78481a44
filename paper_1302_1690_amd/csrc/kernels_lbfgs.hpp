// Vector work of the limited-memory BFGS step (Results, the steel data set: LBFGS): the two-loop
// recursion over the stored pairs, as a chain of launches.  A launch first adds up the partial
// dot products the launch before it left (every workgroup adds all of them, in the same fixed
// order, so all hold the same scalar and no grid-wide wait is needed), applies its update to its
// own stretch of the working vector and leaves the partial sums of the next dot product over
// that stretch.  Sums are fp64 and ordered: the direction does not depend on timing.
#pragma once
#include <hip/hip_runtime.h>

namespace mpcnn {

constexpr int kLbBlocks = 64;   // workgroups = partial sums per dot product

// fixed-order sum of this workgroup's 256 thread values; result in every thread
__device__ inline double lb_block_sum(double v, double* red)
{
    red[threadIdx.x] = v;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
        __syncthreads();
    }
    const double s = red[0];
    __syncthreads();
    return s;
}

struct LbArgs {
    float* q;               // working vector (ends as the direction p)
    const float* src;       // mode 0: q = src
    const float* v;         // the update's vector: y_i (mode 1), s_i (mode 2)
    const float* u;         // vector of the dot product left for the next launch (null: none)
    const double* part_in;  // [kLbBlocks] partial sums of the launch before
    double* part_out;       // [kLbBlocks]
    double* alpha;          // first-loop coefficients, one per pair
    double rho;             // 1 / s.y of the update's pair
    double scale;           // factor on q after the update (H_0 at the turn, -1 at the end)
    int mode;               // 0: q = src;  1: a = rho*dot, q -= a v;  2: b = rho*dot, q += (a - b) v
    int idx;                // which alpha
    long n;
};

__global__ __launch_bounds__(256) void lb_update_kernel(LbArgs a)
{
    __shared__ double red[256];
    double coef = 0.0;
    if (a.mode != 0) {
        const double dot = lb_block_sum((int)threadIdx.x < kLbBlocks ? a.part_in[threadIdx.x] : 0.0, red);
        if (a.mode == 1) {
            coef = -(a.rho * dot);
            if (blockIdx.x == 0 && threadIdx.x == 0) a.alpha[a.idx] = a.rho * dot;
        } else {
            coef = a.alpha[a.idx] - a.rho * dot;
        }
    }
    const long chunk = (a.n + kLbBlocks - 1) / kLbBlocks;
    const long e0 = (long)blockIdx.x * chunk, e1 = e0 + chunk < a.n ? e0 + chunk : a.n;
    double part = 0.0;
    for (long e = e0 + threadIdx.x; e < e1; e += 256) {
        double x = a.mode == 0 ? (double)a.src[e] : (double)a.q[e] + coef * (double)a.v[e];
        x *= a.scale;
        const float xf = (float)x;
        a.q[e] = xf;
        if (a.u) part += (double)a.u[e] * (double)xf;
    }
    part = lb_block_sum(part, red);
    if (threadIdx.x == 0) a.part_out[blockIdx.x] = part;
}

// s = theta - theta_prev, y = g - g_prev into a free slot, with the partial sums of s.y, y.y, s.s
__global__ __launch_bounds__(256) void lb_pair_kernel(const float* __restrict__ theta, const float* __restrict__ theta_prev,
                                                      const float* __restrict__ g, const float* __restrict__ g_prev,
                                                      float* __restrict__ s_out, float* __restrict__ y_out,
                                                      double* __restrict__ part, long n)
{
    __shared__ double red[256];
    const long chunk = (n + kLbBlocks - 1) / kLbBlocks;
    const long e0 = (long)blockIdx.x * chunk, e1 = e0 + chunk < n ? e0 + chunk : n;
    double sy = 0.0, yy = 0.0, ss = 0.0;
    for (long e = e0 + threadIdx.x; e < e1; e += 256) {
        const float s = theta[e] - theta_prev[e], y = g[e] - g_prev[e];
        s_out[e] = s; y_out[e] = y;
        sy += (double)s * (double)y; yy += (double)y * (double)y; ss += (double)s * (double)s;
    }
    sy = lb_block_sum(sy, red); yy = lb_block_sum(yy, red); ss = lb_block_sum(ss, red);
    if (threadIdx.x == 0) {
        part[blockIdx.x] = sy; part[kLbBlocks + blockIdx.x] = yy; part[2 * kLbBlocks + blockIdx.x] = ss;
    }
}

// out[j] = sum of part[j][0..kLbBlocks), j < count (one workgroup)
__global__ __launch_bounds__(256) void lb_sum_kernel(const double* __restrict__ part, int count, double* __restrict__ out)
{
    __shared__ double red[256];
    for (int j = 0; j < count; ++j) {
        const double s = lb_block_sum((int)threadIdx.x < kLbBlocks ? part[j * kLbBlocks + threadIdx.x] : 0.0, red);
        if (threadIdx.x == 0) out[j] = s;
    }
}

}  // namespace mpcnn
