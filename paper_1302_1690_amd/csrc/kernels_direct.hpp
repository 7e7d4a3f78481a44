// Direct (one thread per output element) kernels: the fallbacks that accept any layer
// shape (channel counts that are not multiples of 4, class layers the fused kernel does
// not cover, tiles that do not fit LDS), plus the staging, softmax and SGD kernels.
//
// Tensors are dense whole-image maps in channels-last order [B][rows][cols][C].
// A layer that follows pooling by a cumulative factor d reads taps d elements
// apart (Method, MPF layer: the k*k pooling offsets become the residues mod d).
// Weights are stored [tap = u*k+v][c][o] followed by the bias row [o].
//
// The steps of one training pass, as the comments in these files number them:
//   a0 image to channels-last storage      a1 convolution / FC forward + bias + squashing function
//   a2 max filter + argmax tap codes        a3 class layer: logits, softmax, loss
//   a4 its backward (delta of the logits)   a5 parameter gradient of a layer
//   a6 data gradient of a layer             a7 routing of the delta through a pooling layer
//   a8 parameter update
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "storage.hpp"

namespace mpcnn {

// a0: planar fp32 [B][C][Hs][Ws] -> channels-last [B][H][W][C] in the storage type.  The
// destination may be larger than the source: it then starts `top` rows above and `left`
// columns left of it, and what lies outside the source is its mirror image with the edge
// pixel repeated (Experiments: borders of test images synthesised by mirroring).
template <typename T>
__global__ void stage_input_kernel(const float* __restrict__ src, T* __restrict__ dst, int B,
                                   int C, int H, int W, int Hs, int Ws, int top, int left)
{
    long total = (long)B * C * H * W;
    for (long e = (long)blockIdx.x * blockDim.x + threadIdx.x; e < total;
         e += (long)gridDim.x * blockDim.x) {
        int c = (int)(e % C);
        long p = e / C;
        int x = (int)(p % W);
        long q = p / W;
        int y = (int)(q % H);
        int b = (int)(q / H);
        int ys = y - top, xs = x - left;
        ys = ys < 0 ? -1 - ys : (ys >= Hs ? 2 * Hs - 1 - ys : ys);
        xs = xs < 0 ? -1 - xs : (xs >= Ws ? 2 * Ws - 1 - xs : xs);
        store1(dst + e, src[(((long)b * C + c) * Hs + ys) * Ws + xs]);
    }
}

// a6: dA[b,y,x,c] = sum_{u<k,v<k2,o} W[u,v,c,o] * dY[b, y-u*d, x-v*d2, o]  (terms outside dY dropped;
// k2, d2: columns of the kernel and their spacing, which differ from the rows' after a rectangular pool),
// times (1 - A^2) when A is the tanh output of the layer below.
template <bool TANHP, typename T = float>
__global__ void conv_dgrad_direct_kernel(const T* __restrict__ dY, const float* __restrict__ Wk,
                                         const T* __restrict__ A, T* __restrict__ dA, int B,
                                         int Hi, int Wi, int Ci, int Ho, int Wo, int Co, int k, int k2, int d, int d2,
                                         int logistic)
{
    long total = (long)B * Hi * Wi * Ci;
    for (long e = (long)blockIdx.x * blockDim.x + threadIdx.x; e < total;
         e += (long)gridDim.x * blockDim.x) {
        int c = (int)(e % Ci);
        long p = e / Ci;
        int x = (int)(p % Wi);
        long q = p / Wi;
        int y = (int)(q % Hi);
        int b = (int)(q / Hi);
        float acc = 0.f;
        for (int u = 0; u < k; ++u) {
            int yy = y - u * d;
            if (yy < 0 || yy >= Ho) continue;
            for (int v = 0; v < k2; ++v) {
                int xx = x - v * d2;
                if (xx < 0 || xx >= Wo) continue;
                const T* g = dY + (((long)b * Ho + yy) * Wo + xx) * Co;
                const float* w = Wk + ((long)(u * k2 + v) * Ci + c) * Co;
                for (int o = 0; o < Co; ++o) acc = fmaf(load1(g + o), w[o], acc);
            }
        }
        if (TANHP) {
            float a = load1(A + e);
            acc *= squash_slope(a, logistic);
        }
        store1(dA + e, acc);
    }
}

// a5: partial[chunk][(tap*Ci + c)*Co + o] = sum over the chunk's rows of
//     dY[b,y,x,o] * A[b, y+u*d, x+v*d, c];  row kk = k*k*Ci is the bias row (A = 1).
// One chunk = `rows_per_chunk` output rows (b,y); a later pass adds the chunks
// in index order (Alg. 2: the gradient is the sum over all fragments).
template <typename T = float>
__global__ void conv_wgrad_direct_kernel(const T* __restrict__ A, const T* __restrict__ dY,
                                         float* __restrict__ partial, int B, int Hi, int Wi, int Ci,
                                         int Ho, int Wo, int Co, int k, int k2, int d, int d2,
                                         int rows_per_chunk)
{
    const long KN = ((long)k * k2 * Ci + 1) * Co;
    long e = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= KN) return;
    int o = (int)(e % Co);
    int kk = (int)(e / Co);
    const bool is_bias = kk == k * k2 * Ci;
    int c = kk % Ci, tap = kk / Ci;
    int u = tap / k2, v = tap % k2;
    long row0 = (long)blockIdx.y * rows_per_chunk;
    long row1 = row0 + rows_per_chunk;
    if (row1 > (long)B * Ho) row1 = (long)B * Ho;
    float acc = 0.f;
    for (long r = row0; r < row1; ++r) {
        int b = (int)(r / Ho), y = (int)(r % Ho);
        const T* g = dY + (r * Wo) * Co + o;
        if (is_bias) {
            for (int x = 0; x < Wo; ++x) acc += load1(g + (long)x * Co);
        } else {
            const T* a = A + (((long)b * Hi + (y + u * d)) * Wi + v * d2) * Ci + c;
            for (int x = 0; x < Wo; ++x) acc = fmaf(load1(g + (long)x * Co), load1(a + (long)x * Ci), acc);
        }
    }
    partial[(long)blockIdx.y * KN + e] = acc;
}

// a2: stride-1 max filter with taps d apart, plus the argmax tap code of the FIRST
// maximum in row-major (u,v) order (Alg. 3: MP_fwd on every offset, mpIDXS).
template <typename T = float>
__global__ void maxfilter_fwd_direct_kernel(const T* __restrict__ A, T* __restrict__ O,
                                            uint8_t* __restrict__ code, int B, int Hi, int Wi, int C,
                                            int Ho, int Wo, int p, int p2, int d, int d2)
{
    long total = (long)B * Ho * Wo * C;
    for (long e = (long)blockIdx.x * blockDim.x + threadIdx.x; e < total;
         e += (long)gridDim.x * blockDim.x) {
        int c = (int)(e % C);
        long q = e / C;
        int x = (int)(q % Wo);
        long r = q / Wo;
        int y = (int)(r % Ho);
        int b = (int)(r / Ho);
        float best = 0.f;
        int bi = -1;
        for (int u = 0; u < p; ++u)
            for (int v = 0; v < p2; ++v) {
                float a = load1(A + (((long)b * Hi + (y + u * d)) * Wi + (x + v * d2)) * C + c);
                if (bi < 0 || a > best) {
                    best = a;
                    bi = u * p2 + v;
                }
            }
        store1(O + e, best);   // a value read back unchanged: exact in either storage type
        if (code) code[e] = (uint8_t)bi;
    }
}

// a7: routing by argmax as a gather (Alg. 4): an input element collects dO of every
// window that chose it, in fixed (u,v) order; times (1 - A^2) when A is a tanh output.
template <bool TANHP, typename T = float>
__global__ void maxfilter_bwd_direct_kernel(const T* __restrict__ dO,
                                            const uint8_t* __restrict__ code,
                                            const T* __restrict__ A, T* __restrict__ dA,
                                            int B, int Hi, int Wi, int C, int Ho, int Wo, int p, int p2, int d, int d2,
                                            int logistic)
{
    long total = (long)B * Hi * Wi * C;
    for (long e = (long)blockIdx.x * blockDim.x + threadIdx.x; e < total;
         e += (long)gridDim.x * blockDim.x) {
        int c = (int)(e % C);
        long q = e / C;
        int x = (int)(q % Wi);
        long r = q / Wi;
        int y = (int)(r % Hi);
        int b = (int)(r / Hi);
        float acc = 0.f;
        for (int u = 0; u < p; ++u) {
            int yy = y - u * d;
            if (yy < 0 || yy >= Ho) continue;
            for (int v = 0; v < p2; ++v) {
                int xx = x - v * d2;
                if (xx < 0 || xx >= Wo) continue;
                long s = (((long)b * Ho + yy) * Wo + xx) * C + c;
                if (code[s] == (uint8_t)(u * p2 + v)) acc += load1(dO + s);
            }
        }
        if (TANHP) {
            float a = load1(A + e);
            acc *= squash_slope(a, logistic);
        }
        store1(dA + e, acc);
    }
}

constexpr int kMaxClasses = 16;

// a3 (second half): softmax over the class logits of every pixel, probabilities out in
// planar [B][n_cls][Ho][Wo]; with labels: delta = w (p - onehot) and the block's share of
// the summed cross-entropy (Results: MCCE per pixel; Method: first step of back-prop).
// mse != 0: linear outputs and half the squared error instead (Method: the derivative of
// the mean squared error w.r.t. the output image is x^ - t); `probs` then gets the outputs.
template <typename T = float>
__global__ void softmax_ce_kernel(const T* __restrict__ Z, float* __restrict__ probs,
                                  const int32_t* __restrict__ labels, const float* __restrict__ pixw,
                                  T* __restrict__ dZ, double* __restrict__ loss_partial, int B,
                                  int Ho, int Wo, int H, int W, int ctr, int n_cls, int mse, int probs_rows)
{
    __shared__ double red[256];
    long total = (long)B * Ho * Wo;
    double my_loss = 0.0;
    for (long m = (long)blockIdx.x * blockDim.x + threadIdx.x; m < total;
         m += (long)gridDim.x * blockDim.x) {
        int j = (int)(m % Wo);
        long q = m / Wo;
        int i = (int)(q % Ho);
        int b = (int)(q / Ho);
        float z[kMaxClasses];
        float zmax = -INFINITY;
        for (int o = 0; o < n_cls; ++o) {
            z[o] = load1(Z + m * n_cls + o);
            zmax = fmaxf(zmax, z[o]);
        }
        float sum = 0.f;
        float zt = 0.f;  // logit of the labelled class, relative to the maximum
        for (int o = 0; o < n_cls; ++o) {
            z[o] -= zmax;
            sum += expf(z[o]);
        }
        float inv = 1.f / sum;
        int t = -1;
        float w = 0.f;
        if (labels) {
            long lp = ((long)b * H + (i + ctr)) * W + (j + ctr);
            t = labels[lp];
            if (t < 0 || t >= n_cls) t = -1;
            else w = pixw ? pixw[lp] : 1.f;
        }
        float sq = 0.f;
        for (int o = 0; o < n_cls; ++o) {
            float p = mse ? z[o] + zmax : expf(z[o]) * inv;
            if (probs) probs[(((long)b * n_cls + o) * probs_rows + i) * Wo + j] = p;
            const float e = p - (o == t ? 1.f : 0.f);
            if (dZ) store1(dZ + m * n_cls + o, (t >= 0) ? w * e : 0.f);
            if (o == t) zt = z[o];
            sq += e * e;
        }
        if (t >= 0) my_loss += mse ? (double)w * 0.5 * (double)sq
                                   : (double)w * ((double)logf(sum) - (double)zt);  // -log p[t]
    }
    if (loss_partial) {
        red[threadIdx.x] = my_loss;
        __syncthreads();
        for (int s = blockDim.x / 2; s > 0; s >>= 1) {
            if ((int)threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
            __syncthreads();
        }
        if (threadIdx.x == 0) loss_partial[blockIdx.x] = red[0];
    }
}

// a8: theta -= step * g
__global__ void sgd_kernel(float* __restrict__ theta, const float* __restrict__ g, float step,
                           long n)
{
    long e = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (e < n) theta[e] = fmaf(-step, g[e], theta[e]);
}

// Pieces of the safeguarded gradient step: |g|^2 in fp64 by one workgroup (fixed order), and
// theta = theta0 - step * g from a kept copy of the parameters.
__global__ __launch_bounds__(1024) void sqnorm_kernel(const float* __restrict__ g, long n, double* __restrict__ out)
{
    __shared__ double red[1024];
    double s = 0.0;
    for (long e = threadIdx.x; e < n; e += 1024) s += (double)g[e] * (double)g[e];
    red[threadIdx.x] = s;
    __syncthreads();
    for (int w = 512; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) *out = red[0];
}
__global__ void step_from_kernel(float* __restrict__ theta, const float* __restrict__ theta0,
                                 const float* __restrict__ g, float step, long n)
{
    long e = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (e < n) theta[e] = fmaf(-step, g[e], theta0[e]);
}

// Per-class balanced weights (Experiments, steel defects: the loss is minimised per class):
// counts[k] = number of output pixels whose label (read at the patch centre) is k, then
// w = 1 / counts[k] at those pixels and 0 everywhere else.  Integer atomics: exact.
__global__ void label_count_kernel(const int32_t* __restrict__ labels, unsigned* __restrict__ counts,
                                   int B, int H, int W, int Ho, int Wo, int ctr, int n_cls)
{
    __shared__ unsigned hist[kMaxClasses];
    if (threadIdx.x < kMaxClasses) hist[threadIdx.x] = 0;
    __syncthreads();
    const long total = (long)B * Ho * Wo;
    for (long m = (long)blockIdx.x * blockDim.x + threadIdx.x; m < total; m += (long)gridDim.x * blockDim.x) {
        const int j = (int)(m % Wo);
        const long q = m / Wo;
        const int i = (int)(q % Ho), b = (int)(q / Ho);
        const int t = labels[((long)b * H + (i + ctr)) * W + (j + ctr)];
        if (t >= 0 && t < n_cls) atomicAdd(&hist[t], 1u);
    }
    __syncthreads();
    if ((int)threadIdx.x < n_cls && hist[threadIdx.x]) atomicAdd(&counts[threadIdx.x], hist[threadIdx.x]);
}
__global__ void balance_fill_kernel(const int32_t* __restrict__ labels, const unsigned* __restrict__ counts,
                                    float* __restrict__ pixw, int B, int H, int W, int Ho, int Wo, int ctr,
                                    int n_cls)
{
    const long total = (long)B * H * W;
    for (long e = (long)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (long)gridDim.x * blockDim.x) {
        const int x = (int)(e % W);
        const long q = e / W;
        const int y = (int)(q % H);
        const int i = y - ctr, j = x - ctr;
        const int t = labels[e];
        float w = 0.f;
        if (i >= 0 && i < Ho && j >= 0 && j < Wo && t >= 0 && t < n_cls) w = 1.f / (float)counts[t];
        pixw[e] = w;
    }
}
__global__ void clear_counts_kernel(unsigned* counts) { if (threadIdx.x < kMaxClasses) counts[threadIdx.x] = 0; }

// bf16 storage: the kernels read parameters rounded to bf16 (kept as fp32 values); the fp32
// originals stay the optimiser's state.
__global__ void round_params_kernel(const float* __restrict__ theta, float* __restrict__ rounded, long n)
{
    for (long e = (long)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += (long)gridDim.x * blockDim.x)
        rounded[e] = (float)(bf16)theta[e];
}

}  // namespace mpcnn
