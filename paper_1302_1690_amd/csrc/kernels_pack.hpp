// Repacking of a layer's parameters into the operand order of the matrix-core convolution
// kernels (forward and data gradient; Method, forward and backward of layer C).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "storage.hpp"

namespace mpcnn {

// Repack W[tap][c][o] (+ bias row) into the operand order of conv_mfma_kernel, G lane groups:
//   forward : reduce over c, outputs o:  P[tap*nch + ch][g][o][s]  = W[tap][4G*ch+4g+s][o]
//   dgrad   : reduce over o, outputs c:  P[tap'*nch + ch][g][c][s] = W[k*k-1-tap'][c][4G*ch+4g+s]
// (taps reversed: the data gradient at x collects deltas at x - u*d).  Padding is zero.
__global__ void pack_weights_kernel(const float* __restrict__ W, float* __restrict__ P, int kk,
                                    int Ci, int Co, int RPad, int OPad, int G, int dgrad)
{
    const int nch = RPad / (4 * G);
    long total = (long)kk * nch * G * OPad * 4;
    for (long e = (long)blockIdx.x * blockDim.x + threadIdx.x; e < total;
         e += (long)gridDim.x * blockDim.x) {
        int s = (int)(e & 3);
        long q = e >> 2;
        int oo = (int)(q % OPad); q /= OPad;
        int g = (int)(q % G); q /= G;
        int ch = (int)(q % nch);
        int tap = (int)(q / nch);
        int r = 4 * G * ch + 4 * g + s;  // index along the reduced dimension
        float v = 0.f;
        if (!dgrad) {
            if (r < Ci && oo < Co) v = W[((long)tap * Ci + r) * Co + oo];
        } else {
            if (r < Co && oo < Ci) v = W[((long)(kk - 1 - tap) * Ci + oo) * Co + r];
        }
        P[e] = v;
    }
}

// The same packs for the bf16 matrix instruction (v_mfma_f32_32x32x16_bf16: lane l supplies
// 8 consecutive reduction indices, 8*(l/32) .. +7, of row / column l%32): 8 channels per item,
//   P[tap*nch + ch][g][o][s] = W[..][16*ch + 8*g + s][..], s < 8, as bf16.
__global__ void pack_weights_bf16_kernel(const float* __restrict__ W, bf16* __restrict__ P, int kk,
                                         int Ci, int Co, int RPad, int OPad, int dgrad)
{
    const int nch = RPad / 16;
    long total = (long)kk * nch * 2 * OPad * 8;
    for (long e = (long)blockIdx.x * blockDim.x + threadIdx.x; e < total;
         e += (long)gridDim.x * blockDim.x) {
        int s = (int)(e & 7);
        long q = e >> 3;
        int oo = (int)(q % OPad); q /= OPad;
        int g = (int)(q & 1); q >>= 1;
        int ch = (int)(q % nch);
        int tap = (int)(q / nch);
        int r = 16 * ch + 8 * g + s;  // index along the reduced dimension
        float v = 0.f;
        if (!dgrad) {
            if (r < Ci && oo < Co) v = W[((long)tap * Ci + r) * Co + oo];
        } else {
            if (r < Co && oo < Ci) v = W[((long)(kk - 1 - tap) * Ci + oo) * Co + r];
        }
        P[e] = (bf16)v;
    }
}

}  // namespace mpcnn
