// The image layer with fp32 storage on v_mfma_f32_32x32x2_f32: conv + bias + squashing function over
// 1 or 3 input channels at spacing 1 (Background, layer C).  The reduction, k*k*C values, is far too
// short for the general kernel's channel tiling, and on the vector ALU the layer runs at a tenth of the
// matrix rate (49 taps x 32 maps of multiply-adds per position).
//
// The product is [maps] x [k rows of k*C values] x [positions].  A window row's k*C values are contiguous
// in a channels-last image, so with the image tile in LDS as rows of (32 + k - 1)*C floats a lane's share
// of the positions' operand at step (u, j) - values 2j and 2j + 1 of window row u, one per lane half -
// is the word at  lane base + u * (row pitch) + 2j, an immediate offset: the loop holds one LDS read and
// one matrix instruction per position tile and nothing else.  An odd k*C is padded by one value that
// meets a zero weight.  The maps' operand, the whole filter bank, stays in registers (one word per step).
// A workgroup's tile is 4 MP rows x 32 columns of positions: wave w owns rows w*MP .. w*MP + MP - 1,
// a lane one column.  Result layout and epilogue as in conv_ts_kernel.
#pragma once
#include "kernels_mfma.hpp"

namespace mpcnn {

struct FirstMfmaArgs {
    const float* in;      // [B][Hi][Wi][C] channels-last image
    const float* Wk;      // [k*k*C][Co] then bias [Co]
    float* out;           // [B][Ho][Wo][Co]
    int B, Hi, Wi, Ho, Wo, Co;
    int squash;           // 0 linear, 1 tanh, 2 logistic
    int ntx, nty;         // tiles per image
};

template <int K, int C, int MP>
__global__ __launch_bounds__(256) void first_layer_mfma_kernel(FirstMfmaArgs a)
{
    constexpr int R = K * C, RP = (R + 1) & ~1, SR = RP / 2, STEPS = K * SR;
    constexpr int TY = 4 * MP, TX = 32;
    constexpr int HH = TY + K - 1, HWC = (TX + K - 1) * C + (RP - R);   // floats per LDS row (+ the padding value)
    __shared__ float tile[HH * HWC];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lt = lane & 31, lg = lane >> 5;
    int bid = blockIdx.x;
    const int txi = bid % a.ntx; bid /= a.ntx;
    const int tyi = bid % a.nty;
    const int b = bid / a.nty;
    const int y0 = tyi * TY, x0 = txi * TX;
    const int oc0 = 32 * blockIdx.y;

    // ---- the maps' operand: lane (map lt, half lg) holds value 2j + lg of window row u for step u*SR + j
    float w[STEPS];
#pragma unroll
    for (int u = 0; u < K; ++u)
#pragma unroll
        for (int j = 0; j < SR; ++j) {
            const int r = 2 * j + lg;
            w[u * SR + j] = (r < R && oc0 + lt < a.Co) ? a.Wk[(long)(u * R + r) * a.Co + oc0 + lt] : 0.f;
        }
    v4f bias4[4];
#pragma unroll
    for (int n = 0; n < 4; ++n)
#pragma unroll
        for (int z = 0; z < 4; ++z) {
            const int c = oc0 + 8 * n + 4 * lg + z;
            bias4[n][z] = a.Wk[(long)K * R * a.Co + (c < a.Co ? c : a.Co - 1)];
        }

    // ---- the image tile; outside the image, and the padding value of each row: zeros
    const float* img = a.in + (long)b * a.Hi * a.Wi * C;
    for (int e = tid; e < HH * HWC; e += 256) {
        const int hy = e / HWC, hx = e - hy * HWC;
        const int iy = y0 + hy, ie = x0 * C + hx;
        tile[e] = (iy < a.Hi && ie < a.Wi * C && hx < (TX + K - 1) * C) ? img[(long)iy * a.Wi * C + ie] : 0.f;
    }
    __syncthreads();

    v16f acc[MP];
#pragma unroll
    for (int p = 0; p < MP; ++p)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[p][r] = 0.f;
    const float* base = tile + (wave * MP) * HWC + lt * C + lg;
#pragma unroll
    for (int u = 0; u < K; ++u)
#pragma unroll
        for (int j = 0; j < SR; ++j)
#pragma unroll
            for (int p = 0; p < MP; ++p)
                acc[p] = mfma_f32<32>(w[u * SR + j], base[(p + u) * HWC + 2 * j], acc[p]);

    // ---- epilogue: register 4n + z of position tile p is map oc0 + 8n + 4lg + z of position (row w*MP + p, column lt)
    const int x = x0 + lt;
#pragma unroll
    for (int p = 0; p < MP; ++p) {
        const int y = y0 + wave * MP + p;
        if (y >= a.Ho || x >= a.Wo) continue;
        float* o = a.out + (((long)b * a.Ho + y) * a.Wo + x) * a.Co;
#pragma unroll
        for (int n = 0; n < 4; ++n) {
            const int oc = oc0 + 8 * n + 4 * lg;
            if (oc >= a.Co) continue;
            v4f s = (v4f){acc[p][4 * n], acc[p][4 * n + 1], acc[p][4 * n + 2], acc[p][4 * n + 3]} + bias4[n];
            if (a.squash) {
#pragma unroll
                for (int z = 0; z < 4; ++z) s[z] = squash(s[z], a.squash == 2);
            }
            const int nv = a.Co - oc < 4 ? a.Co - oc : 4;
            if (nv == 4 && (a.Co & 3) == 0) store4(o + oc, s);
            else for (int z = 0; z < nv; ++z) o[oc + z] = s[z];
        }
    }
}

}  // namespace mpcnn
