// First layer with bf16 storage on v_mfma_f32_32x32x16_bf16: a convolution over at most 4 input
// channels (the image), spacing 1, filter side at most 8, at most 64 output maps.  The layer
// is a product [positions] x [k*k*C] x [maps] with a short reduction, far too short for the
// general kernel's channel tiling, and on the vector ALU it is the slowest layer of an RGB net.
//
// Reduction index: a window row is padded to 8 pixels of 4 channels, 32 values = two
// instructions of 16; the padding meets zero weights.  A workgroup stages its image tile in LDS
// as [row][pixel][4 channels] (8 bytes per pixel), so that a lane's share of an A operand -
// two neighbouring pixels - is one aligned 64-bit word whatever the column (an LDS read off its
// natural alignment is served lane by lane).  The B operands, the whole filter bank, stay in
// registers: 2k sets of four per column tile.  One wave = 32 neighbouring positions of a row.
#pragma once
#include "storage.hpp"

namespace mpcnn {

typedef __bf16 fl_bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned fl_u32x2 __attribute__((ext_vector_type(2)));

constexpr int kFirstBmTy = 16, kFirstBmTx = 32;   // output tile of a workgroup; wave w takes rows w, w+4, ...

struct FirstBmArgs {
    const bf16* in;       // [B][Hi][Wi][Ci] channels-last image
    const float* Wk;      // [k*k*Ci][Co] then bias [Co] (values representable in bf16)
    bf16* out;            // [B][Ho][Wo][Co]
    int B, Hi, Wi, Ci, Ho, Wo, Co, k;
    int squash;           // 0 linear, 1 tanh, 2 logistic
    int ntx, nty;
};

template <int NT, int K>   // NT column tiles of 32 maps; K = filter side
__global__ __launch_bounds__(256) void first_layer_bm_kernel(FirstBmArgs a)
{
    constexpr int LW = kFirstBmTx + 8;                 // pixels per LDS row: a window row reads 8 from its column
    constexpr int LH = kFirstBmTy + K - 1;
    __shared__ __attribute__((aligned(16))) fl_u32x2 tile[LH * LW];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lm = lane & 31, lh = lane >> 5;

    // ---- B operands: lane (map lm, half lh) holds, for step s, the weights of window row s/2,
    // pixels 4*(s%2) + 2*lh and the next, 4 channels each
    fl_bf16x8 wv[NT][2 * K];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int o = 32 * t + lm;
#pragma unroll
        for (int s = 0; s < 2 * K; ++s) {
            const int u = s >> 1;
#pragma unroll
            for (int z = 0; z < 8; ++z) {
                const int v = 4 * (s & 1) + 2 * lh + (z >> 2), c = z & 3;
                float w = 0.f;
                if (v < K && c < a.Ci && o < a.Co) w = a.Wk[(long)((u * K + v) * a.Ci + c) * a.Co + o];
                wv[t][s][z] = (bf16)w;
            }
        }
    }
    float bias[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) bias[t] = 32 * t + lm < a.Co ? a.Wk[(long)K * K * a.Ci * a.Co + 32 * t + lm] : 0.f;

    // the workgroups share the tiles out among themselves: the filter bank is fetched once
    const int tiles = a.B * a.nty * a.ntx;
    for (int tidx = blockIdx.x; tidx < tiles; tidx += gridDim.x) {
    unsigned bid = tidx;
    const int txi = bid % a.ntx; bid /= a.ntx;
    const int tyi = bid % a.nty;
    const int b = bid / a.nty;
    const int y0 = tyi * kFirstBmTy, x0 = txi * kFirstBmTx;

    // ---- stage the tile: pixel (y0 + r, x0 + p), clamped to the image; channels past Ci are zero
    const bf16* img = a.in + (long)b * a.Hi * a.Wi * a.Ci;
    for (int e = tid; e < LH * LW; e += 256) {
        const int r = e / LW, p = e - r * LW;
        int iy = y0 + r, ix = x0 + p;
        iy = iy < a.Hi ? iy : a.Hi - 1;
        ix = ix < a.Wi ? ix : a.Wi - 1;
        const bf16* px = img + ((long)iy * a.Wi + ix) * a.Ci;
        unsigned short c[4] = {0, 0, 0, 0};
#pragma unroll
        for (int z = 0; z < 4; ++z)
            if (z < a.Ci) c[z] = __builtin_bit_cast(unsigned short, px[z]);
        tile[e] = (fl_u32x2){(unsigned)c[0] | ((unsigned)c[1] << 16), (unsigned)c[2] | ((unsigned)c[3] << 16)};
    }
    __syncthreads();

    for (int r = wave; r < kFirstBmTy; r += 4) {
        const int y = y0 + r;
        if (y >= a.Ho) break;                         // uniform per wave
        v16f acc[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int z = 0; z < 16; ++z) acc[t][z] = 0.f;
#pragma unroll
        for (int s = 0; s < 2 * K; ++s) {
            // A operand: position column lm, pixels lm + 4*(s%2) + 2*lh and the next of window row s/2
            const fl_u32x2* p = tile + (r + (s >> 1)) * LW + lm + 4 * (s & 1) + 2 * lh;
            const fl_u32x2 p0 = p[0], p1 = p[1];
            const unsigned q[4] = {p0[0], p0[1], p1[0], p1[1]};
            const fl_bf16x8 av = __builtin_bit_cast(fl_bf16x8, q);
#pragma unroll
            for (int t = 0; t < NT; ++t)
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, wv[t][s], acc[t], 0, 0, 0);
        }
        // result register z: position column 8*(z/4) + 4*lh + z%4, map lm of the column tile
        bf16* orow = a.out + (((long)b * a.Ho + y) * a.Wo + x0) * a.Co;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int o = 32 * t + lm;
#pragma unroll
            for (int z = 0; z < 16; ++z) {
                const int i = 8 * (z >> 2) + 4 * lh + (z & 3);
                if (x0 + i < a.Wo && o < a.Co) {
                    const float v = acc[t][z] + bias[t];
                    orow[(long)i * a.Co + o] = (bf16)(a.squash ? squash(v, a.squash == 2) : v);
                }
            }
        }
    }
    __syncthreads();   // every wave is done with the tile before the next one is staged
    }
}

}  // namespace mpcnn
