// Weight and bias gradient of the image layer (1 or 3 input channels, spacing 1, filter side 3, 5 or 7,
// Method: step 3 of back-propagation, Alg. 2 for the sum over positions) on v_mfma_f32_32x32x2_f32, in
// either storage type.  The general weight-gradient kernels tile the input by channel quads or octets;
// with an image's few channels most of what they stage and multiply is padding (12-58 TFLOP/s).
//
// The gradient is the product [k rows of k*C values] x [positions] x [maps], contracted over positions.
// A window row's k*C values are contiguous in a channels-last image, so gradient row m = u*(k*C) + r (which
// is the parameter row (u*k + v)*C + c itself) reads, for the position pair (2s, 2s + 1) of a tile row, the
// word at  lane base + (u row pitch + r) + (2s + half)*C  of the image tile in LDS: per 32 gradient rows one
// 32-bit LDS read at an immediate offset and one matrix instruction; the maps' operand is one read of the
// delta tile, [position][map] in LDS, shared by all row tiles.  Both tiles are staged as fp32.
// A workgroup walks tiles of 8 rows x 32 columns of positions (wave w: rows 2w, 2w + 1) and keeps its sums
// in accumulators; at the end the four waves' sums meet in LDS in a fixed order and the workgroup writes
// one partial result in parameter order, bias row last (added by reduce_all_kernel, flat segments).
#pragma once
#include "kernels_mfma.hpp"

namespace mpcnn {

constexpr int kL0wTy = 8, kL0wTx = 32;

struct L0WgradArgs {
    const void* in;       // [B][Hi][Wi][C] channels-last image (T)
    const void* dY;       // [B][Ho][Wo][Co] delta at the layer's output (T)
    float* partial;       // [workgroups][(k*k*C + 1) * Co]
    int B, Hi, Wi, Ho, Wo, Co;
    int ntx, nty, tiles_total;
};

template <int K, int C, typename T>
__global__ __launch_bounds__(256) void l0_wgrad_mfma_kernel(L0WgradArgs a)
{
    constexpr int R = K * C, ROWS = K * R, MT = (ROWS + 31) / 32;
    constexpr int TY = kL0wTy, TX = kL0wTx, HH = TY + K - 1, HWC = (TX + K - 1) * C;
    constexpr int XT = (HH * HWC + 3) & ~3;                // floats of the image tile
    __shared__ __attribute__((aligned(16))) float smem[XT + TY * TX * 32];
    float* xt = smem;                                       // [HH][HWC]
    float* dt = smem + XT;                                  // [TY*TX][32 maps]
    const T* in_t = static_cast<const T*>(a.in);
    const T* dy_t = static_cast<const T*>(a.dY);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lt = lane & 31, lg = lane >> 5;
    const int oc0 = 32 * blockIdx.y;
    const int nco = a.Co - oc0 < 32 ? a.Co - oc0 : 32;      // maps of this slice

    // gradient row of this lane in row tile mt: offset of its value for position 0 of tile row 0
    int roff[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int m = 32 * mt + lt;
        roff[mt] = m < ROWS ? (m / R) * HWC + (m % R) : 0;  // rows past the last: any in-bounds word, never stored
    }
    v16f acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[mt][r] = 0.f;
    float bsum = 0.f;

    // A tile's values wait in registers while the tile before it is multiplied: the loads are issued
    // before the matrix instructions of the current tile and written to LDS after them.
    constexpr int XN = (HH * HWC + 255) / 256;              // image values per thread
    float xr[XN];
    v4f dr[8];                                              // 8 quads of deltas, or 32 single ones
    const bool quads = (a.Co & 3) == 0;
    auto fetch = [&](int t) {
        int bid = t;
        const int txi = bid % a.ntx; bid /= a.ntx;
        const int tyi = bid % a.nty;
        const int b = bid / a.nty;
        const int y0 = tyi * TY, x0 = txi * TX;
        // outside the image: zeros; outside the map, and maps past the last: zeros (a zero delta
        // contributes nothing whatever the image value)
        const T* img = in_t + (long)b * a.Hi * a.Wi * C;
#pragma unroll
        for (int i = 0; i < XN; ++i) {
            const int e = tid + 256 * i;
            const int hy = e / HWC, hx = e - hy * HWC;
            const int iy = y0 + hy, ie = x0 * C + hx;
            const bool ok = e < HH * HWC && iy < a.Hi && ie < a.Wi * C;
            xr[i] = load1(img + (ok ? (long)iy * a.Wi * C + ie : 0));
            if (!ok) xr[i] = 0.f;
        }
        const T* dyb = dy_t + (long)b * a.Ho * a.Wo * a.Co;
        if (quads) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int e = tid + 256 * i, pos = e >> 3, q = e & 7;
                const int y = y0 + pos / TX, x = x0 + pos % TX;
                const bool ok = y < a.Ho && x < a.Wo && 4 * q < nco;
                dr[i] = load4(dyb + (ok ? ((long)y * a.Wo + x) * a.Co + oc0 + 4 * q : 0));
                if (!ok) dr[i] = (v4f){0.f, 0.f, 0.f, 0.f};
            }
        } else {
#pragma unroll
            for (int i = 0; i < 32; ++i) {
                const int e = tid + 256 * i, pos = e >> 5, o = e & 31;
                const int y = y0 + pos / TX, x = x0 + pos % TX;
                const bool ok = y < a.Ho && x < a.Wo && o < nco;
                const float v = load1(dyb + (ok ? ((long)y * a.Wo + x) * a.Co + oc0 + o : 0));
                dr[i >> 2][i & 3] = ok ? v : 0.f;
            }
        }
    };
    auto deposit = [&]() {
#pragma unroll
        for (int i = 0; i < XN; ++i)
            if (tid + 256 * i < HH * HWC) xt[tid + 256 * i] = xr[i];
        if (quads) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int e = tid + 256 * i;
                *reinterpret_cast<v4f*>(dt + (e >> 3) * 32 + 4 * (e & 7)) = dr[i];
            }
        } else {
#pragma unroll
            for (int i = 0; i < 32; ++i) dt[tid + 256 * i] = dr[i >> 2][i & 3];
        }
    };
    fetch(blockIdx.x);                                      // (the launch has no more workgroups than tiles)
    for (int t = blockIdx.x; t < a.tiles_total; t += gridDim.x) {
        deposit();
        __syncthreads();
        const int tn = t + gridDim.x;
        fetch(tn < a.tiles_total ? tn : t);                 // (a last tile fetches itself again: same loads on every path)
        // ---- this wave's two tile rows: 16 position pairs each, MT matrix instructions per pair
#pragma unroll
        for (int rw = 0; rw < 2; ++rw) {
            const int ty = 2 * wave + rw;
            const float* xa = xt + ty * HWC + lg * C;
            const float* db = dt + (ty * TX + lg) * 32 + lt;
#pragma unroll
            for (int s = 0; s < TX / 2; ++s) {
                const float bv = db[2 * s * 32];
                bsum += bv;
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) acc[mt] = mfma_f32<32>(xa[roff[mt] + 2 * s * C], bv, acc[mt]);
            }
        }
        __syncthreads();
    }

    // ---- the four waves' sums meet in LDS, wave after wave; then one partial result in parameter order
    float* red = smem;                                      // [MT*32 rows][32 maps], then the bias row
    static_assert(MT * 1024 + 32 <= XT + TY * TX * 32, "the sums fit the tiles' space");
    bsum += __shfl_xor(bsum, 32, 64);                       // both position halves of a map
    for (int w = 0; w < 4; ++w) {
        if (wave == w) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = 32 * mt + 8 * (r >> 2) + 4 * lg + (r & 3);   // register 4n + z: row 8n + 4lg + z, column lt
                    float* p = red + row * 32 + lt;
                    *p = w == 0 ? acc[mt][r] : *p + acc[mt][r];
                }
            if (lg == 0) {
                float* p = red + MT * 1024 + lt;
                *p = w == 0 ? bsum : *p + bsum;
            }
        }
        __syncthreads();
    }
    // partial results: workgroup (x, y) owns slot x; slice y fills its own maps of that slot
    float* part = a.partial + (long)blockIdx.x * ((long)ROWS + 1) * a.Co;
    for (int e = tid; e < (ROWS + 1) * 32; e += 256) {
        const int row = e >> 5, o = e & 31;
        if (o < nco) part[(long)row * a.Co + oc0 + o] = row < ROWS ? red[row * 32 + o] : red[MT * 1024 + o];
    }
}

}  // namespace mpcnn
