// Fixed-order second stage of the split reductions (Alg. 2: the gradients of all fragments
// are summed): adds the per-workgroup partial sums of every layer, and the loss shares.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "storage.hpp"

namespace mpcnn {

// Second stage of the split reductions, all layers in one launch: out = sum over the n
// partial results of a segment.  64 items per workgroup, the n partials dealt to 4 thread
// rows; each adds its share in ascending order, then the 4 sums are added in a fixed order -
// the result does not depend on timing.  A flat segment's item is one float; a tiled
// segment (written by wgrad_mfma_kernel) has 128-bit items = 4 consecutive rows of one
// column, scattered to the parameter order [tap*Ci + c][o], bias row last.
constexpr int kMaxReduceSegs = 49;   // 48 layers and the loss
struct ReduceSeg {
    const float* partial;
    float* out;
    long plen;          // floats per partial
    int items, n, block0;
    int tiled, Nt, rows_total, Co;   // tiled: 0 flat, 1 tiled, 2 the per-workgroup loss shares (fp64), 3 tiled with the bias as row rows_total
};
struct ReduceArgs {
    ReduceSeg seg[kMaxReduceSegs];
    int n_seg, total_blocks;
    int accumulate;     // add to what `out` holds (the image comes in bands) instead of replacing it
};

__global__ __launch_bounds__(256) void reduce_all_kernel(ReduceArgs a)
{
    __shared__ double red[4][64][4];
    int si = 0;
    while (si + 1 < a.n_seg && (int)blockIdx.x >= a.seg[si + 1].block0) ++si;
    const ReduceSeg& sg = a.seg[si];
    const float* __restrict__ partial = sg.partial;
    const long plen = sg.plen;
    const int n = sg.n;
    const int col = threadIdx.x & 63, row = threadIdx.x >> 6;
    if (sg.tiled == 2) {
        // the summed loss: one workgroup adds the n fp64 shares in a fixed (tree) order
        double* tree = &red[0][0][0];   // 1024 doubles, 256 used
        const double* share = reinterpret_cast<const double*>(partial);
        double s = 0.0;
        for (int i = threadIdx.x; i < n; i += 256) s += share[i];
        tree[threadIdx.x] = s;
        __syncthreads();
        for (int w = 128; w > 0; w >>= 1) {
            if ((int)threadIdx.x < w) tree[threadIdx.x] += tree[threadIdx.x + w];
            __syncthreads();
        }
        if (threadIdx.x == 0) {
            double* o = reinterpret_cast<double*>(sg.out);
            *o = a.accumulate ? *o + tree[0] : tree[0];
        }
        return;
    }
    const int e = ((int)blockIdx.x - sg.block0) * 64 + col;
    const int per = (n + 3) >> 2;
    const int i0 = row * per, i1 = (i0 + per < n) ? i0 + per : n;
    if (!sg.tiled) {
        double s = 0.0;
        if (e < sg.items) {
            // the sum is bound by the round trips to memory: 8 loads in flight, 4 chains
            double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
            int i = i0;
            for (; i + 7 < i1; i += 8) {
                float u[8];
#pragma unroll
                for (int z = 0; z < 8; ++z) u[z] = partial[(long)(i + z) * plen + e];
                s0 += (double)u[0]; s1 += (double)u[1]; s2 += (double)u[2]; s3 += (double)u[3];
                s0 += (double)u[4]; s1 += (double)u[5]; s2 += (double)u[6]; s3 += (double)u[7];
            }
            for (; i < i1; ++i) s0 += (double)partial[(long)i * plen + e];
            s = (s0 + s1) + (s2 + s3);
        }
        red[row][col][0] = s;
        __syncthreads();
        if (row == 0 && e < sg.items) {
            const float r = (float)((red[0][col][0] + red[1][col][0]) + (red[2][col][0] + red[3][col][0]));
            sg.out[e] = a.accumulate ? sg.out[e] + r : r;
        }
        return;
    }
    double s[4] = {0.0, 0.0, 0.0, 0.0};
    if (e < sg.items) {
        double t[4] = {0.0, 0.0, 0.0, 0.0};
        const v4f* p4 = reinterpret_cast<const v4f*>(partial) + e;
        const long pl4 = plen >> 2;
        int i = i0;
        for (; i + 7 < i1; i += 8) {   // bound by the round trips to memory: 8 loads in flight
            v4f u[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) u[q] = p4[(long)(i + q) * pl4];
#pragma unroll
            for (int q = 0; q < 8; q += 2)
#pragma unroll
                for (int z = 0; z < 4; ++z) { s[z] += (double)u[q][z]; t[z] += (double)u[q + 1][z]; }
        }
        for (; i + 1 < i1; i += 2) {
            const v4f u = p4[(long)i * pl4], v = p4[(long)(i + 1) * pl4];
#pragma unroll
            for (int z = 0; z < 4; ++z) { s[z] += (double)u[z]; t[z] += (double)v[z]; }
        }
        if (i < i1) {
            const v4f u = p4[(long)i * pl4];
#pragma unroll
            for (int z = 0; z < 4; ++z) s[z] += (double)u[z];
        }
#pragma unroll
        for (int z = 0; z < 4; ++z) s[z] += t[z];
    }
#pragma unroll
    for (int z = 0; z < 4; ++z) red[row][col][z] = s[z];
    __syncthreads();
    if (row == 0 && e < sg.items) {
        float r[4];
#pragma unroll
        for (int z = 0; z < 4; ++z)
            r[z] = (float)((red[0][col][z] + red[1][col][z]) + (red[2][col][z] + red[3][col][z]));
        // the bias sums follow the result tiles, or (tiled == 3) are the row after the last
        const int tile_items = sg.tiled == 3 ? sg.items : sg.items - sg.Nt * 8;
        const int rows_out = sg.rows_total + (sg.tiled == 3 ? 1 : 0);
        if (e < tile_items) {
            const int tile = e >> 8, r4 = (e >> 6) & 3, l = e & 63;
            const int mt = tile / sg.Nt, nt = tile - mt * sg.Nt;
            const int row0 = 32 * mt + 8 * r4 + 4 * (l >> 5), oc = 32 * nt + (l & 31);
            if (oc < sg.Co)
#pragma unroll
                for (int z = 0; z < 4; ++z)
                    if (row0 + z < rows_out) {
                        float* o = sg.out + (long)(row0 + z) * sg.Co + oc;
                        *o = a.accumulate ? *o + r[z] : r[z];
                    }
        } else {
            const int oc = 4 * (e - tile_items);
#pragma unroll
            for (int z = 0; z < 4; ++z)
                if (oc + z < sg.Co) {
                    float* o = sg.out + (long)sg.rows_total * sg.Co + oc + z;
                    *o = a.accumulate ? *o + r[z] : r[z];
                }
        }
    }
}

}  // namespace mpcnn
