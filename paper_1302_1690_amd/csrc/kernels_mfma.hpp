// Matrix-core (MFMA, fp32) kernels for the dilated convolutions of the whole-image pass:
// forward and data gradient share one kernel, the weight gradient has its own.
//
// Tiling rule.  A layer whose taps are d elements apart never mixes the d*d residue
// classes (y mod d, x mod d) of its dense map - each class is one "fragment" of the
// paper's MPF storage (Method, MPF layer) and, seen alone, an ordinary undilated
// convolution.  So a workgroup takes a Ty x Tx tile of ONE class: its (Ty+k-1) x (Tx+k-1)
// input halo is staged once in LDS, each element a contiguous channel vector in the
// channels-last tensor, and is reused by all k*k taps.
//
// MFMA operand layout (v_mfma_f32_16x16x4_f32, 64 lanes): lane l supplies A[l%16][l/16] and
// B[l/16][l%16], and receives D[4*(l/16)+r][l%16] in register r.  The contraction index may
// be permuted freely as long as A and B agree, so every lane fetches FOUR consecutive
// channels with one 128-bit load and feeds them to four successive MFMAs.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mpcnn {

typedef float v4f __attribute__((ext_vector_type(4)));

enum ConvMode { kFwdTanh = 0, kFwdLinear = 1, kDgradTanh = 2, kDgradPlain = 3 };

struct ConvArgs {
    const float* in;     // [B][Hi][Wi][Cr]   tensor the taps read (activations, or deltas for dgrad)
    const v4f* wpack;    // [steps][4][CoPad] x 4 channels, steps = k*k*CrPad/16
    const float* bias;   // [Co]   (forward modes)
    const float* act;    // [B][Ho][Wo][Co] tanh output at the positions written (kDgradTanh)
    float* out;          // [B][Ho][Wo][Co]
    int B, Hi, Wi, Cr, CrPad;
    int Ho, Wo, Co, CoPad;
    int k, d;
    int origin;          // halo origin in fragment units relative to the tile: 0 forward, -(k-1) dgrad
    int Ty, Tx, nty, ntx;
    int mode;
};

// Repack W[tap][c][o] (+ bias row) into the operand order of conv_mfma_kernel.
//   forward : reduce over c, outputs o:  P[tap*nch + ch][g][o][s]  = W[tap][16ch+4g+s][o]
//   dgrad   : reduce over o, outputs c:  P[tap'*nch + ch][g][c][s] = W[k*k-1-tap'][c][16ch+4g+s]
// (taps reversed: the data gradient at x collects deltas at x - u*d).  Padding is zero.
__global__ void pack_weights_kernel(const float* __restrict__ W, float* __restrict__ P, int kk,
                                    int Ci, int Co, int RPad, int OPad, int dgrad)
{
    const int nch = RPad / 16;
    long total = (long)kk * nch * 4 * OPad * 4;
    for (long e = (long)blockIdx.x * blockDim.x + threadIdx.x; e < total;
         e += (long)gridDim.x * blockDim.x) {
        int s = (int)(e & 3);
        long q = e >> 2;
        int oo = (int)(q % OPad); q /= OPad;
        int g = (int)(q & 3); q >>= 2;
        int ch = (int)(q % nch);
        int tap = (int)(q / nch);
        int r = 16 * ch + 4 * g + s;  // index along the reduced dimension
        float v = 0.f;
        if (!dgrad) {
            if (r < Ci && oo < Co) v = W[((long)tap * Ci + r) * Co + oo];
        } else {
            if (r < Co && oo < Ci) v = W[((long)(kk - 1 - tap) * Ci + oo) * Co + r];
        }
        P[e] = v;
    }
}

// Forward / data gradient of one dilated convolution as an implicit GEMM.
// Workgroup = 256 threads = 4 waves; tile = 16*PT positions of one residue class x 16*OT
// output channels (blockIdx.y selects the group of OT channel tiles).  All four waves hold
// the full tile in accumulators and each sums a quarter of the k*k*CrPad/16 reduction
// steps; the four partial tiles meet in LDS, where all 256 threads add them in wave order,
// apply the epilogue and store.  Summation order is the same for every position, so equal
// inputs give bit-equal outputs (exact pooling ties stay exact).
template <int OT, int PT>
__global__ __launch_bounds__(256, 2) void conv_mfma_kernel(ConvArgs a)
{
    extern __shared__ __attribute__((aligned(16))) float lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 15, lg = lane >> 4;

    int bid = blockIdx.x;
    const int txi = bid % a.ntx; bid /= a.ntx;
    const int tyi = bid % a.nty; bid /= a.nty;
    const int rx = bid % a.d; bid /= a.d;
    const int ry = bid % a.d;
    const int b = bid / a.d;
    const int fh = ry < a.Ho ? (a.Ho - ry + a.d - 1) / a.d : 0;  // extent of this residue class
    const int fw = rx < a.Wo ? (a.Wo - rx + a.d - 1) / a.d : 0;
    const int ty0 = tyi * a.Ty, tx0 = txi * a.Tx;
    if (ty0 >= fh || tx0 >= fw) return;  // uniform for the workgroup

    const int hw = a.Tx + a.k - 1, hh = a.Ty + a.k - 1;
    const int Cs = a.CrPad + 4;  // row pitch of the halo in floats (pad: bank spread)
    const int cq = a.CrPad >> 2;

    // ---- stage the halo: zero outside the tensor and in the channel padding
    for (int it = tid; it < hh * hw * cq; it += 256) {
        const int pos = it / cq, q = it - pos * cq;
        const int ha = pos / hw, hb = pos - ha * hw;
        const int fy = ty0 + ha + a.origin, fx = tx0 + hb + a.origin;
        const int iy = fy * a.d + ry, ix = fx * a.d + rx;
        v4f v = {0.f, 0.f, 0.f, 0.f};
        if (fy >= 0 && fx >= 0 && iy < a.Hi && ix < a.Wi && 4 * q < a.Cr)
            v = *reinterpret_cast<const v4f*>(a.in + (((long)b * a.Hi + iy) * a.Wi + ix) * a.Cr + 4 * q);
        *reinterpret_cast<v4f*>(lds + pos * Cs + 4 * q) = v;
    }

    // ---- per-lane halo offsets of the PT positions this lane feeds as the B operand
    int lbase[PT];
#pragma unroll
    for (int pt = 0; pt < PT; ++pt) {
        int m = 16 * pt + li;
        int ty = m / a.Tx, tx = m - ty * a.Tx;
        if (ty >= a.Ty) { ty = 0; tx = 0; }  // padding position: any in-bounds address
        lbase[pt] = (ty * hw + tx) * Cs + 4 * lg;
    }

    const int nch = a.CrPad >> 4;
    const int steps = a.k * a.k * nch;
    const int t0 = (steps * wave) >> 2, t1 = (steps * (wave + 1)) >> 2;
    const int ot0 = blockIdx.y * OT;
    const v4f* wp = a.wpack + (long)lg * a.CoPad + 16 * ot0 + li;

    v4f acc[OT][PT];
#pragma unroll
    for (int o = 0; o < OT; ++o)
#pragma unroll
        for (int p = 0; p < PT; ++p) acc[o][p] = (v4f){0.f, 0.f, 0.f, 0.f};

    __syncthreads();

    // step t = tap * nch + chunk; the running tap offset avoids divisions
    int tap = t0 / nch, chunk = t0 - tap * nch;
    int ta = tap / a.k, tb = tap - ta * a.k;
    // weights come from global memory (long latency): fetched one step ahead into a second
    // register set; activations come from LDS and are fetched just before use
    v4f wv[OT], wn[OT], av[PT];
#pragma unroll
    for (int o = 0; o < OT; ++o) wn[o] = wv[o] = (v4f){0.f, 0.f, 0.f, 0.f};
    if (t0 < t1) {
#pragma unroll
        for (int o = 0; o < OT; ++o) wv[o] = wp[(long)t0 * 4 * a.CoPad + 16 * o];
    }
    for (int t = t0; t < t1; ++t) {
        if (t + 1 < t1) {
#pragma unroll
            for (int o = 0; o < OT; ++o) wn[o] = wp[(long)(t + 1) * 4 * a.CoPad + 16 * o];
        }
        const int soff = (ta * hw + tb) * Cs + 16 * chunk;
#pragma unroll
        for (int p = 0; p < PT; ++p) av[p] = *reinterpret_cast<const v4f*>(lds + lbase[p] + soff);
        if (++chunk == nch) { chunk = 0; if (++tb == a.k) { tb = 0; ++ta; } }
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int o = 0; o < OT; ++o)
#pragma unroll
                for (int p = 0; p < PT; ++p)
                    acc[o][p] = __builtin_amdgcn_mfma_f32_16x16x4f32(wv[o][s], av[p][s], acc[o][p], 0, 0, 0);
#pragma unroll
        for (int o = 0; o < OT; ++o) wv[o] = wn[o];
    }

    // ---- meet in LDS: part[wave][ot][pos li][quad lg] as 128-bit items, one position tile per round
    v4f* part = reinterpret_cast<v4f*>(lds);
#pragma unroll
    for (int pt = 0; pt < PT; ++pt) {
        __syncthreads();  // halo (or the previous round) no longer needed
#pragma unroll
        for (int o = 0; o < OT; ++o) part[((wave * OT + o) * 16 + li) * 4 + lg] = acc[o][pt];
        __syncthreads();
        for (int e = tid; e < OT * 64; e += 256) {
            const int o = e >> 6, rem = e & 63, i = rem >> 2, g = rem & 3;
            const int m = 16 * pt + i;
            const int ty = m / a.Tx, tx = m - ty * a.Tx;
            const int fy = ty0 + ty, fx = tx0 + tx;
            if (ty >= a.Ty || fy >= fh || fx >= fw) continue;
            v4f s = part[((0 * OT + o) * 16 + i) * 4 + g];
            s += part[((1 * OT + o) * 16 + i) * 4 + g];
            s += part[((2 * OT + o) * 16 + i) * 4 + g];
            s += part[((3 * OT + o) * 16 + i) * 4 + g];
            const int oc = 16 * (ot0 + o) + 4 * g;
            if (oc >= a.Co) continue;
            const long off = (((long)b * a.Ho + (fy * a.d + ry)) * a.Wo + (fx * a.d + rx)) * a.Co + oc;
            const int nv = a.Co - oc < 4 ? a.Co - oc : 4;
            float r[4] = {s[0], s[1], s[2], s[3]};
            if (a.mode == kFwdTanh) {
                for (int q = 0; q < nv; ++q) r[q] = tanhf(r[q] + a.bias[oc + q]);
            } else if (a.mode == kFwdLinear) {
                for (int q = 0; q < nv; ++q) r[q] += a.bias[oc + q];
            } else if (a.mode == kDgradTanh) {
                for (int q = 0; q < nv; ++q) {
                    float y = a.act[off + q];
                    r[q] *= 1.f - y * y;
                }
            }
            if (nv == 4 && (a.Co & 3) == 0) {
                *reinterpret_cast<v4f*>(a.out + off) = (v4f){r[0], r[1], r[2], r[3]};
            } else {
                for (int q = 0; q < nv; ++q) a.out[off + q] = r[q];
            }
        }
    }
}

struct WgradArgs {
    const float* in;     // [B][Hi][Wi][Ci]  layer input (activations)
    const float* dY;     // [B][Ho][Wo][Co]  delta w.r.t. the layer's pre-activation
    float* partial;      // [slabs][(k*k*Ci + 1) * Co]
    int B, Hi, Wi, Ci;
    int Ho, Wo, Co;
    int k, d;
    int Ty, Tx, nty, ntx;  // Ty*Tx <= 64
    int tiles_total, tiles_per_slab;
    int rtiles_total;      // ceil(k*k*Ci / 16) tiles of 16 gradient rows, row = tap*Ci + c
    int rtiles_per_group;  // row tiles handled by one blockIdx.y
};

// Weight gradient dW[tap][c][o] = sum over positions of in[pos + tap][c] * dY[pos][o]
// (Alg. 2: the same gradient function applied to every fragment, results summed).
// MFMA rows = 16 consecutive gradient rows (tap, c) in parameter order, columns = 16 output
// channels, contraction over positions.  blockIdx.x = slab of position tiles (partial sums,
// added later in slab order), blockIdx.y = group of row tiles, blockIdx.z = group of OT
// output tiles.  Inside a workgroup the row tiles are dealt round-robin to the 4 waves; each
// wave keeps NP x OT accumulator tiles in registers across its whole slab.
template <int NP, int OT>
__global__ __launch_bounds__(256, 1) void wgrad_mfma_kernel(WgradArgs a)
{
    extern __shared__ __attribute__((aligned(16))) float lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 15, lg = lane >> 4;
    const int hw = a.Tx + a.k - 1, hh = a.Ty + a.k - 1;
    const int Cs = a.Ci | 1;           // halo pitch (floats): odd, spreads the 4 positions read together
    const int Ds = 16 * OT + 1;        // delta tile pitch
    float* halo = lds;
    float* dtile = halo + hh * hw * Cs;
    int* hbt = reinterpret_cast<int*>(dtile + 64 * Ds);  // position -> halo index

    const int rows_total = a.k * a.k * a.Ci;
    const int ot0 = blockIdx.z * OT;
    const int rt0 = blockIdx.y * a.rtiles_per_group;
    int rend = rt0 + a.rtiles_per_group;
    if (rend > a.rtiles_total) rend = a.rtiles_total;
    // this wave's row tiles: rt0 + wave + 4*p; this lane feeds row 16*tile + li of each
    int poff[NP];   // LDS offset of that row's (tap, c) relative to a position's halo slot
    int np = 0;
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        const int q = rt0 + wave + 4 * p;
        poff[p] = 0;
        if (q < rend) {
            np = p + 1;
            const int row = 16 * q + li;
            if (row < rows_total) {
                const int tap = row / a.Ci, c = row - tap * a.Ci;
                const int ta = tap / a.k, tb = tap - ta * a.k;
                poff[p] = (ta * hw + tb) * Cs + c;
            }
        }
    }
    if (tid < 64) {
        int ty = tid / a.Tx, tx = tid - ty * a.Tx;
        hbt[tid] = (ty < a.Ty) ? (ty * hw + tx) * Cs : 0;
    }

    v4f acc[NP][OT];
#pragma unroll
    for (int p = 0; p < NP; ++p)
#pragma unroll
        for (int o = 0; o < OT; ++o) acc[p][o] = (v4f){0.f, 0.f, 0.f, 0.f};
    float bsum[OT];
#pragma unroll
    for (int o = 0; o < OT; ++o) bsum[o] = 0.f;

    const int tile_begin = blockIdx.x * a.tiles_per_slab;
    int tile_end = tile_begin + a.tiles_per_slab;
    if (tile_end > a.tiles_total) tile_end = a.tiles_total;
    const int cq = (a.Ci + 3) >> 2;
    const bool vec_in = (a.Ci & 3) == 0, vec_dy = (a.Co & 3) == 0;

    for (int tile = tile_begin; tile < tile_end; ++tile) {
        int bid = tile;
        const int txi = bid % a.ntx; bid /= a.ntx;
        const int tyi = bid % a.nty; bid /= a.nty;
        const int rx = bid % a.d; bid /= a.d;
        const int ry = bid % a.d;
        const int b = bid / a.d;
        const int fh = ry < a.Ho ? (a.Ho - ry + a.d - 1) / a.d : 0;
        const int fw = rx < a.Wo ? (a.Wo - rx + a.d - 1) / a.d : 0;
        const int ty0 = tyi * a.Ty, tx0 = txi * a.Tx;
        if (ty0 >= fh || tx0 >= fw) continue;  // uniform
        __syncthreads();                        // previous tile fully consumed
        // input halo: zero outside the input tensor
        for (int it = tid; it < hh * hw * cq; it += 256) {
            const int pos = it / cq, q = it - pos * cq;
            const int ha = pos / hw, hb = pos - ha * hw;
            const int iy = (ty0 + ha) * a.d + ry, ix = (tx0 + hb) * a.d + rx;
            float v[4] = {0.f, 0.f, 0.f, 0.f};
            const int nv = a.Ci - 4 * q < 4 ? a.Ci - 4 * q : 4;
            if (iy < a.Hi && ix < a.Wi) {
                const float* src = a.in + (((long)b * a.Hi + iy) * a.Wi + ix) * a.Ci + 4 * q;
                if (vec_in) {
                    v4f t = *reinterpret_cast<const v4f*>(src);
                    v[0] = t[0]; v[1] = t[1]; v[2] = t[2]; v[3] = t[3];
                } else {
                    for (int z = 0; z < nv; ++z) v[z] = src[z];
                }
            }
            float* dst = halo + pos * Cs + 4 * q;
            for (int z = 0; z < nv; ++z) dst[z] = v[z];
        }
        // delta tile: zero for padding positions and padding channels
        for (int it = tid; it < 64 * 4 * OT; it += 256) {
            const int m = it / (4 * OT), q = it - m * (4 * OT);
            const int ty = m / a.Tx, tx = m - ty * a.Tx;
            const int fy = ty0 + ty, fx = tx0 + tx;
            const int oc = 16 * ot0 + 4 * q;
            float v[4] = {0.f, 0.f, 0.f, 0.f};
            if (ty < a.Ty && fy < fh && fx < fw && oc < a.Co) {
                const float* src = a.dY + (((long)b * a.Ho + (fy * a.d + ry)) * a.Wo + (fx * a.d + rx)) * a.Co + oc;
                if (vec_dy) {
                    v4f t = *reinterpret_cast<const v4f*>(src);
                    v[0] = t[0]; v[1] = t[1]; v[2] = t[2]; v[3] = t[3];
                } else {
                    for (int z = 0; z < 4; ++z) if (oc + z < a.Co) v[z] = src[z];
                }
            }
            float* dst = dtile + m * Ds + 4 * q;
            dst[0] = v[0]; dst[1] = v[1]; dst[2] = v[2]; dst[3] = v[3];
        }
        __syncthreads();
#pragma unroll 2
        for (int kk = 0; kk < 16; ++kk) {
            const int m = 4 * kk + lg;  // the position this lane contributes to the contraction
            const int hb = hbt[m];
            float bop[OT];
#pragma unroll
            for (int o = 0; o < OT; ++o) {
                bop[o] = dtile[m * Ds + 16 * o + li];
                bsum[o] += bop[o];
            }
#pragma unroll
            for (int p = 0; p < NP; ++p) {
                if (p < np) {
                    const float aop = halo[hb + poff[p]];
#pragma unroll
                    for (int o = 0; o < OT; ++o)
                        acc[p][o] = __builtin_amdgcn_mfma_f32_16x16x4f32(aop, bop[o], acc[p][o], 0, 0, 0);
                }
            }
        }
    }

    // ---- write this slab's partial sums in parameter order (row-major [tap*Ci + c][o]), bias row last
    const long plen = ((long)rows_total + 1) * a.Co;
    float* out = a.partial + (long)blockIdx.x * plen;
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        if (p < np) {
            const int q = rt0 + wave + 4 * p;
#pragma unroll
            for (int o = 0; o < OT; ++o) {
                const int oc = 16 * (ot0 + o) + li;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int row = 16 * q + 4 * lg + r;
                    if (row < rows_total && oc < a.Co) out[(long)row * a.Co + oc] = acc[p][o][r];
                }
            }
        }
    }
    // bias gradient = column sums of the delta tiles; one wave of the first row group owns it
    if (blockIdx.y == 0) {
        __syncthreads();
        float* red = lds;  // [4 lane groups][16*OT]
        if (wave == 0) {
#pragma unroll
            for (int o = 0; o < OT; ++o) red[lg * 16 * OT + 16 * o + li] = bsum[o];
        }
        __syncthreads();
        if (tid < 16 * OT) {
            const int oc = 16 * ot0 + tid;
            if (oc < a.Co)
                out[(long)rows_total * a.Co + oc] =
                    (red[tid] + red[16 * OT + tid]) + (red[32 * OT + tid] + red[48 * OT + tid]);
        }
    }
}

// Second stage of the split reductions: out[e] = sum_{i<n} partial[i][e].  64 columns per
// workgroup, the n rows dealt to 4 thread rows; each adds its rows in ascending order, then
// the 4 sums are added in a fixed order - the result does not depend on timing.
__global__ __launch_bounds__(256) void reduce_rows_kernel(const float* __restrict__ partial,
                                                          float* __restrict__ out, long len, int n)
{
    __shared__ double red[4][64];
    const int col = threadIdx.x & 63, row = threadIdx.x >> 6;
    const long e = (long)blockIdx.x * 64 + col;
    double s = 0.0;
    if (e < len) {
        const int per = (n + 3) >> 2;
        const int i0 = row * per, i1 = (i0 + per < n) ? i0 + per : n;
        double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;  // independent chains: loads in flight
        int i = i0;
        for (; i + 3 < i1; i += 4) {
            s0 += (double)partial[(long)i * len + e];
            s1 += (double)partial[(long)(i + 1) * len + e];
            s2 += (double)partial[(long)(i + 2) * len + e];
            s3 += (double)partial[(long)(i + 3) * len + e];
        }
        for (; i < i1; ++i) s0 += (double)partial[(long)i * len + e];
        s = (s0 + s1) + (s2 + s3);
    }
    red[row][col] = s;
    __syncthreads();
    if (row == 0 && e < len) out[e] = (float)((red[0][col] + red[1][col]) + (red[2][col] + red[3][col]));
}

}  // namespace mpcnn
