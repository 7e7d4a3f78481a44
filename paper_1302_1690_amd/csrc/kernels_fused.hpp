// Bandwidth-bound steps of the whole-image pass, each written so that every tensor is
// read or written once, in channels-last order [B][rows][cols][C]:
//   first_layer_kernel   conv + bias + tanh for a layer with very few input channels (shapes the
//                        matrix-instruction kernels of the image layer do not take)
//   maxfilter_fwd4 / maxfilter_bwd4   stride-1 max filter / routing by argmax, 4 channels per thread
//   class_layer_kernel   last FC (1x1) + softmax + cross-entropy + its own backward
// (step numbers a0 .. a8 in the comments: see the list at the top of kernels_direct.hpp)
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels_mfma.hpp"

namespace mpcnn {

// Conv + bias + tanh when the input has too few channels for the matrix cores (the image
// itself: 1 or 3 channels).  One thread = one position x 4 output channels, the quads of a
// position in neighbouring lanes: a wave's stores are contiguous, its tap loads are shared
// by the lanes of a position, and there are enough waves to hide the load latency.  The taps
// of one filter row are fetched together, without branches.  The weights (a few KB) sit in
// LDS, zero-padded to whole quads, bias row last; if they do not fit (`w_in_lds` = 0) they
// are read from global memory.
constexpr int kFirstLayerBatch = 8;   // taps of a filter row fetched together
template <typename T>
__global__ __launch_bounds__(256) void first_layer_kernel(const T* __restrict__ A,
                                                          const float* __restrict__ Wk,
                                                          T* __restrict__ Y, int B, int Hi, int Wi,
                                                          int Ci, int Ho, int Wo, int Co, int k, int k2, int d,
                                                          int d2, int tanh_out, int w_in_lds)
{
    extern __shared__ __attribute__((aligned(16))) float wl[];   // [(k*k*Ci + 1)][CoP]
    const int OG = (Co + 3) >> 2, CoP = 4 * OG;
    const int rows = k * k2 * Ci + 1;
    if (w_in_lds) {
        for (int e = threadIdx.x; e < rows * CoP; e += 256) {
            const int r = e / CoP, o = e - r * CoP;
            wl[e] = o < Co ? Wk[(long)r * Co + o] : 0.f;
        }
        __syncthreads();
    }
    const long total = (long)B * Ho * Wo * OG;
    const long e = (long)blockIdx.x * 256 + threadIdx.x;
    if (e >= total) return;
    const long m = e / OG;                            // position
    const int o0 = 4 * (int)(e - m * OG);
    const int b = (int)(m / ((long)Ho * Wo));
    const int r = (int)(m - (long)b * Ho * Wo);       // position within the image: 32-bit from here on
    const int y = r / Wo, x = r - y * Wo;
    v4f acc = {0.f, 0.f, 0.f, 0.f};
    for (int u = 0; u < k; ++u) {
        const T* arow = A + (((long)b * Hi + (y + u * d)) * Wi + x) * Ci;
        for (int c = 0; c < Ci; ++c)
            for (int v0 = 0; v0 < k2; v0 += kFirstLayerBatch) {
                // no branches around the loads (they would be waited for one by one): taps past
                // the filter's edge read the last tap again and count as zero
                float av[kFirstLayerBatch];
                v4f w[kFirstLayerBatch];
#pragma unroll
                for (int j = 0; j < kFirstLayerBatch; ++j) {
                    const int v = v0 + j < k2 ? v0 + j : k2 - 1;
                    av[j] = load1(arow + (long)v * d2 * Ci + c);
                    const int wr = (u * k2 + v) * Ci + c;
                    if (w_in_lds) w[j] = *reinterpret_cast<const v4f*>(wl + wr * CoP + o0);
                    else {
#pragma unroll
                        for (int z = 0; z < 4; ++z) w[j][z] = o0 + z < Co ? Wk[(long)wr * Co + o0 + z] : 0.f;
                    }
                }
#pragma unroll
                for (int j = 0; j < kFirstLayerBatch; ++j) {
                    const float xj = v0 + j < k2 ? av[j] : 0.f;
#pragma unroll
                    for (int z = 0; z < 4; ++z) acc[z] = fmaf(xj, w[j][z], acc[z]);
                }
            }
    }
#pragma unroll
    for (int z = 0; z < 4; ++z) {
        const int o = o0 + z < Co ? o0 + z : Co - 1;
        const float s = acc[z] + (w_in_lds ? wl[(rows - 1) * CoP + o] : Wk[(long)(rows - 1) * Co + o]);
        acc[z] = tanh_out ? squash(s, tanh_out == 2) : s;   // 0 linear, 1 tanh, 2 logistic
    }
    T* out = Y + m * Co + o0;
    if ((Co & 3) == 0) store4(out, acc);
    else {
#pragma unroll
        for (int z = 0; z < 4; ++z)
            if (o0 + z < Co) store1(out + z, acc[z]);
    }
}

// Index plumbing of the two max-filter kernels.  A workgroup takes 256 consecutive
// (column, channel quad) items of one map row.  Workgroups are handed to the 8 XCDs in
// turn, so the launch index is first turned into a position in eight contiguous bands of
// the row sequence, one per XCD.  The sequence walks an image's rows one residue class
// (row mod d) after the other - rows r, r + d, r + 2d, ..: the two rows a window straddles
// (d apart) are then neighbours in the sequence, so the second row of one window is still
// in that XCD's L2 when it comes up as the first row of the next (in plain row order d rows
// of the map lie between the two uses, which at d = 8 and 128 channels is more than an L2
// holds: every row was fetched from memory twice).
// All divisions are by launch constants: multiply-high with ceil(2^32 / x) (exact for
// n * x < 2^32, x > 1).
struct RowGrid {
    int gx;            // workgroups per map row
    int rows;          // B * (rows of the map the threads walk)
    int h;             // rows per image
    int C4;            // channel quads
    unsigned mg_gx, mg_h, mg_c4;
    int d;             // tap spacing (row order: residue classes mod d, one after the other)
    int n1, rem;       // the first `rem` classes have n1 = ceil(h / d) rows, the others n1 - 1
    unsigned mg_n1, mg_n0;
};
__device__ __forceinline__ unsigned rg_div(unsigned n, unsigned magic, unsigned x)
{
    return x == 1 ? n : __umulhi(n, magic);
}
// -> false if this thread has no item; else image b, row y, column x, channel quad c4
__device__ __forceinline__ bool rg_locate(const RowGrid& g, int width, int* b, int* y, int* x, int* c4)
{
    const unsigned nb = gridDim.x, i = blockIdx.x;
    const unsigned q = nb >> 3, r = nb & 7, xcd = i & 7;
    const unsigned lb = xcd * q + (xcd < r ? xcd : r) + (i >> 3);   // band of this XCD, then its turn
    const unsigned row = rg_div(lb, g.mg_gx, g.gx), bx = lb - row * g.gx;
    const unsigned it = bx * 256 + threadIdx.x;
    if (it >= (unsigned)(width * g.C4)) return false;
    const unsigned xx = rg_div(it, g.mg_c4, g.C4);
    const unsigned bb = rg_div(row, g.mg_h, g.h);
    unsigned t = row - bb * g.h;                     // place in the image's row sequence -> row
    if (g.d > 1) {
        const unsigned big = (unsigned)(g.rem * g.n1);
        if (t < big) {
            const unsigned r = rg_div(t, g.mg_n1, g.n1);
            t = r + (t - r * g.n1) * g.d;
        } else {
            const unsigned n0 = g.n1 - 1, u = t - big;
            const unsigned r = rg_div(u, g.mg_n0, n0);
            t = g.rem + r + (u - r * n0) * g.d;
        }
    }
    *b = (int)bb; *y = (int)t; *x = (int)xx; *c4 = (int)(it - xx * g.C4);
    return true;
}

// Q quads of channels at consecutive addresses: one 128-bit access for 4 floats or 8 bf16
template <int Q, typename T>
__device__ __forceinline__ void load_quads(const T* p, v4f (&v)[Q])
{
    if constexpr (Q == 2 && sizeof(T) == 2) {
        typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
        const bf16x8_t raw = *reinterpret_cast<const bf16x8_t*>(p);
        v[0] = __builtin_convertvector(raw.lo, v4f);
        v[1] = __builtin_convertvector(raw.hi, v4f);
    } else {
#pragma unroll
        for (int q = 0; q < Q; ++q) v[q] = load4(p + 4 * q);
    }
}
template <int Q, typename T>
__device__ __forceinline__ void store_quads(T* p, const v4f (&v)[Q])
{
    if constexpr (Q == 2 && sizeof(T) == 2) {
        typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
        bf16x8_t raw;
        raw.lo = __builtin_convertvector(v[0], bf16x4);
        raw.hi = __builtin_convertvector(v[1], bf16x4);
        *reinterpret_cast<bf16x8_t*>(p) = raw;
    } else {
#pragma unroll
        for (int q = 0; q < Q; ++q) store4(p + 4 * q, v[q]);
    }
}

// a2, 4 Q channels per thread (C % 4Q == 0; Q = 2 with bf16 storage keeps the accesses 128 bits
// wide - these kernels run at a fixed rate of elements, not of bytes): O = max over the p x p2 taps
// (rows x columns) d rows / d2 columns apart, code = tap of the FIRST maximum in row-major (u,v)
// order (strict > while scanning), 4 packed codes per quad.  RowGrid.C4 counts the threads' channel groups.
template <typename T, int Q>
__global__ __launch_bounds__(256) void maxfilter_fwd4_kernel(const T* __restrict__ A,
                                                             T* __restrict__ O,
                                                             uint8_t* __restrict__ code, RowGrid g,
                                                             int Hi, int Wi, int C, int Ho, int Wo,
                                                             int p, int p2, int d, int d2)
{
    int b, y, x, c4;
    if (!rg_locate(g, Wo, &b, &y, &x, &c4)) return;
    const long e = ((((long)b * Ho + y) * Wo + x) * g.C4 + c4) * (4 * Q);
    const T* base = A + (((long)b * Hi + y) * Wi + x) * C + 4 * Q * c4;
    v4f best[Q];
    load_quads<Q>(base, best);
    uint32_t bi[Q][4];
#pragma unroll
    for (int q = 0; q < Q; ++q)
#pragma unroll
        for (int z = 0; z < 4; ++z) bi[q][z] = 0;
    for (int u = 0; u < p; ++u)
        for (int v = (u == 0 ? 1 : 0); v < p2; ++v) {
            v4f a[Q];
            load_quads<Q>(base + ((long)u * d * Wi + v * d2) * C, a);
            const uint32_t t = u * p2 + v;
#pragma unroll
            for (int q = 0; q < Q; ++q)
#pragma unroll
                for (int z = 0; z < 4; ++z)
                    if (a[q][z] > best[q][z]) { best[q][z] = a[q][z]; bi[q][z] = t; }
        }
    store_quads<Q>(O + e, best);   // a value read back unchanged: exact in either storage type
    if (code) {
        uint32_t packed[Q];
#pragma unroll
        for (int q = 0; q < Q; ++q) packed[q] = bi[q][0] | (bi[q][1] << 8) | (bi[q][2] << 16) | (bi[q][3] << 24);
        if constexpr (Q == 2) *reinterpret_cast<uint2*>(code + e) = make_uint2(packed[0], packed[1]);
        else *reinterpret_cast<uint32_t*>(code + e) = packed[0];
    }
}

// a2 for 2 x 2 windows, 2 x 2 outputs per thread: outputs (y, x), (y, x+d), (y+d, x), (y+d, x+d) share
// 9 input elements, so a thread loads 9 instead of 16 (every input element is then fetched 2.25
// times by the threads, not 4: the other fetches were L2 hits, but L2 hits are not free).  A
// thread's rows y and y+d are neighbours in the row sequence: the sequence walks the rows of
// one residue class mod d two at a time (y = r + 2 d j), class after class; columns likewise in
// blocks of 2 d.  Outputs whose row or column lies outside the map are skipped (their loads are
// clamped to valid addresses).  Same values and codes as maxfilter_fwd4_kernel.
struct PairGrid {
    int gx;            // workgroups per row pair
    int rows;          // B * S, S = row pairs per image
    int S, C4;         // row pairs per image, channel groups
    int Sx;            // column pairs per row
    int d;
    int nbig, q1;      // the first nbig residue classes have q1 row pairs, the others q1 - 1
    unsigned mg_gx, mg_S, mg_c4, mg_q1, mg_q0, mg_d;
};
template <typename T, int Q>
__global__ __launch_bounds__(256) void maxfilter_fwd2x2_kernel(const T* __restrict__ A, T* __restrict__ O,
                                                               uint8_t* __restrict__ code, PairGrid g,
                                                               int Hi, int Wi, int C, int Ho, int Wo)
{
    const unsigned nb = gridDim.x, i = blockIdx.x;
    const unsigned q = nb >> 3, r8 = nb & 7, xcd = i & 7;
    const unsigned lb = xcd * q + (xcd < r8 ? xcd : r8) + (i >> 3);   // band of this XCD, then its turn
    const unsigned row = rg_div(lb, g.mg_gx, g.gx), bx = lb - row * g.gx;
    const unsigned it = bx * 256 + threadIdx.x;
    if (it >= (unsigned)(g.Sx * g.C4)) return;
    const unsigned sx = rg_div(it, g.mg_c4, g.C4), c4 = it - sx * g.C4;
    const unsigned b = rg_div(row, g.mg_S, g.S);
    unsigned t = row - b * g.S, rc, j;
    const unsigned big = (unsigned)(g.nbig * g.q1);
    if (t < big) { rc = rg_div(t, g.mg_q1, g.q1); j = t - rc * g.q1; }
    else { const unsigned u = t - big, q0 = g.q1 - 1; const unsigned rr = rg_div(u, g.mg_q0, q0); rc = g.nbig + rr; j = u - rr * q0; }
    const int d = g.d;
    const int y0 = (int)(rc + j * 2 * d);
    const unsigned xb = rg_div(sx, g.mg_d, d);
    const int x0 = (int)(xb * 2 * d + (sx - xb * d));
    const bool row1 = y0 + d < Ho, col1 = x0 + d < Wo;
    // the 3 x 3 inputs (rows y0, +d, +2d; columns x0, +d, +2d), coordinates clamped into the map
    int ys[3], xs[3];
#pragma unroll
    for (int k = 0; k < 3; ++k) {
        ys[k] = y0 + k * d < Hi ? y0 + k * d : Hi - 1;
        xs[k] = x0 + k * d < Wi ? x0 + k * d : Wi - 1;
    }
    const T* img = A + (long)b * Hi * Wi * C + 4 * Q * c4;
    v4f in[3][3][Q];
#pragma unroll
    for (int u = 0; u < 3; ++u)
#pragma unroll
        for (int v = 0; v < 3; ++v) load_quads<Q>(img + ((long)ys[u] * Wi + xs[v]) * C, in[u][v]);
#pragma unroll
    for (int oy = 0; oy < 2; ++oy)
#pragma unroll
        for (int ox = 0; ox < 2; ++ox) {
            if ((oy && !row1) || (ox && !col1)) continue;
            v4f best[Q];
            uint32_t packed[Q];
#pragma unroll
            for (int qq = 0; qq < Q; ++qq) {
                best[qq] = in[oy][ox][qq];
                uint32_t bi[4] = {0, 0, 0, 0};
#pragma unroll
                for (int tap = 1; tap < 4; ++tap) {
                    const v4f a = in[oy + (tap >> 1)][ox + (tap & 1)][qq];
#pragma unroll
                    for (int z = 0; z < 4; ++z)
                        if (a[z] > best[qq][z]) { best[qq][z] = a[z]; bi[z] = tap; }   // strict >: the first maximum wins
                }
                packed[qq] = bi[0] | (bi[1] << 8) | (bi[2] << 16) | (bi[3] << 24);
            }
            const long e = ((((long)b * Ho + (y0 + oy * d)) * Wo + (x0 + ox * d)) * g.C4 + c4) * (4 * Q);
            store_quads<Q>(O + e, best);
            if (code) {
                if constexpr (Q == 2) *reinterpret_cast<uint2*>(code + e) = make_uint2(packed[0], packed[1]);
                else *reinterpret_cast<uint32_t*>(code + e) = packed[0];
            }
        }
}

// a7, 4 Q channels per thread: dA = sum over the windows that chose this element (gather in
// fixed (u,v) order, no atomics), times the squashing function's slope when A is its output.
template <bool TANHP, typename T, int Q>
__global__ __launch_bounds__(256) void maxfilter_bwd4_kernel(const T* __restrict__ dO,
                                                             const uint8_t* __restrict__ code,
                                                             const T* __restrict__ A,
                                                             T* __restrict__ dA, RowGrid g,
                                                             int Hi, int Wi, int C, int Ho, int Wo,
                                                             int p, int p2, int d, int d2, int logistic)
{
    int b, y, x, c4;
    if (!rg_locate(g, Wi, &b, &y, &x, &c4)) return;
    const long e = ((((long)b * Hi + y) * Wi + x) * g.C4 + c4) * (4 * Q);
    v4f acc[Q];
#pragma unroll
    for (int q = 0; q < Q; ++q) acc[q] = (v4f){0.f, 0.f, 0.f, 0.f};
    for (int u = 0; u < p; ++u) {
        const int yy = y - u * d;
        if (yy < 0 || yy >= Ho) continue;
        for (int v = 0; v < p2; ++v) {
            const int xx = x - v * d2;
            if (xx < 0 || xx >= Wo) continue;
            const long s = (((long)b * Ho + yy) * Wo + xx) * C + 4 * Q * c4;
            uint32_t cd[Q];
            if constexpr (Q == 2) {
                const uint2 c2 = *reinterpret_cast<const uint2*>(code + s);
                cd[0] = c2.x; cd[1] = c2.y;
            } else {
                cd[0] = *reinterpret_cast<const uint32_t*>(code + s);
            }
            v4f gr[Q];
            load_quads<Q>(dO + s, gr);
            const uint32_t t = u * p2 + v;
#pragma unroll
            for (int q = 0; q < Q; ++q)
#pragma unroll
                for (int z = 0; z < 4; ++z)
                    if (((cd[q] >> (8 * z)) & 255u) == t) acc[q][z] += gr[q][z];
        }
    }
    if (TANHP) {
        v4f a[Q];
        load_quads<Q>(A + e, a);
#pragma unroll
        for (int q = 0; q < Q; ++q)
#pragma unroll
            for (int z = 0; z < 4; ++z) acc[q][z] *= squash_slope(a[q][z], logistic);
    }
    store_quads<Q>(dA + e, acc);
}

// a7 for 2 x 2 windows, 2 x 2 input elements per thread (the layout of maxfilter_fwd2x2_kernel, over
// the pool's INPUT map): elements (y, x), (y, x+d), (y+d, x), (y+d, x+d) collect from the pooled
// positions in rows y-d, y, y+d and columns x-d, x, x+d - 9 of them instead of 16.  Same sums in
// the same (u,v) order as maxfilter_bwd4_kernel.
template <bool TANHP, typename T, int Q>
__global__ __launch_bounds__(256) void maxfilter_bwd2x2_kernel(const T* __restrict__ dO,
                                                               const uint8_t* __restrict__ code,
                                                               const T* __restrict__ A, T* __restrict__ dA,
                                                               PairGrid g, int Hi, int Wi, int C, int Ho, int Wo,
                                                               int logistic)
{
    const unsigned nb = gridDim.x, i = blockIdx.x;
    const unsigned q = nb >> 3, r8 = nb & 7, xcd = i & 7;
    const unsigned lb = xcd * q + (xcd < r8 ? xcd : r8) + (i >> 3);
    const unsigned row = rg_div(lb, g.mg_gx, g.gx), bx = lb - row * g.gx;
    const unsigned it = bx * 256 + threadIdx.x;
    if (it >= (unsigned)(g.Sx * g.C4)) return;
    const unsigned sx = rg_div(it, g.mg_c4, g.C4), c4 = it - sx * g.C4;
    const unsigned b = rg_div(row, g.mg_S, g.S);
    unsigned t = row - b * g.S, rc, j;
    const unsigned big = (unsigned)(g.nbig * g.q1);
    if (t < big) { rc = rg_div(t, g.mg_q1, g.q1); j = t - rc * g.q1; }
    else { const unsigned u = t - big, q0 = g.q1 - 1; const unsigned rr = rg_div(u, g.mg_q0, q0); rc = g.nbig + rr; j = u - rr * q0; }
    const int d = g.d;
    const int y0 = (int)(rc + j * 2 * d);
    const unsigned xb = rg_div(sx, g.mg_d, d);
    const int x0 = (int)(xb * 2 * d + (sx - xb * d));
    // pooled positions in rows y0 - d, y0, y0 + d and columns x0 - d, x0, x0 + d (clamped; `ok` says which exist)
    int ys[3], xs[3];
    bool yok[3], xok[3];
#pragma unroll
    for (int k = 0; k < 3; ++k) {
        const int yy = y0 + (k - 1) * d, xx = x0 + (k - 1) * d;
        yok[k] = yy >= 0 && yy < Ho; xok[k] = xx >= 0 && xx < Wo;
        ys[k] = yy < 0 ? 0 : (yy < Ho ? yy : Ho - 1);
        xs[k] = xx < 0 ? 0 : (xx < Wo ? xx : Wo - 1);
    }
    const long cb = (long)b * Ho * Wo * C + 4 * Q * c4;
    v4f gr[3][3][Q];
    uint32_t cd[3][3][Q];
#pragma unroll
    for (int u = 0; u < 3; ++u)
#pragma unroll
        for (int v = 0; v < 3; ++v) {
            const long s = cb + ((long)ys[u] * Wo + xs[v]) * C;
            if constexpr (Q == 2) {
                const uint2 c2 = *reinterpret_cast<const uint2*>(code + s);
                cd[u][v][0] = c2.x; cd[u][v][1] = c2.y;
            } else {
                cd[u][v][0] = *reinterpret_cast<const uint32_t*>(code + s);
            }
            load_quads<Q>(dO + s, gr[u][v]);
        }
#pragma unroll
    for (int iy = 0; iy < 2; ++iy)
#pragma unroll
        for (int ix = 0; ix < 2; ++ix) {
            const int Y = y0 + iy * d, X = x0 + ix * d;
            if (Y >= Hi || X >= Wi) continue;
            const long e = ((((long)b * Hi + Y) * Wi + X) * g.C4 + c4) * (4 * Q);
            v4f acc[Q];
#pragma unroll
            for (int qq = 0; qq < Q; ++qq) acc[qq] = (v4f){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int v = 0; v < 2; ++v) {
                    const int ry = iy + 1 - u, rx = ix + 1 - v;   // the window (Y - u d, X - v d)
                    if (!yok[ry] || !xok[rx]) continue;
                    const uint32_t tap = u * 2 + v;
#pragma unroll
                    for (int qq = 0; qq < Q; ++qq)
#pragma unroll
                        for (int z = 0; z < 4; ++z)
                            if (((cd[ry][rx][qq] >> (8 * z)) & 255u) == tap) acc[qq][z] += gr[ry][rx][qq][z];
                }
            if (TANHP) {
                v4f a[Q];
                load_quads<Q>(A + e, a);
#pragma unroll
                for (int qq = 0; qq < Q; ++qq)
#pragma unroll
                    for (int z = 0; z < 4; ++z) acc[qq][z] *= squash_slope(a[qq][z], logistic);
            }
            store_quads<Q>(dA + e, acc);
        }
}

struct ClassArgs {
    const void* h;         // [M][K] input of the class layer (storage type T)
    const float* Wk;       // [K][NCLS] then bias [NCLS]
    float* probs;          // [B][NCLS][Ho][Wo] or null
    const int32_t* labels; // [B][H][W]      (training)
    const float* pixw;     // [B][H][W] or null
    const float* pixw_any; // pixw, or with none the labels (as many elements: fetched with them, not used)
    void* dH;              // [M][K]         (training) delta w.r.t. the pre-activation below (T)
    float* partial;        // [blocks][(K+1)*NCLS]  (training) this block's share of dW, db
    double* loss_partial;  // [blocks] or null
    int B, Ho, Wo, H, W, ctr, K, tanh_below;
    int probs_rows;        // rows of the probs array (Ho, or the whole image's when this call covers a band)
    int mse;               // linear outputs + half the squared error instead of softmax + cross-entropy
};

// a3 + a4 in one pass over h: class logits z = W h + b, softmax, probabilities out; in
// training also delta_z = w (p - onehot), the block's share of the summed cross-entropy,
// dW += h delta_z^T, db += delta_z, and dH = (W^T delta_z) (1 - h^2)   (Results: MCCE per
// pixel; Method: first step of back-propagation; Alg. 2 for the sums).
// 16 lanes share one position: lane j holds KV quads of channels, quad v = channels
// 4Q(j + 16(v/Q)) + 4(v%Q) .. +3 - with Q = 1 every quad is a 128-bit access of its own (fp32), with
// Q = 2 two neighbouring quads are one (8 bf16 values; K a multiple of 8); dot products meet
// by xor-shuffles in a fixed order.  A workgroup walks 16 positions at a time.
// Q quads as they come from memory (expanded to fp32 only when their turn comes)
template <int Q, typename T> struct RawQuads { typedef v4f type; };
template <> struct RawQuads<1, bf16> { typedef bf16x4 type; };
template <> struct RawQuads<2, bf16> { typedef __bf16 type __attribute__((ext_vector_type(8))); };
template <int Q>
__device__ __forceinline__ void expand_quads(const typename RawQuads<Q, float>::type& r, v4f (&v)[Q]) { v[0] = r; }
template <int Q>
__device__ __forceinline__ void expand_quads(const typename RawQuads<Q, bf16>::type& r, v4f (&v)[Q])
{
    if constexpr (Q == 2) {
        v[0] = __builtin_convertvector(r.lo, v4f);
        v[1] = __builtin_convertvector(r.hi, v4f);
    } else {
        v[0] = __builtin_convertvector(r, v4f);
    }
}
// Sum over each aligned group of 16 lanes, left in all of them: four rotations inside the row of the
// data-parallel-primitive modifier (no LDS round trip).  Every lane's additions pair the same partial
// sums as a butterfly over lane ^ 8, 4, 2, 1 would, so all 16 results are the same bits.
template <int CTRL>
__device__ __forceinline__ float row_rotated(float x)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, true));
}
__device__ __forceinline__ float row16_sum(float x)
{
    x += row_rotated<0x128>(x);   // row_ror:8
    x += row_rotated<0x124>(x);   // row_ror:4
    x += row_rotated<0x122>(x);   // row_ror:2
    x += row_rotated<0x121>(x);   // row_ror:1
    return x;
}
// positions fetched ahead per 16-lane group: the pass keeps only two waves per SIMD, and what bounds it
// is the number of bytes those waves have in flight (about 40-50 KB per compute unit with these
// depths); one less where the weights and their sums leave no registers for it
template <typename T, int NCLS, int KV>
constexpr int kClassAhead = (sizeof(T) == 2 ? 3 : 2) - (NCLS * KV >= 16 ? 1 : 0);
template <int NCLS, int KV, bool TRAIN, typename T, int Q = 1>
__global__ __launch_bounds__(256, 2) void class_layer_kernel(ClassArgs a)
{
    static_assert(KV % Q == 0, "whole accesses");
    static_assert(Q == 1 || sizeof(T) == 2, "pairs of quads: 2-byte storage only");
    auto chan = [](int lane16, int v) { return 4 * Q * (lane16 + 16 * (v / Q)) + 4 * (v % Q); };
    const T* h_t = static_cast<const T*>(a.h);
    T* dh_t = static_cast<T*>(a.dH);
    __shared__ float red[4][KV * 4 * NCLS + NCLS][16];
    __shared__ double lred[16];
    const int tid = threadIdx.x, j = tid & 15, grp = tid >> 4, wave = tid >> 6;
    const long M = (long)a.B * a.Ho * a.Wo;
    float w[KV][4][NCLS];
    float gw[KV][4][NCLS];
    float gb[NCLS], bias[NCLS];
#pragma unroll
    for (int v = 0; v < KV; ++v)
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int o = 0; o < NCLS; ++o) {
                const int c = chan(j, v) + s;
                w[v][s][o] = c < a.K ? a.Wk[(long)c * NCLS + o] : 0.f;
                gw[v][s][o] = 0.f;
            }
#pragma unroll
    for (int o = 0; o < NCLS; ++o) { bias[o] = a.Wk[(long)a.K * NCLS + o]; gb[o] = 0.f; }
    double my_loss = 0.0;
    // slope of the squashing function below in terms of its output y, as sl0 + y (sl1 + y sl2):
    // none 1, tanh 1 - y^2, logistic y (1 - y) - the same roundings as the direct forms, no selects
    const float sl0 = a.tanh_below == 2 ? 0.f : 1.f, sl1 = a.tanh_below == 2 ? 1.f : 0.f,
                sl2 = a.tanh_below ? -1.f : 0.f;

    // the pass is a chain of dependent steps per position (load, dot products, shuffles, exp,
    // stores): the h of the next few positions is fetched before the current one is worked on.
    // The loads sit behind no branch (every path then has the same number in flight and the waits
    // stay exact): a position past the end reads the last one again, a channel group past K reads
    // group 0 - its weights are zero, and nothing of it is stored.
    typedef typename RawQuads<Q, T>::type Raw;
    constexpr int AH = kClassAhead<T, NCLS, KV>;
    const long stride = (long)gridDim.x * 16;
    Raw ring[AH][KV / Q];
    int coff[KV / Q];
#pragma unroll
    for (int v = 0; v < KV / Q; ++v) coff[v] = chan(j, v * Q) < a.K ? chan(j, v * Q) : 0;
    // position m as (image b, row iy, column jx), advanced by the stride's own (images, rows,
    // columns) instead of dividing a 64-bit index at every position; (fb, fy, fx) runs AH steps ahead
    const long m0 = (long)blockIdx.x * 16 + grp;
    int jx = (int)(m0 % a.Wo), iy = (int)((m0 / a.Wo) % a.Ho), b = (int)(m0 / a.Wo / a.Ho);
    const int sx = (int)(stride % a.Wo), sy = (int)((stride / a.Wo) % a.Ho), sb = (int)(stride / a.Wo / a.Ho);
    int fx = jx, fy = iy, fb = b;
    // the label and pixel weight travel with h: loads return in issue order, so a label fetched when
    // its position comes up would have to wait for everything fetched ahead
    int ring_t[AH];
    float ring_w[AH];
    const long jplane = (long)j * a.probs_rows * a.Wo;   // this lane's class plane of the probabilities
    // element offsets of the position worked on and of the one being fetched, advanced by additions
    const long hstep = stride * a.K, last_off = (M - 1) * a.K;
    long hoff = m0 * a.K, foff = hoff;
    auto fetch_h = [&](long m, Raw (&dst)[KV / Q], int& t, float& wt) {
        const bool in = m < M;
        const T* row = h_t + (in ? foff : last_off);
        foff += hstep;
#pragma unroll
        for (int v = 0; v < KV / Q; ++v) dst[v] = *reinterpret_cast<const Raw*>(row + coff[v]);
        if (TRAIN) {
            // (image and row in 32 bits: B * H rows exist as an array index on the host already)
            const long lp = in ? (long)(fb * a.H + fy + a.ctr) * a.W + (fx + a.ctr) : 0;
            t = a.labels[lp];
            wt = a.pixw_any[lp];
        }
        fx += sx;
        if (fx >= a.Wo) { fx -= a.Wo; ++fy; }
        fy += sy;
        if (fy >= a.Ho) { fy -= a.Ho; ++fb; }
        fb += sb;
    };
#pragma unroll
    for (int i = 0; i < AH; ++i) fetch_h(m0 + i * stride, ring[i], ring_t[i], ring_w[i]);
    // (the ring's slots are taken in turn by an unrolled inner loop: moving a slot's registers
    // along would wait for its load; a turn past the last position works on the last position
    // again with label "ignore" and stores nothing - no exit from the middle of the round)
    for (long mo = m0; mo < M; mo += AH * stride)
#pragma unroll
    for (int slot = 0; slot < AH; ++slot) {
        const long m = mo + slot * stride;
        const bool live = m < M;
        v4f hv[KV];
        float z[NCLS];
#pragma unroll
        for (int o = 0; o < NCLS; ++o) z[o] = 0.f;
#pragma unroll
        for (int v = 0; v < KV / Q; ++v) expand_quads<Q>(ring[slot][v], *reinterpret_cast<v4f(*)[Q]>(&hv[v * Q]));
        int t = ring_t[slot];
        const float wt_in = ring_w[slot];
        fetch_h(m + AH * stride, ring[slot], ring_t[slot], ring_w[slot]);
#pragma unroll
        for (int v = 0; v < KV; ++v) {
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int o = 0; o < NCLS; ++o) z[o] = fmaf(hv[v][s], w[v][s][o], z[o]);
        }
#pragma unroll
        for (int o = 0; o < NCLS; ++o) {
            z[o] = row16_sum(z[o]) + bias[o];
        }
        float zmax = z[0];
#pragma unroll
        for (int o = 1; o < NCLS; ++o) zmax = fmaxf(zmax, z[o]);
        float sum = 0.f, pr[NCLS];
#pragma unroll
        for (int o = 0; o < NCLS; ++o) {   // arguments <= 0: the hardware exp2 neither overflows nor needs a range check
            z[o] -= zmax;
            pr[o] = __builtin_amdgcn_exp2f(1.4426950408889634f * z[o]);
            sum += pr[o];
        }
        const float inv = a.mse ? 1.f : __builtin_amdgcn_rcpf(sum);
        if (a.mse) {   // the outputs themselves (Method: mean squared error with linear outputs)
#pragma unroll
            for (int o = 0; o < NCLS; ++o) pr[o] = z[o] + zmax;
        }
#pragma unroll
        for (int o = 0; o < NCLS; ++o) pr[o] *= inv;
        if (a.probs) {   // lane o of the 16 writes class o: one store, at this lane's plane
            float pj = pr[0];
#pragma unroll
            for (int o = 1; o < NCLS; ++o) pj = j == o ? pr[o] : pj;
            if (j < NCLS && live) a.probs[(long)(b * NCLS * a.probs_rows + iy) * a.Wo + jx + jplane] = pj;
        }
        if (TRAIN) {
            float wt = 0.f;
            if (t < 0 || t >= NCLS || !live) t = -1;
            else wt = a.pixw ? wt_in : 1.f;
            float dz[NCLS];
            float zt = 0.f, sq = 0.f;
#pragma unroll
            for (int o = 0; o < NCLS; ++o) {
                const float e = pr[o] - (o == t ? 1.f : 0.f);
                dz[o] = t >= 0 ? wt * e : 0.f;
                if (o == t) zt = z[o];
                gb[o] += dz[o];
                sq += e * e;
            }
            if (t >= 0 && j == 0)
                my_loss += a.mse ? (double)wt * 0.5 * (double)sq : (double)wt * ((double)logf(sum) - (double)zt);
            v4f dh[KV];
#pragma unroll
            for (int v = 0; v < KV; ++v) {
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    float g = 0.f;
#pragma unroll
                    for (int o = 0; o < NCLS; ++o) {
                        g = fmaf(w[v][s][o], dz[o], g);
                        gw[v][s][o] = fmaf(hv[v][s], dz[o], gw[v][s][o]);
                    }
                    dh[v][s] = g * fmaf(hv[v][s], fmaf(hv[v][s], sl2, sl1), sl0);
                }
            }
            if (dh_t && live)   // (no delta buffer: loss only)
#pragma unroll
                for (int v = 0; v < KV; v += Q) {
                    const int c = chan(j, v);
                    if (c < a.K) store_quads<Q>(dh_t + hoff + c, *reinterpret_cast<const v4f(*)[Q]>(&dh[v]));
                }
        }
        hoff += hstep;
        jx += sx;
        if (jx >= a.Wo) { jx -= a.Wo; ++iy; }
        iy += sy;
        if (iy >= a.Ho) { iy -= a.Ho; ++b; }
        b += sb;
    }
    if (TRAIN) {
        // sum the 16 position groups of the workgroup: 4 per wave by shuffles, waves through LDS
        constexpr int NV = KV * 4 * NCLS + NCLS;
        float vals[NV];
#pragma unroll
        for (int v = 0; v < KV; ++v)
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int o = 0; o < NCLS; ++o) vals[(v * 4 + s) * NCLS + o] = gw[v][s][o];
#pragma unroll
        for (int o = 0; o < NCLS; ++o) vals[KV * 4 * NCLS + o] = gb[o];
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            vals[i] += __shfl_xor(vals[i], 16, 64);
            vals[i] += __shfl_xor(vals[i], 32, 64);
            if ((tid & 63) < 16) red[wave][i][j] = vals[i];
        }
        my_loss += __shfl_xor(my_loss, 16, 64);   // only lanes with j == 0 hold a share
        my_loss += __shfl_xor(my_loss, 32, 64);
        if ((tid & 63) == 0) lred[wave] = my_loss;
        __syncthreads();
        float* out = a.partial + (long)blockIdx.x * ((long)a.K + 1) * NCLS;
        for (int e = tid; a.partial && e < NV * 16; e += 256) {
            const int i = e >> 4, jj = e & 15;
            const float s = (red[0][i][jj] + red[1][i][jj]) + (red[2][i][jj] + red[3][i][jj]);
            if (i < KV * 4 * NCLS) {
                const int o = i % NCLS, vs = i / NCLS, sidx = vs & 3, v = vs >> 2;
                const int c = chan(jj, v) + sidx;
                if (c < a.K) out[(long)c * NCLS + o] = s;
            } else if (jj == 0) {
                out[(long)a.K * NCLS + (i - KV * 4 * NCLS)] = s;
            }
        }
        if (tid == 0 && a.loss_partial)
            a.loss_partial[blockIdx.x] = (lred[0] + lred[1]) + (lred[2] + lred[3]);
    }
}

// Routing through the first pooling layer and the first layer's parameter gradient in one pass
// (a7 + a5 for the image layer).  The delta at the first convolution's output is needed by that
// layer's weight gradient only (the image gets no gradient), so it is formed tile by tile in LDS -
// gathered from the pooled delta by the tap codes, times the squashing function's slope - and
// multiplied with the image tile right there, instead of being written out and read back.  A
// workgroup walks tiles of kL0Rows x 16 positions and keeps its sums in registers, thread e owns
// outputs e, e + 256, .. of the layer's [(k k Ci + 1) x C1] block (bias row last); the per-workgroup
// sums are added by reduce_all_kernel.  For small blocks (at most 8 outputs per thread).
constexpr int kL0Rows = 8, kL0Cols = 16, kL0MaxPerThread = 8;
struct L0Args {
    const void* in;        // [B][Hi][Wi][Ci] image, channels-last (T)
    const void* act1;      // [B][H1][W1][C1] output of the first layer (T)
    const void* dP;        // [B][Hp][Wp][C1] delta at the pooling layer's output (T)
    const uint8_t* code;   // same shape: tap codes of the pooling layer
    float* partial;        // [workgroups][(k*k*Ci + 1) * C1]
    int B, Hi, Wi, Ci, H1, W1, C1, k, Hp, Wp;
    int nty, ntx;
    int slope;             // 0: no squashing function, 1 tanh, 2 logistic
};

template <typename T, int P>   // P = side of the pooling window
__global__ __launch_bounds__(256) void l0_wgrad_fused_kernel(L0Args a)
{
    extern __shared__ __attribute__((aligned(16))) float l0_lds[];
    constexpr int NP = kL0Rows * kL0Cols;
    const T* in_t = static_cast<const T*>(a.in);
    const T* act_t = static_cast<const T*>(a.act1);
    const T* dp_t = static_cast<const T*>(a.dP);
    const int hw = kL0Cols + a.k - 1, hh = kL0Rows + a.k - 1;
    float* dl = l0_lds;                    // [NP][C1]
    float* hl = l0_lds + NP * a.C1;        // [hh][hw][Ci]
    const int tid = threadIdx.x;
    const int rows_total = a.k * a.k * a.Ci, E = (rows_total + 1) * a.C1;
    const int Q = a.C1 >> 2;
    float acc[kL0MaxPerThread];
#pragma unroll
    for (int j = 0; j < kL0MaxPerThread; ++j) acc[j] = 0.f;
    // what each of this thread's outputs reads: halo offset of its tap and channel, delta column
    int hoff[kL0MaxPerThread], ocol[kL0MaxPerThread];
#pragma unroll
    for (int j = 0; j < kL0MaxPerThread; ++j) {
        const int e = tid + 256 * j;
        hoff[j] = -2; ocol[j] = 0;
        if (e < E) {
            const int r = e / a.C1;
            ocol[j] = e - r * a.C1;
            if (r == rows_total) hoff[j] = -1;             // the bias row: the input is 1
            else {
                const int tap = r / a.Ci, c = r - tap * a.Ci, u = tap / a.k, v = tap - u * a.k;
                hoff[j] = (u * hw + v) * a.Ci + c;
            }
        }
    }
    const int tiles = a.B * a.nty * a.ntx;
    for (int tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
        int t = tile;
        const int txi = t % a.ntx; t /= a.ntx;
        const int tyi = t % a.nty;
        const int b = t / a.nty;
        const int y0 = tyi * kL0Rows, x0 = txi * kL0Cols;
        // the image tile (clamped at the border: those positions carry a zero delta)
        for (int e = tid; e < hh * hw * a.Ci; e += 256) {
            const int c = e % a.Ci, q = e / a.Ci, hx = q % hw, hy = q / hw;
            int iy = y0 + hy, ix = x0 + hx;
            iy = iy < a.Hi ? iy : a.Hi - 1;
            ix = ix < a.Wi ? ix : a.Wi - 1;
            hl[e] = load1(in_t + (((long)b * a.Hi + iy) * a.Wi + ix) * a.Ci + c);
        }
        // the delta tile: gather over the <= P*P windows that contain the element, fixed (u,v)
        // order.  Every load is issued, at a clamped address, before the first use: the tile is
        // small and the round trips to memory are what this phase costs.
#pragma unroll 2
        for (int it = tid; it < NP * Q; it += 256) {
            const int pos = it / Q, q4 = it - pos * Q;
            const int y = y0 + pos / kL0Cols, x = x0 + pos % kL0Cols;
            const bool inside = y < a.H1 && x < a.W1;
            const int yc = inside ? y : 0, xc = inside ? x : 0;
            uint32_t cd[P * P];
            v4f gr[P * P];
            bool ok[P * P];
#pragma unroll
            for (int u = 0; u < P; ++u)
#pragma unroll
                for (int v = 0; v < P; ++v) {
                    const int yy = yc - u, xx = xc - v;
                    ok[u * P + v] = inside && yy >= 0 && yy < a.Hp && xx >= 0 && xx < a.Wp;
                    const int ys = yy < 0 ? 0 : (yy < a.Hp ? yy : a.Hp - 1), xs = xx < 0 ? 0 : (xx < a.Wp ? xx : a.Wp - 1);
                    const long s = (((long)b * a.Hp + ys) * a.Wp + xs) * a.C1 + 4 * q4;
                    cd[u * P + v] = *reinterpret_cast<const uint32_t*>(a.code + s);
                    gr[u * P + v] = load4(dp_t + s);
                }
            v4f y1 = {0.f, 0.f, 0.f, 0.f};
            if (a.slope) y1 = load4(act_t + (((long)b * a.H1 + yc) * a.W1 + xc) * a.C1 + 4 * q4);
            v4f d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int t = 0; t < P * P; ++t)
#pragma unroll
                for (int z = 0; z < 4; ++z)
                    if (ok[t] && ((cd[t] >> (8 * z)) & 255u) == (uint32_t)t) d[z] += gr[t][z];
            if (a.slope)
#pragma unroll
                for (int z = 0; z < 4; ++z) d[z] *= squash_slope(y1[z], a.slope == 2);
            *reinterpret_cast<v4f*>(dl + pos * a.C1 + 4 * q4) = d;
        }
        __syncthreads();
#pragma unroll
        for (int j = 0; j < kL0MaxPerThread; ++j) {
            if (hoff[j] < -1) continue;
            const float* dcol = dl + ocol[j];
            float s0 = 0.f, s1 = 0.f;
            if (hoff[j] < 0) {
                for (int pos = 0; pos < NP; pos += 2) { s0 += dcol[pos * a.C1]; s1 += dcol[(pos + 1) * a.C1]; }
            } else {
                const float* hp = hl + hoff[j];
                for (int py = 0; py < kL0Rows; ++py)
#pragma unroll
                    for (int px = 0; px < kL0Cols; px += 2) {
                        s0 = fmaf(dcol[(py * kL0Cols + px) * a.C1], hp[(py * hw + px) * a.Ci], s0);
                        s1 = fmaf(dcol[(py * kL0Cols + px + 1) * a.C1], hp[(py * hw + px + 1) * a.Ci], s1);
                    }
            }
            acc[j] += s0 + s1;
        }
        __syncthreads();
    }
    float* out = a.partial + (long)blockIdx.x * E;
#pragma unroll
    for (int j = 0; j < kL0MaxPerThread; ++j)
        if (hoff[j] >= -1) out[tid + 256 * j] = acc[j];
}

}  // namespace mpcnn
