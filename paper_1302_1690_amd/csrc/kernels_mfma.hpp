// Matrix-core (MFMA, fp32) kernel for the dilated convolutions of the whole-image pass:
// forward and data gradient share it; the weight gradient has its own file.
//
// Tiling rule.  A layer whose taps are d elements apart never mixes the d*d residue
// classes (y mod d, x mod d) of its dense map - each class is one "fragment" of the
// paper's MPF storage (Method, MPF layer) and, seen alone, an ordinary undilated
// convolution.  So a workgroup takes a Ty x Tx tile of ONE class: its (Ty+k-1) x (Tx+k-1)
// input halo is staged once in LDS, each element a contiguous channel vector in the
// channels-last tensor, and is reused by all k*k taps.
//
// MFMA operand layouts (64 lanes, W = tile side, G = 64 / W lane groups):
//   v_mfma_f32_32x32x2_f32: lane l supplies A[l%32][l/32], B[l/32][l%32]; register r of the
//     result is D[8*(r/4) + 4*(l/32) + r%4][l%32]              (W = 32, G = 2, 16 registers)
//   v_mfma_f32_16x16x4_f32: lane l supplies A[l%16][l/16], B[l/16][l%16]; register r is
//     D[4*(l/16) + r][l%16]                                     (W = 16, G = 4, 4 registers)
// The contraction index may be permuted freely as long as A and B agree, so every lane
// fetches FOUR consecutive channels with one 128-bit load and feeds them to four successive
// MFMAs; one reduction step therefore covers 4*G channels of one tap.  The 32-wide form
// sustains the full fp32 matrix rate, the 16-wide one about 0.87 of it; the 16-wide form is
// kept for channel counts that would waste more than that in 32-wide tiles.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "storage.hpp"

namespace mpcnn {

enum ConvMode { kFwdTanh = 0, kFwdLinear = 1, kDgradTanh = 2, kDgradPlain = 3 };

struct ConvArgs {
    // tensors are fp32 or bf16 (the kernel's template parameter T)
    const void* in;      // [B][Hi][Wi][Cr]   tensor the taps read (activations, or deltas for dgrad)
    const v4f* wpack;    // [steps][G][CoPad] x 4 channels, steps = k*k*CrPad/(4G)
    const float* bias;   // [Co]   (forward modes)
    const void* act;     // [B][Ho][Wo][Co] tanh output at the positions written (kDgradTanh)
    void* out;           // [B][Ho][Wo][Co]
    int B, Hi, Wi, Cr, CrPad;   // CrPad: Cr rounded up to a multiple of 16
    int Ho, Wo, Co, CoPad;
    int k, d;            // filter rows and the spacing of rows
    int k2, d2;          // filter columns and the spacing of columns (they differ from k, d behind a rectangular pool)
    int origin, origin2; // halo origin (rows, columns) in fragment units relative to the tile: 0 forward, -(k-1), -(k2-1) dgrad
    int Ty, Tx, nty, ntx;
    int mode;
    int logistic;        // squashing function of the Tanh modes: 0 tanh, 1 logistic
    // persistent kernels (conv_tp_kernel): number of tiles to walk, and ceil(2^32 / x) of the
    // divisors they use (n / x == umulhi(n, magic) for n * x < 2^32, x > 1)
    int tiles_total;
    unsigned mg_cq, mg_hw, mg_tx, mg_ntx, mg_nty, mg_d;
};

template <int W> struct MfmaAcc;
template <> struct MfmaAcc<16> { typedef v4f type; };
template <> struct MfmaAcc<32> { typedef v16f type; };

template <int W>
__device__ __forceinline__ typename MfmaAcc<W>::type mfma_f32(float a, float b, typename MfmaAcc<W>::type c)
{
    if constexpr (W == 32) return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
    else return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

// Forward / data gradient of one dilated convolution as an implicit GEMM.
// Workgroup = NW waves (4 or 8); tile = W*PT positions of one residue class x W*OT output
// channels (blockIdx.y selects the group of OT channel tiles).  All waves hold the full
// tile in accumulators and each sums 1/NW of the reduction steps; the partial tiles meet in
// LDS, where all threads add them in wave order, apply the epilogue and store.  With 8
// waves one workgroup fills a CU (two waves per SIMD that are always in the same phase).  Summation order is the same for every position, so equal inputs
// give bit-equal outputs (exact pooling ties stay exact).
template <int W, int OT, int PT, int NW, typename T>
__global__ __launch_bounds__(64 * NW, 2) void conv_mfma_kernel(ConvArgs a)
{
    constexpr int CU = 4;              // channels per 128-bit halo / pack item
    const T* in_t = static_cast<const T*>(a.in);
    const T* act_t = static_cast<const T*>(a.act);
    T* out_t = static_cast<T*>(a.out);
    constexpr int G = 64 / W;          // lane groups = contraction index of one MFMA
    constexpr int QT = W / 4;          // 4-channel quads per output tile
    constexpr int NQ = W * W / 256;    // quads one lane holds of one result tile
    constexpr int ITEMS = OT * W * QT; // (position, quad) items of one epilogue round
    constexpr int NT = 64 * NW;        // threads per workgroup
    constexpr int NIT = (ITEMS + NT - 1) / NT;
    typedef typename MfmaAcc<W>::type acc_t;
    extern __shared__ __attribute__((aligned(16))) float lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: loop control stays scalar
    const int lt = lane % W, lg = lane / W;

    int bid = blockIdx.x;
    const int txi = bid % a.ntx; bid /= a.ntx;
    const int tyi = bid % a.nty; bid /= a.nty;
    const int rx = bid % a.d2; bid /= a.d2;
    const int ry = bid % a.d;
    const int b = bid / a.d;
    const int fh = ry < a.Ho ? (a.Ho - ry + a.d - 1) / a.d : 0;  // extent of this residue class
    const int fw = rx < a.Wo ? (a.Wo - rx + a.d2 - 1) / a.d2 : 0;
    const int ty0 = tyi * a.Ty, tx0 = txi * a.Tx;
    if (ty0 >= fh || tx0 >= fw) return;  // uniform for the workgroup

    const int hw = a.Tx + a.k2 - 1, hh = a.Ty + a.k - 1;
    const int cq = a.CrPad / CU;
    const int Cs4 = cq + 1;              // pitch of one halo position in 128-bit units (+1: bank spread)
    const int ot0 = blockIdx.y * OT;
    v4f* lds4 = reinterpret_cast<v4f*>(lds);

    // ---- stage the halo: zero outside the tensor and in the channel padding.  Eight loads
    // per thread are issued before the first is stored, so their latencies overlap.
    {
        const int total = hh * hw * cq;
        constexpr int U = 8;
        for (int base = tid; base < total; base += NT * U) {
            v4f v[U];
            int dst[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int it = base + NT * u;
                v[u] = (v4f){0.f, 0.f, 0.f, 0.f};
                dst[u] = -1;
                if (it < total) {
                    const int pos = it / cq, q = it - pos * cq;
                    const int ha = pos / hw, hb = pos - ha * hw;
                    const int fy = ty0 + ha + a.origin, fx = tx0 + hb + a.origin2;
                    const int iy = fy * a.d + ry, ix = fx * a.d2 + rx;
                    dst[u] = pos * Cs4 + q;
                    if (fy >= 0 && fx >= 0 && iy < a.Hi && ix < a.Wi && CU * q < a.Cr) {
                        const T* src = in_t + (((long)b * a.Hi + iy) * a.Wi + ix) * a.Cr + CU * q;
                        v[u] = load4(src);
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (dst[u] >= 0) lds4[dst[u]] = v[u];
        }
    }

    // ---- what each thread will need in the epilogue, fetched now: the bias of its quads
    // (clamped addresses instead of branches, so that the loads are issued back to back)
    v4f bias4[NIT];
#pragma unroll
    for (int it = 0; it < NIT; ++it) bias4[it] = (v4f){0.f, 0.f, 0.f, 0.f};
    if (a.mode <= kFwdLinear) {
        constexpr int SLOTS_ = W * QT, TPS_ = NT / SLOTS_ > 0 ? NT / SLOTS_ : 1;
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            const int oc = W * (ot0 + tid / SLOTS_ + TPS_ * it) + 4 * ((tid % SLOTS_) % QT);
#pragma unroll
            for (int z = 0; z < 4; ++z) {
                const int c = oc + z < a.Co ? oc + z : a.Co - 1;
                bias4[it][z] = a.bias[c];
            }
        }
    }

    // ---- per-lane halo offsets of the PT positions this lane feeds as the B operand
    int lbase[PT];
#pragma unroll
    for (int pt = 0; pt < PT; ++pt) {
        int m = W * pt + lt;
        int ty = m / a.Tx, tx = m - ty * a.Tx;
        if (ty >= a.Ty) { ty = 0; tx = 0; }  // padding position: any in-bounds address
        lbase[pt] = (ty * hw + tx) * Cs4 + lg;
    }

    const int nch = a.CrPad / (CU * G);
    const int steps = a.k * a.k2 * nch;
    const int t0 = steps * wave / NW, t1 = steps * (wave + 1) / NW;
    const int lane_w = lg * a.CoPad + W * ot0 + lt;   // this lane's offset inside one step of the pack

    // MFMA results kept in AccVGPRs: an (empty) asm operand in an AccVGPR makes the compiler
    // select the AccVGPR form of the MFMAs.
    { float agpr_hint = 0.f; asm volatile("" : "+a"(agpr_hint)); }
    acc_t acc[OT][PT];
#pragma unroll
    for (int o = 0; o < OT; ++o)
#pragma unroll
        for (int p = 0; p < PT; ++p)
#pragma unroll
            for (int r = 0; r < 4 * NQ; ++r) acc[o][p][r] = 0.f;

    __syncthreads();

    // step t = tap * nch + chunk; the running tap offset avoids divisions
    int tap = t0 / nch, chunk = t0 - tap * nch;
    int ta = tap / a.k2, tb = tap - ta * a.k2;
    // Operands are fetched one step ahead into one of two register sets (A, B) that the loop
    // alternates between, so no register is copied and the loop holds next to no vector-ALU
    // work: on this chip such instructions are not overlapped with the MFMAs of the same
    // wave.  Weights come from global memory, activations from LDS.
    v4f wA[OT], wB[OT], aA[PT], aB[PT];
    auto fetch = [&](v4f (&wr)[OT], v4f (&ar)[PT], int t) {
        const v4f* wq = a.wpack + (long)t * G * a.CoPad;   // uniform part of the address
#pragma unroll
        for (int o = 0; o < OT; ++o) wr[o] = wq[lane_w + W * o];
        const int soff = (ta * hw + tb) * Cs4 + G * chunk;
#pragma unroll
        for (int p = 0; p < PT; ++p) ar[p] = lds4[lbase[p] + soff];
        if (++chunk == nch) { chunk = 0; if (++tb == a.k2) { tb = 0; ++ta; } }
    };
    auto mfmas = [&](const v4f (&wr)[OT], const v4f (&ar)[PT]) {
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int o = 0; o < OT; ++o)
#pragma unroll
                for (int p = 0; p < PT; ++p) acc[o][p] = mfma_f32<W>(wr[o][s], ar[p][s], acc[o][p]);
    };
#pragma unroll
    for (int o = 0; o < OT; ++o) wA[o] = wB[o] = (v4f){0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int p = 0; p < PT; ++p) aA[p] = aB[p] = (v4f){0.f, 0.f, 0.f, 0.f};
    if (t0 < t1) fetch(wA, aA, t0);
    int t = t0;
    for (; t + 2 <= t1; t += 2) {
        fetch(wB, aB, t + 1);
        mfmas(wA, aA);
        if (t + 2 < t1) fetch(wA, aA, t + 2);
        mfmas(wB, aB);
    }
    if (t < t1) mfmas(wA, aA);

    // ---- meet in LDS, one position tile per round: part[wave][ot][quad][position] as 128-bit
    // items with a pitch of W+1 positions, which keeps both the writes (a lane group writes
    // consecutive positions) and the reads (consecutive threads read consecutive quads of one
    // position, so that the global stores are contiguous) free of bank conflicts.  This
    // lane's n-th quad of a tile is quad n*G + lg of position lt.  Every thread then owns
    // one (position, quad) slot per group of 256 items and walks the output tiles.
    constexpr int WP = W + 1;
    constexpr int SLOTS = W * QT;              // (position, quad) slots of one output tile
    constexpr int TPS = NT / SLOTS > 0 ? NT / SLOTS : 1;   // output tiles covered by the workgroup at once
    const int slot = tid % SLOTS, osub = tid / SLOTS;
    const int ei = slot / QT, eq = slot % QT;  // position in tile, quad
#pragma unroll
    for (int pt = 0; pt < PT; ++pt) {
        __syncthreads();  // halo (or the previous round) no longer needed
#pragma unroll
        for (int o = 0; o < OT; ++o)
#pragma unroll
            for (int n = 0; n < NQ; ++n)
                lds4[((wave * OT + o) * QT + n * G + lg) * WP + lt] =
                    (v4f){acc[o][pt][4 * n], acc[o][pt][4 * n + 1], acc[o][pt][4 * n + 2], acc[o][pt][4 * n + 3]};
        __syncthreads();
        const int m = W * pt + ei;
        const int ty = m / a.Tx, tx = m - ty * a.Tx;
        const int fy = ty0 + ty, fx = tx0 + tx;
        const bool pos_ok = ty < a.Ty && fy < fh && fx < fw;
        const long pos_off = (((long)b * a.Ho + (fy * a.d + ry)) * a.Wo + (fx * a.d2 + rx)) * a.Co;
        // all LDS reads (and, for the data gradient, the activation loads) of this thread's
        // items are issued before the first is used, so their latencies overlap
        v4f part[NIT][NW], yv[NIT];
        bool live[NIT];
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            const int o = osub + TPS * it;
            const int oc = W * (ot0 + o) + 4 * eq;
            live[it] = o < OT && pos_ok && oc < a.Co;
            const int oo = o < OT ? o : 0;
#pragma unroll
            for (int w = 0; w < NW; ++w) part[it][w] = lds4[((w * OT + oo) * QT + eq) * WP + ei];
            yv[it] = (v4f){0.f, 0.f, 0.f, 0.f};
            if (a.mode == kDgradTanh && live[it]) {
                const long off = pos_off + oc;
                if ((a.Co & 3) == 0) yv[it] = load4(act_t + off);
                else for (int z = 0; z < 4; ++z) if (oc + z < a.Co) yv[it][z] = load1(act_t + off + z);
            }
        }
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            if (!live[it]) continue;
            const int oc = W * (ot0 + osub + TPS * it) + 4 * eq;
            const long off = pos_off + oc;
            const int nv = a.Co - oc < 4 ? a.Co - oc : 4;
            v4f s = part[it][0];
#pragma unroll
            for (int w = 1; w < NW; ++w) s += part[it][w];   // fixed wave order
            if (a.mode == kFwdTanh) {
#pragma unroll
                for (int z = 0; z < 4; ++z) s[z] = squash(s[z] + bias4[it][z], a.logistic);
            } else if (a.mode == kFwdLinear) {
                s += bias4[it];
            } else if (a.mode == kDgradTanh) {
#pragma unroll
                for (int z = 0; z < 4; ++z) s[z] *= squash_slope(yv[it][z], a.logistic);
            }
            if (nv == 4 && (a.Co & 3) == 0) store4(out_t + off, s);
            else for (int z = 0; z < nv; ++z) store1(out_t + off + z, s[z]);
        }
    }
}

// The same product with the result tiles dealt out to the waves instead of the reduction
// (fp32 matrix instruction; W-wide tiles, 32 or - for layers with 16 outputs or fewer - 16).  The
// workgroup's tile is W*PT positions x W*OT output channels; each of its OT*PT/MP waves owns MP position tiles of ONE channel tile and
// runs through all k*k*C/8 reduction steps for them, so no partial tiles meet anywhere: the
// epilogue goes from the accumulators straight to memory (a lane holds 4 consecutive channels
// of one position per register quad, one 128-bit store each).  A step feeds only 4*MP MFMAs, so
// the operands are fetched through a ring D steps deep to cover the weights' trip from L2.
// Summation order is the step order for every output element, whatever the tiling: equal
// inputs give bit-equal outputs, and a position's value does not depend on how the map is cut.
template <int OT, int PT, int MP, typename T, int W = 32>
__global__ __launch_bounds__(64 * OT * PT / MP) void conv_ts_kernel(ConvArgs a)
{
    static_assert(PT % MP == 0 && (OT * PT / MP == 4 || OT * PT / MP == 8), "4 or 8 waves");
    static_assert(W == 32 || W == 16, "tile side of the matrix instruction");
    constexpr int G = 64 / W;                      // lane groups = contraction index of one matrix instruction
    constexpr int NQ = W * W / 256;                // register quads one lane holds of a result tile
    typedef typename MfmaAcc<W>::type acc_t;
    constexpr int NW = OT * PT / MP, NT = 64 * NW;
    constexpr int D = MP == 1 ? 6 : 4;             // steps in flight
    const T* in_t = static_cast<const T*>(a.in);
    const T* act_t = static_cast<const T*>(a.act);
    T* out_t = static_cast<T*>(a.out);
    extern __shared__ __attribute__((aligned(16))) float lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lt = lane % W, lg = lane / W;
    // channel tile (turned by the workgroup's index: where the last tile of the last group holds no channel at
    // all - 200 maps in 8 tiles - its wave leaves after the staging, and the idle wave should not be the same
    // SIMD's in every workgroup of a compute unit); the first of the wave's MP position tiles is wp*MP
    const int wo = (wave + (int)(blockIdx.x % OT)) % OT, wp = wave / OT;

    int bid = blockIdx.x;
    const int txi = bid % a.ntx; bid /= a.ntx;
    const int tyi = bid % a.nty; bid /= a.nty;
    const int rx = bid % a.d2; bid /= a.d2;
    const int ry = bid % a.d;
    const int b = bid / a.d;
    const int fh = ry < a.Ho ? (a.Ho - ry + a.d - 1) / a.d : 0;  // extent of this residue class
    const int fw = rx < a.Wo ? (a.Wo - rx + a.d2 - 1) / a.d2 : 0;
    const int ty0 = tyi * a.Ty, tx0 = txi * a.Tx;
    if (ty0 >= fh || tx0 >= fw) return;  // uniform for the workgroup

    const int hw = a.Tx + a.k2 - 1, hh = a.Ty + a.k - 1;
    const int cq = a.CrPad / 4;
    const int Cs4 = cq + 1;              // pitch of one halo position in 128-bit units (+1: bank spread)
    const int oc0 = W * (blockIdx.y * OT + wo);   // first channel of this wave's tile
    v4f* lds4 = reinterpret_cast<v4f*>(lds);

    // ---- stage the halo: eight loads in flight per thread.  A workgroup stages while its neighbour on the compute
    // unit streams matrix instructions, and beside such a stream a wave's vector-ALU instructions are issued at a
    // fraction of their usual rate (measured: the staging below, written with two integer divisions per item, took
    // 28 us of a workgroup's 100 us there, 4.6 us alone).  Where the thread count is a multiple of the channel quads
    // per position (every power-of-two channel count) a thread keeps ONE channel quad and walks positions a fixed
    // distance apart: coordinates, source offset and LDS index all advance by additions.
    if (NT % cq == 0) {
        constexpr int U = 8;
        const int q = tid % cq, dpos = NT / cq, npos = hh * hw;
        const int dA = dpos / hw, dB = dpos - dA * hw;              // uniform
        int pos = tid / cq;
        const int ha0 = pos / hw;
        int hb = pos - ha0 * hw;
        int iy = (ty0 + ha0 + a.origin) * a.d + ry, ix = (tx0 + hb + a.origin2) * a.d2 + rx;
        const int diy = dA * a.d, dix = dB * a.d2, wrapx = hw * a.d2;
        const long row = (long)a.Wi * a.Cr;
        long off = (long)iy * row + (long)ix * a.Cr + 4 * q;        // (negative above / left of the tensor: never used then)
        const long dstep = (long)diy * row + (long)dix * a.Cr, dwrap = (long)a.d * row - (long)wrapx * a.Cr;
        const T* img = in_t + (long)b * a.Hi * a.Wi * a.Cr;
        const bool qok = 4 * q < a.Cr;
        int dst = pos * Cs4 + q;
        const int ddst = dpos * Cs4;
        while (pos < npos) {
            v4f v[U];
            int dsts[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const bool mine = pos < npos;
                v[u] = (v4f){0.f, 0.f, 0.f, 0.f};
                dsts[u] = mine ? dst : -1;
                // (iy >= 0 exactly when the fragment row is: 0 <= ry < d)
                if (mine && qok && (unsigned)iy < (unsigned)a.Hi && (unsigned)ix < (unsigned)a.Wi) v[u] = load4(img + off);
                pos += dpos; dst += ddst; hb += dB; iy += diy; ix += dix; off += dstep;
                if (hb >= hw) { hb -= hw; iy += a.d; ix -= wrapx; off += dwrap; }
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (dsts[u] >= 0) lds4[dsts[u]] = v[u];
        }
    } else {
        const int total = hh * hw * cq;
        constexpr int U = 8;
        for (int base = tid; base < total; base += NT * U) {
            v4f v[U];
            int dst[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int it = base + NT * u;
                v[u] = (v4f){0.f, 0.f, 0.f, 0.f};
                dst[u] = -1;
                if (it < total) {
                    const int pos = it / cq, q = it - pos * cq;
                    const int ha = pos / hw, hb = pos - ha * hw;
                    const int fy = ty0 + ha + a.origin, fx = tx0 + hb + a.origin2;
                    const int iy = fy * a.d + ry, ix = fx * a.d2 + rx;
                    dst[u] = pos * Cs4 + q;
                    if (fy >= 0 && fx >= 0 && iy < a.Hi && ix < a.Wi && 4 * q < a.Cr)
                        v[u] = load4(in_t + (((long)b * a.Hi + iy) * a.Wi + ix) * a.Cr + 4 * q);
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (dst[u] >= 0) lds4[dst[u]] = v[u];
        }
    }

    // ---- the bias of this lane's channel quads (channels oc0 + 4G n + 4lg .. +3)
    v4f bias4[NQ];
#pragma unroll
    for (int n = 0; n < NQ; ++n) {
        bias4[n] = (v4f){0.f, 0.f, 0.f, 0.f};
        if (a.mode <= kFwdLinear)
#pragma unroll
            for (int z = 0; z < 4; ++z) {
                const int c = oc0 + 4 * G * n + 4 * lg + z;
                bias4[n][z] = a.bias[c < a.Co ? c : a.Co - 1];
            }
    }

    // ---- per-lane halo offsets of the positions this lane feeds as the B operand
    int lbase[MP];
#pragma unroll
    for (int p = 0; p < MP; ++p) {
        const int m = W * (wp * MP + p) + lt;
        int ty = m / a.Tx, tx = m - ty * a.Tx;
        if (ty >= a.Ty) { ty = 0; tx = 0; }  // padding position: any in-bounds address
        lbase[p] = (ty * hw + tx) * Cs4 + lg;
    }

    const int nch = a.CrPad / (4 * G);
    const int steps = a.k * a.k2 * nch;
    const int lane_w = lg * a.CoPad + oc0 + lt;   // this lane's offset inside one step of the pack

    { float agpr_hint = 0.f; asm volatile("" : "+a"(agpr_hint)); }
    acc_t acc[MP];
#pragma unroll
    for (int p = 0; p < MP; ++p)
#pragma unroll
        for (int r = 0; r < 4 * NQ; ++r) acc[p][r] = 0.f;

    __syncthreads();

    if (oc0 >= a.Co) return;             // a tile past the last channel (uniform for the wave; no barrier follows)

    // the ring: slot i holds the operands of step t with t % D == i; fetches run in step order.
    // The weights come through a buffer descriptor: the lane's byte offset in a step never changes and the step's
    // offset is a scalar, so a fetch costs no vector-ALU instruction (a 64-bit address formed per lane and step
    // did: every such instruction takes an issue slot from the matrix instructions of the SIMD - measured on the
    // bare loop, two waves per SIMD: 132.7 TFLOP/s with per-lane addresses, 145.1 with the descriptor).
    int chunk = 0, ta = 0, tb = 0, tf = 0;
    v4f wr[D], ar[D][MP];
    typedef unsigned v4u __attribute__((ext_vector_type(4)));
    const __amdgpu_buffer_rsrc_t wrsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<v4f*>(a.wpack), 0, steps * G * a.CoPad * 16, 0x00020000);   // (raw 32-bit data, range-checked)
    const int wlane = lane_w * 16, wstep = G * a.CoPad * 16;                    // bytes
    auto fetch = [&](int i) {
        wr[i] = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(wrsrc, wlane, tf * wstep, 0));
        const int soff = (ta * hw + tb) * Cs4 + G * chunk;
#pragma unroll
        for (int p = 0; p < MP; ++p) ar[i][p] = lds4[lbase[p] + soff];
        ++tf;
        if (++chunk == nch) { chunk = 0; if (++tb == a.k2) { tb = 0; ++ta; } }
    };
    // The first D fetches are issued on every path (a reduction shorter than D steps fetches step
    // 0 again into the slots it does not use): with a fetch count that depended on a branch the
    // compiler no longer knows how many loads are in flight when the loop starts, and waits for
    // ALL of them at the top of every round of D steps - the ring then hides nothing.
    auto fetch_first = [&](int i) {
        const bool real = i < steps;
        wr[i] = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(wrsrc, wlane, (real ? tf : 0) * wstep, 0));
        const int soff = real ? (ta * hw + tb) * Cs4 + G * chunk : 0;
#pragma unroll
        for (int p = 0; p < MP; ++p) ar[i][p] = lds4[lbase[p] + soff];
        if (real) {
            ++tf;
            if (++chunk == nch) { chunk = 0; if (++tb == a.k2) { tb = 0; ++ta; } }
        }
    };
    auto mfmas = [&](int i) {
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int p = 0; p < MP; ++p) acc[p] = mfma_f32<W>(wr[i][s], ar[i][p][s], acc[p]);
    };
#pragma unroll
    for (int i = 0; i < D; ++i) fetch_first(i);
    int t = 0;
    for (; t + 2 * D <= steps; t += D) {          // every step of the group has a successor D ahead
#pragma unroll
        for (int i = 0; i < D; ++i) { mfmas(i); fetch(i); }
    }
#pragma unroll
    for (int i = 0; i < D; ++i)
        if (t + i < steps) { mfmas(i); if (t + i + D < steps) fetch(i); }
#pragma unroll
    for (int i = 0; i < D; ++i)
        if (t + D + i < steps) mfmas(i);

    // ---- epilogue from the accumulators: register 4n + z of position tile p is channel
    // oc0 + 4G n + 4lg + z of position W*(wp*MP + p) + lt
#pragma unroll
    for (int p = 0; p < MP; ++p) {
        const int m = W * (wp * MP + p) + lt;
        const int ty = m / a.Tx, tx = m - ty * a.Tx;
        const int fy = ty0 + ty, fx = tx0 + tx;
        const bool pos_ok = ty < a.Ty && fy < fh && fx < fw;
        const long pos_off = (((long)b * a.Ho + (fy * a.d + ry)) * a.Wo + (fx * a.d2 + rx)) * a.Co;
        v4f yv[NQ];
#pragma unroll
        for (int n = 0; n < NQ; ++n) {
            const int oc = oc0 + 4 * G * n + 4 * lg;
            yv[n] = (v4f){0.f, 0.f, 0.f, 0.f};
            if (a.mode == kDgradTanh && pos_ok && oc < a.Co) {
                if ((a.Co & 3) == 0) yv[n] = load4(act_t + pos_off + oc);
                else for (int z = 0; z < 4; ++z) if (oc + z < a.Co) yv[n][z] = load1(act_t + pos_off + oc + z);
            }
        }
#pragma unroll
        for (int n = 0; n < NQ; ++n) {
            const int oc = oc0 + 4 * G * n + 4 * lg;
            if (!pos_ok || oc >= a.Co) continue;
            v4f s = (v4f){acc[p][4 * n], acc[p][4 * n + 1], acc[p][4 * n + 2], acc[p][4 * n + 3]};
            if (a.mode == kFwdTanh) {
#pragma unroll
                for (int z = 0; z < 4; ++z) s[z] = squash(s[z] + bias4[n][z], a.logistic);
            } else if (a.mode == kFwdLinear) {
                s += bias4[n];
            } else if (a.mode == kDgradTanh) {
#pragma unroll
                for (int z = 0; z < 4; ++z) s[z] *= squash_slope(yv[n][z], a.logistic);
            }
            const int nv = a.Co - oc < 4 ? a.Co - oc : 4;
            if (nv == 4 && (a.Co & 3) == 0) store4(out_t + pos_off + oc, s);
            else for (int z = 0; z < nv; ++z) store1(out_t + pos_off + oc + z, s[z]);
        }
    }
}

}  // namespace mpcnn
