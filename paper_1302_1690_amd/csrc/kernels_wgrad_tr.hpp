// Weight gradient with bf16 storage on v_mfma_f32_32x32x16_bf16, operands fetched with the
// transposing LDS read of gfx950 (ds_read_b64_tr_b16).  Same decomposition as wgrad_bm_kernel
// (kernels_wgrad_bf16.hpp: slabs of 4-row tiles of one residue class, PM x 2 result tiles per
// wave kept in accumulators, four multiplying and four loading waves, double-buffered LDS,
// partial sums in register layout, the bias gradient as one more gradient row), for layers
// whose input channel count is a multiple of 32.
//
// The instruction contracts 16 positions; a lane supplies 8 of them for ONE gradient row
// (A: one (tap, channel)) or ONE output channel (B).  The tensors are channels-last, so a plain
// read gives a lane 8 channels of one position instead.  wgrad_bm_kernel therefore transposes
// both tiles on their way into LDS (vector-ALU packing and 32-bit stores in the loading waves)
// and then reads the A operand at a 2-byte-aligned address (the tap shifts it), which the LDS
// serves lane by lane: 8 times the cost of an aligned read, the LDS 80 % busy, the matrix
// pipes 19 %.  Here both tiles are raw 128-bit copies, laid out in planes of 32 channels,
//     halo  [channel / 32][halo row][halo col][32 channels]      (64 bytes per position)
//     delta [channel / 32][tile row][tile col][32 channels]
// and the transposing read does the rest: within each group of 16 lanes, lane r names 4
// channels (r % 4) of one position (r / 4), and lane i receives channel i % 4 of quad i / 4 at
// the group's 4 positions.  Two such reads (positions +0..3 and +4..7) give a lane its 8
// positions of one channel; lanes 16-31 take the upper 16 channels, lanes 32-63 the other 8
// positions.  A tap shifts the address by whole positions (64 bytes): every read is aligned,
// a row's reads differ by immediates only (no address arithmetic inside a tile row), and
// the 32 lanes served together touch 256 consecutive bytes.
//
// Gradient rows are (tap, channel) in parameter order, so with C a multiple of 32 a result row
// tile is 32 channels of one tap = one plane at one shift.  The bias row's tile reads a block
// of constant "positions" whose channel 0 is 1 (and does not move with the tile row).
#pragma once
#include "kernels_wgrad.hpp"
#include <utility>

namespace mpcnn {

typedef __bf16 tr_bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 tr_bf16x8 __attribute__((ext_vector_type(8)));

constexpr int kTrStageH = 12;  // 128-bit halo items per loading thread and tile
constexpr int kTrStageD = 8;   // ... of the delta tile
constexpr int kWgTrMaxTiles = 5;

// LDS geometry shared by the kernel and the host's plan (bytes)
struct TrGeom {
    int hwp, hh;         // halo: columns, rows
    int hplane, dplane;  // positions per plane (the count is 1 mod 4: the loading waves' 128-bit
                         // stores of one position's planes then fall on different banks)
    int nhp, ndp;        // planes of the halo / of the delta tile
    int halo_b, ones_b, buf_b;   // byte offsets in a buffer of the halo (the delta tile is first)
                                 // and of the constant block; size of a buffer
};
__host__ __device__ inline TrGeom tr_geom(int nch, int k, int Ci, int wn)
{
    TrGeom g;
    const int TxP = 16 * nch;
    g.hh = 4 + k - 1; g.hwp = TxP + k - 1;
    g.hplane = ((g.hh * g.hwp + 3) & ~3) + 1;
    g.dplane = 4 * TxP + 1;
    g.nhp = Ci / 32; g.ndp = 2 * wn;
    g.halo_b = g.ndp * g.dplane * 64;
    g.ones_b = g.halo_b + g.nhp * g.hplane * 64;
    g.buf_b = (g.ones_b + (TxP + 8) * 64 + 255) & ~255;
    return g;
}

// one operand: 8 positions of this lane's channel, from two transposing reads 4 positions apart
template <int OFF>
__device__ __forceinline__ tr_bf16x8 tr_fetch(unsigned addr)
{
    typedef tr_bf16x4 __attribute__((address_space(3))) * lds_ptr;
    const tr_bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_ptr)(uintptr_t)(addr + OFF));
    const tr_bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_ptr)(uintptr_t)(addr + OFF + 256));
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

template <int PM, int NCH>
__global__ __launch_bounds__(512, 1) void wgrad_tr_kernel(WgradArgs a)
{
    constexpr int HL = kTrStageH, DL = kTrStageD, PN = 2;
    constexpr int TxP = 16 * NCH;
    extern __shared__ __attribute__((aligned(16))) float lds[];
    char* ldsb = reinterpret_cast<char*>(lds);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave8 = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool loader = wave8 >= 4;             // uniform per wave
    const int wave = wave8 & 3, ltid = tid & 255;
    const int wn = a.wn;                        // 1, 2 or 4 pairs of column tiles
    const int nidx = wave & (wn - 1);
    const int midx = __builtin_amdgcn_readfirstlane((wave / wn) % a.wm);
    const int kidx = __builtin_amdgcn_readfirstlane(wave / (wn * a.wm));
    const int rpw = a.wk == 4 ? 1 : (a.wk == 2 ? 2 : 4);   // tile rows per wave
    const TrGeom g = tr_geom(NCH, a.k, a.Ci, wn);
    const int hwp = g.hwp, hh = g.hh;

    const int rows_total = a.k * a.k * a.Ci;    // a multiple of 32; row rows_total is the bias row
    const int mt0 = blockIdx.y * (a.wm * PM) + midx * PM;
    int np = a.Mt - mt0;
    np = __builtin_amdgcn_readfirstlane(np < 0 ? 0 : (np > PM ? PM : np));
    const int nt0 = (blockIdx.z * wn + nidx) * PN;
    const bool active = !loader && np > 0 && nt0 < a.Nt;

    v16f acc[PM][PN];
#pragma unroll
    for (int p = 0; p < PM; ++p)
#pragma unroll
        for (int j = 0; j < PN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[p][j][r] = 0.f;

    const int tile_begin = blockIdx.x * a.tiles_per_slab;
    int tile_end = tile_begin + a.tiles_per_slab;
    if (tile_end > a.tiles_total) tile_end = a.tiles_total;

    // the constant block of each buffer: "positions" whose channel 0 is 1, the others 0
    for (int i = tid; i < 2 * (TxP + 8) * 32; i += 512) {
        const int b = i >= (TxP + 8) * 32, e = i - b * (TxP + 8) * 32;
        reinterpret_cast<bf16*>(ldsb + b * g.buf_b + g.ones_b)[e] = (bf16)((e & 31) == 0 ? 1.f : 0.f);
    }

    struct TileGeom { int b, ry, rx, ty0, tx0, rows, cols; };
    auto decode = [&](int tile) {
        TileGeom t;
        unsigned bid = tile;
        unsigned qd = magic_div(bid, a.mg_ntx, a.ntx);
        const int txi = bid - qd * a.ntx; bid = qd;
        qd = magic_div(bid, a.mg_nty, a.nty);
        const int tyi = bid - qd * a.nty; bid = qd;
        qd = magic_div(bid, a.mg_d, a.d);
        t.rx = bid - qd * a.d; bid = qd;
        qd = magic_div(bid, a.mg_d, a.d);
        t.ry = bid - qd * a.d;
        t.b = qd;
        const int fh = t.ry < a.Ho ? (int)magic_div(a.Ho - t.ry + a.d - 1, a.mg_d, a.d) : 0;
        const int fw = t.rx < a.Wo ? (int)magic_div(a.Wo - t.rx + a.d - 1, a.mg_d, a.d) : 0;
        t.ty0 = tyi * 4; t.tx0 = txi * a.Tx;
        t.rows = fh - t.ty0; t.cols = fw - t.tx0;
        return t;
    };

    if (loader) {
        // ================= loading waves: global memory -> LDS, raw 128-bit copies, one tile ahead =================
        const int cq = a.Ci >> 3;                       // 8-channel items per input position
        const int dq_shift = 3 + (wn >> 1);             // 8 wn items of output channels per position
        const int h_items = hh * hwp * cq;
        const int d_items = (4 * TxP) << dq_shift;
        const bool vec_dy = (a.Co & 7) == 0;
        // items decoded once: they are the same for every tile
        unsigned h_yx[HL];   // (halo row * d) << 16 | halo col * d
        int h_dst[HL];       // byte offset in a buffer, -1 = none
        unsigned h_off[HL];  // byte offset of the item from the halo's first element
        unsigned d_tyx[DL];  // tile row << 16 | tile col
        int d_rel[DL];       // byte offset of the item from the tile's first delta (0 where there is none)
        int d_dst[DL];       // byte offset in a buffer, -1 = none (or never inside: zeroed once, below)
#pragma unroll
        for (int u = 0; u < HL; ++u) {
            const unsigned it = ltid + 256 * u;
            h_yx[u] = 0; h_dst[u] = -1; h_off[u] = 0;
            if (it < (unsigned)h_items) {
                const unsigned pos = magic_div(it, a.mg_cq, cq), q = it - pos * cq;
                const unsigned ha = magic_div(pos, a.mg_hwp, hwp), hb = pos - ha * hwp;
                h_yx[u] = ((ha * a.d) << 16) | (hb * a.d);
                h_dst[u] = (int)(g.halo_b + ((q >> 2) * g.hplane + pos) * 64 + (q & 3) * 16);
                h_off[u] = (((ha * a.d) * a.Wi + hb * a.d) * a.Ci + 8 * q) * 2u;   // in bytes
            }
        }
#pragma unroll
        for (int u = 0; u < DL; ++u) {
            const unsigned it = ltid + 256 * u;
            d_tyx[u] = 0; d_rel[u] = 0; d_dst[u] = -1;
            if (it < (unsigned)d_items) {
                const unsigned m = it >> dq_shift, q = it - (m << dq_shift);
                const unsigned ty = m / TxP, tx = m - ty * TxP;
                const int oc = 64 * blockIdx.z * wn + 8 * q;
                d_tyx[u] = (ty << 16) | tx;
                d_dst[u] = (int)(((q >> 2) * g.dplane + m) * 64 + (q & 3) * 16);
                if (tx < (unsigned)a.Tx && oc < a.Co) d_rel[u] = 2 * ((int)((ty * a.d * a.Wo + tx * a.d) * a.Co) + oc);
                else {
                    // never inside (a column past the tile's width, a channel past the last): zero in both
                    // buffers now, never stored again
                    typedef unsigned z32x4 __attribute__((ext_vector_type(4)));
                    *reinterpret_cast<z32x4*>(ldsb + d_dst[u]) = (z32x4){0u, 0u, 0u, 0u};
                    *reinterpret_cast<z32x4*>(ldsb + g.buf_b + d_dst[u]) = (z32x4){0u, 0u, 0u, 0u};
                    d_dst[u] = -1;
                }
            }
        }
        typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
        auto load8 = [](const bf16* p, bool vec, int nvalid) -> u32x4 {   // nvalid: channels that exist
            if (vec) return *reinterpret_cast<const u32x4*>(p);
            u32x4 r = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int z = 0; z < 8; ++z)
                if (z < nvalid) r[z >> 1] |= (unsigned)__builtin_bit_cast(unsigned short, p[z]) << (16 * (z & 1));
            return r;
        };
        const int halo_h = (hh - 1) * a.d, halo_w = (hwp - 1) * a.d;   // reach of the halo below / right of its first element
        auto stage = [&](int tile, char* buf) {
            const TileGeom t = decode(tile);
            const bf16* in_b = static_cast<const bf16*>(a.in) + (long)t.b * a.Hi * a.Wi * a.Ci;
            const bf16* dy_b = static_cast<const bf16*>(a.dY) + (long)t.b * a.Ho * a.Wo * a.Co;
            const int y0 = t.ty0 * a.d + t.ry, x0 = t.tx0 * a.d + t.rx;
            const int dbase = (y0 * a.Wo + x0) * a.Co;
            u32x4 hr[HL], dr[DL];
            const bool inside = y0 + halo_h < a.Hi && x0 + halo_w < a.Wi;     // uniform
            // all loads of the tile first: one trip to memory.  A halo element outside the input
            // meets only zero deltas, so any finite value will do for it: clamped coordinates.
            if (inside) {
                // through a buffer descriptor of this image's tensor (under 4 GiB, the host sees to it): the
                // address is the thread's fixed byte offset plus a scalar - no vector-ALU instruction per load
                // on these waves, which share their SIMDs with the multiplying ones
                const __amdgpu_buffer_rsrc_t in_r = __builtin_amdgcn_make_buffer_rsrc(
                    const_cast<bf16*>(in_b), 0, (int)((unsigned)(a.Hi * a.Wi * a.Ci) * 2u), 0x00020000);
                const unsigned in_s = (unsigned)(y0 * a.Wi + x0) * a.Ci * 2u;
#pragma unroll
                for (int u = 0; u < HL; ++u)
                    hr[u] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(in_r, (int)h_off[u], (int)in_s, 0));
            } else {
#pragma unroll
                for (int u = 0; u < HL; ++u) {
                    int iy = y0 + (int)(h_yx[u] >> 16), ix = x0 + (int)(h_yx[u] & 0xffffu);
                    iy = iy < a.Hi ? iy : a.Hi - 1;
                    ix = ix < a.Wi ? ix : a.Wi - 1;
                    const unsigned it = ltid + 256 * u;
                    const unsigned q = h_dst[u] < 0 ? 0u : it - magic_div(it, a.mg_cq, cq) * cq;
                    hr[u] = *reinterpret_cast<const u32x4*>(in_b + (unsigned)(iy * a.Wi + ix) * a.Ci + 8 * q);
                }
            }
            if (vec_dy && t.rows >= 4 && t.cols >= a.Tx) {
                // the whole tile lies inside its residue class: every item that is ever stored is valid
                const __amdgpu_buffer_rsrc_t dy_r = __builtin_amdgcn_make_buffer_rsrc(
                    const_cast<bf16*>(dy_b), 0, (int)((unsigned)(a.Ho * a.Wo * a.Co) * 2u), 0x00020000);
                const unsigned dy_s = (unsigned)dbase * 2u;
#pragma unroll
                for (int u = 0; u < DL; ++u)
                    dr[u] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(
                                                          dy_r, d_rel[u], (int)dy_s, 0));
            } else
#pragma unroll
            for (int u = 0; u < DL; ++u) {
                const int ty = (int)(d_tyx[u] >> 16), tx = (int)(d_tyx[u] & 0xffffu);
                const bool ok = d_dst[u] >= 0 && ty < t.rows && tx < t.cols;
                const unsigned off = ok ? (unsigned)(dbase + (d_rel[u] >> 1)) : 0u;
                if (vec_dy) dr[u] = *reinterpret_cast<const u32x4*>(dy_b + off);
                else dr[u] = load8(dy_b + off, false, ok ? a.Co - (d_rel[u] >> 1) % a.Co : 0);   // (rare: channel count not a multiple of 8)
                if (!ok) dr[u] = (u32x4){0u, 0u, 0u, 0u};
            }
#pragma unroll
            for (int u = 0; u < HL; ++u)
                if (h_dst[u] >= 0) *reinterpret_cast<u32x4*>(buf + h_dst[u]) = hr[u];
#pragma unroll
            for (int u = 0; u < DL; ++u)
                if (d_dst[u] >= 0) *reinterpret_cast<u32x4*>(buf + d_dst[u]) = dr[u];
        };
        __builtin_amdgcn_s_setprio(3);
        if (tile_begin < tile_end) stage(tile_begin, ldsb);
        __syncthreads();
        int cur = 0;
        for (int tile = tile_begin; tile < tile_end; ++tile, cur ^= 1) {
            if (tile + 1 < tile_end) stage(tile + 1, ldsb + (cur ^ 1) * g.buf_b);
            __syncthreads();
        }
    } else {
        // ================= multiplying waves =================
        const unsigned lds_base = (unsigned)reinterpret_cast<size_t>(lds);
        const int grp = lane >> 4, r16 = lane & 15;
        // this lane's part of every operand address: position 8 (grp / 2) + r16 / 4 of a chunk,
        // channels 16 (grp % 2) + 4 (r16 % 4) .. +3 of a plane
        const unsigned lane_b = (unsigned)((8 * (grp >> 1) + (r16 >> 2)) * 64 + (16 * (grp & 1) + 4 * (r16 & 3)) * 2);
        unsigned ap[PM];      // A operand of row tile p: buffer 0, tile row 0, chunk 0
        unsigned arow[PM];    // bytes from a tile row to the next (0 for the bias row's tile: it reads the constant block)
#pragma unroll
        for (int p = 0; p < PM; ++p) {
            const unsigned row = 32u * (mt0 + p);
            unsigned o = g.ones_b;
            arow[p] = 0;
            if (row < (unsigned)rows_total) {
                const unsigned tap = magic_div(row, a.mg_ci, a.Ci), c = row - tap * a.Ci;
                const unsigned ta = magic_div(tap, a.mg_k2, a.k2), tb = tap - ta * a.k2;   // (square filters only: k2 == k)
                o = g.halo_b + ((c >> 5) * g.hplane + ta * hwp + tb) * 64;
                arow[p] = 64u * hwp;
            }
            ap[p] = lds_base + o + lane_b;
        }
        const unsigned bp0 = lds_base + (unsigned)(2 * nidx * g.dplane * 64) + lane_b;   // B operand: first column tile, tile row 0
        const unsigned BJ = (unsigned)g.dplane * 64u;                                     // bytes to the wave's second column tile
        constexpr unsigned row_b = 64u * TxP;

        // One tile: per row NCH chunks of 16 positions, 2 PM instructions per chunk.  Operands of
        // the next chunk are fetched while the current one is multiplied (two register sets).
        auto multiply = [&](int cur) {
            unsigned av[PM], bv = bp0 + (unsigned)(cur * g.buf_b) + (unsigned)(kidx * rpw) * row_b;
#pragma unroll
            for (int p = 0; p < PM; ++p) av[p] = ap[p] + (unsigned)(cur * g.buf_b) + (unsigned)(kidx * rpw) * arow[p];
            tr_bf16x8 A0[PM], A1[PM], B0[PN], B1[PN];
            auto fetch = [&](tr_bf16x8 (&A)[PM], tr_bf16x8 (&Bq)[PN], auto imm) {
                constexpr int IMM = decltype(imm)::value;
                Bq[0] = tr_fetch<IMM>(bv);
#pragma unroll
                for (int p = 0; p < PM; ++p) A[p] = tr_fetch<IMM>(av[p]);
                Bq[1] = tr_fetch<IMM>(bv + BJ);
            };
            auto mfmas = [&](const tr_bf16x8 (&A)[PM], const tr_bf16x8 (&Bq)[PN]) {
#pragma unroll
                for (int j = 0; j < PN; ++j)
#pragma unroll
                    for (int p = 0; p < PM; ++p)
                        acc[p][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[p], Bq[j], acc[p][j], 0, 0, 0);
            };
            auto next_row = [&]() {
#pragma unroll
                for (int p = 0; p < PM; ++p) av[p] += arow[p];
                bv += row_b;
            };
            // chunks c = 0 .. NCH-1 of a row at immediates 1024 c; sets alternate chunk by chunk
            fetch(A0, B0, std::integral_constant<int, 0>());
            for (int row = 0; row < rpw; ++row) {
                const bool more = row + 1 < rpw;   // uniform
                if constexpr (NCH == 1) {
                    if (more) { next_row(); fetch(A1, B1, std::integral_constant<int, 0>()); }
                    mfmas(A0, B0);
                    if (more) {
#pragma unroll
                        for (int p = 0; p < PM; ++p) A0[p] = A1[p];
                        B0[0] = B1[0]; B0[1] = B1[1];
                    }
                } else if constexpr (NCH == 2) {
                    fetch(A1, B1, std::integral_constant<int, 1024>());
                    mfmas(A0, B0);
                    if (more) { next_row(); fetch(A0, B0, std::integral_constant<int, 0>()); }
                    mfmas(A1, B1);
                } else if constexpr (NCH == 3) {
                    fetch(A1, B1, std::integral_constant<int, 1024>());
                    mfmas(A0, B0);
                    fetch(A0, B0, std::integral_constant<int, 2048>());
                    mfmas(A1, B1);
                    if (more) { next_row(); fetch(A1, B1, std::integral_constant<int, 0>()); }
                    mfmas(A0, B0);
                    if (more) {
#pragma unroll
                        for (int p = 0; p < PM; ++p) A0[p] = A1[p];
                        B0[0] = B1[0]; B0[1] = B1[1];
                    }
                } else {
                    fetch(A1, B1, std::integral_constant<int, 1024>());
                    mfmas(A0, B0);
                    fetch(A0, B0, std::integral_constant<int, 2048>());
                    mfmas(A1, B1);
                    fetch(A1, B1, std::integral_constant<int, 3072>());
                    mfmas(A0, B0);
                    if (more) { next_row(); fetch(A0, B0, std::integral_constant<int, 0>()); }
                    mfmas(A1, B1);
                }
            }
        };

        __syncthreads();   // first tile staged
        int cur = 0;
        for (int tile = tile_begin; tile < tile_end; ++tile, cur ^= 1) {
            if (active) multiply(cur);
            __syncthreads();
        }
    }

    // ---- partial sums of the waves that shared result tiles (wk > 1) meet in LDS
    v4f* lds4 = reinterpret_cast<v4f*>(lds);
    for (int s = a.wk >> 1; s >= 1; s >>= 1) {
        if (active && kidx >= s && kidx < 2 * s) {
            v4f* dst = lds4 + ((((kidx - s) * a.wm + midx) * wn + nidx) * (PM * PN * 4)) * 64 + lane;
#pragma unroll
            for (int p = 0; p < PM; ++p)
#pragma unroll
                for (int j = 0; j < PN; ++j)
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4)
                        dst[((p * PN + j) * 4 + r4) * 64] =
                            (v4f){acc[p][j][4 * r4], acc[p][j][4 * r4 + 1], acc[p][j][4 * r4 + 2], acc[p][j][4 * r4 + 3]};
        }
        __syncthreads();
        if (active && kidx < s) {
            const v4f* src = lds4 + (((kidx * a.wm + midx) * wn + nidx) * (PM * PN * 4)) * 64 + lane;
#pragma unroll
            for (int p = 0; p < PM; ++p)
#pragma unroll
                for (int j = 0; j < PN; ++j)
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4) {
                        const v4f v = src[((p * PN + j) * 4 + r4) * 64];
                        acc[p][j][4 * r4] += v[0]; acc[p][j][4 * r4 + 1] += v[1];
                        acc[p][j][4 * r4 + 2] += v[2]; acc[p][j][4 * r4 + 3] += v[3];
                    }
        }
        __syncthreads();
    }

    // partial result of this slab: result tiles in register layout (the bias row is row k*k*Ci)
    const long plen = (long)a.Mt * a.Nt * 1024;
    float* out = a.partial + (long)blockIdx.x * plen;
    if (active && kidx == 0) {
#pragma unroll
        for (int p = 0; p < PM; ++p)
#pragma unroll
            for (int j = 0; j < PN; ++j)
                if (p < np && nt0 + j < a.Nt) {
                    v4f* dst = reinterpret_cast<v4f*>(out + ((long)(mt0 + p) * a.Nt + nt0 + j) * 1024) + lane;
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4)
                        dst[r4 * 64] = (v4f){acc[p][j][4 * r4], acc[p][j][4 * r4 + 1], acc[p][j][4 * r4 + 2], acc[p][j][4 * r4 + 3]};
                }
    }
}

}  // namespace mpcnn
