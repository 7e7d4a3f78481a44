// Weight gradient with bf16 storage on v_mfma_f32_32x32x16_bf16: the decomposition of
// wgrad_mfma_kernel (slabs of 4-row tiles of one residue class, result tiles kept in
// accumulators, four multiplying and four loading waves, double-buffered LDS, partial sums
// in register layout), with 16 positions contracted per instruction: lane l supplies the 8
// consecutive columns 8*(l/32) .. +7 of a chunk of 16 for gradient row l%32 (A) and for
// output channel l%32 (B).
//
// An operand of this instruction is 1 KB per wave and the instruction takes 32 cycles, so a
// wave that fetched one operand per instruction would, with its three neighbours, ask the
// LDS for all it can deliver.  Each wave therefore owns PM x 2 result tiles: PM + 2 operand
// fetches feed 2 PM instructions.
//
// Both operands must be contiguous along the columns: the halo sits in LDS channel-major,
// [c][halo row][halo col], and the delta tile is transposed to [o][tile row][col] on its way
// in.  The loading threads take two neighbouring positions of 8 channels each (two 128-bit
// loads) and write 8 words of two positions.  An A operand starts at any element (the tap
// shifts it), i.e. these 128-bit LDS reads are only 2-byte aligned.
//
// The bias gradient is one more gradient row: its "input" is a run of ones kept in each
// buffer, so the sum of the deltas falls out of the same instructions as row k*k*Ci.
// Every tile is multiplied in full (4 rows, NCH chunks): deltas outside the image are staged
// as zeros, halo values outside it are clamped copies, so the padding adds nothing.
#pragma once
#include "kernels_wgrad.hpp"

namespace mpcnn {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef bf16x8 __attribute__((aligned(2))) bf16x8_u;   // read at any element offset
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

constexpr int kBmStageH = 8;   // halo items (2 positions x 8 channels) per loading thread
constexpr int kBmStageD = 8;   // delta items per loading thread

// LDS geometry shared by the kernel and the host's plan (elements of 2 bytes)
struct BmGeom {
    int hwp, HPb, DPb, dt_e, ones_e, buf_e;
};
__host__ __device__ inline BmGeom bm_geom(int nch, int k, int Ci, int wn)
{
    BmGeom g;
    const int TxP = 16 * nch, hh = 4 + k - 1;
    g.hwp = (TxP + k) & ~1;                       // halo row pitch: TxP + k - 1, rounded up to even
    // plane pitches are an odd number of 16-byte units (neighbouring channels = neighbouring
    // lanes of an operand read start 16 bytes further round the banks); every 8 channels the
    // planes shift by another 16 bytes, which spreads the loading threads' words
    g.HPb = 8 * (((hh * g.hwp + 7) >> 3) | 1);
    g.DPb = 8 * ((8 * nch) | 1);
    g.dt_e = 64 * wn * g.DPb + 8 * (8 * wn);      // delta tile first: 64 wn output channels
    g.ones_e = g.dt_e + Ci * g.HPb + 8 * ((Ci + 7) >> 3);
    g.buf_e = g.ones_e + ((5 * g.hwp + 16 * nch + 16 + 7) & ~7);
    return g;
}

// 128-bit LDS read at byte address addr + OFF (2-byte aligned), not waited for: the caller
// pairs it with lds_wait before the first use of the value.
template <int OFF>
__device__ __forceinline__ bf16x8 lds_fetch16(unsigned addr)
{
    bf16x8 r;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFF) : "memory");
    return r;
}
// waits until at most N LDS operations issued after x's fetch are outstanding; x is tied to
// the wait so that its users stay behind it
template <int N>
__device__ __forceinline__ void lds_wait(bf16x8& x, std::integral_constant<int, N>)
{
    asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(x) : "n"(N) : "memory");
}

template <int... I, class F>
__device__ __forceinline__ void static_for(std::integer_sequence<int, I...>, F&& f)
{
    (f(std::integral_constant<int, I>()), ...);
}

template <int PM, int NCH>
__global__ __launch_bounds__(512, 1) void wgrad_bm_kernel(WgradArgs a)
{
    constexpr int HL = kBmStageH, DL = kBmStageD, PN = 2;
    constexpr int TxP = 16 * NCH, TxP2 = TxP / 2;
    extern __shared__ __attribute__((aligned(16))) float lds[];
    bf16* ldsh = reinterpret_cast<bf16*>(lds);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave8 = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool loader = wave8 >= 4;             // uniform per wave
    const int wave = wave8 & 3, ltid = tid & 255;
    const int lm = lane & 31, lk = lane >> 5;
    const int wn = a.wn;                        // 1, 2 or 4 pairs of column tiles
    const int nidx = wave & (wn - 1);
    const int midx = __builtin_amdgcn_readfirstlane((wave / wn) % a.wm);
    const int kidx = __builtin_amdgcn_readfirstlane(wave / (wn * a.wm));
    const int rpw = a.wk == 4 ? 1 : (a.wk == 2 ? 2 : 4);   // tile rows per wave
    const BmGeom g = bm_geom(NCH, a.k, a.Ci, wn);
    const int hwp = g.hwp, hwp2 = hwp >> 1, hh = 4 + a.k - 1;
    const int HPb = g.HPb, dt_e = g.dt_e, buf_e = g.buf_e;
    constexpr int DPb = 8 * ((8 * NCH) | 1);

    const int rows_total = a.k * a.k * a.Ci;    // row rows_total is the bias row
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

    // the run of ones behind each buffer's halo
    for (int i = tid; i < 2 * (buf_e - g.ones_e); i += 512) {
        const int b = i >= buf_e - g.ones_e;
        ldsh[b * buf_e + g.ones_e + (i - b * (buf_e - g.ones_e))] = (bf16)1.f;
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
        // ================= loading waves: global memory -> LDS (transposed), one tile ahead =================
        const int cq = (a.Ci + 7) >> 3;                 // channel octets of the input
        const int dq_shift = 3 + (wn >> 1);             // 8 wn octets of output channels per position
        const int h_items = hh * hwp2 * cq;
        const int d_items = (4 * TxP2) << dq_shift;
        const bool vec_in = (a.Ci & 7) == 0, vec_dy = (a.Co & 7) == 0;
        // items decoded once: they are the same for every tile
        unsigned h_yx[HL];   // halo row * d << 16 | first halo column * d
        int h_dst[HL];       // first channel << 20 | element index in a buffer, -1 = none
        unsigned d_tyx[DL];  // tile row << 16 | first tile column
        int d_rel[DL];       // element offset of the item from the tile's first delta, -1 = never inside
        int d_dst[DL];       // element index in a buffer, -1 = none
#pragma unroll
        for (int u = 0; u < HL; ++u) {
            const unsigned it = ltid + 256 * u;
            h_yx[u] = 0; h_dst[u] = -1;
            if (it < (unsigned)h_items) {
                const unsigned pos = magic_div(it, a.mg_cq, cq), q = it - pos * cq;
                const unsigned ha = magic_div(pos, a.mg_hwp, hwp2), hb = 2 * (pos - ha * hwp2);
                h_yx[u] = ((ha * a.d) << 16) | (hb * a.d);
                h_dst[u] = (int)((8 * q) << 20 | (dt_e + 8 * q * HPb + 8 * q + ha * hwp + hb));
            }
        }
#pragma unroll
        for (int u = 0; u < DL; ++u) {
            const unsigned it = ltid + 256 * u;
            d_tyx[u] = 0; d_rel[u] = -1; d_dst[u] = -1;
            if (it < (unsigned)d_items) {
                const unsigned m = it >> dq_shift, q = it - (m << dq_shift);
                const unsigned ty = m / TxP2, tx = 2 * (m - ty * TxP2);
                const int oc = 64 * blockIdx.z * wn + 8 * q;
                d_tyx[u] = (ty << 16) | tx;
                d_dst[u] = (int)(8 * q * DPb + 8 * q + ty * TxP + tx);
                if (tx < (unsigned)a.Tx && oc < a.Co) d_rel[u] = (int)((ty * a.d * a.Wo + tx * a.d) * a.Co) + oc;
            }
        }
        // word z of the pair: channel z of the first position below channel z of the second
        auto pair_word = [](const u32x4& lo, const u32x4& hi, int z) -> unsigned {
            const unsigned a0 = lo[z >> 1], a1 = hi[z >> 1];
            return (z & 1) ? ((a0 >> 16) | (a1 & 0xffff0000u)) : ((a0 & 0xffffu) | (a1 << 16));
        };
        auto load8 = [](const bf16* p, bool vec, int nvalid) -> u32x4 {   // nvalid: channels that exist
            if (vec) return *reinterpret_cast<const u32x4*>(p);
            u32x4 r = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int z = 0; z < 8; ++z)
                if (z < nvalid) r[z >> 1] |= (unsigned)__builtin_bit_cast(unsigned short, p[z]) << (16 * (z & 1));
            return r;
        };
        auto stage = [&](int tile, bf16* buf) {
            const TileGeom t = decode(tile);
            const bf16* in_b = static_cast<const bf16*>(a.in) + (long)t.b * a.Hi * a.Wi * a.Ci;
            const bf16* dy_b = static_cast<const bf16*>(a.dY) + (long)t.b * a.Ho * a.Wo * a.Co;
            const int y0 = t.ty0 * a.d + t.ry, x0 = t.tx0 * a.d + t.rx;
            const int dbase = (y0 * a.Wo + x0) * a.Co;
            u32x4 hr[HL][2], dr[DL][2];
#pragma unroll
            for (int u = 0; u < HL; ++u) {
                int iy = y0 + (int)(h_yx[u] >> 16), ix = x0 + (int)(h_yx[u] & 0xffffu), ix1 = ix + a.d;
                iy = iy < a.Hi ? iy : a.Hi - 1;
                ix = ix < a.Wi ? ix : a.Wi - 1;
                ix1 = ix1 < a.Wi ? ix1 : a.Wi - 1;
                const int q8 = h_dst[u] < 0 ? 0 : h_dst[u] >> 20;
                hr[u][0] = load8(in_b + (unsigned)(iy * a.Wi + ix) * a.Ci + q8, vec_in, a.Ci - q8);
                hr[u][1] = load8(in_b + (unsigned)(iy * a.Wi + ix1) * a.Ci + q8, vec_in, a.Ci - q8);
            }
#pragma unroll
            for (int u = 0; u < DL; ++u) {
                const int ty = (int)(d_tyx[u] >> 16), tx = (int)(d_tyx[u] & 0xffffu);
                const bool ok0 = d_rel[u] >= 0 && ty < t.rows && tx < t.cols;
                const bool ok1 = ok0 && tx + 1 < t.cols && tx + 1 < a.Tx;
                const int oc = d_rel[u] < 0 ? 0 : (64 * (int)blockIdx.z * wn + ((d_dst[u] / (8 * DPb + 8)) << 3));
                const unsigned off0 = ok0 ? (unsigned)(dbase + d_rel[u]) : 0u;
                const unsigned off1 = ok1 ? off0 + (unsigned)(a.d * a.Co) : 0u;
                const int nv = vec_dy ? 8 : a.Co - oc;
                dr[u][0] = load8(dy_b + off0, vec_dy, ok0 ? nv : 0);
                dr[u][1] = load8(dy_b + off1, vec_dy, ok1 ? nv : 0);
                if (!ok0) dr[u][0] = (u32x4){0u, 0u, 0u, 0u};
                if (!ok1) dr[u][1] = (u32x4){0u, 0u, 0u, 0u};
            }
#pragma unroll
            for (int u = 0; u < HL; ++u) {
                if (h_dst[u] >= 0) {
                    unsigned* p = reinterpret_cast<unsigned*>(buf + (h_dst[u] & 0xfffff));
                    const int q8 = h_dst[u] >> 20;
#pragma unroll
                    for (int z = 0; z < 8; ++z)
                        if (vec_in || q8 + z < a.Ci) p[z * (HPb >> 1)] = pair_word(hr[u][0], hr[u][1], z);
                }
            }
#pragma unroll
            for (int u = 0; u < DL; ++u) {
                if (d_dst[u] >= 0) {
                    unsigned* p = reinterpret_cast<unsigned*>(buf + d_dst[u]);
#pragma unroll
                    for (int z = 0; z < 8; ++z) p[z * (DPb >> 1)] = pair_word(dr[u][0], dr[u][1], z);
                }
            }
        };
        __builtin_amdgcn_s_setprio(3);
        if (tile_begin < tile_end) stage(tile_begin, ldsh);
        __syncthreads();
        int cur = 0;
        for (int tile = tile_begin; tile < tile_end; ++tile, cur ^= 1) {
            if (tile + 1 < tile_end) stage(tile + 1, ldsh + (cur ^ 1) * buf_e);
            __syncthreads();
        }
    } else {
        // ================= multiplying waves =================
        // LDS byte address of the buffers (the low half of the array's flat address)
        const unsigned lds_base = (unsigned)reinterpret_cast<size_t>(lds);
        // byte offset in a buffer of this lane's A operand: its (tap, c) at tile row 0, column 8*lk
        unsigned ap[PM];
#pragma unroll
        for (int p = 0; p < PM; ++p) {
            const unsigned row = 32u * (mt0 + p) + lm;
            unsigned o = g.ones_e;
            if (row < (unsigned)rows_total) {
                const unsigned tap = magic_div(row, a.mg_ci, a.Ci), c = row - tap * a.Ci;
                const unsigned ta = magic_div(tap, a.mg_k2, a.k2), tb = tap - ta * a.k2;   // (square filters only: k2 == k)
                o = dt_e + c * HPb + (c >> 3) * 8 + ta * hwp + tb;
            }
            ap[p] = lds_base + 2u * (o + 8 * lk);
        }
        const unsigned brow = 64 * nidx + lm;
        const unsigned boff = lds_base + 2u * (brow * DPb + (brow >> 3) * 8 + 8 * lk);   // B operand: columns 8*lk.. of row 0
        constexpr int BJ = 2 * (32 * DPb + 32);                                // bytes to the wave's second column tile
        const unsigned row_a = 2u * hwp, row_b = 2u * TxP;                     // bytes from a row to the next

        // One tile: per row NCH chunks of 16 columns, 2 PM instructions per chunk, column tile
        // by column tile.  Each operand register set is refilled for the next chunk right
        // behind its last use; at a row's end the address registers move first.  The fetches
        // are written as instructions (the compiler would gather a row's fetches at the top of
        // the row loop and wait there), so the waits are written too: LDS returns in order, and
        // each wait names how many younger fetches may still be in flight.
        auto multiply = [&](int cur) {
            unsigned moved = 2u * (unsigned)(cur * buf_e + kidx * rpw * hwp);
            unsigned bp = boff + 2u * (unsigned)(cur * buf_e + kidx * rpw * TxP);
#pragma unroll
            for (int p = 0; p < PM; ++p) { ap[p] += moved; asm volatile("" : "+v"(ap[p])); }
            asm volatile("" : "+v"(bp));
            bf16x8 av[PM], bv[PN];
            // issue order of a chunk's fetches: B0, A0 .. A(PM-1), B1
            bv[0] = lds_fetch16<0>(bp);
#pragma unroll
            for (int p = 0; p < PM; ++p) av[p] = lds_fetch16<0>(ap[p]);
            bv[1] = lds_fetch16<BJ>(bp);
            auto step = [&](auto imm) {
                constexpr int IMM = decltype(imm)::value;
                static_for(std::make_integer_sequence<int, PM>(), [&](auto pc) {
                    constexpr int p = decltype(pc)::value;
                    lds_wait(av[p], std::integral_constant<int, PM - p>());   // A(p+1).., B1 may be pending
                    acc[p][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[p], bv[0], acc[p][0], 0, 0, 0);
                });
                bv[0] = lds_fetch16<IMM>(bp);
                lds_wait(bv[1], std::integral_constant<int, 1>());            // only the new B0 may be pending
#pragma unroll
                for (int p = 0; p < PM; ++p) {
                    acc[p][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[p], bv[1], acc[p][1], 0, 0, 0);
                    av[p] = lds_fetch16<IMM>(ap[p]);
                }
                bv[1] = lds_fetch16<BJ + IMM>(bp);
            };
            for (int row = 0; row < rpw; ++row) {
                if constexpr (NCH > 1) step(std::integral_constant<int, 32>());
                if constexpr (NCH > 2) step(std::integral_constant<int, 64>());
                if constexpr (NCH > 3) step(std::integral_constant<int, 96>());
                // last chunk: its successor is the next row's first chunk (after the last row
                // that fetch reads on inside the buffer and is dropped)
#pragma unroll
                for (int p = 0; p < PM; ++p) { ap[p] += row_a; asm volatile("" : "+v"(ap[p])); }
                bp += row_b; asm volatile("" : "+v"(bp));
                moved += row_a;
                step(std::integral_constant<int, 0>());
            }
            // the dropped fetches must have landed before their registers are used again
            lds_wait(bv[1], std::integral_constant<int, 0>());
#pragma unroll
            for (int p = 0; p < PM; ++p) asm volatile("" : "+v"(av[p]));
            asm volatile("" : "+v"(bv[0]));
#pragma unroll
            for (int p = 0; p < PM; ++p) ap[p] -= moved;
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
