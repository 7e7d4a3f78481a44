// Weight gradient of one dilated convolution on the fp32 matrix cores, and the fixed-order
// second stage that adds the per-workgroup partial sums of all layers.
//
//   dW[tap][c][o] = sum over positions of in[pos + tap][c] * dY[pos][o]        (Alg. 2: the
//   same gradient function applied to every fragment, the results summed)
//
// Seen as a GEMM the result is tiny (k*k*Ci rows x Co columns) and the contraction runs
// over every position of the dense map, so the positions are split over the workgroups
// (blockIdx.x = slab of tiles) and each workgroup keeps its share of the result in
// accumulator registers for its whole slab.  v_mfma_f32_32x32x2_f32 contracts two
// positions per instruction: lane l supplies A[row l%32][position l/32] and
// B[position l/32][column l%32].
//
// Tile = 4 rows x Tx columns of one residue class (one fragment of the MPF storage).  Its
// input halo sits in LDS as [channel quad][halo row][halo col][4 channels] with an odd number
// of positions per quad plane, so the 32 lanes of an A operand (32 consecutive gradient rows =
// consecutive channels of a tap) hit 32 different banks, successive columns are 16 bytes apart,
// and the loading waves write a 128-bit global item with one 128-bit LDS store; the delta tile sits as
// [tile row][32-column block of the result][col][32].  The number of result tiles per wave (MW) is a template parameter so
// that the multiply loop has no branches; tiles beyond the gradient's last row tile compute
// on valid addresses and are never stored.  The four waves split the 32 x 32 result tiles along rows (wm),
// columns (wn) and tile rows (wk, partial sums met in LDS at the end, fixed order).
// A workgroup has eight waves, two per SIMD: waves 0-3 multiply, waves 4-7 only move data.
// LDS is double buffered: while the multiplying waves work on tile t, the loading waves bring
// tile t+1 from global memory into the other buffer; one barrier per tile.  The matrix cores
// of a SIMD thus see nothing of the staging (a wave's own vector ALU and memory instructions
// are not overlapped with its MFMAs, another wave's are).
#pragma once
#include "kernels_mfma.hpp"
#include <type_traits>

namespace mpcnn {

constexpr int kWgBmMaxTiles = 5;  // row tiles per wave of wgrad_bm_kernel, which owns two column tiles for each
constexpr int kWgMaxTiles = 11;   // 32x32 result tiles per wave (16 accumulator registers each; two waves share a SIMD's 512)
constexpr int kWgStageH = 8;      // 128-bit items of the input halo one thread stages per tile, or twice as many (template parameter)
constexpr int kWgStageD = 8;      // ... of the delta tile

struct WgradArgs {
    const void* in;      // [B][Hi][Wi][Ci]  layer input (activations), fp32 or bf16 (template parameter T)
    const void* dY;      // [B][Ho][Wo][Co]  delta w.r.t. the layer's pre-activation, same type
    float* partial;      // [slabs][Mt*Nt result tiles][4][64 lanes][4] then [Nt*32] bias sums
    int B, Hi, Wi, Ci;
    int Ho, Wo, Co;
    int k, d;
    int Tx, TxP;           // tile = 4 rows x Tx columns of one residue class; TxP = Tx rounded up to 4
    int nty, ntx;
    int tiles_total, tiles_per_slab;
    int Mt, Nt;            // 32-row / 32-column tiles of the gradient matrix (row = tap*Ci + c)
    int wm, wn, wk;        // multiplying waves along result rows, result columns, tile rows (wm*wn*wk = 4)
    int mw;                // row tiles per wave (<= kWgMaxTiles); blockIdx.y covers wm*mw of them
    // ceil(2^32 / x): n / x == umulhi(n, magic) for n * x < 2^32, x > 1
    unsigned mg_cq, mg_hwp, mg_txp, mg_ci, mg_k, mg_ntx, mg_nty, mg_d;
};

__device__ __forceinline__ unsigned magic_div(unsigned n, unsigned magic, unsigned x)
{
    return x == 1 ? n : __umulhi(n, magic);
}

template <int MW, int HLT, typename T>   // HLT: halo items per loading thread and tile (kWgStageH or twice that)
__global__ __launch_bounds__(512, 1) void wgrad_mfma_kernel(WgradArgs a)
{
    constexpr int HL = HLT, DL = kWgStageD;
    extern __shared__ __attribute__((aligned(16))) float lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave8 = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool loader = wave8 >= 4;             // uniform per wave
    const int wave = wave8 & 3, ltid = tid & 255;
    const int lm = lane & 31, lk = lane >> 5;
    // (uniform values that come out of a division are pinned to scalar registers by hand)
    const int wn = a.wn;                        // 1, 2 or 4
    const int nidx = wave & (wn - 1);
    const int midx = __builtin_amdgcn_readfirstlane((wave / wn) % a.wm);
    const int kidx = __builtin_amdgcn_readfirstlane(wave / (wn * a.wm));
    const int rpw = a.wk == 4 ? 1 : (a.wk == 2 ? 2 : 4);   // tile rows per wave
    const int hwp = a.TxP + a.k - 1;            // halo row pitch
    const int hh = 4 + a.k - 1;
    const int QP = 4 * ((hh * hwp) | 1);        // pitch of a channel quad's plane in the halo (floats; odd number of positions)
    const int cq = (a.Ci + 3) >> 2;
    // delta tile [tile row][block of 32 columns of the result][col][32]: a wave's B operands of
    // successive columns are 128 bytes apart whatever wn is; 32 floats of padding per block keep
    // the 128-bit staging writes of neighbouring blocks on different banks
    const int OB = a.TxP * 32 + 32, RB = wn * OB;
    const int dt_f = 4 * RB;                    // delta tile first (128-bit aligned), halo behind it
    const int buf_f = dt_f + cq * QP;
    const int trash_f = 2 * buf_f + 16;         // 16 bytes that nobody reads, behind the slack of the second buffer

    const int rows_total = a.k * a.k * a.Ci;
    // ---- a multiplying wave's result tiles: rows 32*(mt0 + p), p < np; columns 32*nt
    const int mt0 = blockIdx.y * (a.wm * a.mw) + midx * a.mw;
    int np = a.Mt - mt0;
    np = __builtin_amdgcn_readfirstlane(np < 0 ? 0 : (np > a.mw ? a.mw : np));
    const int nt = blockIdx.z * wn + nidx;
    const bool active = !loader && np > 0 && nt < a.Nt;

    // MFMA results kept in AccVGPRs (an empty asm operand in one makes the compiler select
    // that form): the matrix pipe then leaves the ArchVGPR ports to the loading waves
    if constexpr (MW <= 7) { float agpr_hint = 0.f; asm volatile("" : "+a"(agpr_hint)); }
    v16f acc[MW];
#pragma unroll
    for (int p = 0; p < MW; ++p)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[p][r] = 0.f;
    float bsum = 0.f;

    const int tile_begin = blockIdx.x * a.tiles_per_slab;
    int tile_end = tile_begin + a.tiles_per_slab;
    if (tile_end > a.tiles_total) tile_end = a.tiles_total;

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
        // extent of this residue class
        const int fh = t.ry < a.Ho ? (int)magic_div(a.Ho - t.ry + a.d - 1, a.mg_d, a.d) : 0;
        const int fw = t.rx < a.Wo ? (int)magic_div(a.Wo - t.rx + a.d - 1, a.mg_d, a.d) : 0;
        t.ty0 = tyi * 4; t.tx0 = txi * a.Tx;
        t.rows = fh - t.ty0; t.cols = fw - t.tx0;
        return t;
    };

    if (loader) {
        // ================= loading waves: global memory -> LDS, one tile ahead =================
        const int h_items = hh * hwp * cq;
        const int dq_shift = 3 + (wn >> 1);     // 8 * wn 128-bit items per delta position
        const int d_items = (4 * a.TxP) << dq_shift;
        const bool vec_in = (a.Ci & 3) == 0, vec_dy = (a.Co & 3) == 0;
        const int h_full = h_items >> 8, d_full = d_items >> 8;   // rounds in which every thread has an item
        // Thread ltid stages the 128-bit items ltid + 256*u of the halo and of the delta tile.
        // Which items those are never changes, so they are decoded once; per tile only the
        // global addresses are formed (these waves share their SIMD's issue slots with the
        // multiplying waves: the less vector ALU work here, the better).  Halo coordinates
        // outside the input are clamped (any finite value will do there: the matching deltas
        // are zero); delta items outside the class are loaded from a safe address and zeroed on
        // the way to LDS.
        // Tiles whose halo and delta lie inside the tensors (all but those on the lower / right
        // border) take every load at a fixed per-thread offset from a per-tile scalar base: the
        // multiplying waves wait for these waves at every tile's barrier, so what a tile costs
        // here beyond its trip to memory is kept as small as possible.
        unsigned h_yx[HL];   // (halo row * d) << 16 | halo col * d
        int h_dst[HL];       // channel 4q << 20 | float index in a buffer of the item (its quad plane, its position), -1 = none
        unsigned h_off[HL];  // element offset of the item from the halo's first element (0 if none)
        unsigned d_tyx[DL];  // tile row << 16 | tile col
        int d_rel[DL];       // float offset of the item from the tile's first delta, -1 = never inside
        int d_dst[DL];       // float index in a buffer (of the 16 unread bytes for items never inside: added to either buffer's base it stays there), -1 = none
#pragma unroll
        for (int u = 0; u < HL; ++u) {
            const unsigned it = ltid + 256 * u;
            h_yx[u] = 0; h_dst[u] = -1; h_off[u] = 0;
            if (it < (unsigned)h_items) {
                const unsigned pos = magic_div(it, a.mg_cq, cq), q = it - pos * cq;
                const unsigned ha = magic_div(pos, a.mg_hwp, hwp), hb = pos - ha * hwp;
                h_yx[u] = ((ha * a.d) << 16) | (hb * a.d);
                h_dst[u] = (int)((4 * q) << 20 | (dt_f + q * QP + 4 * (ha * hwp + hb)));
                h_off[u] = ((ha * a.d) * a.Wi + hb * a.d) * a.Ci + 4 * q;
            }
        }
#pragma unroll
        for (int u = 0; u < DL; ++u) {
            const unsigned it = ltid + 256 * u;
            d_tyx[u] = 0; d_rel[u] = -1; d_dst[u] = -1;
            if (it < (unsigned)d_items) {
                const unsigned m = it >> dq_shift, q = it - (m << dq_shift);
                const unsigned ty = magic_div(m, a.mg_txp, a.TxP), tx = m - ty * a.TxP;
                const int oc = 32 * blockIdx.z * wn + 4 * q;
                d_tyx[u] = (ty << 16) | tx;
                d_dst[u] = (int)((q >> 3) * OB + 4 * (q & 7) + ty * RB + tx * 32);
                if (tx < (unsigned)a.Tx && oc < a.Co) d_rel[u] = (int)((ty * a.d * a.Wo + tx * a.d) * a.Co) + oc;
                else {
                    // never inside: zero in both buffers now, and from here on the item's store
                    // goes to the unread bytes
                    const v4f z4 = {0.f, 0.f, 0.f, 0.f};
                    *reinterpret_cast<v4f*>(lds + d_dst[u]) = z4;
                    *reinterpret_cast<v4f*>(lds + buf_f + d_dst[u]) = z4;
                    d_dst[u] = -2;
                }
            }
        }
        const int halo_h = (hh - 1) * a.d, halo_w = (hwp - 1) * a.d;   // reach of the halo below / right of its first element
        auto stage = [&](int tile, float* buf) {
            const TileGeom t = decode(tile);
            const T* in_b = static_cast<const T*>(a.in) + (long)t.b * a.Hi * a.Wi * a.Ci;
            const T* dy_b = static_cast<const T*>(a.dY) + (long)t.b * a.Ho * a.Wo * a.Co;
            const int y0 = t.ty0 * a.d + t.ry, x0 = t.tx0 * a.d + t.rx;
            const int dbase = (y0 * a.Wo + x0) * a.Co;
            v4f hr[HL], dr[DL];
            unsigned okmask = 0;
            const bool inside = vec_in && vec_dy && t.rows >= 4 && t.cols >= a.Tx &&
                                y0 + halo_h < a.Hi && x0 + halo_w < a.Wi;     // uniform
            // all loads of the tile first: one trip to memory
            if (inside) {
                const T* in_t0 = in_b + (unsigned)(y0 * a.Wi + x0) * a.Ci;
                const T* dy_t0 = dy_b + dbase;
#pragma unroll
                for (int u = 0; u < HL; ++u) hr[u] = load4(in_t0 + h_off[u]);
#pragma unroll
                for (int u = 0; u < DL; ++u) dr[u] = load4(dy_t0 + (d_rel[u] < 0 ? 0 : d_rel[u]));
                okmask = ~0u;
            } else {
            if (vec_in) {
                // a halo element outside the input meets only zero deltas, so any finite value
                // will do for it: the offset is merely kept inside this image's tensor
                const unsigned base = (unsigned)(y0 * a.Wi + x0) * a.Ci, last = (unsigned)(a.Hi * a.Wi * a.Ci) - 4u;
#pragma unroll
                for (int u = 0; u < HL; ++u) {
                    const unsigned off = base + h_off[u];
                    hr[u] = load4(in_b + (off < last ? off : last));
                }
            } else {
#pragma unroll
            for (int u = 0; u < HL; ++u) {
                int iy = y0 + (int)(h_yx[u] >> 16), ix = x0 + (int)(h_yx[u] & 0xffffu);
                iy = iy < a.Hi ? iy : a.Hi - 1;
                ix = ix < a.Wi ? ix : a.Wi - 1;
                const int q4 = h_dst[u] < 0 ? 0 : h_dst[u] >> 20;
                const unsigned off = (unsigned)(iy * a.Wi + ix) * a.Ci + q4;   // in elements
#pragma unroll
                for (int z = 0; z < 4; ++z) hr[u][z] = q4 + z < a.Ci ? load1(in_b + off + z) : 0.f;
            }
            }
#pragma unroll
            for (int u = 0; u < DL; ++u) {
                const bool ok = d_rel[u] >= 0 && (int)(d_tyx[u] >> 16) < t.rows && (int)(d_tyx[u] & 0xffffu) < t.cols;
                okmask |= ok ? (1u << u) : 0u;
                const unsigned off = ok ? (unsigned)(dbase + d_rel[u]) : 0u;   // in elements
                if (vec_dy) dr[u] = load4(dy_b + off);
                else {
                    const int oc = ok ? d_rel[u] % a.Co : 0;   // rare path: Co not a multiple of 4
#pragma unroll
                    for (int z = 0; z < 4; ++z) dr[u][z] = (ok && oc + z < a.Co) ? load1(dy_b + off + z) : 0.f;
                }
            }
            }
#pragma unroll
            for (int u = 0; u < HL; ++u)
                if (u < h_full || h_dst[u] >= 0)        // first test is uniform: whole rounds store unmasked
                    *reinterpret_cast<v4f*>(buf + (h_dst[u] & 0xfffff)) = hr[u];
            float* const trash = lds + trash_f;
#pragma unroll
            for (int u = 0; u < DL; ++u) {
                if (u < d_full || d_dst[u] != -1) {
                    const v4f z4 = {0.f, 0.f, 0.f, 0.f};
                    float* dst = d_dst[u] == -2 ? trash : buf + d_dst[u];
                    if (inside) *reinterpret_cast<v4f*>(dst) = dr[u];
                    else *reinterpret_cast<v4f*>(dst) = ((okmask >> u) & 1u) ? dr[u] : z4;
                }
            }
        };
        // these waves issue little and must not wait behind the MFMA stream of their SIMD
        __builtin_amdgcn_s_setprio(3);
        if (tile_begin < tile_end) stage(tile_begin, lds);
        __syncthreads();
        int cur = 0;
        for (int tile = tile_begin; tile < tile_end; ++tile, cur ^= 1) {
            if (tile + 1 < tile_end) stage(tile + 1, lds + (cur ^ 1) * buf_f);
            __syncthreads();
        }
    } else {
    // ================= multiplying waves =================
    // byte offset in a buffer of this lane's A operand: its (tap, c) at tile row 0, column lk
    unsigned aoff[MW];
#pragma unroll
    for (int p = 0; p < MW; ++p) {
        const unsigned row = 32u * (mt0 + p) + lm;
        unsigned o = dt_f + 4 * lk;
        if (p < np && row < (unsigned)rows_total) {
            const unsigned tap = magic_div(row, a.mg_ci, a.Ci), c = row - tap * a.Ci;
            const unsigned ta = magic_div(tap, a.mg_k, a.k), tb = tap - ta * a.k;
            o += (c >> 2) * QP + (c & 3) + 4 * (ta * hwp + tb);
        }
        aoff[p] = 4u * o;
    }
    const unsigned boff = 4u * (nidx * OB + lk * 32 + lm);   // B operand: column lk of row 0

    // ---- one tile on the matrix cores: chunks of 2 columns (lane group lk takes column lk),
    // one MFMA per row tile and chunk; the operands of the next chunk are fetched while the
    // current one is multiplied.  Operand addresses are a lane register + an immediate; the
    // registers move once per block of 8 / 4 / 2 chunks, at a row's end straight to the next
    // row, so the chain of MFMAs is never interrupted inside a tile.
    const char* ldsb = reinterpret_cast<const char*>(lds);
    auto multiply = [&](int cur, int rows_valid, int nch) {   // nch: chunks per row, even
        const int r0 = kidx * rpw;
        int r1 = r0 + rpw;
        r1 = r1 < rows_valid ? r1 : rows_valid;
        if (r0 >= r1 || nch <= 0) return;
        float aA[MW], aB[MW], bA, bB;
        unsigned moved = 0;   // what aoff[] has been moved by
        unsigned bp = boff + 4u * (unsigned)(cur * buf_f + r0 * RB);
        // (the empty asm keeps the compiler from folding the moves back into base + counter,
        // which would cost an add per read; vector ALU work is not overlapped with the wave's
        // own MFMAs, so the loop holds none but these moves and the bias sum)
        auto move = [&](unsigned da, unsigned db) {
#pragma unroll
            for (int p = 0; p < MW; ++p) { aoff[p] += da; asm volatile("" : "+v"(aoff[p])); }
            bp += db; asm volatile("" : "+v"(bp));
            moved += da;
        };
        // multiply the chunk in `cur` while the operands of chunk `chunk` (relative to the
        // address registers) arrive in `nxt`: one LDS read behind every MFMA, no branches
        auto step = [&](const float (&cur)[MW], float bcur, float (&nxt)[MW], float& bnxt, int chunk) {
            bnxt = *reinterpret_cast<const float*>(ldsb + bp + chunk * 256);
#pragma unroll
            for (int p = 0; p < MW; ++p) {
                acc[p] = __builtin_amdgcn_mfma_f32_32x32x2f32(cur[p], bcur, acc[p], 0, 0, 0);
                nxt[p] = *reinterpret_cast<const float*>(ldsb + aoff[p] + chunk * 32);
            }
            bsum += bcur;
        };
        // N chunks (N even): N - 1 steps on immediates, the move, the last step fetching the
        // first chunk behind it
        auto block = [&](auto nc, unsigned da, unsigned db) {
            constexpr int N = decltype(nc)::value;
#pragma unroll
            for (int q = 1; q < N; q += 2) {
                step(aA, bA, aB, bB, q);
                if (q + 1 < N) step(aB, bB, aA, bA, q + 1);
            }
            // last chunk of the block: first the move and the reads behind it, then the MFMAs
            move(da, db);
            bA = *reinterpret_cast<const float*>(ldsb + bp);
#pragma unroll
            for (int p = 0; p < MW; ++p) aA[p] = *reinterpret_cast<const float*>(ldsb + aoff[p]);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int p = 0; p < MW; ++p)
                acc[p] = __builtin_amdgcn_mfma_f32_32x32x2f32(aB[p], bB, acc[p], 0, 0, 0);
            bsum += bB;
        };
        move(4u * (unsigned)(cur * buf_f) + 16u * (unsigned)(r0 * hwp), 0);
        bA = *reinterpret_cast<const float*>(ldsb + bp);
#pragma unroll
        for (int p = 0; p < MW; ++p) aA[p] = *reinterpret_cast<const float*>(ldsb + aoff[p]);
        const unsigned row_a = 16u * hwp, row_b = 4u * RB;   // bytes from a row to the next
        for (int row = r0; row < r1; ++row) {
            const bool jump = row + 1 < r1;   // at the row's end fetch the next row's first chunk
            int left = nch;
            unsigned pa = 0, pb = 0;          // bytes moved within this row
            while (left >= 8) {
                left -= 8;
                const bool end = left == 0 && jump;
                block(std::integral_constant<int, 8>(), end ? row_a - pa : 256u, end ? row_b - pb : 2048u);
                pa += 256; pb += 2048;
            }
            if (left & 4) {
                left -= 4;
                const bool end = left == 0 && jump;
                block(std::integral_constant<int, 4>(), end ? row_a - pa : 128u, end ? row_b - pb : 1024u);
                pa += 128; pb += 1024;
            }
            if (left & 2) {
                block(std::integral_constant<int, 2>(), jump ? row_a - pa : 64u, jump ? row_b - pb : 512u);
            }
        }
#pragma unroll
        for (int p = 0; p < MW; ++p) aoff[p] -= moved;
    };

    __syncthreads();   // first tile staged
    int cur = 0;
    for (int tile = tile_begin; tile < tile_end; ++tile, cur ^= 1) {
        if (active) {
            const TileGeom t = decode(tile);
            const int rows_valid = t.rows < 4 ? t.rows : 4;
            int cols = t.cols < a.Tx ? t.cols : a.Tx;
            multiply(cur, rows_valid, ((cols + 3) >> 2) * 2);
        }
        __syncthreads();
    }
    }   // multiplying waves

    // ---- partial sums of the waves that shared result tiles (wk > 1) meet in LDS: the upper
    // half of the tile-row groups hands its tiles to the lower half, twice if wk = 4
    v4f* lds4 = reinterpret_cast<v4f*>(lds);
    for (int s = a.wk >> 1; s >= 1; s >>= 1) {
        if (active && kidx >= s && kidx < 2 * s) {
            v4f* dst = lds4 + ((((kidx - s) * a.wm + midx) * wn + nidx) * a.mw * 4) * 64 + lane;
#pragma unroll
            for (int p = 0; p < MW; ++p)
                if (p < np)
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4)
                        dst[(p * 4 + r4) * 64] = (v4f){acc[p][4 * r4], acc[p][4 * r4 + 1], acc[p][4 * r4 + 2], acc[p][4 * r4 + 3]};
        }
        __syncthreads();
        if (active && kidx < s) {
            const v4f* src = lds4 + (((kidx * a.wm + midx) * wn + nidx) * a.mw * 4) * 64 + lane;
#pragma unroll
            for (int p = 0; p < MW; ++p)
                if (p < np)
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4) {
                        const v4f v = src[(p * 4 + r4) * 64];
                        acc[p][4 * r4] += v[0]; acc[p][4 * r4 + 1] += v[1];
                        acc[p][4 * r4 + 2] += v[2]; acc[p][4 * r4 + 3] += v[3];
                    }
        }
        __syncthreads();
    }

    // ---- this slab's partial sums, result tiles as the accumulator registers hold them:
    // [tile (mt, nt)][r / 4][lane][r % 4], register r of lane l = row 8*(r/4) + 4*(l/32) + r%4, column l%32
    const long plen = (long)a.Mt * a.Nt * 1024 + a.Nt * 32;
    float* out = a.partial + (long)blockIdx.x * plen;
    if (active && kidx == 0) {
#pragma unroll
        for (int p = 0; p < MW; ++p)
            if (p < np) {
                v4f* dst = reinterpret_cast<v4f*>(out + ((long)(mt0 + p) * a.Nt + nt) * 1024) + lane;
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4)
                    dst[r4 * 64] = (v4f){acc[p][4 * r4], acc[p][4 * r4 + 1], acc[p][4 * r4 + 2], acc[p][4 * r4 + 3]};
            }
    }
    // bias gradient = column sums of the delta tiles, from the waves of the first row group
    if (blockIdx.y == 0) {
        if (!loader) lds[wave * 64 + lane] = bsum;
        __syncthreads();
        if (tid < 32 * wn) {
            const int ni = tid >> 5, n = tid & 31;
            const int bt = blockIdx.z * wn + ni;
            float s = 0.f;
            for (int kk = 0; kk < a.wk; ++kk) {
                const int w = (kk * a.wm) * wn + ni;
                s += lds[w * 64 + n] + lds[w * 64 + 32 + n];
            }
            if (bt < a.Nt) out[(long)a.Mt * a.Nt * 1024 + bt * 32 + n] = s;
        }
    }
}

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
