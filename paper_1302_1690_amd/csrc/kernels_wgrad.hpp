// Weight gradient of one dilated convolution on the fp32 matrix cores (its per-workgroup
// partial sums are added by reduce_all_kernel, kernels_reduce.hpp).
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
    int k, d;              // filter rows and the spacing of rows
    int k2, d2;            // filter columns and the spacing of columns (they differ from k, d behind a rectangular pool)
    int Tx, TxP;           // tile = 4 rows x Tx columns of one residue class; TxP = Tx rounded up to 4
    int nty, ntx;
    int tiles_total, tiles_per_slab;
    int Mt, Nt;            // 32-row / 32-column tiles of the gradient matrix (row = tap*Ci + c)
    int wm, wn, wk;        // multiplying waves along result rows, result columns, tile rows (wm*wn*wk = 4)
    int mw;                // row tiles per wave (<= kWgMaxTiles); blockIdx.y covers wm*mw of them
    // ceil(2^32 / x): n / x == umulhi(n, magic) for n * x < 2^32, x > 1
    unsigned mg_cq, mg_hwp, mg_txp, mg_ci, mg_k2, mg_ntx, mg_nty, mg_d, mg_d2;
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
    const int hwp = a.TxP + a.k2 - 1;           // halo row pitch
    const int hh = 4 + a.k - 1;
    const int QP = 4 * ((hh * hwp) | 1);        // pitch of a channel quad's plane in the halo (floats; odd number of positions)
    const int cq = (a.Ci + 3) >> 2;
    // delta tile [tile row][block of 32 columns of the result][col][32]: a wave's B operands of
    // successive columns are 128 bytes apart whatever wn is; 32 floats of padding per block keep
    // the 128-bit staging writes of neighbouring blocks on different banks
    const int OB = a.TxP * 32 + 32, RB = wn * OB;
    const int dt_f = 4 * RB;                    // delta tile first (128-bit aligned), halo behind it
    const int buf_f = dt_f + cq * QP;

    const int rows_total = a.k * a.k2 * a.Ci;
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
        qd = magic_div(bid, a.mg_d2, a.d2);
        t.rx = bid - qd * a.d2; bid = qd;
        qd = magic_div(bid, a.mg_d, a.d);
        t.ry = bid - qd * a.d;
        t.b = qd;
        // extent of this residue class
        const int fh = t.ry < a.Ho ? (int)magic_div(a.Ho - t.ry + a.d - 1, a.mg_d, a.d) : 0;
        const int fw = t.rx < a.Wo ? (int)magic_div(a.Wo - t.rx + a.d2 - 1, a.mg_d2, a.d2) : 0;
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
        int h_dst[HL];       // float index in a buffer of the item (its quad plane, its position), -1 = none
        unsigned h_off[HL];  // BYTE offset of the item from the halo's first element (0 if none)
        unsigned d_tyx[DL];  // tile row << 16 | tile col
        int d_rel[DL];       // BYTE offset of the item from the tile's first delta (0 for items never inside)
        int d_dst[DL];       // float index in a buffer (items never inside: in the unread padding of their block), -1 = none
#pragma unroll
        for (int u = 0; u < HL; ++u) {
            const unsigned it = ltid + 256 * u;
            h_yx[u] = 0; h_dst[u] = -1; h_off[u] = 0;
            if (it < (unsigned)h_items) {
                const unsigned pos = magic_div(it, a.mg_cq, cq), q = it - pos * cq;
                const unsigned ha = magic_div(pos, a.mg_hwp, hwp), hb = pos - ha * hwp;
                h_yx[u] = ((ha * a.d) << 16) | (hb * a.d2);
                h_dst[u] = (int)(dt_f + q * QP + 4 * (ha * hwp + hb));
                h_off[u] = (((ha * a.d) * a.Wi + hb * a.d2) * a.Ci + 4 * q) * (unsigned)sizeof(T);
            }
        }
#pragma unroll
        for (int u = 0; u < DL; ++u) {
            const unsigned it = ltid + 256 * u;
            d_tyx[u] = 0; d_rel[u] = 0; d_dst[u] = -1;
            if (it < (unsigned)d_items) {
                const unsigned m = it >> dq_shift, q = it - (m << dq_shift);
                const unsigned ty = magic_div(m, a.mg_txp, a.TxP), tx = m - ty * a.TxP;
                const int oc = 32 * blockIdx.z * wn + 4 * q;
                d_tyx[u] = (ty << 16) | tx;
                d_dst[u] = (int)((q >> 3) * OB + 4 * (q & 7) + ty * RB + tx * 32);
                if (tx < (unsigned)a.Tx && oc < a.Co) d_rel[u] = ((int)((ty * a.d * a.Wo + tx * a.d2) * a.Co) + oc) * (int)sizeof(T);
                else {
                    // never inside: zero in both buffers now, and from here on the item's store
                    // goes to the unread bytes
                    const v4f z4 = {0.f, 0.f, 0.f, 0.f};
                    *reinterpret_cast<v4f*>(lds + d_dst[u]) = z4;
                    *reinterpret_cast<v4f*>(lds + buf_f + d_dst[u]) = z4;
                    d_dst[u] = (int)((q >> 3) * OB + ty * RB + a.TxP * 32 + 4 * (q & 7));   // the block's 32 floats of padding
                }
            }
        }
        const int halo_h = (hh - 1) * a.d, halo_w = (hwp - 1) * a.d2;   // reach of the halo below / right of its first element
        auto stage = [&](int tile, float* buf) {
            const TileGeom t = decode(tile);
            const T* in_b = static_cast<const T*>(a.in) + (long)t.b * a.Hi * a.Wi * a.Ci;
            const T* dy_b = static_cast<const T*>(a.dY) + (long)t.b * a.Ho * a.Wo * a.Co;
            const int y0 = t.ty0 * a.d + t.ry, x0 = t.tx0 * a.d2 + t.rx;
            const int dbase = (y0 * a.Wo + x0) * a.Co;
            v4f hr[HL], dr[DL];
            unsigned okmask = 0;
            const bool inside = vec_in && vec_dy && t.rows >= 4 && t.cols >= a.Tx &&
                                y0 + halo_h < a.Hi && x0 + halo_w < a.Wi;     // uniform
            // all loads of the tile first: one trip to memory
            if (inside) {
                // through buffer descriptors of this image's two tensors (the host keeps them under 4 GiB): a
                // load's address is the thread's fixed byte offset plus a scalar, so these waves, which share
                // their SIMDs with the multiplying ones, spend no vector-ALU instruction on it
                const __amdgpu_buffer_rsrc_t in_r = __builtin_amdgcn_make_buffer_rsrc(
                    const_cast<T*>(in_b), 0, (int)((unsigned)(a.Hi * a.Wi * a.Ci) * (unsigned)sizeof(T)), 0x00020000);
                const __amdgpu_buffer_rsrc_t dy_r = __builtin_amdgcn_make_buffer_rsrc(
                    const_cast<T*>(dy_b), 0, (int)((unsigned)(a.Ho * a.Wo * a.Co) * (unsigned)sizeof(T)), 0x00020000);
                const unsigned in_s = (unsigned)(y0 * a.Wi + x0) * a.Ci * (unsigned)sizeof(T);
                const unsigned dy_s = (unsigned)dbase * (unsigned)sizeof(T);
#pragma unroll
                for (int u = 0; u < HL; ++u) hr[u] = buffer_load4<T>(in_r, h_off[u], in_s);
#pragma unroll
                for (int u = 0; u < DL; ++u) dr[u] = buffer_load4<T>(dy_r, (unsigned)d_rel[u], dy_s);
                okmask = ~0u;
            } else {
            if (vec_in) {
                // a halo element outside the input meets only zero deltas, so any finite value
                // will do for it: the offset is merely kept inside this image's tensor
                const unsigned base = (unsigned)(y0 * a.Wi + x0) * a.Ci * (unsigned)sizeof(T);
                const unsigned last = ((unsigned)(a.Hi * a.Wi * a.Ci) - 4u) * (unsigned)sizeof(T);
#pragma unroll
                for (int u = 0; u < HL; ++u) {
                    const unsigned off = base + h_off[u];                       // in bytes
                    hr[u] = load4(reinterpret_cast<const T*>(reinterpret_cast<const char*>(in_b) + (off < last ? off : last)));
                }
            } else {
#pragma unroll
            for (int u = 0; u < HL; ++u) {
                int iy = y0 + (int)(h_yx[u] >> 16), ix = x0 + (int)(h_yx[u] & 0xffffu);
                iy = iy < a.Hi ? iy : a.Hi - 1;
                ix = ix < a.Wi ? ix : a.Wi - 1;
                const unsigned it = ltid + 256 * u;
                const int q4 = h_dst[u] < 0 ? 0 : (int)(4 * (it - magic_div(it, a.mg_cq, cq) * cq));
                const unsigned off = (unsigned)(iy * a.Wi + ix) * a.Ci + q4;   // in elements
#pragma unroll
                for (int z = 0; z < 4; ++z) hr[u][z] = q4 + z < a.Ci ? load1(in_b + off + z) : 0.f;
            }
            }
#pragma unroll
            for (int u = 0; u < DL; ++u) {
                const bool ok = d_dst[u] >= 0 && (int)(d_tyx[u] >> 16) < t.rows && (int)(d_tyx[u] & 0xffffu) < t.cols;
                okmask |= ok ? (1u << u) : 0u;
                const unsigned off = ok ? (unsigned)(dbase + d_rel[u] / (int)sizeof(T)) : 0u;   // in elements
                if (vec_dy) dr[u] = load4(dy_b + off);
                else {
                    const int oc = ok ? (d_rel[u] / (int)sizeof(T)) % a.Co : 0;   // rare path: Co not a multiple of 4
#pragma unroll
                    for (int z = 0; z < 4; ++z) dr[u][z] = (ok && oc + z < a.Co) ? load1(dy_b + off + z) : 0.f;
                }
            }
            }
#pragma unroll
            for (int u = 0; u < HL; ++u)
                if (u < h_full || h_dst[u] >= 0)        // first test is uniform: whole rounds store unmasked
                    *reinterpret_cast<v4f*>(buf + h_dst[u]) = hr[u];
#pragma unroll
            for (int u = 0; u < DL; ++u) {
                if (u < d_full || d_dst[u] >= 0) {
                    const v4f z4 = {0.f, 0.f, 0.f, 0.f};
                    float* dst = buf + d_dst[u];
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
            const unsigned ta = magic_div(tap, a.mg_k2, a.k2), tb = tap - ta * a.k2;
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

}  // namespace mpcnn
