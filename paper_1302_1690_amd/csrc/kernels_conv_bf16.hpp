// Forward / data gradient of one dilated convolution on the bf16 matrix instruction
// (v_mfma_f32_32x32x16_bf16; bf16 storage, channel counts that are multiples of 8): the
// tile-per-wave product of conv_ts_kernel (kernels_mfma.hpp) - a workgroup's tile is 32*PT
// positions of ONE residue class x 32*OT output channels, each wave owns MP position tiles of one
// channel tile and runs through all k*k*C/16 reduction steps for them - reorganised around what
// that instruction's speed leaves exposed.  One instruction takes 32 cycles, an eighth of the
// fp32 form's time per flop, so a tile's matrix work (a few thousand cycles) is no longer long
// against the rest of a workgroup's life: measured per workgroup on the 2 x 3 x 2048 x 2048
// workload, staging the halo took 11-16 K cycles (two rounds of loads, each item's address formed
// with two integer divisions at 4 cycles per vector instruction), the reduction 14 K, the stores
// 14 K.  Hence:
//   * workgroups are persistent: each walks tiles t = blockIdx.x, + gridDim.x, ..; what never
//     changes from tile to tile is computed once - which 128-bit halo items a thread stages, where
//     they go in LDS, their offset from the halo's first element, the bias, the lanes' operand
//     and result positions;
//   * a tile whose halo lies inside the tensor (most) is loaded at those fixed offsets from one
//     scalar base, with no per-item arithmetic; the others check every item's coordinates;
//   * the next tile's halo is loaded into registers right after the reduction loop, so the loads
//     travel while the epilogue computes and stores (loads issued before or inside the reduction
//     would hold up its weight fetches: a wave's loads return in order), and is written to LDS
//     once every wave has left the current tile;
//   * two workgroups share a compute unit: one multiplies while the other stores and stages.
// Summation order is the step order for every output element whatever the tiling, as in
// conv_ts_kernel: equal inputs give bit-equal outputs.
#pragma once
#include <type_traits>

#include "kernels_mfma.hpp"

namespace mpcnn {

// 128-bit halo items one thread stages per tile, at most (they wait in registers while the
// epilogue runs; a wave with 4 accumulator tiles has room for fewer)
__host__ __device__ constexpr int tp_items(int MP) { return MP >= 4 ? 8 : 12; }

__device__ __forceinline__ unsigned tp_div(unsigned n, unsigned magic, unsigned x)
{
    return x == 1 ? n : __umulhi(n, magic);   // n / x for n * x < 2^32, magic = ceil(2^32 / x)
}

template <int OT, int PT, int MP>
__global__ __launch_bounds__(64 * OT * PT / MP, 2) void conv_tp_kernel(ConvArgs a)
{
    static_assert(PT % MP == 0 && (OT * PT / MP == 4 || OT * PT / MP == 8), "4 or 8 waves");
    constexpr int W = 32, G = 2, CU = 8, SI = tp_items(MP);
    constexpr int NW = OT * PT / MP, NT = 64 * NW;
    constexpr int DW = 8, DA = 2;                  // reduction steps in flight: weights, activations
    typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
    const bf16* in_t = static_cast<const bf16*>(a.in);
    const bf16* act_t = static_cast<const bf16*>(a.act);
    bf16* out_t = static_cast<bf16*>(a.out);
    extern __shared__ __attribute__((aligned(16))) float lds[];
    v4f* lds4 = reinterpret_cast<v4f*>(lds);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lt = lane & 31, lg = lane >> 5;
    // channel tile, turned by the workgroup's index (a wave whose tile lies past the last channel - 200 maps in
    // 8 tiles - only stages and waits: it should not sit on the same SIMD in both workgroups of a compute unit);
    // the first of the wave's MP position tiles is wp*MP
    const int wo = (wave + (int)(blockIdx.x % OT)) % OT, wp = wave / OT;

    const int hw = a.Tx + a.k - 1, hh = a.Ty + a.k - 1;
    const int cq = a.CrPad / CU;
    const int Cs4 = cq + 1;                        // pitch of one halo position in 128-bit units (+1: bank spread)
    const int n_items = hh * hw * cq;              // <= SI * NT (the host's plan sees to it)
    const int oc0 = W * (blockIdx.y * OT + wo);    // first channel of this wave's tile
    const bool wave_live = oc0 < a.Co;             // uniform for the wave
    const v4f zero4 = {0.f, 0.f, 0.f, 0.f};

    // ---- what this thread stages of every tile: item it = tid + NT*u is channels 8q.. of halo
    // position pos = (ha, hb); i_dst = its place in LDS (-1: none), i_off = its element offset from
    // the halo's first element.  Channel padding (8q >= C) is zeroed once and never touched again.
    unsigned i_dst2[SI / 2];                       // two 16-bit LDS indices each (the halo has < 65535 items)
    unsigned i_off[SI];
#pragma unroll
    for (int u = 0; u < SI; ++u) {
        const unsigned it = tid + NT * u;
        unsigned dst = 0xffffu;
        i_off[u] = 0;
        if (it < (unsigned)n_items) {
            const unsigned pos = tp_div(it, a.mg_cq, cq), q = it - pos * cq;
            const unsigned ha = tp_div(pos, a.mg_hw, hw), hb = pos - ha * hw;
            if (CU * q < (unsigned)a.Cr) {
                dst = pos * Cs4 + q;
                i_off[u] = ((ha * a.d) * a.Wi + hb * a.d) * a.Cr + CU * q;
            } else {
                lds4[pos * Cs4 + q] = zero4;
            }
        }
        if (u & 1) i_dst2[u >> 1] |= dst << 16;
        else i_dst2[u >> 1] = dst;
    }
    auto i_dst = [&](int u) { return (int)((i_dst2[u >> 1] >> (16 * (u & 1))) & 0xffffu); };

    // ---- per lane: the halo offset of the positions it feeds as the B operand, and their place
    // in the tile (row << 16 | column; 0xffff: a padding position of the last tile)
    int lbase[MP];
    unsigned e_tyx[MP];
#pragma unroll
    for (int p = 0; p < MP; ++p) {
        const unsigned m = W * (wp * MP + p) + lt;
        unsigned ty = tp_div(m, a.mg_tx, a.Tx), tx = m - ty * a.Tx;
        e_tyx[p] = (ty << 16) | tx;
        if (ty >= (unsigned)a.Ty) { ty = 0; tx = 0; e_tyx[p] = 0xffff0000u; }   // any in-bounds address
        lbase[p] = (int)((ty * hw + tx) * Cs4) + lg;
    }

    const int nch = a.CrPad / (CU * G);
    const int steps = a.k * a.k * nch;
    const int lane_w = lg * a.CoPad + oc0 + lt;    // this lane's offset inside one step of the pack
    typedef unsigned v4u __attribute__((ext_vector_type(4)));
    const __amdgpu_buffer_rsrc_t wrsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<v4f*>(a.wpack), 0, steps * G * a.CoPad * 16, 0x00020000);   // (raw data, range-checked)
    const int wlane = lane_w * 16;                 // bytes

    struct Tile { int b, ry, rx, ty0, tx0, fh, fw; bool live; };
    auto decode = [&](int t) {
        Tile g;
        unsigned bid = t;
        unsigned qd = tp_div(bid, a.mg_ntx, a.ntx);
        const int txi = bid - qd * a.ntx; bid = qd;
        qd = tp_div(bid, a.mg_nty, a.nty);
        const int tyi = bid - qd * a.nty; bid = qd;
        qd = tp_div(bid, a.mg_d, a.d);
        g.rx = bid - qd * a.d; bid = qd;
        qd = tp_div(bid, a.mg_d, a.d);
        g.ry = bid - qd * a.d;
        g.b = qd;
        g.fh = g.ry < a.Ho ? (int)tp_div(a.Ho - g.ry + a.d - 1, a.mg_d, a.d) : 0;  // extent of this residue class
        g.fw = g.rx < a.Wo ? (int)tp_div(a.Wo - g.rx + a.d - 1, a.mg_d, a.d) : 0;
        g.ty0 = tyi * a.Ty; g.tx0 = txi * a.Tx;
        g.live = g.ty0 < g.fh && g.tx0 < g.fw;      // uniform for the workgroup
        return g;
    };
    // loads of tile g's halo into v (nothing waits for them here)
    auto issue = [&](const Tile& g, v4f (&v)[SI]) {
        const int iy0 = (g.ty0 + a.origin) * a.d + g.ry, ix0 = (g.tx0 + a.origin) * a.d + g.rx;
        const bf16* img = in_t + (long)g.b * a.Hi * a.Wi * a.Cr;
        const bool inside = iy0 >= 0 && ix0 >= 0 && iy0 + (hh - 1) * a.d < a.Hi && ix0 + (hw - 1) * a.d < a.Wi;
        if (inside) {
            const bf16* base = img + (unsigned)(iy0 * a.Wi + ix0) * a.Cr;
#pragma unroll
            for (int u = 0; u < SI; ++u) v[u] = *reinterpret_cast<const v4f*>(base + i_off[u]);   // (items without a place: element 0)
        } else {
#pragma unroll
            for (int u = 0; u < SI; ++u) {
                const unsigned it = tid + NT * u;
                const unsigned pos = tp_div(it, a.mg_cq, cq), q = it - pos * cq;
                const unsigned ha = tp_div(pos, a.mg_hw, hw), hb = pos - ha * hw;
                const int iy = iy0 + (int)(ha * a.d), ix = ix0 + (int)(hb * a.d);
                const bool ok = i_dst(u) != 0xffff && iy >= 0 && ix >= 0 && iy < a.Hi && ix < a.Wi;
                const unsigned off = ok ? (unsigned)(iy * a.Wi + ix) * a.Cr + CU * q : 0u;
                v[u] = *reinterpret_cast<const v4f*>(img + off);
                if (!ok) v[u] = zero4;             // outside the tensor: the zero padding of the data gradient
            }
        }
    };

    // (no AccVGPR hint here: a kernel that may use AccVGPRs gets half of its 256 registers as such,
    // and this one needs about 190 ordinary ones beside the 16 MP accumulators)
    const int total = a.tiles_total;
    auto to_lds = [&](const v4f (&v)[SI]) {
#pragma unroll
        for (int u = 0; u < SI; ++u)
            if (i_dst(u) != 0xffff) lds4[i_dst(u)] = v[u];
    };
    int t = blockIdx.x;
    Tile cur = decode(t < total ? t : 0);
    if (t >= total) cur.live = false;
    if (cur.live) {
        v4f first[SI];
        issue(cur, first);
        to_lds(first);
    }
    __syncthreads();
    for (; t < total; t += gridDim.x) {
        v16f acc[MP];
#pragma unroll
        for (int p = 0; p < MP; ++p)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[p][r] = 0.f;
        if (cur.live && wave_live) {
            // Two rings.  The weights come from L2 (a layer's pack is far larger than the vector
            // cache), a trip of 1-2 K cycles under load, and a step lasts 32 MP cycles: DW = 8 steps
            // of weights are in flight.  The activations come from LDS: DA = 2.  Slot s % DW (s % DA)
            // holds the operand of step s; fetches run in step order.
            // (weights through a buffer descriptor: the lane's byte offset is fixed, the step's is a scalar - no
            // vector-ALU instruction per fetch, which would take an issue slot from the matrix instructions)
            int chunk = 0, ta = 0, tb = 0;
            int wq = 0;                                // byte offset of the next step in the pack
            const int wstep = G * a.CoPad * 16;
            v4f wr[DW], ar[DA][MP];
            auto fetch_w = [&](int i) {
                wr[i] = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(wrsrc, wlane, wq, 0));
                wq += wstep;
            };
            auto fetch_a = [&](int i) {
                const int soff = (ta * hw + tb) * Cs4 + G * chunk;
#pragma unroll
                for (int p = 0; p < MP; ++p) ar[i][p] = lds4[lbase[p] + soff];
                if (++chunk == nch) { chunk = 0; if (++tb == a.k) { tb = 0; ++ta; } }
            };
            auto mfmas = [&](int iw, int ia) {
#pragma unroll
                for (int p = 0; p < MP; ++p)
                    acc[p] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, wr[iw]),
                                                                     __builtin_bit_cast(bf16x8, ar[ia][p]), acc[p], 0, 0, 0);
            };
            // The first fetches are issued on every path (a reduction shorter than the rings
            // fetches step 0 again into the slots it does not use): were their number to depend on
            // a branch, the compiler would no longer know how many loads are in flight when the
            // loop starts and would wait for ALL of them at the top of every round.
#pragma unroll
            for (int i = 0; i < DW; ++i) {
                wr[i] = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(wrsrc, wlane, wq, 0));
                wq += i + 1 < steps ? wstep : 0;
            }
#pragma unroll
            for (int i = 0; i < DA; ++i) {
                const bool real = i < steps;
                const int soff = real ? (ta * hw + tb) * Cs4 + G * chunk : 0;
#pragma unroll
                for (int p = 0; p < MP; ++p) ar[i][p] = lds4[lbase[p] + soff];
                if (real && ++chunk == nch) { chunk = 0; if (++tb == a.k) { tb = 0; ++ta; } }
            }
            int s = 0;
            for (; s + 2 * DW <= steps; s += DW) {     // every step of the group has successors DW and DA ahead
#pragma unroll
                for (int i = 0; i < DW; ++i) { mfmas(i, i % DA); fetch_w(i); fetch_a(i % DA); }
            }
            for (; s < steps; s += DW) {               // the last one or two groups: fetches stop at the end
#pragma unroll
                for (int i = 0; i < DW; ++i)
                    if (s + i < steps) {
                        mfmas(i, i % DA);
                        if (s + i + DW < steps) fetch_w(i);
                        if (s + i + DA < steps) fetch_a(i % DA);
                    }
            }
        }

        // ---- the next tile's halo starts its trip now
        const int tn = t + gridDim.x;
        Tile nxt = decode(tn < total ? tn : 0);
        if (tn >= total) nxt.live = false;
        v4f pre[SI];
        if (nxt.live) issue(nxt, pre);

        // ---- epilogue from the accumulators: register 4n + z of position tile p is channel
        // oc0 + 8n + 4lg + z of position 32*(wp*MP + p) + lt.  One copy of the code per mode, picked once
        // per tile: with the mode tested per value the scalar branches cost as much as the arithmetic.
        auto epilogue = [&](auto mode_tag) {
            constexpr int mode = decltype(mode_tag)::value;
#pragma unroll
            for (int p = 0; p < MP; ++p) {
                const int ty = (int)(e_tyx[p] >> 16), tx = (int)(e_tyx[p] & 0xffffu);
                const int fy = cur.ty0 + ty, fx = cur.tx0 + tx;
                const bool pos_ok = ty != 0xffff && fy < cur.fh && fx < cur.fw;
                const long pos_off = (((long)cur.b * a.Ho + (fy * a.d + cur.ry)) * a.Wo + (fx * a.d + cur.rx)) * a.Co;
                // what the epilogue reads: the layer's output at these positions (data gradient: its
                // slope), or the bias of the lane's channel quads (a few cached bytes per tile)
                v4f yv[4];
#pragma unroll
                for (int n = 0; n < 4; ++n) {
                    const int oc = oc0 + 8 * n + 4 * lg;
                    yv[n] = zero4;
                    if (mode != kDgradPlain && pos_ok && oc < a.Co) {
                        if (mode == kDgradTanh) yv[n] = load4(act_t + pos_off + oc);
                        else yv[n] = *reinterpret_cast<const v4f*>(a.bias + oc);
                    }
                }
#pragma unroll
                for (int n = 0; n < 4; ++n) {
                    const int oc = oc0 + 8 * n + 4 * lg;
                    if (!pos_ok || oc >= a.Co) continue;
                    v4f s4 = (v4f){acc[p][4 * n], acc[p][4 * n + 1], acc[p][4 * n + 2], acc[p][4 * n + 3]};
                    if (mode == kFwdTanh) {
#pragma unroll
                        for (int z = 0; z < 4; ++z) s4[z] = squash(s4[z] + yv[n][z], a.logistic);
                    } else if (mode == kFwdLinear) {
                        s4 += yv[n];
                    } else if (mode == kDgradTanh) {
#pragma unroll
                        for (int z = 0; z < 4; ++z) s4[z] *= squash_slope(yv[n][z], a.logistic);
                    }
                    store4(out_t + pos_off + oc, s4);   // (channel counts are multiples of 4)
                }
            }
        };
        if (cur.live && wave_live) {
            if (a.mode == kFwdTanh) epilogue(std::integral_constant<int, kFwdTanh>{});
            else if (a.mode == kDgradTanh) epilogue(std::integral_constant<int, kDgradTanh>{});
            else if (a.mode == kFwdLinear) epilogue(std::integral_constant<int, kFwdLinear>{});
            else epilogue(std::integral_constant<int, kDgradPlain>{});
        }
        __syncthreads();   // every wave has left this tile's halo
        if (nxt.live) to_lds(pre);
        __syncthreads();
        cur = nxt;
    }
}

}  // namespace mpcnn
