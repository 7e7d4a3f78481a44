// libmpcnn: host side of the whole-image MPCNN forward / backward (see include/mpcnn.h).
//
// The paper keeps each layer's data as a set of fragments, k*k new ones per pooling
// layer (Method, Notation and MPF layer).  Here the whole set is ONE dense tensor per
// layer, [B][rows][cols][channels]: element (r,s) of the patch with top-left (i,j) sits at
// (i + r*d, j + s*d), d = product of the pooling factors so far, so fragment (a,b) of the
// paper is the sub-lattice {y = a mod d, x = b mod d}.  Pooling becomes a stride-1 max
// filter with taps d apart, later C / FC kernels read taps d apart, and the first FC is
// a convolution whose kernel covers the q x q map that remains of a patch.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <memory>
#include <mutex>
#include <new>
#include <type_traits>
#include <vector>

#include "../../include/mpcnn.h"
#include "kernels_direct.hpp"
#include "launchers.hpp"
#include "kernels_conv_bf16.hpp"    // tp_items
#include "kernels_wgrad_tr.hpp"     // its LDS geometry
#include "kernels_wgrad_bf16.hpp"   // its LDS geometry, which the planner shares (no instance is built here)
#include "kernels_pack.hpp"
#include "kernels_reduce.hpp"
#include "kernels_lbfgs.hpp"
#include "kernels_first_bf16.hpp"
#include "kernels_first_f32.hpp"
#include "kernels_l0_wgrad.hpp"
#include "kernels_fused.hpp"

// Device memory of mpcnn_seg_forward_static: a fixed array in the library's device image, so that
// the call needs no allocation.  Every GPU the library runs on holds its own copy, at its own
// address, until the process ends.  In host code the name below is only a handle for
// hipGetSymbolAddress; the kernels are given the address that call returns.
static __device__ __align__(256) unsigned char scratch[MPCNN_STATIC_WORKSPACE_BYTES];

namespace {

thread_local char g_err[512] = "";

mpcnn_status fail(mpcnn_status st, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return st;
}

#define HIP_TRY(expr)                                                                      \
    do {                                                                                   \
        hipError_t e_ = (expr);                                                            \
        if (e_ != hipSuccess)                                                              \
            return fail(MPCNN_EHIP, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), \
                        __FILE__, __LINE__);                                               \
    } while (0)

constexpr int kLossBlocks = 2048;         // most per-workgroup loss shares (= most workgroups of the class-layer kernel)
constexpr int kSoftmaxBlocks = 512;       // workgroups of the unfused softmax kernel
constexpr int kDirectWgradChunks = 512;   // split of the position reduction, direct kernel
constexpr size_t kConvLdsCap = 64 * 1024; // halo bytes per workgroup (two workgroups per CU)
constexpr size_t kWgradLdsCap = 144 * 1024;
constexpr int kNumCU = 256;

inline size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }
inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

// Output-channel tiling of the MFMA kernels: tiles of W channels, OT tiles per workgroup,
// `split` groups of them (blockIdx.y / z), `pad` = channels covered.
struct ChanTiling { int W, OT, split, pad; };
ChanTiling tile_channels(int channels, int W, const int* allowed, int n_allowed)
{
    const int max_ot = allowed[n_allowed - 1];
    const int tiles = ceil_div(channels, W);
    const int split = ceil_div(tiles, max_ot);
    const int per = ceil_div(tiles, split);
    int OT = max_ot;
    for (int i = 0; i < n_allowed; ++i) if (allowed[i] >= per) { OT = allowed[i]; break; }
    return {W, OT, split, OT * split * W};
}
ChanTiling chan_tiling_w(int channels, int W)   // forward / data-gradient kernel instances
{
    static const int allowed[] = {1, 2, 4};
    return tile_channels(channels, W, allowed, 3);
}
// 32-wide MFMA tiles run at the full fp32 matrix rate, 16-wide ones at about 0.87 of it:
// take whichever wastes less once its padding is counted.
ChanTiling chan_tiling(int channels)
{
    const ChanTiling a = chan_tiling_w(channels, 16), b = chan_tiling_w(channels, 32);
    return (a.pad / 0.87 < b.pad) ? a : b;
}

struct Layer {
    int kind;     // mpcnn_kind
    int k;        // kernel side (C, FC) or pooling side (MP)
    int cin, cout;
    int dil;      // spacing of this layer's taps in its input map
    int drop = 0; // MP: trailing rows / columns of the patch-level map that no window covers (side mod k)
    // columns, where they differ from the rows (a rectangular pool, and every layer after it):
    int k2 = 0, dil2 = 0, drop2 = 0;
    bool rect = false;   // k2 != k or dil2 != dil: the fp32 matrix instruction's kernels and the direct kernels take such a layer
    bool tanh_out;
    size_t p_off; // offset of this layer's [(k*k*cin + 1) x cout] block in the parameter buffer
    size_t p_len;
    // matrix-core paths (decided once from the channel counts)
    bool fwd_mfma = false, dgrad_mfma = false, wgrad_mfma = false;
    bool class_fused = false;             // last FC handled by class_layer_kernel
    ChanTiling fwd_ct{}, dgrad_ct{};
    bool fwd_bm = false, dgrad_bm = false; // bf16 storage: multiply on the bf16 matrix instruction
    int fwd_rpad = 0, dgrad_rpad = 0;     // reduced channels padded to 16
    size_t fwd_pack_off = 0, fwd_pack_len = 0, dgrad_pack_off = 0, dgrad_pack_len = 0;
};

struct TilePlan {
    int PT = 0, NW = 4, Ty = 0, Tx = 0, nty = 0, ntx = 0;
    int MP = 0;           // > 0: conv_ts_kernel (result tiles dealt out to the waves), MP position tiles per wave
    size_t lds = 0;
    bool ok = false;
};
struct WgradPlan {
    bool ok = false;
    bool bm = false;      // bf16 storage: the bf16 matrix instruction, 16 positions per MFMA
    bool tr = false;      // ... with operands from the transposing LDS read (wgrad_tr_kernel)
    int Tx = 0, TxP = 0, nty = 0, ntx = 0, tiles_total = 0, tiles_per_slab = 0, slabs = 0;
    int Mt = 0, Nt = 0, wm = 0, wn = 0, wk = 0, mw = 0, gm = 0, gn = 0;
    size_t lds = 0;
    size_t plen = 0;      // floats per partial result (tiled layout)
    int hl = 0;           // halo items per loading thread and tile (fp32 matrix instruction kernel)
    // direct kernel fallback
    int rows_per_chunk = 0, chunks = 0;
    bool l0m = false;     // the image layer's own kernel (l0_wgrad_mfma_kernel): `chunks` workgroups, flat partial results
};

// Per-call geometry: dense map sizes, launch plans and workspace offsets.
struct Geom {
    int B = 0, H = 0, W = 0;
    bool training = false;
    std::vector<int> rows, cols;      // output map of layer l
    std::vector<size_t> act_off;      // byte offset of layer l's output in the workspace
    std::vector<size_t> code_off;     // MP layers: byte offset of the argmax map
    std::vector<TilePlan> fwd, dgrad;
    std::vector<WgradPlan> wgrad;
    int pad_top = 0, pad_left = 0;    // same-size forward: H, W are the mirrored image's, which starts
    int src_h = 0, src_w = 0;         //   this far above / left of the caller's src_h x src_w image
    bool staged = false;              // the image is copied to channels-last storage first
    int label_h = 0, probs_rows = 0;  // rows of the label / weight arrays and of the probs array (bands: the whole image's)
    bool accumulate = false;          // gradients and loss are added to what the net holds (bands after the first)
    bool fixed_partials = false;      // partial-sum buffers sized by bounds that hold for every map size (bands)
    size_t staged_off = 0;            // that copy (C0 > 1, or bf16 storage)
    size_t delta_off[2] = {0, 0};     // two delta buffers, each as large as the largest map
    std::vector<size_t> partial_off;  // per parametrised layer: its slab / block partial sums
    std::vector<int> partial_n;
    std::vector<size_t> partial_len;  // floats per partial result
    size_t loss_partial_off = 0;
    // first convolution followed by a pool: routing through the pool and the convolution's
    // parameter gradient run as one kernel (l0_wgrad_fused_kernel), in l0_blocks workgroups
    bool l0_fused = false;
    int l0_blocks = 0, l0_nty = 0, l0_ntx = 0;
    size_t l0_lds = 0;
    size_t total = 0;
};

struct ProfSite {
    char name[48];
    int layer, step, launches;
    double ms, flops, bytes;
};
struct ProfPending { int site; hipEvent_t e0, e1; };

// Plans are kept per (sizes, mode, tiling hints): a call with sizes seen before plans nothing.
struct GeomKey {
    int B, H, W, training, same, hint_pt, hint_mp;
    bool operator==(const GeomKey& o) const
    {
        return B == o.B && H == o.H && W == o.W && training == o.training && same == o.same &&
               hint_pt == o.hint_pt && hint_mp == o.hint_mp;
    }
};
constexpr size_t kGeomCacheSize = 8;

}  // namespace

struct mpcnn_net {
    std::vector<Layer> layers;
    int in_ch = 0, patch = 0, n_cls = 0;
    size_t n_params = 0, pack_len = 0;
    int loss_kind = MPCNN_LOSS_MCCE;
    int loss_shares = 0;          // per-workgroup loss shares the forward left for the closing reduce
    double* loss_out = nullptr;   // where that reduce puts their sum
    bool bf16 = false;            // activations and deltas stored in bf16 (arithmetic stays fp32)
    float* d_params = nullptr;
    float* d_params0 = nullptr;   // copy of the parameters a safeguarded step starts from
    double* d_scalar = nullptr;   // fp64 results of that step's reductions (8)
    int logistic = 0;             // squashing function of C and hidden FC layers: 0 tanh, 1 logistic
    int hint_pt = 0, hint_mp = 0; // mpcnn_set_conv_tiling: 0 = the planner's choice
    int class_max_blocks = 512;   // workgroups of the class-layer kernel's training form resident on the chip
    // limited-memory BFGS: pairs in a ring of lb_m + 1 slots (one always free for the candidate)
    int lb_m = 0, lb_head = 0, lb_count = 0;
    bool lb_have_prev = false;
    float *d_lb_S = nullptr, *d_lb_Y = nullptr;            // [lb_m + 1][n_params]
    float *d_lb_theta_prev = nullptr, *d_lb_g_prev = nullptr, *d_lb_p = nullptr;
    double *d_lb_part = nullptr, *d_lb_alpha = nullptr;    // partial sums (5 x kLbBlocks), first-loop coefficients
    std::vector<double> lb_sy, lb_yy;                      // per slot
    float* d_wread = nullptr;     // what the kernels read: d_params, or its copy rounded to bf16 values
    bool wread_stale = true;
    float* d_grads = nullptr;
    float* d_packs = nullptr;
    bool packs_stale = true;
    int device = -1;
    bool lds_attr_set = false;
    // plans of the sizes seen so far (oldest dropped first)
    mutable std::vector<std::pair<GeomKey, std::shared_ptr<const Geom>>> geoms;
    // what the last forward / backward left behind (for the test hooks)
    std::shared_ptr<const Geom> last;
    void* last_ws = nullptr;
    // profiling
    bool prof_on = false;
    std::vector<ProfSite> sites;
    std::vector<ProfPending> pending;
    std::vector<hipEvent_t> pool;
};

namespace {

// ------------------------------------------------------------------ profiling
struct ProfScope {
    mpcnn_net* net;
    hipStream_t st;
    hipEvent_t e1 = nullptr;
    ProfScope(mpcnn_net* n, hipStream_t s, const char* name, int layer, int step, double flops,
              double bytes) : net(n), st(s)
    {
        if (!net->prof_on) return;
        int site = -1;
        for (size_t i = 0; i < net->sites.size(); ++i)
            if (net->sites[i].layer == layer && strcmp(net->sites[i].name, name) == 0) { site = (int)i; break; }
        if (site < 0) {
            ProfSite ps{};
            snprintf(ps.name, sizeof ps.name, "%s", name);
            ps.layer = layer; ps.step = step;
            net->sites.push_back(ps);
            site = (int)net->sites.size() - 1;
        }
        net->sites[site].flops = flops;
        net->sites[site].bytes = bytes;
        hipEvent_t e0 = take(), e = take();
        if (!e0 || !e) return;
        (void)hipEventRecord(e0, st);
        e1 = e;
        net->pending.push_back({site, e0, e1});
    }
    ~ProfScope() { if (e1) (void)hipEventRecord(e1, st); }
    hipEvent_t take()
    {
        if (!net->pool.empty()) { hipEvent_t e = net->pool.back(); net->pool.pop_back(); return e; }
        hipEvent_t e = nullptr;
        if (hipEventCreate(&e) != hipSuccess) return nullptr;
        return e;
    }
};
#define LAUNCH(name, layer, step, flops, bytes, ...)                                  \
    do {                                                                              \
        ProfScope ps_(net, st, name, (int)(layer), step, (double)(flops), (double)(bytes)); \
        __VA_ARGS__;                                                                  \
    } while (0)

// ------------------------------------------------------------------ planning
// Ty x Tx tile (<= max_pos positions) of a residue class with extents fh x fw: fewest
// tiles first, then the smallest halo; the halo must fit `lds_cap`.
bool choose_tile(int fh, int fw, int max_pos, int k, int k2, size_t pitch_bytes, size_t extra_bytes,
                 size_t lds_cap, int* Ty, int* Tx)
{
    long best_tiles = -1, best_halo = 0;
    for (int ty = 1; ty <= std::min(fh, max_pos); ++ty) {
        for (int tx = 1; tx <= std::min(fw, max_pos / ty); ++tx) {
            long halo = (long)(ty + k - 1) * (tx + k2 - 1);
            if ((size_t)halo * pitch_bytes + extra_bytes > lds_cap) continue;
            long tiles = (long)ceil_div(fh, ty) * ceil_div(fw, tx);
            if (best_tiles < 0 || tiles < best_tiles || (tiles == best_tiles && halo < best_halo)) {
                best_tiles = tiles; best_halo = halo; *Ty = ty; *Tx = tx;
            }
        }
    }
    return best_tiles > 0;
}

// Tile plan of the convolution kernels for a map of out_r x out_c positions, a k x k2 filter (rows x columns)
// with taps d rows / d2 columns apart (k2 != k or d2 != d: a rectangular pool, or a layer behind one).
TilePlan plan_conv_tiles(int B, int out_r, int out_c, int d, int d2, int k, int k2, int rpad, const ChanTiling& ct, bool bm,
                         int hint_pt = 0, int hint_mp = 0)
{
    TilePlan best;
    double best_cost = 0;
    const int fh = ceil_div(out_r, d), fw = ceil_div(out_c, d2);
    const size_t pitch = bm ? 16 * (size_t)(rpad / 8 + 1) : sizeof(float) * (rpad + 4);   // one halo position in LDS
    if (!bm && (ct.W == 32 || ct.OT == 1)) {
        // conv_ts_kernel: W*PT positions x W*OT channels, OT*PT/MP waves (16-wide: one channel tile, 32 cycles
        // per instruction; 32-wide: 64 cycles).  Cost of the busiest CU:
        // its workgroups' matrix instructions one after the other, plus, once per round of
        // co-resident workgroups, what is not hidden behind another's multiplications
        // (staging the halo at ~8 bytes per cycle, a memory round trip, the stores).
        const bool w16 = ct.W == 16;
        const int steps = k * k2 * (rpad / (w16 ? 16 : 8));
        for (int PT : {2, 4, 8, 16})
            for (int MP : {1, 2, 4}) {
                const int NW = ct.OT * PT / MP;
                if (PT % MP || (NW != 4 && NW != 8)) continue;
                const bool built4 = (ct.OT == 4 && (PT == 4 || PT == 8)) || (ct.OT == 2 && PT == 8) || (ct.OT == 1 && PT == 16);
                if (w16 ? PT < 4 : (MP == 4 ? !built4 : PT > 8)) continue;   // (the instances that are built)
                // four tiles per wave pay where the reduction is long: with 64 steps (2 x 2 taps of 128 channels) the
                // longer epilogue and the fewer workgroups per compute unit cost more than the weight fetches saved
                // (measured: 2012 -> 2074 us; 9 taps of 64 channels, 72 steps: 1242 -> 1185 us)
                if (!w16 && MP == 4 && steps < 72 && hint_mp != 4) continue;
                if ((hint_pt && PT != hint_pt) || (hint_mp && MP != hint_mp)) continue;
                // measured: a wave with one tile spends ~12 % more per instruction on operand
                // fetches than one with two
                const double t_mul1 = (double)steps * 4 * ct.OT * PT * (w16 ? 32 : 64) / 4 * (MP >= 4 ? 0.94 : (MP >= 2 ? 1.0 : 1.12));   // (a weight fetch per 4 MP instructions: each costs the matrix pipe about 100 cycles)
                for (int ty = 1; ty <= std::min(fh, ct.W * PT); ++ty)
                    for (int tx = 1; tx <= std::min(fw, ct.W * PT / ty); ++tx) {
                        const size_t lds = std::max((size_t)(ty + k - 1) * (tx + k2 - 1) * pitch, (size_t)1024);
                        if (lds > (size_t)150 * 1024) break;
                        const int nty = ceil_div(fh, ty), ntx = ceil_div(fw, tx);
                        const double wgs = (double)B * d * d2 * nty * ntx * ct.split;
                        const int together = (int)std::max<size_t>(1, std::min<size_t>(16 / NW, (size_t)(160 * 1024) / lds));
                        const double per_cu = std::ceil(wgs / kNumCU);
                        // fewer than 8 waves on the CU leave SIMDs idle in every wait
                        const double t_mul = t_mul1 * (NW * std::min<double>(together, per_cu) >= 8 ? 1.0 : 1.25);
                        const double t_rest = 4000.0 + (double)lds / 8;
                        const double cost = per_cu * t_mul + std::ceil(per_cu / together) * t_rest;
                        if (!best.ok || cost < best_cost) {
                            best.PT = PT; best.NW = NW; best.MP = MP; best.Ty = ty; best.Tx = tx;
                            best.nty = nty; best.ntx = ntx; best.lds = lds; best.ok = true;
                            best_cost = cost;
                        }
                    }
            }
        if (best.ok) return best;
    }
    if (bm) {
        // conv_ts_kernel on the bf16 matrix instruction (32 cycles per instruction, 16 channels
        // of a tap per step).  The instruction stream of a workgroup is an eighth of the fp32
        // one, so staging and stores weigh 8 times more: large tiles, MP = 4 where possible (a wave
        // with 2 position tiles asks the vector cache for twice the weights per instruction: the
        // cache, not the matrix pipe, then sets the pace), two workgroups per compute unit.
        const int steps = k * k * (rpad / 16);
        // (the kernel forms element offsets inside one image in 32 bits)
        if ((size_t)(out_r + (k - 1) * d) * (out_c + (k - 1) * d) * rpad >= (1ull << 31)) return best;
        for (int PT : {2, 4, 8, 16})
            for (int MP : {2, 4}) {
                const int NW = ct.OT * PT / MP;
                if (PT % MP || (NW != 4 && NW != 8)) continue;
                const double t_mul1 = (double)steps * ct.OT * PT * 32 / 4 * (MP == 4 ? 1.0 : 1.6);
                for (int ty = 1; ty <= std::min(fh, 32 * PT); ++ty)
                    for (int tx = 1; tx <= std::min(fw, 32 * PT / ty); ++tx) {
                        const size_t lds = std::max((size_t)(ty + k - 1) * (tx + k - 1) * pitch, (size_t)1024);
                        if (lds > (size_t)150 * 1024) break;
                        // a thread holds its share of the next tile's halo in registers
                        if ((long)(ty + k - 1) * (tx + k - 1) * (rpad / 8) > (long)mpcnn::tp_items(MP) * 64 * NW) break;
                        const int nty = ceil_div(fh, ty), ntx = ceil_div(fw, tx);
                        const double wgs = (double)B * d * d * nty * ntx * ct.split;
                        const int together = (int)std::max<size_t>(1, std::min<size_t>(8 / NW, (size_t)(160 * 1024) / lds));
                        const double per_cu = std::ceil(wgs / kNumCU);
                        const double t_rest = 4000.0 + (double)lds / 8 + 32.0 * ct.OT * PT * 16;   // + the stores
                        // co-resident workgroups hide each other's staging and stores; alone, a
                        // workgroup pays for them in full
                        const double cost = together >= 2 ? per_cu * t_mul1 + std::ceil(per_cu / together) * t_rest
                                                          : per_cu * (t_mul1 + t_rest);
                        if (!best.ok || cost < best_cost) {
                            best.PT = PT; best.NW = NW; best.MP = MP; best.Ty = ty; best.Tx = tx;
                            best.nty = nty; best.ntx = ntx; best.lds = lds; best.ok = true;
                            best_cost = cost;
                        }
                    }
            }
        return best;
    }
    const int regs_per_tile = ct.W * ct.W / 64;
    for (int PT : {64 / ct.W, 128 / ct.W}) {            // 64 or 128 positions per workgroup
        if (ct.OT * PT * regs_per_tile > (ct.W == 16 ? 64 : 128)) continue;  // accumulator registers per lane
        for (int NW : {4, 8}) {
            TilePlan p;
            p.PT = PT; p.NW = NW;
            if (!choose_tile(fh, fw, ct.W * PT, k, k2, pitch, 0, kConvLdsCap, &p.Ty, &p.Tx)) continue;
            p.nty = ceil_div(fh, p.Ty); p.ntx = ceil_div(fw, p.Tx);
            size_t halo = (size_t)(p.Ty + k - 1) * (p.Tx + k2 - 1) * pitch;
            size_t part = (size_t)NW * ct.OT * (ct.W / 4) * (ct.W + 1) * 4 * sizeof(float);
            p.lds = std::max(halo, part);
            if (p.lds > 150 * 1024) continue;
            if (NW == 8 && k * k2 * (rpad / (256 / ct.W)) < 16) continue;   // too few reduction steps to split 8 ways
            p.ok = true;
            // Measured: two co-resident 4-wave workgroups with large tiles (LDS allows no more than
            // two) only overlap well once their phases have drifted apart, i.e. over many rounds;
            // for a few rounds one 8-wave workgroup per CU is faster.  Small tiles: 4 waves.
            const double wgs = (double)B * d * d2 * p.nty * p.ntx * ct.split;
            const double per_cu = wgs / kNumCU;
            const int steps = k * k2 * (rpad / (256 / ct.W));
            const bool want8 = ct.W == 32 && ct.OT * PT >= 4 && steps >= 64 && per_cu < 8;
            if ((NW == 8) != want8) continue;
            const double rounds = NW == 8 ? std::ceil(per_cu) : std::ceil(per_cu / 2);
            const double cost = rounds * (ct.W * PT / 16 + 1.0);
            if (!best.ok || cost < best_cost) { best = p; best_cost = cost; }
        }
    }
    return best;
}

unsigned magic_of(unsigned x) { return x <= 1 ? 0u : (unsigned)(((1ull << 32) + x - 1) / x); }

WgradPlan plan_wgrad(const Layer& ly, int B, int in_r, int in_c, int out_r, int out_c, bool bm)
{
    WgradPlan w;
    const int d = ly.dil, k = ly.k, d2 = ly.dil2, k2 = ly.k2;   // rows; columns
    const int fh = ceil_div(out_r, d), fw = ceil_div(out_c, d2);
    // the kernel forms element offsets inside one image in 32 bits
    // (and, through buffer descriptors, byte offsets inside one image's tensor in 32 bits)
    const size_t es = bm ? 2 : 4;
    const bool fits32 = (size_t)in_r * in_c * ly.cin < (1ull << 31) &&
                        (size_t)out_r * out_c * ly.cout < (1ull << 31) && (k + 3) * d < 65536 &&
                        (size_t)in_r * in_c * ly.cin * es < (1ull << 32) && (size_t)out_r * out_c * ly.cout * es < (1ull << 32);
    // the bf16 instruction's kernels take square filters at one spacing only
    bm = bm && !ly.rect;
    // the bf16 instruction's kernel gives a wave pairs of column tiles: not for 32 maps or fewer
    // - except for an image layer's few channels, where that kernel, half of its instructions wasted,
    // is still ahead of the fp32 instruction's (7 x 7 filters on 2 x 3 x 2048 x 2048, 32 maps: 1.51 -> 1.34 ms)
    bm = bm && (ly.cout > 32 || ly.cin < 8);
    if (bm && ly.wgrad_mfma && fits32 && ly.cin % 32 == 0) {
        // wgrad_tr_kernel: the tiles are raw copies in planes of 32 channels.  Same choices as for
        // wgrad_bm_kernel below: wave split and tile width together, by the busiest workgroup's
        // time - its matrix instructions, or taking the tiles in, whichever is longer.
        const int Mt = k * k * ly.cin / 32 + 1, Nt = ceil_div(ly.cout, 32), Nu = ceil_div(Nt, 2);
        double best = -1;
        for (int wn : {4, 2, 1})
            for (int wm : {1, 2, 4}) {
                if (wm * wn > 4) continue;
                const int wk = 4 / (wm * wn);
                const int gm = ceil_div(Mt, mpcnn::kWgTrMaxTiles * wm), mw = ceil_div(Mt, gm * wm);
                const int gn = ceil_div(Nu, wn);
                const int target = std::max(1, kNumCU / (gm * gn));
                for (int tx = 1; tx <= fw && tx <= 64; ++tx) {
                    const int nch = ceil_div(tx, 16), txp = 16 * nch;
                    const mpcnn::TrGeom tg = mpcnn::tr_geom(nch, k, ly.cin, wn);
                    size_t lds = (size_t)2 * tg.buf_b;
                    if (wk > 1) lds = std::max(lds, (size_t)2 * mw * 2 * 4096);
                    const int h_items = tg.hh * tg.hwp * (ly.cin / 8), d_items = 4 * txp * 8 * wn;
                    if (h_items > mpcnn::kTrStageH * 256 || d_items > mpcnn::kTrStageD * 256 ||
                        lds > kWgradLdsCap || (tg.hwp + 1) * d >= 65536)
                        continue;
                    const int ntx = ceil_div(fw, tx);
                    const long tiles = (long)B * d * d * ceil_div(fh, 4) * ntx;
                    if (tiles * std::max(std::max(ntx, ceil_div(fh, 4)), d) >= (1ll << 31)) continue;
                    const long tps = (tiles + target - 1) / target;
                    const double t_mul = (4.0 / wk) * nch * 2 * mw * 36.0;          // cycles of the instruction stream
                    const double t_load = (h_items + d_items) * 16.0 / 7.0;          // cycles to take the tile in
                    const double cost = (double)tps * (std::max(t_mul, t_load) + 1500.0);
                    if (best < 0 || cost < best) {
                        best = cost;
                        w.wm = wm; w.wn = wn; w.wk = wk; w.mw = mw; w.gm = gm; w.gn = gn;
                        w.Tx = tx; w.TxP = txp; w.lds = std::max(lds, (size_t)1024);
                    }
                }
            }
        if (best >= 0) {
            w.bm = true; w.tr = true; w.Mt = Mt; w.Nt = Nt;
            w.plen = (size_t)Mt * Nt * 1024;
            const int target = std::max(1, kNumCU / (w.gm * w.gn));
            w.nty = ceil_div(fh, 4); w.ntx = ceil_div(fw, w.Tx);
            w.tiles_total = B * d * d * w.nty * w.ntx;
            w.tiles_per_slab = ceil_div(w.tiles_total, target);
            w.slabs = ceil_div(w.tiles_total, w.tiles_per_slab);
            w.ok = true;
            return w;
        }
        w = WgradPlan();
    }
    if (bm && ly.wgrad_mfma && fits32) {
        // wgrad_bm_kernel.  Every group of workgroups (gm x gn of them cover the result) stages
        // all tiles again, and a compute unit takes in roughly 7 bytes per cycle, which at
        // bf16 speed is often the slower side: pick the wave split and the tile width
        // together, by the time of the busiest workgroup.
        const int Mt = ceil_div(k * k * ly.cin + 1, 32), Nt = ceil_div(ly.cout, 32), Nu = ceil_div(Nt, 2);
        const int hh = 4 + k - 1;
        double best = -1;
        for (int wn : {4, 2, 1})
            for (int wm : {1, 2, 4}) {
                if (wm * wn > 4) continue;
                const int wk = 4 / (wm * wn);
                const int gm = ceil_div(Mt, mpcnn::kWgBmMaxTiles * wm), mw = ceil_div(Mt, gm * wm);
                const int gn = ceil_div(Nu, wn);
                const int target = std::max(1, kNumCU / (gm * gn));
                for (int tx = 1; tx <= fw && tx <= 64; ++tx) {
                    const int nch = ceil_div(tx, 16), txp = 16 * nch;
                    const mpcnn::BmGeom bg = mpcnn::bm_geom(nch, k, ly.cin, wn);
                    size_t lds = (size_t)2 * bg.buf_e * 2;
                    if (wk > 1) lds = std::max(lds, (size_t)2 * mw * 2 * 4096);
                    const int h_items = hh * (bg.hwp / 2) * ceil_div(ly.cin, 8), d_items = 4 * (txp / 2) * 8 * wn;
                    if (h_items > mpcnn::kBmStageH * 256 || d_items > mpcnn::kBmStageD * 256 ||
                        lds > kWgradLdsCap || (bg.hwp + 1) * d >= 65536)
                        continue;
                    const int ntx = ceil_div(fw, tx);
                    const long tiles = (long)B * d * d * ceil_div(fh, 4) * ntx;
                    if (tiles * std::max(std::max(ntx, ceil_div(fh, 4)), d) >= (1ll << 31)) continue;
                    const long tps = (tiles + target - 1) / target;
                    const double t_mul = (4.0 / wk) * nch * 2 * mw * 36.0;          // cycles of the instruction stream
                    const double t_load = (h_items + d_items) * 32.0 / 7.0;          // cycles to take the tile in
                    const double cost = (double)tps * (std::max(t_mul, t_load) + 1500.0);
                    if (best < 0 || cost < best) {
                        best = cost;
                        w.wm = wm; w.wn = wn; w.wk = wk; w.mw = mw; w.gm = gm; w.gn = gn;
                        w.Tx = tx; w.TxP = txp; w.lds = std::max(lds, (size_t)1024);
                    }
                }
            }
        if (best >= 0) {
            w.bm = true; w.Mt = Mt; w.Nt = Nt;
            w.plen = (size_t)Mt * Nt * 1024;
            const int target = std::max(1, kNumCU / (w.gm * w.gn));
            w.nty = ceil_div(fh, 4); w.ntx = ceil_div(fw, w.Tx);
            w.tiles_total = B * d * d * w.nty * w.ntx;
            w.tiles_per_slab = ceil_div(w.tiles_total, target);
            w.slabs = ceil_div(w.tiles_total, w.tiles_per_slab);
            w.ok = true;
            return w;
        }
        w = WgradPlan();
    }
    if (ly.wgrad_mfma && fits32) {
        // split of the four waves over result rows / columns / tile rows: least padded work,
        // then fewest workgroup groups (each group stages the tiles again)
        const int Mt = ceil_div(k * k2 * ly.cin, 32), Nt = ceil_div(ly.cout, 32);
        long best_pad = -1; int best_groups = 0;
        for (int wn : {4, 2, 1})
            for (int wm : {1, 2, 4}) {
                if (wm * wn > 4) continue;
                const int wk = 4 / (wm * wn);
                const int gm = ceil_div(Mt, mpcnn::kWgMaxTiles * wm), mw = ceil_div(Mt, gm * wm);
                const int gn = ceil_div(Nt, wn);
                const long pad = (long)gm * wm * mw * gn * wn;
                // (equal on both counts: the split with fewer waves along the tile's rows - measured 3 % ahead
                // on a 16 x 7 tile result, their partial tiles need no meeting in LDS)
                if (best_pad < 0 || pad < best_pad || (pad == best_pad && gm * gn < best_groups) ||
                    (pad == best_pad && gm * gn == best_groups && wk < w.wk)) {
                    best_pad = pad; best_groups = gm * gn;
                    w.wm = wm; w.wn = wn; w.wk = wk; w.mw = mw; w.gm = gm; w.gn = gn;
                }
            }
        w.Mt = Mt; w.Nt = Nt;
        w.plen = (size_t)Mt * Nt * 1024 + (size_t)Nt * 32;
        // tile = 4 rows x Tx columns of a residue class: fewest matrix-core ticks of the busiest
        // workgroup (a tile's work grows with Tx rounded up to 4, plus a fixed cost per tile)
        const int cq = ceil_div(ly.cin, 4), hh = 4 + k - 1;
        const int target = std::max(1, kNumCU / (w.gm * w.gn));
        const double col_ticks = (4.0 / w.wk) * w.mw * 32.0;
        // The loading threads hold a tile's items in registers: 8 halo items each, or, where
        // that keeps the tile narrower than 16 columns (many channels, large filters), 16 -
        // the wider instance issues 8 more loads per tile whether it needs them or not.
        // Staging time of a tile (estimate used to compare the two instances): one trip to
        // memory plus a few hundred cycles per round of 256 items.
        auto tile_time = [&](int txp, bool with_load) {
            const double t_load = 3000.0 + 6.0 * 64.0 * ceil_div(hh * (txp + k2 - 1) * cq + 4 * txp * 8 * w.wn, 256);
            return (with_load ? std::max(txp * col_ticks, t_load) : txp * col_ticks) + 1500.0;
        };
        struct Pick { double cost = -1; int Tx = 0, TxP = 0; size_t lds = 0; long tps = 0; };
        auto pass = [&](int hl, bool with_load) {
            Pick pk;
            for (int tx = 1; tx <= fw; ++tx) {
                const int txp = ceil_div(tx, 4) * 4, hwp = txp + k2 - 1;
                const size_t buf = (size_t)4 * w.wn * (txp * 32 + 32) + (size_t)4 * cq * ((hh * hwp) | 1);
                size_t lds = 2 * buf * sizeof(float) + 128;  // slack: the operand prefetch runs one chunk ahead; 16 unread bytes behind it
                if (w.wk > 1) lds = std::max(lds, (size_t)2 * w.mw * 4096);
                lds = std::max(lds, (size_t)1024);
                if (hh * hwp * cq > hl * 256 || 4 * txp * 8 * w.wn > mpcnn::kWgStageD * 256 || lds > kWgradLdsCap)
                    continue;
                const int ntx = ceil_div(fw, tx);
                const long tiles = (long)B * d * d2 * ceil_div(fh, 4) * ntx;
                if (tiles * std::max(std::max(ntx, ceil_div(fh, 4)), std::max(d, d2)) >= (1ll << 31) || (long)hwp * d2 >= 65536) continue;
                const long tps = (tiles + target - 1) / target;
                const double cost = (double)tps * tile_time(txp, with_load);
                if (pk.cost < 0 || cost <= pk.cost) { pk.cost = cost; pk.Tx = tx; pk.TxP = txp; pk.lds = lds; pk.tps = tps; }
            }
            return pk;
        };
        Pick pk = pass(mpcnn::kWgStageH, false);
        w.hl = mpcnn::kWgStageH;
        if (pk.cost < 0 || (pk.TxP < 16 && pk.Tx < fw)) {
            const Pick wide = pass(2 * mpcnn::kWgStageH, true);
            if (wide.cost >= 0 && (pk.cost < 0 || wide.cost < (double)pk.tps * tile_time(pk.TxP, true))) {
                pk = wide; w.hl = 2 * mpcnn::kWgStageH;
            }
        }
        const double best = pk.cost;
        w.Tx = pk.Tx; w.TxP = pk.TxP; w.lds = pk.lds;
        if (best >= 0) {
            w.nty = ceil_div(fh, 4); w.ntx = ceil_div(fw, w.Tx);
            w.tiles_total = B * d * d2 * w.nty * w.ntx;
            w.tiles_per_slab = ceil_div(w.tiles_total, target);
            w.slabs = ceil_div(w.tiles_total, w.tiles_per_slab);
            w.ok = true;
            return w;
        }
    }
    w = WgradPlan();
    long rows_total = (long)B * out_r;
    w.rows_per_chunk = (int)std::max<long>(1, (rows_total + kDirectWgradChunks - 1) / kDirectWgradChunks);
    w.chunks = (int)((rows_total + w.rows_per_chunk - 1) / w.rows_per_chunk);
    w.plen = ly.p_len;
    return w;
}

// Workgroups of the class-layer kernel: as many as are resident at once (a second, partly
// filled round would double its time; it is a chain of dependent steps per position and lives
// on the bytes in flight), fewer on small maps, whose shares the closing reduce has to add.
int class_blocks(const mpcnn_net* net, long positions)
{
    const long want = std::min<long>(net->class_max_blocks, std::max<long>(512, positions / 1024));
    return (int)std::min<long>(want, (positions + 15) / 16);
}

bool make_geom(const mpcnn_net* net, int B, int H, int W, bool training, Geom* g, bool mirrored = false,
               bool fixed_partials = false)
{
    g->fixed_partials = fixed_partials;
    if (B < 1 || H < net->patch || W < net->patch) return false;
    const size_t L = net->layers.size();
    g->B = B; g->H = H; g->W = W; g->training = training;
    g->rows.assign(L, 0); g->cols.assign(L, 0);
    g->act_off.assign(L, 0); g->code_off.assign(L, 0);
    g->fwd.assign(L, TilePlan()); g->dgrad.assign(L, TilePlan()); g->wgrad.assign(L, WgradPlan());
    g->partial_off.assign(L, 0); g->partial_n.assign(L, 0); g->partial_len.assign(L, 0);
    size_t off = 0, max_act = 0;
    const size_t es = net->bf16 ? 2 : 4;   // bytes per stored activation / delta element
    g->src_h = H; g->src_w = W;
    g->staged = net->in_ch > 1 || net->bf16 || mirrored;
    if (g->staged) {
        g->staged_off = off;
        off = align_up(off + es * (size_t)B * H * W * net->in_ch);
    }
    int r = H, c = W;
    for (size_t l = 0; l < L; ++l) {
        const Layer& ly = net->layers[l];
        const int in_r = r, in_c = c;
        // a pool that leaves `drop` trailing rows of every patch's map unused shortens the
        // whole-image map by as many rows of this spacing
        r -= (ly.k - 1 + ly.drop) * ly.dil;
        c -= (ly.k2 - 1 + ly.drop2) * ly.dil2;
        if (r < 1 || c < 1) return false;
        g->rows[l] = r; g->cols[l] = c;
        size_t bytes = es * (size_t)B * r * c * ly.cout;
        max_act = std::max(max_act, bytes);
        if (ly.kind == MPCNN_MP) continue;
        if (ly.fwd_mfma) g->fwd[l] = plan_conv_tiles(B, r, c, ly.dil, ly.dil2, ly.k, ly.k2, ly.fwd_rpad, ly.fwd_ct, ly.fwd_bm, net->hint_pt, net->hint_mp);
        if (training && ly.class_fused) {
            g->partial_n[l] = class_blocks(net, (long)B * r * c);
            g->partial_len[l] = ly.p_len;
        } else if (training) {
            if (ly.dgrad_mfma && l > 0)
                g->dgrad[l] = plan_conv_tiles(B, in_r, in_c, ly.dil, ly.dil2, ly.k, ly.k2, ly.dgrad_rpad, ly.dgrad_ct, ly.dgrad_bm, net->hint_pt, net->hint_mp);
            g->wgrad[l] = plan_wgrad(ly, B, in_r, in_c, r, c, net->bf16);
            const WgradPlan& w = g->wgrad[l];
            g->partial_n[l] = w.ok ? w.slabs : w.chunks;
            g->partial_len[l] = w.plen;
        }
    }
    if (r != H - net->patch + 1 || c != W - net->patch + 1) return false;
    g->l0_fused = false;
    if (training && L >= 2) {
        const Layer& l0 = net->layers[0];
        const Layer& l1 = net->layers[1];
        const size_t lds = sizeof(float) * ((size_t)mpcnn::kL0Rows * mpcnn::kL0Cols * l0.cout +
                                            (size_t)(mpcnn::kL0Rows + l0.k - 1) * (mpcnn::kL0Cols + l0.k - 1) * l0.cin);
        if (l0.kind != MPCNN_MP && !l0.class_fused && !l0.rect && l0.dil == 1 && l1.kind == MPCNN_MP && !l1.rect &&
            l1.dil == 1 && l1.k >= 2 && l1.k <= 4 && l0.cout % 4 == 0 && l0.p_len <= (size_t)mpcnn::kL0MaxPerThread * 256 && lds <= 64 * 1024 &&
            (long)B * ceil_div(g->rows[0], mpcnn::kL0Rows) * ceil_div(g->cols[0], mpcnn::kL0Cols) <= 2 * kNumCU) {
            // small images only (one tile per workgroup, where the two separate launches are
            // bound by their round trips to memory): the kernel multiplies on the vector ALU,
            // and on a large image the matrix-core kernel behind a separate routing pass is faster
            g->l0_fused = true;
            g->l0_nty = ceil_div(g->rows[0], mpcnn::kL0Rows); g->l0_ntx = ceil_div(g->cols[0], mpcnn::kL0Cols);
            g->l0_blocks = B * g->l0_nty * g->l0_ntx;
            g->l0_lds = lds;
            g->wgrad[0] = WgradPlan();
            g->partial_n[0] = g->l0_blocks;
            g->partial_len[0] = l0.p_len;
        }
    }
    if (training && !g->l0_fused) {
        // the image layer's weight gradient on its own matrix-instruction kernel
        const Layer& l0 = net->layers[0];
        if (l0.kind != MPCNN_MP && !l0.class_fused && !l0.rect && l0.dil == 1 && (l0.cin == 1 || l0.cin == 3) &&
            (l0.k == 3 || l0.k == 5 || l0.k == 7)) {
            WgradPlan w;
            w.l0m = true;
            const long tiles = (long)B * ceil_div(g->rows[0], mpcnn::kL0wTy) * ceil_div(g->cols[0], mpcnn::kL0wTx);
            w.tiles_total = (int)tiles;
            // two workgroups per compute unit are resident with the largest filter banks (140 registers):
            // a third, waiting its turn, would walk its tiles alone at the end
            w.chunks = (int)std::min<long>(tiles, 2L * kNumCU);
            w.plen = l0.p_len;
            if (tiles < (1l << 30)) {
                g->wgrad[0] = w;
                g->partial_n[0] = w.chunks;
                g->partial_len[0] = l0.p_len;
            }
        }
    }
    if (training) {
        for (size_t l = 0; l < L; ++l) {
            const Layer& ly = net->layers[l];
            size_t elems = (size_t)B * g->rows[l] * g->cols[l] * ly.cout;
            g->act_off[l] = off;
            off = align_up(off + es * elems);
            if (ly.kind == MPCNN_MP) {
                g->code_off[l] = off;
                off = align_up(off + elems);
            }
        }
        g->delta_off[0] = off; off = align_up(off + max_act);
        g->delta_off[1] = off; off = align_up(off + max_act);
        for (size_t l = 0; l < L; ++l) {
            if (!g->partial_n[l]) continue;
            g->partial_off[l] = off;
            // A pass over bands sizes the buffers of the partial sums by bounds that do not depend
            // on the map's size: the number of slabs a plan ends up with is not monotonic in it (a
            // map with a few tiles more than workgroups gets half as many slabs of two tiles),
            // and the workspace is sized by the tallest band, the last one being shorter.  A
            // one-piece pass takes what its plan needs.  (The class layer's share count depends
            // on an occupancy query made when the net first touches the device, which may be
            // after the caller asked for the workspace size: always the bound.)
            const Layer& ly = net->layers[l];
            size_t alloc_f;
            if (ly.class_fused) alloc_f = (size_t)kLossBlocks * g->partial_len[l];
            else if (!fixed_partials) alloc_f = (size_t)g->partial_n[l] * g->partial_len[l];
            else {
                const size_t rows_w = (size_t)ly.k * ly.k2 * ly.cin, Nt = ceil_div(ly.cout, 32);
                const size_t tiled = std::max((size_t)ceil_div((int)rows_w, 32) * Nt * 1024 + Nt * 32,
                                              (size_t)ceil_div((int)rows_w + 1, 32) * Nt * 1024);
                alloc_f = std::max((size_t)kNumCU * tiled,
                                   (size_t)std::max(kDirectWgradChunks, 2 * kNumCU) * ly.p_len);
                alloc_f = std::max(alloc_f, (size_t)g->partial_n[l] * g->partial_len[l]);
            }
            off = align_up(off + sizeof(float) * alloc_f);
        }
    } else {
        // forward only: layers alternate between two buffers, nothing is kept
        size_t buf[2];
        buf[0] = off; off = align_up(off + max_act);
        buf[1] = off; off = align_up(off + max_act);
        for (size_t l = 0; l < L; ++l) g->act_off[l] = buf[l & 1];
    }
    g->loss_partial_off = off; off = align_up(off + sizeof(double) * kLossBlocks);
    g->total = off;
    g->label_h = H; g->probs_rows = r; g->accumulate = false;
    return true;
}


// Launch geometry of the max-filter kernels: 256 (column, channel quad) items of one map row
// per workgroup.  False if the map is too large for their 32-bit index arithmetic.
bool row_grid(int B, int h, int w, int C4, int d, mpcnn::RowGrid* g)
{
    const long per_row = (long)w * C4, gx = (per_row + 255) / 256, rows = (long)B * h;
    if (gx * rows >= (1l << 31) || gx * rows * gx >= (1l << 32) || (gx * 256) * C4 >= (1l << 32) ||
        rows * h >= (1l << 32))
        return false;
    g->gx = (int)gx; g->rows = (int)rows; g->h = h; g->C4 = C4;
    g->mg_gx = magic_of((unsigned)gx); g->mg_h = magic_of((unsigned)h); g->mg_c4 = magic_of((unsigned)C4);
    // row order: residue classes mod d (h rows: the first h mod d classes have one row more)
    g->d = d < h ? d : 1;
    g->rem = h % g->d; g->n1 = h / g->d + (g->rem ? 1 : 0);
    if (g->rem == 0) g->rem = g->d;          // all classes have n1 rows
    g->mg_n1 = magic_of((unsigned)g->n1); g->mg_n0 = magic_of((unsigned)(g->n1 - 1));
    return true;
}

// Launch geometry of maxfilter_fwd2x2_kernel: row pairs (y, y + d) of one residue class mod d, column
// pairs in blocks of 2 d columns.  False if the map is too large for 32-bit index arithmetic.
bool pair_grid(int B, int h, int w, int C4, int d, mpcnn::PairGrid* g)
{
    const int D2 = 2 * d, q = h / D2, rem = h % D2;
    const int nbig = std::min(rem, d);
    const long S = (long)nbig * (q + 1) + (long)(d - nbig) * q;
    const long Sx = (long)(w / D2) * d + std::min(w % D2, d);
    if (S < 1 || Sx < 1) return false;
    const long per_row = Sx * C4, gx = (per_row + 255) / 256, rows = (long)B * S;
    if (gx * rows >= (1l << 31) || gx * rows * gx >= (1l << 32) || (gx * 256) * C4 >= (1l << 32) ||
        rows * S >= (1l << 32) || (long)h * D2 >= (1l << 31))
        return false;
    g->gx = (int)gx; g->rows = (int)rows; g->S = (int)S; g->C4 = C4; g->Sx = (int)Sx; g->d = d;
    g->nbig = nbig; g->q1 = q + 1;
    g->mg_gx = magic_of((unsigned)gx); g->mg_S = magic_of((unsigned)S); g->mg_c4 = magic_of((unsigned)C4);
    g->mg_q1 = magic_of((unsigned)(q + 1)); g->mg_q0 = magic_of((unsigned)q); g->mg_d = magic_of((unsigned)d);
    return true;
}

inline int grid_for(long total, int block = 256, int cap = 1 << 20)
{
    long g = (total + block - 1) / block;
    return (int)std::min<long>(std::max<long>(g, 1), cap);
}

// ------------------------------------------------------------------ MFMA launches
// conv_tp_kernel: workgroups walk the tiles, two of them per compute unit; its divisors' magic numbers
void persistent_grid(mpcnn::ConvArgs* a, dim3* grid, int split)
{
    a->tiles_total = (int)grid->x;
    a->mg_cq = magic_of((unsigned)(a->CrPad / 8)); a->mg_hw = magic_of((unsigned)(a->Tx + a->k - 1));
    a->mg_tx = magic_of((unsigned)a->Tx); a->mg_ntx = magic_of((unsigned)a->ntx);
    a->mg_nty = magic_of((unsigned)a->nty); a->mg_d = magic_of((unsigned)a->d);
    grid->x = (unsigned)std::min<long>(grid->x, std::max(1, 2 * kNumCU / split));
}

// (the kernel instances live in launch_*.hip, one translation unit per family)
template <typename T>
bool launch_conv_mfma(const mpcnn::ConvArgs& a, const ChanTiling& ct, const TilePlan& tp, dim3 grid,
                      hipStream_t st, bool bm = false)
{
    if (bm) return ct.W == 32 && mpcnn::launch_conv_bm(a, ct.OT, tp.PT, tp.NW, tp.MP, grid, tp.lds, st);
    if constexpr (std::is_same<T, float>::value)
        return mpcnn::launch_conv_f32(a, ct.W, ct.OT, tp.PT, tp.NW, tp.MP, grid, tp.lds, st);
    else
        return mpcnn::launch_conv_b16(a, ct.W, ct.OT, tp.PT, tp.NW, tp.MP, grid, tp.lds, st);
}
template <typename T>
bool launch_wgrad_mfma(const mpcnn::WgradArgs& a, int hl, dim3 grid, size_t lds, hipStream_t st)
{
    if constexpr (std::is_same<T, float>::value) return mpcnn::launch_wgrad_f32(a, hl, grid, lds, st);
    else return mpcnn::launch_wgrad_b16(a, hl, grid, lds, st);
}
void launch_first_bm(const mpcnn::FirstBmArgs& a, unsigned wgs, hipStream_t st)
{
    const int nt = a.Co <= 32 ? 1 : 2;
#define CASE(n, kk) if (nt == n && a.k == kk) { mpcnn::first_layer_bm_kernel<n, kk><<<wgs, 256, 0, st>>>(a); return; }
    CASE(1, 3) CASE(1, 5) CASE(1, 7) CASE(2, 3) CASE(2, 5) CASE(2, 7)
#undef CASE
}
// fp32 storage, the image layer on the fp32 matrix instruction: instance by filter side, channels and rows per wave
bool launch_first_mfma(const mpcnn::FirstMfmaArgs& a0, int k, int ci, int B, hipStream_t st)
{
    mpcnn::FirstMfmaArgs a = a0;
    const int ct = ceil_div(a.Co, 32);
    int mp = 4;   // rows per wave: as many as still give every compute unit two workgroups
    while (mp > 1 && (long)B * ceil_div(a.Ho, 4 * mp) * ceil_div(a.Wo, 32) * ct < 2L * kNumCU) mp >>= 1;
    a.nty = ceil_div(a.Ho, 4 * mp); a.ntx = ceil_div(a.Wo, 32);
    const dim3 grid((unsigned)(B * a.nty * a.ntx), (unsigned)ct);
#define CASE(kk, cc, mm) if (k == kk && ci == cc && mp == mm) { mpcnn::first_layer_mfma_kernel<kk, cc, mm><<<grid, 256, 0, st>>>(a); return true; }
#define CASES(kk, cc) CASE(kk, cc, 1) CASE(kk, cc, 2) CASE(kk, cc, 4)
    CASES(3, 1) CASES(5, 1) CASES(7, 1) CASES(3, 3) CASES(5, 3) CASES(7, 3)
#undef CASES
#undef CASE
    return false;
}
template <typename T>
bool launch_l0_wgrad(const mpcnn::L0WgradArgs& a, int k, int ci, dim3 grid, hipStream_t st)
{
#define CASE(kk, cc) if (k == kk && ci == cc) { mpcnn::l0_wgrad_mfma_kernel<kk, cc, T><<<grid, 256, 0, st>>>(a); return true; }
    CASE(3, 1) CASE(5, 1) CASE(7, 1) CASE(3, 3) CASE(5, 3) CASE(7, 3)
#undef CASE
    return false;
}
// Kernels that may ask for more than 64 KiB of dynamic LDS must say so once.
mpcnn_status set_lds_attrs(bool bf16_storage)
{
    if (bf16_storage) { HIP_TRY(mpcnn::conv_attrs_b16()); HIP_TRY(mpcnn::wgrad_attrs_b16()); }
    else { HIP_TRY(mpcnn::conv_attrs_f32()); HIP_TRY(mpcnn::wgrad_attrs_f32()); }
    return MPCNN_OK;
}

// bf16 storage with a multiple of 8 channels: 8 channels per 128-bit access (Q = 2)
template <int NCLS, int KV, typename T>
void launch_class_inst(const mpcnn::ClassArgs& a, bool train, int blocks, hipStream_t st)
{
    constexpr bool kPairs = sizeof(T) == 2;
    if (kPairs && a.K % 8 == 0) {
        if (train) mpcnn::class_layer_kernel<NCLS, KV, true, T, kPairs ? 2 : 1><<<blocks, 256, 0, st>>>(a);
        else mpcnn::class_layer_kernel<NCLS, KV, false, T, kPairs ? 2 : 1><<<blocks, 256, 0, st>>>(a);
    } else {
        if (train) mpcnn::class_layer_kernel<NCLS, KV, true, T><<<blocks, 256, 0, st>>>(a);
        else mpcnn::class_layer_kernel<NCLS, KV, false, T><<<blocks, 256, 0, st>>>(a);
    }
}
template <int NCLS, int KV, typename T>
int class_occupancy_inst(int K)
{
    constexpr bool kPairs = sizeof(T) == 2;
    int n = 0;
    hipError_t e;
    if (kPairs && K % 8 == 0)
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, mpcnn::class_layer_kernel<NCLS, KV, true, T, kPairs ? 2 : 1>, 256, 0);
    else
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, mpcnn::class_layer_kernel<NCLS, KV, true, T>, 256, 0);
    return e == hipSuccess ? n : 0;
}
// workgroups of the training form that one CU holds at once (0 if unknown)
template <typename T>
int class_occupancy(int ncls, int KV, int K)
{
#define CASE(n, v) if (ncls == n && KV == v) return class_occupancy_inst<n, v, T>(K)
    CASE(2, 2); CASE(3, 2); CASE(4, 2); CASE(2, 4); CASE(3, 4); CASE(4, 4);
#undef CASE
    return 0;
}
template <typename T>
void launch_class(const mpcnn::ClassArgs& a, int ncls, int KV, bool train, int blocks, hipStream_t st)
{
#define CASE(n, v) if (ncls == n && KV == v) return launch_class_inst<n, v, T>(a, train, blocks, st)
    CASE(2, 2); CASE(3, 2); CASE(4, 2); CASE(2, 4); CASE(3, 4); CASE(4, 4);
#undef CASE
}

mpcnn_status refresh_packs(mpcnn_net* net, hipStream_t st)
{
    if (net->bf16 && net->wread_stale) {
        const long n = (long)net->n_params;
        LAUNCH("round_params", -1, 0, 0, 8.0 * n,
               mpcnn::round_params_kernel<<<grid_for(n), 256, 0, st>>>(net->d_params, net->d_wread, n));
    }
    net->wread_stale = false;
    if (!net->packs_stale || !net->d_packs) { net->packs_stale = false; return MPCNN_OK; }
    for (size_t l = 0; l < net->layers.size(); ++l) {
        const Layer& ly = net->layers[l];
        if (ly.kind == MPCNN_MP) continue;
        const float* Wc = net->d_wread + ly.p_off;
        if (ly.fwd_mfma && ly.fwd_bm)
            LAUNCH("pack_weights", l, 0, 0, 6.0 * ly.fwd_pack_len,
                   mpcnn::pack_weights_bf16_kernel<<<grid_for((long)ly.fwd_pack_len), 256, 0, st>>>(
                       Wc, (mpcnn::bf16*)(net->d_packs + ly.fwd_pack_off), ly.k * ly.k2, ly.cin, ly.cout,
                       ly.fwd_rpad, ly.fwd_ct.pad, 0));
        else if (ly.fwd_mfma)
            LAUNCH("pack_weights", l, 0, 0, 8.0 * ly.fwd_pack_len,
                   mpcnn::pack_weights_kernel<<<grid_for((long)ly.fwd_pack_len), 256, 0, st>>>(
                       Wc, net->d_packs + ly.fwd_pack_off, ly.k * ly.k2, ly.cin, ly.cout, ly.fwd_rpad,
                       ly.fwd_ct.pad, 64 / ly.fwd_ct.W, 0));
        if (ly.dgrad_mfma && l > 0 && ly.dgrad_bm)
            LAUNCH("pack_weights", l, 0, 0, 6.0 * ly.dgrad_pack_len,
                   mpcnn::pack_weights_bf16_kernel<<<grid_for((long)ly.dgrad_pack_len), 256, 0, st>>>(
                       Wc, (mpcnn::bf16*)(net->d_packs + ly.dgrad_pack_off), ly.k * ly.k2, ly.cin, ly.cout,
                       ly.dgrad_rpad, ly.dgrad_ct.pad, 1));
        else if (ly.dgrad_mfma && l > 0)
            LAUNCH("pack_weights", l, 0, 0, 8.0 * ly.dgrad_pack_len,
                   mpcnn::pack_weights_kernel<<<grid_for((long)ly.dgrad_pack_len), 256, 0, st>>>(
                       Wc, net->d_packs + ly.dgrad_pack_off, ly.k * ly.k2, ly.cin, ly.cout,
                       ly.dgrad_rpad, ly.dgrad_ct.pad, 64 / ly.dgrad_ct.W, 1));
    }
    HIP_TRY(hipGetLastError());
    net->packs_stale = false;
    return MPCNN_OK;
}

// Forward through every layer; in training mode everything is kept for the backward.
// T = storage type of activations and deltas (float, or bf16 with fp32 arithmetic).
template <typename T>
mpcnn_status run_forward(mpcnn_net* net, const Geom& g, const float* image, char* ws,
                         const int32_t* labels, const float* pixw, float* probs, void* dZ_,
                         double* loss_dev, hipStream_t st)
{
    using namespace mpcnn;
    constexpr bool kF32 = std::is_same<T, float>::value;
    constexpr double es = sizeof(T);
    mpcnn_status rc = refresh_packs(net, st);
    if (rc != MPCNN_OK) return rc;
    const int B = g.B;
    T* dZ = static_cast<T*>(dZ_);
    const T* in = nullptr;
    int Hi = g.H, Wi = g.W, Ci = net->in_ch;
    if (g.staged) {
        T* staged = (T*)(ws + g.staged_off);
        long total = (long)B * Ci * Hi * Wi;
        LAUNCH("stage_input", -1, 0, 0, (4.0 + es) * total,
               stage_input_kernel<T><<<grid_for(total), 256, 0, st>>>(image, staged, B, Ci, Hi, Wi, g.src_h,
                                                                       g.src_w, g.pad_top, g.pad_left));
        in = staged;
    } else if constexpr (kF32) {
        in = image;
    }
    const size_t L = net->layers.size();
    double* lp = (double*)(ws + g.loss_partial_off);
    const bool want_loss = labels && loss_dev;
    net->loss_shares = 0; net->loss_out = loss_dev;
    for (size_t l = 0; l < L; ++l) {
        const Layer& ly = net->layers[l];
        T* out = (T*)(ws + g.act_off[l]);
        const int Ho = g.rows[l], Wo = g.cols[l];
        const double n_in = (double)B * Hi * Wi * Ci, n_out = (double)B * Ho * Wo * ly.cout;
        if (ly.kind == MPCNN_MP) {
            uint8_t* code = g.training ? (uint8_t*)(ws + g.code_off[l]) : nullptr;
            long total = (long)B * Ho * Wo * ly.cout;
            mpcnn::RowGrid rg;
            mpcnn::PairGrid pg;
            constexpr int kQ = kF32 ? 1 : 2;   // channels per thread / 4 (bf16: 8 channels = one 128-bit access)
            if (!ly.rect && ly.k == 2 && ly.cout % (4 * kQ) == 0 && pair_grid(B, Ho, Wo, ly.cout / (4 * kQ), ly.dil, &pg))
                LAUNCH("maxfilter_fwd", l, 2, 0, n_out * (2.0 * es + (code ? 1.0 : 0.0)),
                       (maxfilter_fwd2x2_kernel<T, kQ><<<(unsigned)(pg.gx * pg.rows), 256, 0, st>>>(
                           in, out, code, pg, Hi, Wi, ly.cout, Ho, Wo)));
            else if (!kF32 && ly.cout % 8 == 0 && row_grid(B, Ho, Wo, ly.cout / 8, ly.dil, &rg))   // bf16: 8 channels per thread (fp32: measured slower)
                LAUNCH("maxfilter_fwd", l, 2, 0, n_out * (2.0 * es + (code ? 1.0 : 0.0)),
                       (maxfilter_fwd4_kernel<T, kF32 ? 1 : 2><<<(unsigned)(rg.gx * rg.rows), 256, 0, st>>>(
                           in, out, code, rg, Hi, Wi, ly.cout, Ho, Wo, ly.k, ly.k2, ly.dil, ly.dil2)));
            else if (ly.cout % 4 == 0 && row_grid(B, Ho, Wo, ly.cout / 4, ly.dil, &rg))
                LAUNCH("maxfilter_fwd", l, 2, 0, n_out * (2.0 * es + (code ? 1.0 : 0.0)),
                       (maxfilter_fwd4_kernel<T, 1><<<(unsigned)(rg.gx * rg.rows), 256, 0, st>>>(
                           in, out, code, rg, Hi, Wi, ly.cout, Ho, Wo, ly.k, ly.k2, ly.dil, ly.dil2)));
            else
                LAUNCH("maxfilter_fwd", l, 2, 0, n_out * (2.0 * es + (code ? 1.0 : 0.0)),
                       maxfilter_fwd_direct_kernel<T><<<grid_for(total), 256, 0, st>>>(
                           in, out, code, B, Hi, Wi, ly.cout, Ho, Wo, ly.k, ly.k2, ly.dil, ly.dil2));
        } else if (ly.class_fused) {
            // last FC + softmax + cross-entropy (+ its own backward when labels are given)
            const long M = (long)B * Ho * Wo;
            ClassArgs a{};
            a.h = in; a.Wk = net->d_wread + ly.p_off; a.probs = probs;
            a.labels = labels; a.pixw = pixw; a.pixw_any = pixw ? pixw : reinterpret_cast<const float*>(labels); a.dH = dZ;
            a.partial = g.training ? (float*)(ws + g.partial_off[l]) : nullptr;   // loss only: no gradient shares
            a.loss_partial = want_loss ? lp : nullptr;
            a.B = B; a.Ho = Ho; a.Wo = Wo; a.H = g.label_h; a.W = g.W; a.ctr = (net->patch - 1) / 2;
            a.probs_rows = g.probs_rows;
            a.K = Ci; a.tanh_below = (l > 0 && net->layers[l - 1].tanh_out) ? 1 + net->logistic : 0;
            a.mse = net->loss_kind == MPCNN_LOSS_MSE;
            const int blocks = class_blocks(net, M);
            const bool train = labels != nullptr;
            const double flops = 2.0 * M * Ci * ly.cout * (train ? 3.0 : 1.0);
            const double bytes = es * n_in * (train ? 2.0 : 1.0) + 4.0 * n_out;
            LAUNCH("class_layer", l, train ? 4 : 3, flops, bytes,
                   launch_class<T>(a, ly.cout, Ci <= 128 ? 2 : 4, train, blocks, st));
            // (in training the shares are added by the reduce launch that ends the backward)
            if (train && want_loss) net->loss_shares = blocks;
        } else {
            const float* Wk = net->d_wread + ly.p_off;
            const double flops = 2.0 * B * Ho * Wo * ly.cout * ly.k * ly.k2 * Ci;
            const double bytes = es * (n_in + n_out) + 4.0 * ly.p_len;
            const int step = (l == L - 1) ? 3 : 1;
            if (ly.fwd_mfma && g.fwd[l].ok) {
                const TilePlan& tp = g.fwd[l];
                ConvArgs a{};
                a.in = in; a.wpack = (const v4f*)(net->d_packs + ly.fwd_pack_off);
                a.bias = Wk + (size_t)ly.k * ly.k2 * Ci * ly.cout; a.act = nullptr; a.out = out;
                a.B = B; a.Hi = Hi; a.Wi = Wi; a.Cr = Ci; a.CrPad = ly.fwd_rpad;
                a.Ho = Ho; a.Wo = Wo; a.Co = ly.cout; a.CoPad = ly.fwd_ct.pad;
                a.k = ly.k; a.d = ly.dil; a.origin = 0; a.k2 = ly.k2; a.d2 = ly.dil2; a.origin2 = 0;
                a.Ty = tp.Ty; a.Tx = tp.Tx; a.nty = tp.nty; a.ntx = tp.ntx;
                a.mode = ly.tanh_out ? kFwdTanh : kFwdLinear; a.logistic = net->logistic;
                dim3 grid((unsigned)(B * ly.dil * ly.dil2 * tp.nty * tp.ntx), (unsigned)ly.fwd_ct.split);
                if (ly.fwd_bm) persistent_grid(&a, &grid, ly.fwd_ct.split);
                bool launched = false;
                LAUNCH(ly.fwd_bm ? "conv_fwd_bm" : "conv_fwd_mfma", l, step, flops, bytes,
                       launched = launch_conv_mfma<T>(a, ly.fwd_ct, tp, grid, st, ly.fwd_bm));
                if (!launched)   // a plan without a kernel instance: a planner bug, never a silent skip
                    return fail(MPCNN_EUNSUPPORTED, "layer %zu: no convolution kernel instance for its forward plan", l);
            } else if (!kF32 && l == 0 && ly.dil == 1 && Ci <= 4 && ly.cout <= 64 && (ly.k == 3 || ly.k == 5 || ly.k == 7)) {
                // bf16 storage, the image layer: short reduction on the bf16 matrix instruction
                FirstBmArgs a{};
                a.in = (const mpcnn::bf16*)in; a.Wk = Wk; a.out = (mpcnn::bf16*)out;
                a.B = B; a.Hi = Hi; a.Wi = Wi; a.Ci = Ci; a.Ho = Ho; a.Wo = Wo; a.Co = ly.cout; a.k = ly.k;
                a.squash = ly.tanh_out ? 1 + net->logistic : 0;
                a.nty = ceil_div(Ho, kFirstBmTy); a.ntx = ceil_div(Wo, kFirstBmTx);
                const unsigned wgs = (unsigned)std::min<long>((long)B * a.nty * a.ntx, 4L * kNumCU);
                LAUNCH("first_layer_bm", l, step, flops, bytes, launch_first_bm(a, wgs, st));
            } else if (kF32 && !ly.rect && ly.dil == 1 && (Ci == 1 || Ci == 3) && (ly.k == 3 || ly.k == 5 || ly.k == 7) &&
                       (long)B * Ho * Wo < (1l << 31) / 32) {
                // fp32 storage, the image layer: short reduction on the fp32 matrix instruction
                FirstMfmaArgs a{};
                a.in = (const float*)in; a.Wk = Wk; a.out = (float*)out;
                a.B = B; a.Hi = Hi; a.Wi = Wi; a.Ho = Ho; a.Wo = Wo; a.Co = ly.cout;
                a.squash = ly.tanh_out ? 1 + net->logistic : 0;
                bool launched = false;
                LAUNCH("first_layer_mfma", l, step, flops, bytes, launched = launch_first_mfma(a, ly.k, Ci, B, st));
                if (!launched) return fail(MPCNN_EUNSUPPORTED, "layer %zu: no image-layer kernel instance", l);
            } else {
                const int og = ceil_div(ly.cout, 4);
                const long total = (long)B * Ho * Wo * og;
                const size_t wbytes = sizeof(float) * ((size_t)ly.k * ly.k2 * Ci + 1) * 4 * og;
                const int w_in_lds = wbytes <= 48 * 1024;
                LAUNCH("first_layer", l, step, flops, bytes,
                       first_layer_kernel<T><<<(unsigned)((total + 255) / 256), 256, w_in_lds ? wbytes : 0, st>>>(
                           in, Wk, out, B, Hi, Wi, Ci, Ho, Wo, ly.cout, ly.k, ly.k2, ly.dil, ly.dil2,
                           ly.tanh_out ? 1 + net->logistic : 0,
                           w_in_lds));
            }
        }
        in = out; Hi = Ho; Wi = Wo; Ci = ly.cout;
    }
    if (!net->layers[L - 1].class_fused) {
        // class logits -> probabilities, deltas, loss
        long total = (long)B * Hi * Wi;
        int blocks = (int)std::min<long>(kSoftmaxBlocks, (total + 255) / 256);
        LAUNCH("softmax_ce", L - 1, 3, 0, total * ((4.0 + 2.0 * es) * net->n_cls + 8.0),
               softmax_ce_kernel<T><<<blocks, 256, 0, st>>>(in, probs, labels, pixw, dZ,
                                                         want_loss ? lp : nullptr, B, Hi, Wi, g.label_h, g.W,
                                                         (net->patch - 1) / 2, net->n_cls,
                                                         net->loss_kind == MPCNN_LOSS_MSE, g.probs_rows));
        if (want_loss) net->loss_shares = blocks;
    }
    HIP_TRY(hipGetLastError());
    return MPCNN_OK;
}

template <typename T>
mpcnn_status run_backward(mpcnn_net* net, const Geom& g, const float* image, char* ws,
                          hipStream_t st)
{
    using namespace mpcnn;
    constexpr bool kF32 = std::is_same<T, float>::value;
    constexpr double es = sizeof(T);
    const int B = g.B;
    const size_t L = net->layers.size();
    const T* in0 = nullptr;
    if (g.staged) in0 = (const T*)(ws + g.staged_off);
    else if constexpr (kF32) in0 = image;
    T* dbuf[2] = {(T*)(ws + g.delta_off[0]), (T*)(ws + g.delta_off[1])};
    int cur = 0;  // dbuf[cur] holds dL/d(pre-activation) of layer l's output (dL/d(output) for MP)
    // a fused class layer has already done its own backward and left the delta below it
    for (size_t li = net->layers[L - 1].class_fused ? L - 1 : L; li-- > 0;) {
        const Layer& ly = net->layers[li];
        const int Ho = g.rows[li], Wo = g.cols[li];
        const T* A = li == 0 ? in0 : (const T*)(ws + g.act_off[li - 1]);
        const int Hi = li == 0 ? g.H : g.rows[li - 1], Wi = li == 0 ? g.W : g.cols[li - 1];
        const int Ci = ly.cin;
        const bool below_tanh = li > 0 && net->layers[li - 1].tanh_out;
        const T* dY = dbuf[cur];
        T* dA = dbuf[cur ^ 1];
        const double n_in = (double)B * Hi * Wi * Ci, n_out = (double)B * Ho * Wo * ly.cout;
        if (ly.kind == MPCNN_MP) {
            if (li == 0) break;  // nothing below has parameters
            const uint8_t* code = (const uint8_t*)(ws + g.code_off[li]);
            if (li == 1 && g.l0_fused) {
                const Layer& l0 = net->layers[0];
                L0Args a{};
                a.in = in0; a.act1 = A; a.dP = dY; a.code = code;
                a.partial = (float*)(ws + g.partial_off[0]);
                a.B = B; a.Hi = g.H; a.Wi = g.W; a.Ci = l0.cin; a.H1 = Hi; a.W1 = Wi; a.C1 = Ci;
                a.k = l0.k; a.Hp = Ho; a.Wp = Wo;
                a.nty = g.l0_nty; a.ntx = g.l0_ntx;
                a.slope = below_tanh ? (net->logistic ? 2 : 1) : 0;
                const double wflops = 2.0 * B * Hi * Wi * Ci * l0.k * l0.k * l0.cin;
                const double wbytes = n_out * (es + 1.0) + n_in * (below_tanh ? es : 0.0) + es * B * g.H * g.W * l0.cin + 4.0 * l0.p_len;
                if (ly.k == 2)
                    LAUNCH("l0_wgrad_fused", 0, 5, wflops, wbytes,
                           (l0_wgrad_fused_kernel<T, 2><<<(unsigned)g.l0_blocks, 256, g.l0_lds, st>>>(a)));
                else if (ly.k == 3)
                    LAUNCH("l0_wgrad_fused", 0, 5, wflops, wbytes,
                           (l0_wgrad_fused_kernel<T, 3><<<(unsigned)g.l0_blocks, 256, g.l0_lds, st>>>(a)));
                else
                    LAUNCH("l0_wgrad_fused", 0, 5, wflops, wbytes,
                           (l0_wgrad_fused_kernel<T, 4><<<(unsigned)g.l0_blocks, 256, g.l0_lds, st>>>(a)));
                break;  // the image needs no gradient
            }
            long total = (long)B * Hi * Wi * Ci;
            const double bytes = n_out * (es + 1.0) + n_in * es * (below_tanh ? 2.0 : 1.0);
            mpcnn::RowGrid rg;
            mpcnn::PairGrid pg;
            // 2 x 2 windows: 2 x 2 elements per thread, 8 channels each (4 where the count is no multiple of 8);
            // not where a position is under one 128-byte line and neighbours are adjacent (measured slower)
            const int pq = Ci % 8 == 0 ? 2 : 1;
            if (!ly.rect && ly.k == 2 && Ci % 4 == 0 && (ly.dil > 1 || Ci * es >= 128) && pair_grid(B, Hi, Wi, Ci / (4 * pq), ly.dil, &pg)) {
                const unsigned wgs = (unsigned)(pg.gx * pg.rows);
#define PAIR_BWD(TP, QQ) LAUNCH("maxfilter_bwd", li, 7, 0, bytes, (maxfilter_bwd2x2_kernel<TP, T, QQ><<<wgs, 256, 0, st>>>( \
                             dY, code, A, dA, pg, Hi, Wi, Ci, Ho, Wo, net->logistic)))
                if (below_tanh && pq == 2) PAIR_BWD(true, 2);
                else if (below_tanh) PAIR_BWD(true, 1);
                else if (pq == 2) PAIR_BWD(false, 2);
                else PAIR_BWD(false, 1);
#undef PAIR_BWD
                cur ^= 1;
                continue;
            }
            const bool octs = Ci % 8 == 0 && row_grid(B, Hi, Wi, Ci / 8, ly.dil, &rg);   // 8 channels per thread (measured faster in both storage types)
            const bool quads = !octs && Ci % 4 == 0 && row_grid(B, Hi, Wi, Ci / 4, ly.dil, &rg);
            if (octs && below_tanh)
                LAUNCH("maxfilter_bwd", li, 7, 0, bytes,
                       (maxfilter_bwd4_kernel<true, T, 2><<<(unsigned)(rg.gx * rg.rows), 256, 0, st>>>(
                           dY, code, A, dA, rg, Hi, Wi, Ci, Ho, Wo, ly.k, ly.k2, ly.dil, ly.dil2, net->logistic)));
            else if (octs)
                LAUNCH("maxfilter_bwd", li, 7, 0, bytes,
                       (maxfilter_bwd4_kernel<false, T, 2><<<(unsigned)(rg.gx * rg.rows), 256, 0, st>>>(
                           dY, code, A, dA, rg, Hi, Wi, Ci, Ho, Wo, ly.k, ly.k2, ly.dil, ly.dil2, net->logistic)));
            else if (quads && below_tanh)
                LAUNCH("maxfilter_bwd", li, 7, 0, bytes,
                       (maxfilter_bwd4_kernel<true, T, 1><<<(unsigned)(rg.gx * rg.rows), 256, 0, st>>>(
                           dY, code, A, dA, rg, Hi, Wi, Ci, Ho, Wo, ly.k, ly.k2, ly.dil, ly.dil2, net->logistic)));
            else if (quads)
                LAUNCH("maxfilter_bwd", li, 7, 0, bytes,
                       (maxfilter_bwd4_kernel<false, T, 1><<<(unsigned)(rg.gx * rg.rows), 256, 0, st>>>(
                           dY, code, A, dA, rg, Hi, Wi, Ci, Ho, Wo, ly.k, ly.k2, ly.dil, ly.dil2, net->logistic)));
            else if (below_tanh)
                LAUNCH("maxfilter_bwd", li, 7, 0, bytes,
                       (maxfilter_bwd_direct_kernel<true, T><<<grid_for(total), 256, 0, st>>>(
                           dY, code, A, dA, B, Hi, Wi, Ci, Ho, Wo, ly.k, ly.k2, ly.dil, ly.dil2, net->logistic)));
            else
                LAUNCH("maxfilter_bwd", li, 7, 0, bytes,
                       (maxfilter_bwd_direct_kernel<false, T><<<grid_for(total), 256, 0, st>>>(
                           dY, code, A, dA, B, Hi, Wi, Ci, Ho, Wo, ly.k, ly.k2, ly.dil, ly.dil2, net->logistic)));
        } else {
            const double flops = 2.0 * B * Ho * Wo * ly.cout * ly.k * ly.k2 * Ci;
            const int wstep = (li == L - 1) ? 4 : 5, dstep = (li == L - 1) ? 4 : 6;
            // parameter gradient: partial sums over slabs of positions, then a fixed-order sum
            const WgradPlan& wp = g.wgrad[li];
            float* partial = (float*)(ws + g.partial_off[li]);
            if (wp.ok) {
                WgradArgs a{};
                a.in = A; a.dY = dY; a.partial = partial;
                a.B = B; a.Hi = Hi; a.Wi = Wi; a.Ci = Ci;
                a.Ho = Ho; a.Wo = Wo; a.Co = ly.cout; a.k = ly.k; a.d = ly.dil; a.k2 = ly.k2; a.d2 = ly.dil2;
                a.Tx = wp.Tx; a.TxP = wp.TxP; a.nty = wp.nty; a.ntx = wp.ntx;
                a.tiles_total = wp.tiles_total; a.tiles_per_slab = wp.tiles_per_slab;
                a.Mt = wp.Mt; a.Nt = wp.Nt; a.wm = wp.wm; a.wn = wp.wn; a.wk = wp.wk; a.mw = wp.mw;
                a.mg_cq = magic_of(ceil_div(Ci, 4)); a.mg_hwp = magic_of(wp.TxP + ly.k2 - 1);
                if (wp.tr) {   // items of one position x 8 channels
                    a.mg_cq = magic_of(Ci / 8);
                    a.mg_hwp = magic_of(mpcnn::tr_geom(wp.TxP / 16, ly.k, Ci, wp.wn).hwp);
                } else if (wp.bm) {   // items of two positions x 8 channels
                    a.mg_cq = magic_of(ceil_div(Ci, 8));
                    a.mg_hwp = magic_of(mpcnn::bm_geom(wp.TxP / 16, ly.k, Ci, wp.wn).hwp / 2);
                }
                a.mg_txp = magic_of(wp.TxP); a.mg_ci = magic_of(Ci); a.mg_k2 = magic_of(ly.k2);
                a.mg_ntx = magic_of(wp.ntx); a.mg_nty = magic_of(wp.nty); a.mg_d = magic_of(ly.dil); a.mg_d2 = magic_of(ly.dil2);
                dim3 grid((unsigned)wp.slabs, (unsigned)wp.gm, (unsigned)wp.gn);
                bool launched = false;
                if (wp.tr)
                    LAUNCH("wgrad_bm", li, wstep, flops, es * (n_in + n_out) + 4.0 * ly.p_len,
                           launched = mpcnn::launch_wgrad_tr(a, wp.TxP / 16, grid, wp.lds, st));
                else if (wp.bm)
                    LAUNCH("wgrad_bm", li, wstep, flops, es * (n_in + n_out) + 4.0 * ly.p_len,
                           launched = mpcnn::launch_wgrad_bm(a, wp.TxP / 16, grid, wp.lds, st));
                else
                    LAUNCH("wgrad_mfma", li, wstep, flops, es * (n_in + n_out) + 4.0 * ly.p_len,
                           launched = launch_wgrad_mfma<T>(a, wp.hl, grid, wp.lds, st));
                if (!launched)
                    return fail(MPCNN_EUNSUPPORTED, "layer %zu: no weight-gradient kernel instance for its plan", li);
            } else if (wp.l0m) {
                L0WgradArgs a{};
                a.in = A; a.dY = dY; a.partial = partial;
                a.B = B; a.Hi = Hi; a.Wi = Wi; a.Ho = Ho; a.Wo = Wo; a.Co = ly.cout;
                a.nty = ceil_div(Ho, mpcnn::kL0wTy); a.ntx = ceil_div(Wo, mpcnn::kL0wTx); a.tiles_total = wp.tiles_total;
                bool launched = false;
                LAUNCH("wgrad_image_mfma", li, wstep, flops, es * (n_in + n_out) + 4.0 * ly.p_len,
                       launched = launch_l0_wgrad<T>(a, ly.k, Ci, dim3((unsigned)wp.chunks, (unsigned)ceil_div(ly.cout, 32)), st));
                if (!launched) return fail(MPCNN_EUNSUPPORTED, "layer 0: no image-layer weight-gradient kernel instance");
            } else {
                dim3 grid((unsigned)((ly.p_len + 255) / 256), (unsigned)wp.chunks);
                LAUNCH("wgrad_direct", li, wstep, flops, es * (n_in + n_out) + 4.0 * ly.p_len,
                       conv_wgrad_direct_kernel<T><<<grid, 256, 0, st>>>(A, dY, partial, B, Hi, Wi, Ci, Ho,
                                                                      Wo, ly.cout, ly.k, ly.k2, ly.dil, ly.dil2,
                                                                      wp.rows_per_chunk));
            }
            if (li == 0) break;  // the image needs no gradient
            const float* Wk = net->d_wread + ly.p_off;
            const double dbytes = es * (n_in * (below_tanh ? 2.0 : 1.0) + n_out) + 4.0 * ly.p_len;
            if (ly.dgrad_mfma && g.dgrad[li].ok) {
                const TilePlan& tp = g.dgrad[li];
                ConvArgs a{};
                a.in = dY; a.wpack = (const v4f*)(net->d_packs + ly.dgrad_pack_off);
                a.bias = nullptr; a.act = A; a.out = dA;
                a.B = B; a.Hi = Ho; a.Wi = Wo; a.Cr = ly.cout; a.CrPad = ly.dgrad_rpad;
                a.Ho = Hi; a.Wo = Wi; a.Co = Ci; a.CoPad = ly.dgrad_ct.pad;
                a.k = ly.k; a.d = ly.dil; a.origin = -(ly.k - 1); a.k2 = ly.k2; a.d2 = ly.dil2; a.origin2 = -(ly.k2 - 1);
                a.Ty = tp.Ty; a.Tx = tp.Tx; a.nty = tp.nty; a.ntx = tp.ntx;
                a.mode = below_tanh ? kDgradTanh : kDgradPlain; a.logistic = net->logistic;
                dim3 grid((unsigned)(B * ly.dil * ly.dil2 * tp.nty * tp.ntx), (unsigned)ly.dgrad_ct.split);
                if (ly.dgrad_bm) persistent_grid(&a, &grid, ly.dgrad_ct.split);
                bool launched = false;
                LAUNCH(ly.dgrad_bm ? "conv_dgrad_bm" : "conv_dgrad_mfma", li, dstep, flops, dbytes,
                       launched = launch_conv_mfma<T>(a, ly.dgrad_ct, tp, grid, st, ly.dgrad_bm));
                if (!launched)
                    return fail(MPCNN_EUNSUPPORTED, "layer %zu: no convolution kernel instance for its data-gradient plan", li);
            } else {
                long total = (long)B * Hi * Wi * Ci;
                if (below_tanh)
                    LAUNCH("conv_dgrad_direct", li, dstep, flops, dbytes,
                           (conv_dgrad_direct_kernel<true, T><<<grid_for(total), 256, 0, st>>>(
                               dY, Wk, A, dA, B, Hi, Wi, Ci, Ho, Wo, ly.cout, ly.k, ly.k2, ly.dil, ly.dil2, net->logistic)));
                else
                    LAUNCH("conv_dgrad_direct", li, dstep, flops, dbytes,
                           (conv_dgrad_direct_kernel<false, T><<<grid_for(total), 256, 0, st>>>(
                               dY, Wk, A, dA, B, Hi, Wi, Ci, Ho, Wo, ly.cout, ly.k, ly.k2, ly.dil, ly.dil2, net->logistic)));
            }
        }
        cur ^= 1;
    }
    // one launch adds the partial sums of every layer in a fixed order (Alg. 2)
    ReduceArgs ra{};
    ra.accumulate = g.accumulate ? 1 : 0;
    double rbytes = 0;
    for (size_t l = 0; l < L; ++l) {
        if (!g.partial_n[l] || ra.n_seg >= kMaxReduceSegs) continue;
        const Layer& ly = net->layers[l];
        ReduceSeg& sg = ra.seg[ra.n_seg++];
        sg.partial = (const float*)(ws + g.partial_off[l]);
        sg.out = net->d_grads + ly.p_off;
        sg.plen = (long)g.partial_len[l]; sg.n = g.partial_n[l];
        const WgradPlan& wp = g.wgrad[l];
        sg.tiled = wp.ok ? (wp.bm ? 3 : 1) : 0;
        sg.items = wp.ok ? wp.Mt * wp.Nt * 256 + (wp.bm ? 0 : wp.Nt * 8) : (int)ly.p_len;
        sg.Nt = wp.Nt; sg.rows_total = ly.k * ly.k2 * ly.cin; sg.Co = ly.cout;
        sg.block0 = ra.total_blocks;
        ra.total_blocks += (sg.items + 63) / 64;
        rbytes += 4.0 * ((double)sg.plen * sg.n + ly.p_len);
    }
    if (net->loss_shares > 0 && net->loss_out && ra.n_seg < kMaxReduceSegs) {
        ReduceSeg& sg = ra.seg[ra.n_seg++];
        sg.partial = (const float*)(ws + g.loss_partial_off);
        sg.out = (float*)net->loss_out;
        sg.plen = 0; sg.n = net->loss_shares; sg.tiled = 2; sg.items = 1;
        sg.block0 = ra.total_blocks;
        ra.total_blocks += 1;
    }
    LAUNCH("reduce_all", -1, 0, 0, rbytes, reduce_all_kernel<<<(unsigned)ra.total_blocks, 256, 0, st>>>(ra));
    HIP_TRY(hipGetLastError());
    return MPCNN_OK;
}

// host parameter order W[o][c][u][v], b[o]  <->  device order W[u][v][c][o], b[o]
void to_device_order(const mpcnn_net* net, const float* host, float* dev_order)
{
    for (const Layer& ly : net->layers) {
        if (ly.kind == MPCNN_MP) continue;
        const int kk = ly.k * ly.k2, ci = ly.cin, co = ly.cout;
        const float* src = host + ly.p_off;
        float* dst = dev_order + ly.p_off;
        for (int o = 0; o < co; ++o)
            for (int c = 0; c < ci; ++c)
                for (int t = 0; t < kk; ++t)
                    dst[((size_t)t * ci + c) * co + o] = src[((size_t)o * ci + c) * kk + t];
        memcpy(dst + (size_t)kk * ci * co, src + (size_t)kk * ci * co, sizeof(float) * co);
    }
}

void to_host_order(const mpcnn_net* net, const float* dev_order, float* host)
{
    for (const Layer& ly : net->layers) {
        if (ly.kind == MPCNN_MP) continue;
        const int kk = ly.k * ly.k2, ci = ly.cin, co = ly.cout;
        const float* src = dev_order + ly.p_off;
        float* dst = host + ly.p_off;
        for (int o = 0; o < co; ++o)
            for (int c = 0; c < ci; ++c)
                for (int t = 0; t < kk; ++t)
                    dst[((size_t)o * ci + c) * kk + t] = src[((size_t)t * ci + c) * co + o];
        memcpy(dst + (size_t)kk * ci * co, src + (size_t)kk * ci * co, sizeof(float) * co);
    }
}

void lbfgs_free(mpcnn_net* net)
{
    (void)hipFree(net->d_lb_S); (void)hipFree(net->d_lb_Y);
    (void)hipFree(net->d_lb_theta_prev); (void)hipFree(net->d_lb_g_prev); (void)hipFree(net->d_lb_p);
    (void)hipFree(net->d_lb_part); (void)hipFree(net->d_lb_alpha);
    net->d_lb_S = net->d_lb_Y = net->d_lb_theta_prev = net->d_lb_g_prev = net->d_lb_p = nullptr;
    net->d_lb_part = net->d_lb_alpha = nullptr;
    net->lb_m = net->lb_head = net->lb_count = 0;
    net->lb_have_prev = false;
}

mpcnn_status read_back(const mpcnn_net* net, const float* dev, float* host, size_t n)
{
    if (!net || !host) return fail(MPCNN_EINVAL, "null argument");
    if (n != net->n_params) return fail(MPCNN_EINVAL, "n = %zu, net has %zu parameters", n, net->n_params);
    if (!dev) return fail(MPCNN_EINVAL, "parameters were never set");
    std::vector<float> tmp(n);
    HIP_TRY(hipSetDevice(net->device));
    HIP_TRY(hipDeviceSynchronize());
    HIP_TRY(hipMemcpy(tmp.data(), dev, sizeof(float) * n, hipMemcpyDeviceToHost));
    to_host_order(net, tmp.data(), host);
    return MPCNN_OK;
}

// The plan for these sizes: from the net's cache, or made now and kept (same != 0: the
// same-size forward, H x W being the caller's image).  Null if the sizes do not fit the net.
std::shared_ptr<const Geom> geom_for(const mpcnn_net* net, int B, int H, int W, bool training, bool same)
{
    const GeomKey key{B, H, W, training ? 1 : 0, same ? 1 : 0, net->hint_pt, net->hint_mp};
    for (auto& kv : net->geoms)
        if (kv.first == key) return kv.second;
    auto g = std::make_shared<Geom>();
    if (same) {
        // the net runs on the image extended by P-1 mirrored rows / columns
        const int c = (net->patch - 1) / 2;
        if (!make_geom(net, B, H + net->patch - 1, W + net->patch - 1, false, g.get(), true)) return nullptr;
        g->pad_top = c; g->pad_left = c; g->src_h = H; g->src_w = W;
    } else if (!make_geom(net, B, H, W, training, g.get())) {
        return nullptr;
    }
    if (net->geoms.size() >= kGeomCacheSize) net->geoms.erase(net->geoms.begin());
    net->geoms.emplace_back(key, g);
    return g;
}

// Address of `scratch` on device `dev`, which must be the current device; looked up once per
// device and kept.
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mu;
mpcnn_status scratch_address(int dev, void** out)
{
    if (dev < 0 || dev >= kMaxDevices) return fail(MPCNN_EINVAL, "device %d: at most %d devices", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(MPCNN_EHIP, "hipGetSymbolAddress returned a null address");
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return MPCNN_OK;
}

}  // namespace

extern "C" {

const char* mpcnn_last_error(void) { return g_err; }

mpcnn_status mpcnn_net_create(const mpcnn_layer_desc* layers, int n_layers, int in_channels,
                              int patch, mpcnn_dtype dtype, mpcnn_net** out)
{
    if (!layers || !out) return fail(MPCNN_EINVAL, "null argument");
    *out = nullptr;
    if (n_layers < 1 || n_layers > 48 || in_channels < 1 || patch < 1)
        return fail(MPCNN_EINVAL, "n_layers=%d in_channels=%d patch=%d", n_layers, in_channels, patch);
    if (dtype != MPCNN_F32 && dtype != MPCNN_BF16) return fail(MPCNN_EINVAL, "unknown dtype %d", (int)dtype);
    mpcnn_net* net = new (std::nothrow) mpcnn_net;
    if (!net) return fail(MPCNN_ENOMEM, "out of host memory");
    net->in_ch = in_channels; net->patch = patch; net->bf16 = dtype == MPCNN_BF16;
    int side = patch, side2 = patch, ch = in_channels, dil = 1, dil2 = 1;   // rows; columns
    bool seen_fc = false;
    size_t off = 0, pack = 0;
    mpcnn_status st = MPCNN_OK;
    for (int l = 0; l < n_layers && st == MPCNN_OK; ++l) {
        const mpcnn_layer_desc& d = layers[l];
        Layer ly{};
        ly.kind = d.kind; ly.cin = ch; ly.dil = dil; ly.dil2 = dil2;
        if (d.kind == MPCNN_C) {
            if (d.maps < 1 || d.k < 1) st = fail(MPCNN_EINVAL, "layer %d: C needs maps >= 1, k >= 1", l);
            else if (seen_fc) st = fail(MPCNN_ESHAPE, "layer %d: C after FC", l);
            else if (side - d.k + 1 < 1 || side2 - d.k + 1 < 1) st = fail(MPCNN_ESHAPE, "layer %d: %dx%d filter on a %dx%d map", l, d.k, d.k, side, side2);
            else { ly.k = ly.k2 = d.k; ly.cout = d.maps; ly.tanh_out = true; side -= d.k - 1; side2 -= d.k - 1; }
        } else if (d.kind == MPCNN_MP) {
            const int pc = d.k2 > 0 ? d.k2 : d.k;   // columns of the window
            if (d.k < 1 || d.k2 < 0) st = fail(MPCNN_EINVAL, "layer %d: MP needs k >= 1, k2 >= 0", l);
            else if (seen_fc) st = fail(MPCNN_ESHAPE, "layer %d: MP after FC", l);
            else if (side / d.k < 1 || side2 / pc < 1) st = fail(MPCNN_ESHAPE, "layer %d: %dx%d pooling on a %dx%d map", l, d.k, pc, side, side2);
            else if (d.k * pc > 255) st = fail(MPCNN_EUNSUPPORTED, "layer %d: pooling window too large for byte tap codes", l);
            else {
                ly.k = d.k; ly.k2 = pc; ly.cout = ch; ly.tanh_out = false;
                ly.drop = side % d.k; ly.drop2 = side2 % pc;
                side /= d.k; side2 /= pc; dil *= d.k; dil2 *= pc;
            }
        } else if (d.kind == MPCNN_FC) {
            if (d.maps < 1) st = fail(MPCNN_EINVAL, "layer %d: FC needs maps >= 1", l);
            else {
                ly.k = seen_fc ? 1 : side; ly.k2 = seen_fc ? 1 : side2;
                ly.cout = d.maps; ly.tanh_out = (l != n_layers - 1); side = side2 = 1; seen_fc = true;
            }
        } else st = fail(MPCNN_EINVAL, "layer %d: unknown kind %d", l, d.kind);
        if (st != MPCNN_OK) break;
        // rows and columns differ (a rectangular pool or anything behind one): the kernels on the fp32
        // matrix instruction take such a layer, the bf16 instruction's kernels and the max-filter
        // kernels with several elements per thread do not
        ly.rect = ly.k2 != ly.k || (ly.dil2 != ly.dil && (ly.k > 1 || ly.k2 > 1));
        if (ly.kind != MPCNN_MP) {
            ly.p_off = off;
            ly.p_len = ((size_t)ly.k * ly.k2 * ly.cin + 1) * ly.cout;
            off += ly.p_len;
            // matrix cores take layers whose reduced channel count is a multiple of 4 and at
            // least 8, and that produce at least 8 channels; the rest run on the direct kernels
            const bool last = l == n_layers - 1;
            ly.class_fused = last && ly.k == 1 && ly.cin % 4 == 0 && ly.cin <= 256 &&
                             ly.cout >= 2 && ly.cout <= 4;
            ly.fwd_mfma = !last && ly.cin % 4 == 0 && ly.cin >= 8 && ly.cout >= 8;
            ly.dgrad_mfma = l > 0 && ly.cout % 4 == 0 && ly.cout >= 8 && ly.cin >= 8;
            ly.wgrad_mfma = !ly.class_fused;   // any shape: gradient rows are tiled in parameter order
            // (the convolution kernels address a layer's weight pack by 32-bit byte offsets)
            const size_t pack_bound = (size_t)ly.k * ly.k2 * (ceil_div(std::max(ly.cin, ly.cout), 32) * 32 + 32) *
                                      (ceil_div(std::max(ly.cin, ly.cout), 32) * 32 + 32) * 4;
            if (pack_bound >= (1ull << 31)) ly.fwd_mfma = ly.dgrad_mfma = false;
            // bf16 storage with channel counts that are multiples of 8: the bf16 matrix instruction
            ly.fwd_bm = net->bf16 && !ly.rect && ly.fwd_mfma && ly.cin % 8 == 0;
            ly.dgrad_bm = net->bf16 && !ly.rect && ly.dgrad_mfma && ly.cout % 8 == 0;
            if (ly.fwd_mfma) {
                ly.fwd_ct = ly.fwd_bm ? chan_tiling_w(ly.cout, 32) : chan_tiling(ly.cout);
                ly.fwd_rpad = ceil_div(ly.cin, 16) * 16;
                ly.fwd_pack_len = (size_t)ly.k * ly.k2 * ly.fwd_rpad * ly.fwd_ct.pad;
                ly.fwd_pack_off = pack; pack += ly.fwd_pack_len;
            }
            if (ly.dgrad_mfma) {
                ly.dgrad_ct = ly.dgrad_bm ? chan_tiling_w(ly.cin, 32) : chan_tiling(ly.cin);
                ly.dgrad_rpad = ceil_div(ly.cout, 16) * 16;
                ly.dgrad_pack_len = (size_t)ly.k * ly.k2 * ly.dgrad_rpad * ly.dgrad_ct.pad;
                ly.dgrad_pack_off = pack; pack += ly.dgrad_pack_len;
            }
        }
        ch = ly.cout;
        net->layers.push_back(ly);
    }
    if (st == MPCNN_OK && layers[n_layers - 1].kind != MPCNN_FC)
        st = fail(MPCNN_ESHAPE, "the last layer must be FC");
    if (st == MPCNN_OK && ch > mpcnn::kMaxClasses)
        st = fail(MPCNN_EUNSUPPORTED, "%d classes, at most %d are built", ch, mpcnn::kMaxClasses);
    if (st != MPCNN_OK) { delete net; return st; }
    net->n_cls = ch; net->n_params = off; net->pack_len = pack;
    *out = net;
    return MPCNN_OK;
}

void mpcnn_net_destroy(mpcnn_net* net)
{
    if (!net) return;
    if (net->d_params || net->d_grads || net->d_packs) {
        (void)hipSetDevice(net->device);
        (void)hipDeviceSynchronize();
        if (net->d_wread && net->d_wread != net->d_params) (void)hipFree(net->d_wread);
        (void)hipFree(net->d_params0);
        (void)hipFree(net->d_scalar);
        lbfgs_free(net);
        (void)hipFree(net->d_params);
        (void)hipFree(net->d_grads);
        (void)hipFree(net->d_packs);
    }
    for (auto& p : net->pending) { (void)hipEventDestroy(p.e0); (void)hipEventDestroy(p.e1); }
    for (auto e : net->pool) (void)hipEventDestroy(e);
    delete net;
}

int mpcnn_net_patch(const mpcnn_net* net) { return net ? net->patch : 0; }
int mpcnn_net_classes(const mpcnn_net* net) { return net ? net->n_cls : 0; }
size_t mpcnn_param_count(const mpcnn_net* net) { return net ? net->n_params : 0; }

mpcnn_status mpcnn_layer_shape(const mpcnn_net* net, int H, int W, int layer, int* rows, int* cols,
                               int* channels, int* spacing)
{
    if (!net) return fail(MPCNN_EINVAL, "null net");
    if (layer < 0 || layer >= (int)net->layers.size()) return fail(MPCNN_EINVAL, "layer %d out of range", layer);
    const auto gp = (H >= net->patch && W >= net->patch) ? geom_for(net, 1, H, W, false, false) : nullptr;
    if (!gp) return fail(MPCNN_ESHAPE, "image %dx%d smaller than the %d patch", H, W, net->patch);
    const Geom& g = *gp;
    const Layer& ly = net->layers[layer];
    if (rows) *rows = g.rows[layer];
    if (cols) *cols = g.cols[layer];
    if (channels) *channels = ly.cout;
    if (spacing) *spacing = ly.kind == MPCNN_MP ? ly.dil * ly.k : ly.dil;
    return MPCNN_OK;
}

mpcnn_status mpcnn_plan_describe(const mpcnn_net* net, int B, int H, int W, int training, char* text_host,
                                 size_t cap)
{
    if (!net || !text_host || cap < 1) return fail(MPCNN_EINVAL, "null argument");
    text_host[0] = 0;
    if (B < 1 || H < net->patch || W < net->patch) return fail(MPCNN_ESHAPE, "image %dx%d smaller than the %d patch", H, W, net->patch);
    const auto gp = geom_for(net, B, H, W, training != 0, false);
    if (!gp) return fail(MPCNN_ESHAPE, "layer plan does not fit a %dx%d image", H, W);
    const Geom& g = *gp;
    size_t used = 0;
    auto put = [&](const char* fmt, ...) {
        if (used + 1 >= cap) return;
        va_list ap;
        va_start(ap, fmt);
        const int n = vsnprintf(text_host + used, cap - used, fmt, ap);
        va_end(ap);
        if (n > 0) used = std::min(cap - 1, used + (size_t)n);
    };
    auto conv = [&](const char* what, const Layer& ly, const TilePlan& tp, const ChanTiling& ct, bool bm) {
        if (!tp.ok) { put("  %s: plain kernel\n", what); return; }
        put("  %s: %s %d-wide x %d channel tiles x %d groups, %d position tiles (%d per wave), %d waves, tile %d x %d of a "
            "residue class, %d x %d tiles, %zu B LDS\n", what,
            bm ? "bf16 MFMA, tile per wave," : (tp.MP > 0 ? "fp32 MFMA, tile per wave," : "fp32 MFMA, split reduction,"),
            ct.W, ct.OT, ct.split, tp.PT, tp.MP, tp.MP > 0 ? ct.OT * tp.PT / tp.MP : tp.NW, tp.Ty, tp.Tx, tp.nty, tp.ntx, tp.lds);
    };
    put("workspace %zu bytes\n", g.total);
    for (size_t l = 0; l < net->layers.size(); ++l) {
        const Layer& ly = net->layers[l];
        put("layer %zu: %s %d -> %d channels, k %d x %d, spacing %d x %d, map %d x %d\n", l,
            ly.kind == MPCNN_MP ? "MP" : (ly.kind == MPCNN_C ? "C" : "FC"), ly.cin, ly.cout, ly.k, ly.k2, ly.dil, ly.dil2,
            g.rows[l], g.cols[l]);
        if (ly.kind == MPCNN_MP) continue;
        if (ly.class_fused) { put("  fused class layer, %d workgroups\n", g.partial_n[l]); continue; }
        const bool img_sides = ly.dil == 1 && !ly.rect && (ly.k == 3 || ly.k == 5 || ly.k == 7);
        if (!g.fwd[l].ok && l == 0 && net->bf16 && img_sides && ly.cin <= 4 && ly.cout <= 64)
            put("  forward: image-layer kernel on the bf16 MFMA\n");
        else if (!g.fwd[l].ok && !net->bf16 && img_sides && (ly.cin == 1 || ly.cin == 3) &&
                 (long)B * g.rows[l] * g.cols[l] < (1l << 31) / 32)
            put("  forward: image-layer kernel on the fp32 MFMA\n");
        else
            conv("forward", ly, g.fwd[l], ly.fwd_ct, ly.fwd_bm);
        if (!training) continue;
        if (l > 0) conv("data gradient", ly, g.dgrad[l], ly.dgrad_ct, ly.dgrad_bm);
        const WgradPlan& w = g.wgrad[l];
        if (l == 0 && g.l0_fused) put("  weight gradient: fused with the routing of the pool above, %d workgroups\n", g.l0_blocks);
        else if (w.l0m) put("  weight gradient: image-layer kernel on the fp32 MFMA, %d tiles of 8 x 32, %d workgroups\n", w.tiles_total, w.chunks);
        else if (!w.ok) put("  weight gradient: plain kernel, %d chunks\n", w.chunks);
        else
            put("  weight gradient: %s MFMA, %d x %d result tiles, waves %d x %d x %d (rows x columns x tile rows), %d row "
                "tiles per wave, %d x %d workgroup groups, tile 4 x %d (%d), %d tiles in %d slabs of %d, %zu B LDS\n",
                w.tr ? "bf16 (transposing reads)" : (w.bm ? "bf16" : "fp32"), w.Mt, w.Nt, w.wm, w.wn, w.wk, w.mw, w.gm, w.gn, w.Tx, w.TxP, w.tiles_total, w.slabs,
                w.tiles_per_slab, w.lds);
    }
    return MPCNN_OK;
}

mpcnn_status mpcnn_set_params(mpcnn_net* net, const float* params_host, size_t n)
{
    if (!net || !params_host) return fail(MPCNN_EINVAL, "null argument");
    if (n != net->n_params) return fail(MPCNN_EINVAL, "n = %zu, net has %zu parameters", n, net->n_params);
    if (!net->d_params) {
        HIP_TRY(hipGetDevice(&net->device));
        HIP_TRY(hipMalloc((void**)&net->d_params, sizeof(float) * n));
        HIP_TRY(hipMalloc((void**)&net->d_grads, sizeof(float) * n));
        HIP_TRY(hipMemset(net->d_grads, 0, sizeof(float) * n));
        if (net->pack_len) HIP_TRY(hipMalloc((void**)&net->d_packs, sizeof(float) * net->pack_len));
        if (net->bf16) HIP_TRY(hipMalloc((void**)&net->d_wread, sizeof(float) * n));
        else net->d_wread = net->d_params;
        mpcnn_status rc = set_lds_attrs(net->bf16);
        if (rc != MPCNN_OK) return rc;
        const Layer& last = net->layers.back();
        if (last.class_fused) {
            const int kv = last.cin <= 128 ? 2 : 4;
            const int occ = net->bf16 ? class_occupancy<mpcnn::bf16>(last.cout, kv, last.cin) : class_occupancy<float>(last.cout, kv, last.cin);
            if (occ > 0) net->class_max_blocks = std::min(kLossBlocks, kNumCU * occ);
        }
        net->geoms.clear();   // plans made before this point counted the class layer's shares differently
        void* unused = nullptr;   // (the static workspace's address on this device, for later calls)
        rc = scratch_address(net->device, &unused);
        if (rc != MPCNN_OK) return rc;
    }
    std::vector<float> tmp(n);
    to_device_order(net, params_host, tmp.data());
    HIP_TRY(hipSetDevice(net->device));
    HIP_TRY(hipDeviceSynchronize());
    HIP_TRY(hipMemcpy(net->d_params, tmp.data(), sizeof(float) * n, hipMemcpyHostToDevice));
    net->packs_stale = true; net->wread_stale = true;
    net->lb_head = net->lb_count = 0; net->lb_have_prev = false;   // a new starting point has no history
    return MPCNN_OK;
}

mpcnn_status mpcnn_set_loss(mpcnn_net* net, mpcnn_loss kind)
{
    if (!net) return fail(MPCNN_EINVAL, "null net");
    if (kind != MPCNN_LOSS_MCCE && kind != MPCNN_LOSS_MSE) return fail(MPCNN_EINVAL, "unknown loss %d", (int)kind);
    net->loss_kind = kind;
    return MPCNN_OK;
}

mpcnn_status mpcnn_set_activation(mpcnn_net* net, mpcnn_activation kind)
{
    if (!net) return fail(MPCNN_EINVAL, "null net");
    if (kind != MPCNN_TANH && kind != MPCNN_LOGISTIC) return fail(MPCNN_EINVAL, "unknown activation %d", (int)kind);
    net->logistic = kind == MPCNN_LOGISTIC ? 1 : 0;
    return MPCNN_OK;
}

mpcnn_status mpcnn_set_conv_tiling(mpcnn_net* net, int position_tiles, int tiles_per_wave)
{
    if (!net) return fail(MPCNN_EINVAL, "null net");
    const bool pt_ok = position_tiles == 0 || position_tiles == 2 || position_tiles == 4 || position_tiles == 8 ||
                       position_tiles == 16;
    const bool mp_ok = tiles_per_wave == 0 || tiles_per_wave == 1 || tiles_per_wave == 2 || tiles_per_wave == 4;
    if (!pt_ok || !mp_ok)
        return fail(MPCNN_EINVAL, "conv tiling (%d, %d): position tiles 0/2/4/8/16, tiles per wave 0/1/2/4", position_tiles, tiles_per_wave);
    net->hint_pt = position_tiles; net->hint_mp = tiles_per_wave;
    net->geoms.clear();
    return MPCNN_OK;
}

mpcnn_status mpcnn_class_balance_weights(const mpcnn_net* net, const int32_t* labels_dev, int B, int H,
                                         int W, float* pixw_dev, void* counts_dev, void* hip_stream)
{
    if (!net || !labels_dev || !pixw_dev || !counts_dev) return fail(MPCNN_EINVAL, "null argument");
    if (B < 1) return fail(MPCNN_EINVAL, "B = %d", B);
    if (H < net->patch || W < net->patch)
        return fail(MPCNN_ESHAPE, "image %dx%d smaller than the %dx%d patch", H, W, net->patch, net->patch);
    hipStream_t st = (hipStream_t)hip_stream;
    const int Ho = H - net->patch + 1, Wo = W - net->patch + 1, ctr = (net->patch - 1) / 2;
    unsigned* counts = (unsigned*)counts_dev;
    mpcnn::clear_counts_kernel<<<1, 64, 0, st>>>(counts);
    mpcnn::label_count_kernel<<<grid_for((long)B * Ho * Wo, 256, 1024), 256, 0, st>>>(labels_dev, counts, B, H, W, Ho,
                                                                                    Wo, ctr, net->n_cls);
    mpcnn::balance_fill_kernel<<<grid_for((long)B * H * W), 256, 0, st>>>(labels_dev, counts, pixw_dev, B, H, W, Ho,
                                                                         Wo, ctr, net->n_cls);
    HIP_TRY(hipGetLastError());
    return MPCNN_OK;
}

mpcnn_status mpcnn_get_params(const mpcnn_net* net, float* params_host, size_t n)
{
    return read_back(net, net ? net->d_params : nullptr, params_host, n);
}

mpcnn_status mpcnn_get_grads(const mpcnn_net* net, float* grads_host, size_t n)
{
    return read_back(net, net ? net->d_grads : nullptr, grads_host, n);
}

size_t mpcnn_workspace_bytes(const mpcnn_net* net, int B, int H, int W, int training)
{
    if (!net || B < 1 || H < net->patch || W < net->patch) return 0;
    const auto g = geom_for(net, B, H, W, training != 0, false);
    return g ? g->total : 0;
}

static mpcnn_status check_call(mpcnn_net* net, const float* image, int B, int H, int W, void* ws,
                               size_t ws_bytes, bool training, std::shared_ptr<const Geom>* g)
{
    if (!net || !image || !ws) return fail(MPCNN_EINVAL, "null argument");
    if (!net->d_params) return fail(MPCNN_EINVAL, "parameters were never set");
    if (B < 1) return fail(MPCNN_EINVAL, "B = %d", B);
    if (H < net->patch || W < net->patch)
        return fail(MPCNN_ESHAPE, "image %dx%d smaller than the %dx%d patch", H, W, net->patch, net->patch);
    *g = geom_for(net, B, H, W, training, false);
    if (!*g) return fail(MPCNN_ESHAPE, "layer plan does not fit a %dx%d image", H, W);
    if (ws_bytes < (*g)->total) return fail(MPCNN_EWORKSPACE, "workspace %zu bytes, need %zu", ws_bytes, (*g)->total);
    if (((uintptr_t)ws & 255u) != 0) return fail(MPCNN_EINVAL, "workspace must be 256-byte aligned");
    if (((uintptr_t)image & 15u) != 0) return fail(MPCNN_EINVAL, "image must be 16-byte aligned");
    return MPCNN_OK;
}

static mpcnn_status forward_with(mpcnn_net* net, const std::shared_ptr<const Geom>& g, const float* image_dev,
                                 float* probs_dev, void* ws_dev, hipStream_t stream)
{
    mpcnn_status st = net->bf16 ? run_forward<mpcnn::bf16>(net, *g, image_dev, (char*)ws_dev, nullptr, nullptr, probs_dev,
                                                           nullptr, nullptr, stream)
                                : run_forward<float>(net, *g, image_dev, (char*)ws_dev, nullptr, nullptr, probs_dev, nullptr,
                                                     nullptr, stream);
    net->last = g; net->last_ws = ws_dev;
    return st;
}

mpcnn_status mpcnn_seg_forward(mpcnn_net* net, const float* image_dev, int B, int H, int W,
                               float* probs_dev, void* ws_dev, size_t ws_bytes, void* hip_stream)
{
    std::shared_ptr<const Geom> g;
    mpcnn_status st = check_call(net, image_dev, B, H, W, ws_dev, ws_bytes, false, &g);
    if (st != MPCNN_OK) return st;
    if (!probs_dev) return fail(MPCNN_EINVAL, "null probs_dev");
    return forward_with(net, g, image_dev, probs_dev, ws_dev, (hipStream_t)hip_stream);
}

mpcnn_status mpcnn_seg_forward_static(mpcnn_net* net, const float* image_dev, int B, int H, int W,
                                      float* probs_dev, void* hip_stream)
{
    if (!net || !image_dev || !probs_dev) return fail(MPCNN_EINVAL, "null argument");
    if (!net->d_params) return fail(MPCNN_EINVAL, "parameters were never set");
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev != net->device)
        return fail(MPCNN_EINVAL, "device %d is current, the net lives on device %d", dev, net->device);
    void* ws = nullptr;
    mpcnn_status st = scratch_address(dev, &ws);
    if (st != MPCNN_OK) return st;
    std::shared_ptr<const Geom> g;
    st = check_call(net, image_dev, B, H, W, ws, (size_t)MPCNN_STATIC_WORKSPACE_BYTES, false, &g);
    if (st == MPCNN_EWORKSPACE)
        return fail(MPCNN_EWORKSPACE, "a %d x %dx%d batch needs %zu bytes of workspace, the static one holds %zu",
                    B, H, W, g->total, (size_t)MPCNN_STATIC_WORKSPACE_BYTES);
    if (st != MPCNN_OK) return st;
    // (the per-launch timing hooks create events: not in a call that must not allocate)
    const bool prof = net->prof_on;
    net->prof_on = false;
    st = forward_with(net, g, image_dev, probs_dev, ws, (hipStream_t)hip_stream);
    net->prof_on = prof;
    return st;
}

size_t mpcnn_workspace_bytes_same(const mpcnn_net* net, int B, int H, int W)
{
    if (!net || B < 1 || H < 1 || W < 1) return 0;
    const auto g = geom_for(net, B, H, W, false, true);
    return g ? g->total : 0;
}

mpcnn_status mpcnn_seg_forward_same(mpcnn_net* net, const float* image_dev, int B, int H, int W,
                                    float* probs_dev, void* ws_dev, size_t ws_bytes, void* hip_stream)
{
    if (!net || !image_dev || !ws_dev || !probs_dev) return fail(MPCNN_EINVAL, "null argument");
    if (!net->d_params) return fail(MPCNN_EINVAL, "parameters were never set");
    if (B < 1) return fail(MPCNN_EINVAL, "B = %d", B);
    const int widest = net->patch - 1 - (net->patch - 1) / 2;
    if (H < 1 || W < 1 || H < widest || W < widest)
        return fail(MPCNN_ESHAPE, "image %dx%d smaller than the %d-pixel mirrored border", H, W, widest);
    const auto g = geom_for(net, B, H, W, false, true);
    if (!g) return fail(MPCNN_ESHAPE, "layer plan does not fit a %dx%d image", H, W);
    if (ws_bytes < g->total) return fail(MPCNN_EWORKSPACE, "workspace %zu bytes, need %zu", ws_bytes, g->total);
    if (((uintptr_t)ws_dev & 255u) != 0) return fail(MPCNN_EINVAL, "workspace must be 256-byte aligned");
    return forward_with(net, g, image_dev, probs_dev, ws_dev, (hipStream_t)hip_stream);
}

mpcnn_status mpcnn_seg_backward(mpcnn_net* net, const float* image_dev, const int32_t* labels_dev,
                                const float* pixw_dev, int B, int H, int W, float* probs_dev,
                                double* loss_dev, void* ws_dev, size_t ws_bytes, void* hip_stream)
{
    std::shared_ptr<const Geom> gp;
    mpcnn_status st = check_call(net, image_dev, B, H, W, ws_dev, ws_bytes, true, &gp);
    if (st != MPCNN_OK) return st;
    if (!labels_dev) return fail(MPCNN_EINVAL, "null labels_dev");
    const Geom& g = *gp;
    hipStream_t stream = (hipStream_t)hip_stream;
    char* ws = (char*)ws_dev;
    void* dZ = ws + g.delta_off[0];
    st = net->bf16 ? run_forward<mpcnn::bf16>(net, g, image_dev, ws, labels_dev, pixw_dev, probs_dev, dZ, loss_dev, stream)
                   : run_forward<float>(net, g, image_dev, ws, labels_dev, pixw_dev, probs_dev, dZ, loss_dev, stream);
    net->last = gp; net->last_ws = ws_dev;
    if (st != MPCNN_OK) return st;
    return net->bf16 ? run_backward<mpcnn::bf16>(net, g, image_dev, ws, stream)
                     : run_backward<float>(net, g, image_dev, ws, stream);
}

// geometry of one band of output rows [row0, row0 + rows) of a B x H x W image
static bool make_geom_band(const mpcnn_net* net, int B, int H, int W, int row0, int rows, Geom* g)
{
    if (!make_geom(net, B, rows + net->patch - 1, W, true, g, true, true)) return false;
    g->pad_top = -row0; g->pad_left = 0; g->src_h = H; g->src_w = W;   // the band starts row0 rows down the image
    g->label_h = H; g->probs_rows = H - net->patch + 1;
    g->accumulate = row0 > 0;
    return true;
}

size_t mpcnn_workspace_bytes_banded(const mpcnn_net* net, int B, int W, int band_rows)
{
    Geom g;
    if (!net || band_rows < 1 || B < 1 || W < net->patch) return 0;
    if (!make_geom_band(net, B, band_rows + net->patch - 1, W, 0, band_rows, &g)) return 0;
    return g.total;
}

mpcnn_status mpcnn_seg_backward_banded(mpcnn_net* net, const float* image_dev, const int32_t* labels_dev,
                                       const float* pixw_dev, int B, int H, int W, int band_rows,
                                       float* probs_dev, double* loss_dev, void* ws_dev, size_t ws_bytes,
                                       void* hip_stream)
{
    if (!net || !image_dev || !ws_dev || !labels_dev) return fail(MPCNN_EINVAL, "null argument");
    if (!net->d_params) return fail(MPCNN_EINVAL, "parameters were never set");
    if (B < 1 || band_rows < 1) return fail(MPCNN_EINVAL, "B = %d, band_rows = %d", B, band_rows);
    if (H < net->patch || W < net->patch)
        return fail(MPCNN_ESHAPE, "image %dx%d smaller than the %dx%d patch", H, W, net->patch, net->patch);
    if (((uintptr_t)ws_dev & 255u) != 0) return fail(MPCNN_EINVAL, "workspace must be 256-byte aligned");
    if (((uintptr_t)image_dev & 15u) != 0) return fail(MPCNN_EINVAL, "image must be 16-byte aligned");
    const int Ho = H - net->patch + 1, Wo = W - net->patch + 1;
    hipStream_t stream = (hipStream_t)hip_stream;
    char* ws = (char*)ws_dev;
    for (int row0 = 0; row0 < Ho; row0 += band_rows) {
        const int rows = std::min(band_rows, Ho - row0);
        auto gp = std::make_shared<Geom>();
        if (!make_geom_band(net, B, H, W, row0, rows, gp.get()))
            return fail(MPCNN_ESHAPE, "layer plan does not fit a band of %d rows", rows);
        const Geom& g = *gp;
        if (ws_bytes < g.total) return fail(MPCNN_EWORKSPACE, "workspace %zu bytes, need %zu", ws_bytes, g.total);
        // the band's labels, weights and probabilities start row0 rows down their arrays
        const int32_t* lab = labels_dev + (size_t)row0 * W;
        const float* pw = pixw_dev ? pixw_dev + (size_t)row0 * W : nullptr;
        float* pr = probs_dev ? probs_dev + (size_t)row0 * Wo : nullptr;
        void* dZ = ws + g.delta_off[0];
        mpcnn_status st =
            net->bf16 ? run_forward<mpcnn::bf16>(net, g, image_dev, ws, lab, pw, pr, dZ, loss_dev, stream)
                      : run_forward<float>(net, g, image_dev, ws, lab, pw, pr, dZ, loss_dev, stream);
        net->last = gp; net->last_ws = ws_dev;
        if (st != MPCNN_OK) return st;
        st = net->bf16 ? run_backward<mpcnn::bf16>(net, g, image_dev, ws, stream)
                       : run_backward<float>(net, g, image_dev, ws, stream);
        if (st != MPCNN_OK) return st;
    }
    return MPCNN_OK;
}

// forward + summed loss, nothing kept (the workspace is a forward-only one)
static mpcnn_status loss_only(mpcnn_net* net, const Geom& g, const float* image_dev, const int32_t* labels_dev,
                              const float* pixw_dev, double* loss_dev, char* ws, hipStream_t st)
{
    mpcnn_status rc = net->bf16 ? run_forward<mpcnn::bf16>(net, g, image_dev, ws, labels_dev, pixw_dev, nullptr,
                                                           nullptr, loss_dev, st)
                                : run_forward<float>(net, g, image_dev, ws, labels_dev, pixw_dev, nullptr, nullptr,
                                                     loss_dev, st);
    if (rc != MPCNN_OK) return rc;
    if (net->loss_shares < 1) return fail(MPCNN_EINVAL, "no loss was computed");
    mpcnn::ReduceArgs ra{};
    mpcnn::ReduceSeg& sg = ra.seg[ra.n_seg++];
    sg.partial = (const float*)(ws + g.loss_partial_off);
    sg.out = (float*)loss_dev;
    sg.n = net->loss_shares; sg.tiled = 2; sg.items = 1; sg.block0 = 0;
    ra.total_blocks = 1;
    LAUNCH("reduce_all", -1, 0, 0, 8.0 * sg.n, mpcnn::reduce_all_kernel<<<1, 256, 0, st>>>(ra));
    HIP_TRY(hipGetLastError());
    return MPCNN_OK;
}

mpcnn_status mpcnn_seg_loss(mpcnn_net* net, const float* image_dev, const int32_t* labels_dev,
                            const float* pixw_dev, int B, int H, int W, double* loss_dev,
                            void* ws_dev, size_t ws_bytes, void* hip_stream)
{
    std::shared_ptr<const Geom> gp;
    mpcnn_status st = check_call(net, image_dev, B, H, W, ws_dev, ws_bytes, false, &gp);
    if (st != MPCNN_OK) return st;
    if (!labels_dev || !loss_dev) return fail(MPCNN_EINVAL, "null argument");
    return loss_only(net, *gp, image_dev, labels_dev, pixw_dev, loss_dev, (char*)ws_dev, (hipStream_t)hip_stream);
}

mpcnn_status mpcnn_armijo_step(mpcnn_net* net, const float* image_dev, const int32_t* labels_dev,
                               const float* pixw_dev, int B, int H, int W, double f0, float alpha0,
                               float grad_scale, float c, float beta, int max_trials, void* ws_dev,
                               size_t ws_bytes, void* hip_stream, float* alpha_host, double* loss_host,
                               int* trials_host)
{
    std::shared_ptr<const Geom> gp;
    mpcnn_status rc = check_call(net, image_dev, B, H, W, ws_dev, ws_bytes, false, &gp);
    if (rc != MPCNN_OK) return rc;
    const Geom& g = *gp;
    if (!labels_dev) return fail(MPCNN_EINVAL, "null labels_dev");
    if (!(alpha0 > 0.f) || !(beta > 0.f && beta < 1.f) || !(c >= 0.f && c < 1.f) || max_trials < 1)
        return fail(MPCNN_EINVAL, "alpha0 = %g, beta = %g, c = %g, max_trials = %d", alpha0, beta, c, max_trials);
    hipStream_t st = (hipStream_t)hip_stream;
    const long n = (long)net->n_params;
    if (!net->d_params0) HIP_TRY(hipMalloc((void**)&net->d_params0, sizeof(float) * n));
    if (!net->d_scalar) HIP_TRY(hipMalloc((void**)&net->d_scalar, 8 * sizeof(double)));
    HIP_TRY(hipMemcpyAsync(net->d_params0, net->d_params, sizeof(float) * n, hipMemcpyDeviceToDevice, st));
    mpcnn::sqnorm_kernel<<<1, 1024, 0, st>>>(net->d_grads, n, net->d_scalar);
    double gg = 0.0;
    HIP_TRY(hipMemcpyAsync(&gg, net->d_scalar, sizeof(double), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    float alpha = alpha0;
    double f = f0;
    int trial = 0;
    bool ok = false;
    while (trial < max_trials) {
        ++trial;
        mpcnn::step_from_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(net->d_params, net->d_params0,
                                                                              net->d_grads, alpha * grad_scale, n);
        net->packs_stale = true; net->wread_stale = true;
        rc = loss_only(net, g, image_dev, labels_dev, pixw_dev, net->d_scalar + 1, (char*)ws_dev, st);
        if (rc != MPCNN_OK) break;
        HIP_TRY(hipMemcpyAsync(&f, net->d_scalar + 1, sizeof(double), hipMemcpyDeviceToHost, st));
        HIP_TRY(hipStreamSynchronize(st));
        if (f <= f0 - (double)c * (double)alpha * (double)grad_scale * gg) { ok = true; break; }
        alpha *= beta;
    }
    if (!ok) {   // also after an error: the parameters the call started from
        HIP_TRY(hipMemcpyAsync(net->d_params, net->d_params0, sizeof(float) * n, hipMemcpyDeviceToDevice, st));
        HIP_TRY(hipStreamSynchronize(st));
        net->packs_stale = true; net->wread_stale = true;
        alpha = 0.f; f = f0;
    }
    if (alpha_host) *alpha_host = alpha;
    if (loss_host) *loss_host = f;
    if (trials_host) *trials_host = trial;
    return rc;
}

mpcnn_status mpcnn_lbfgs_reset(mpcnn_net* net)
{
    if (!net) return fail(MPCNN_EINVAL, "null net");
    net->lb_head = net->lb_count = 0;
    net->lb_have_prev = false;
    return MPCNN_OK;
}

mpcnn_status mpcnn_lbfgs_step(mpcnn_net* net, const float* image_dev, const int32_t* labels_dev,
                              const float* pixw_dev, int B, int H, int W, double f0, int history,
                              float alpha0, float c, float beta, int max_trials, void* ws_dev,
                              size_t ws_bytes, void* hip_stream, float* alpha_host, double* loss_host,
                              int* trials_host, int* pairs_host)
{
    using namespace mpcnn;
    std::shared_ptr<const Geom> gp;
    mpcnn_status rc = check_call(net, image_dev, B, H, W, ws_dev, ws_bytes, false, &gp);
    if (rc != MPCNN_OK) return rc;
    const Geom& g = *gp;
    if (!labels_dev) return fail(MPCNN_EINVAL, "null labels_dev");
    if (!(alpha0 > 0.f) || !(beta > 0.f && beta < 1.f) || !(c >= 0.f && c < 1.f) || max_trials < 1 ||
        history < 1 || history > 64)
        return fail(MPCNN_EINVAL, "alpha0 = %g, beta = %g, c = %g, max_trials = %d, history = %d", alpha0, beta,
                    c, max_trials, history);
    hipStream_t st = (hipStream_t)hip_stream;
    const long n = (long)net->n_params;
    const size_t vec = sizeof(float) * n;
    if (net->lb_m != history) {   // first call, or another history length: start afresh
        lbfgs_free(net);
        HIP_TRY(hipMalloc((void**)&net->d_lb_S, vec * (history + 1)));
        HIP_TRY(hipMalloc((void**)&net->d_lb_Y, vec * (history + 1)));
        HIP_TRY(hipMalloc((void**)&net->d_lb_theta_prev, vec));
        HIP_TRY(hipMalloc((void**)&net->d_lb_g_prev, vec));
        HIP_TRY(hipMalloc((void**)&net->d_lb_p, vec));
        HIP_TRY(hipMalloc((void**)&net->d_lb_part, sizeof(double) * 5 * kLbBlocks));
        HIP_TRY(hipMalloc((void**)&net->d_lb_alpha, sizeof(double) * (history + 1)));
        net->lb_m = history;
        net->lb_sy.assign(history + 1, 0.0); net->lb_yy.assign(history + 1, 0.0);
    }
    if (!net->d_params0) HIP_TRY(hipMalloc((void**)&net->d_params0, vec));
    if (!net->d_scalar) HIP_TRY(hipMalloc((void**)&net->d_scalar, 8 * sizeof(double)));
    const int slots = net->lb_m + 1;
    double* part[2] = {net->d_lb_part, net->d_lb_part + kLbBlocks};

    // 1. the pair (theta - theta_prev, g - g_prev), kept if its curvature s.y is positive
    if (net->lb_have_prev) {
        const int slot = (net->lb_head + net->lb_count) % slots;
        lb_pair_kernel<<<kLbBlocks, 256, 0, st>>>(net->d_params, net->d_lb_theta_prev, net->d_grads, net->d_lb_g_prev,
                                                  net->d_lb_S + (size_t)slot * n, net->d_lb_Y + (size_t)slot * n,
                                                  net->d_lb_part + 2 * kLbBlocks, n);
        lb_sum_kernel<<<1, 256, 0, st>>>(net->d_lb_part + 2 * kLbBlocks, 3, net->d_scalar + 2);
        double r[3];
        HIP_TRY(hipMemcpyAsync(r, net->d_scalar + 2, sizeof(r), hipMemcpyDeviceToHost, st));
        HIP_TRY(hipStreamSynchronize(st));
        if (r[0] > 1e-10 * std::sqrt(r[2] * r[1])) {
            net->lb_sy[slot] = r[0]; net->lb_yy[slot] = r[1];
            if (net->lb_count < net->lb_m) ++net->lb_count;
            else net->lb_head = (net->lb_head + 1) % slots;   // the oldest pair's slot becomes the free one
        }
    }

    // 2. p = -H g by the two-loop recursion, and the slope g.p
    double slope = 0.0;
    for (int attempt = 0; attempt < 2; ++attempt) {
        const int M = net->lb_count;
        auto slot_of = [&](int i) { return (net->lb_head + i) % slots; };   // i = 0 oldest
        LbArgs a{};
        a.q = net->d_lb_p; a.n = n; a.alpha = net->d_lb_alpha;
        int flip = 0;
        a.mode = 0; a.src = net->d_grads; a.part_out = part[flip];
        if (M == 0) { a.scale = -1.0; a.u = net->d_grads; }
        else { a.scale = 1.0; a.u = net->d_lb_S + (size_t)slot_of(M - 1) * n; }
        lb_update_kernel<<<kLbBlocks, 256, 0, st>>>(a);
        for (int i = M - 1; i >= 0; --i) {        // newest to oldest
            const int sl = slot_of(i);
            a.mode = 1; a.idx = i; a.rho = 1.0 / net->lb_sy[sl];
            a.v = net->d_lb_Y + (size_t)sl * n;
            a.part_in = part[flip]; flip ^= 1; a.part_out = part[flip];
            if (i > 0) { a.scale = 1.0; a.u = net->d_lb_S + (size_t)slot_of(i - 1) * n; }
            else {                                  // the turn: r = H_0 q
                const int nw = slot_of(M - 1);
                a.scale = net->lb_sy[nw] / net->lb_yy[nw];
                a.u = net->d_lb_Y + (size_t)slot_of(0) * n;
            }
            lb_update_kernel<<<kLbBlocks, 256, 0, st>>>(a);
        }
        for (int i = 0; i < M; ++i) {              // oldest to newest
            const int sl = slot_of(i);
            a.mode = 2; a.idx = i; a.rho = 1.0 / net->lb_sy[sl];
            a.v = net->d_lb_S + (size_t)sl * n;
            a.part_in = part[flip]; flip ^= 1; a.part_out = part[flip];
            if (i + 1 < M) { a.scale = 1.0; a.u = net->d_lb_Y + (size_t)slot_of(i + 1) * n; }
            else { a.scale = -1.0; a.u = net->d_grads; }
            lb_update_kernel<<<kLbBlocks, 256, 0, st>>>(a);
        }
        lb_sum_kernel<<<1, 256, 0, st>>>(part[flip], 1, net->d_scalar);
        HIP_TRY(hipMemcpyAsync(&slope, net->d_scalar, sizeof(double), hipMemcpyDeviceToHost, st));
        HIP_TRY(hipStreamSynchronize(st));
        if (slope < 0.0 || M == 0) break;
        net->lb_count = 0;                         // not a descent direction: forget the pairs
    }
    const int used = net->lb_count;

    // 3. back-tracking along p
    HIP_TRY(hipMemcpyAsync(net->d_params0, net->d_params, vec, hipMemcpyDeviceToDevice, st));
    float alpha = alpha0;
    double f = f0;
    int trial = 0;
    bool ok = false;
    while (slope < 0.0 && trial < max_trials) {
        ++trial;
        step_from_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(net->d_params, net->d_params0, net->d_lb_p,
                                                                      -alpha, n);
        net->packs_stale = true; net->wread_stale = true;
        rc = loss_only(net, g, image_dev, labels_dev, pixw_dev, net->d_scalar + 1, (char*)ws_dev, st);
        if (rc != MPCNN_OK) break;
        HIP_TRY(hipMemcpyAsync(&f, net->d_scalar + 1, sizeof(double), hipMemcpyDeviceToHost, st));
        HIP_TRY(hipStreamSynchronize(st));
        if (f <= f0 + (double)c * (double)alpha * slope) { ok = true; break; }
        alpha *= beta;
    }
    if (ok) {      // this iterate becomes the previous one
        std::swap(net->d_params0, net->d_lb_theta_prev);
        HIP_TRY(hipMemcpyAsync(net->d_lb_g_prev, net->d_grads, vec, hipMemcpyDeviceToDevice, st));
        HIP_TRY(hipStreamSynchronize(st));
        net->lb_have_prev = true;
    } else {       // also after an error: the parameters the call started from, no history
        HIP_TRY(hipMemcpyAsync(net->d_params, net->d_params0, vec, hipMemcpyDeviceToDevice, st));
        HIP_TRY(hipStreamSynchronize(st));
        net->packs_stale = true; net->wread_stale = true;
        net->lb_count = 0; net->lb_head = 0; net->lb_have_prev = false;
        alpha = 0.f; f = f0;
    }
    if (alpha_host) *alpha_host = alpha;
    if (loss_host) *loss_host = f;
    if (trials_host) *trials_host = trial;
    if (pairs_host) *pairs_host = used;
    return rc;
}

mpcnn_status mpcnn_sgd_step(mpcnn_net* net, float lr, float grad_scale, void* hip_stream)
{
    if (!net) return fail(MPCNN_EINVAL, "null net");
    if (!net->d_params) return fail(MPCNN_EINVAL, "parameters were never set");
    long n = (long)net->n_params;
    hipStream_t st = (hipStream_t)hip_stream;
    LAUNCH("sgd", -1, 8, 2.0 * n, 12.0 * n,
           mpcnn::sgd_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(net->d_params, net->d_grads,
                                                                          lr * grad_scale, n));
    HIP_TRY(hipGetLastError());
    net->packs_stale = true; net->wread_stale = true;
    return MPCNN_OK;
}

mpcnn_status mpcnn_get_activation(const mpcnn_net* net, int layer, float* host, size_t n)
{
    if (!net || !host) return fail(MPCNN_EINVAL, "null argument");
    if (!net->last_ws || !net->last || !net->last->training) return fail(MPCNN_EINVAL, "no backward call has been made");
    if (layer < 0 || layer >= (int)net->layers.size()) return fail(MPCNN_EINVAL, "layer %d out of range", layer);
    const Geom& g = *net->last;
    size_t elems = (size_t)g.B * g.rows[layer] * g.cols[layer] * net->layers[layer].cout;
    if (n != elems) return fail(MPCNN_EINVAL, "n = %zu, layer holds %zu elements", n, elems);
    HIP_TRY(hipSetDevice(net->device));
    HIP_TRY(hipDeviceSynchronize());
    const char* src = (const char*)net->last_ws + g.act_off[layer];
    if (!net->bf16) {
        HIP_TRY(hipMemcpy(host, src, sizeof(float) * elems, hipMemcpyDeviceToHost));
    } else {
        std::vector<uint16_t> tmp(elems);
        HIP_TRY(hipMemcpy(tmp.data(), src, sizeof(uint16_t) * elems, hipMemcpyDeviceToHost));
        for (size_t i = 0; i < elems; ++i) {
            const uint32_t bits = (uint32_t)tmp[i] << 16;   // bf16 = the upper half of an fp32
            memcpy(host + i, &bits, sizeof(float));
        }
    }
    return MPCNN_OK;
}

mpcnn_status mpcnn_get_argmax(const mpcnn_net* net, int layer, uint8_t* host, size_t n)
{
    if (!net || !host) return fail(MPCNN_EINVAL, "null argument");
    if (!net->last_ws || !net->last || !net->last->training) return fail(MPCNN_EINVAL, "no backward call has been made");
    if (layer < 0 || layer >= (int)net->layers.size() || net->layers[layer].kind != MPCNN_MP)
        return fail(MPCNN_EINVAL, "layer %d is not an MP layer", layer);
    const Geom& g = *net->last;
    size_t elems = (size_t)g.B * g.rows[layer] * g.cols[layer] * net->layers[layer].cout;
    if (n != elems) return fail(MPCNN_EINVAL, "n = %zu, layer holds %zu elements", n, elems);
    HIP_TRY(hipSetDevice(net->device));
    HIP_TRY(hipDeviceSynchronize());
    HIP_TRY(hipMemcpy(host, (char*)net->last_ws + g.code_off[layer], elems, hipMemcpyDeviceToHost));
    return MPCNN_OK;
}

mpcnn_status mpcnn_profile_enable(mpcnn_net* net, int on)
{
    if (!net) return fail(MPCNN_EINVAL, "null net");
    net->prof_on = on != 0;
    return MPCNN_OK;
}

mpcnn_status mpcnn_profile_read(mpcnn_net* net, mpcnn_kernel_stat* out_host, int cap, int* n)
{
    if (!net || !n || (cap > 0 && !out_host)) return fail(MPCNN_EINVAL, "null argument");
    for (auto& p : net->pending) {
        HIP_TRY(hipEventSynchronize(p.e1));
        float ms = 0.f;
        HIP_TRY(hipEventElapsedTime(&ms, p.e0, p.e1));
        net->sites[p.site].ms += ms;
        net->sites[p.site].launches += 1;
        net->pool.push_back(p.e0);
        net->pool.push_back(p.e1);
    }
    net->pending.clear();
    *n = (int)net->sites.size();
    for (int i = 0; i < *n && i < cap; ++i) {
        const ProfSite& s = net->sites[i];
        mpcnn_kernel_stat& o = out_host[i];
        memset(&o, 0, sizeof o);
        snprintf(o.name, sizeof o.name, "%s", s.name);
        o.layer = s.layer; o.step = s.step; o.launches = s.launches;
        o.ms_total = s.ms; o.flops = s.flops; o.bytes = s.bytes;
    }
    for (auto& s : net->sites) { s.ms = 0; s.launches = 0; }
    return MPCNN_OK;
}

}  // extern "C"
