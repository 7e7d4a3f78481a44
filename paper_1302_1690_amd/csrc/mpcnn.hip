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
#include <new>
#include <vector>

#include "../../include/mpcnn.h"
#include "kernels_direct.hpp"

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

struct Layer {
    int kind;     // mpcnn_kind
    int k;        // kernel side (C, FC) or pooling side (MP)
    int cin, cout;
    int dil;      // spacing of this layer's taps in its input map
    bool tanh_out;
    size_t p_off; // offset of this layer's [(k*k*cin + 1) x cout] block in the parameter buffer
    size_t p_len;
};

// Per-call geometry: dense map sizes and workspace offsets.
struct Geom {
    int B = 0, H = 0, W = 0;
    bool training = false;
    std::vector<int> rows, cols;      // output map of layer l
    std::vector<size_t> act_off;      // byte offset of layer l's output in the workspace
    std::vector<size_t> code_off;     // MP layers: byte offset of the argmax map
    size_t staged_off = 0;            // channels-last copy of the image (C0 > 1 only)
    size_t delta_off[2] = {0, 0};     // two delta buffers, each as large as the largest map
    size_t partial_off = 0, partial_bytes = 0;
    size_t loss_partial_off = 0;
    size_t total = 0;
};

constexpr int kLossBlocks = 256;
constexpr int kWgradChunkTarget = 512;  // split of the position reduction

inline size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }

}  // namespace

struct mpcnn_net {
    std::vector<Layer> layers;
    int in_ch = 0, patch = 0, n_cls = 0;
    size_t n_params = 0;
    float* d_params = nullptr;
    float* d_grads = nullptr;
    int device = -1;
    // what the last forward / backward left behind (for the test hooks)
    Geom last;
    void* last_ws = nullptr;
};

namespace {

bool make_geom(const mpcnn_net* net, int B, int H, int W, bool training, Geom* g)
{
    if (B < 1 || H < net->patch || W < net->patch) return false;
    const size_t L = net->layers.size();
    g->B = B; g->H = H; g->W = W; g->training = training;
    g->rows.assign(L, 0); g->cols.assign(L, 0);
    g->act_off.assign(L, 0); g->code_off.assign(L, 0);
    size_t off = 0, max_act = 0, max_partial = 0;
    if (net->in_ch > 1) {
        g->staged_off = off;
        off = align_up(off + sizeof(float) * (size_t)B * H * W * net->in_ch);
    }
    int r = H, c = W;
    for (size_t l = 0; l < L; ++l) {
        const Layer& ly = net->layers[l];
        r -= (ly.k - 1) * ly.dil;
        c -= (ly.k - 1) * ly.dil;
        if (r < 1 || c < 1) return false;
        g->rows[l] = r; g->cols[l] = c;
        size_t bytes = sizeof(float) * (size_t)B * r * c * ly.cout;
        max_act = std::max(max_act, bytes);
        if (ly.kind != MPCNN_MP) {
            long rows_total = (long)B * r;
            long rpc = std::max<long>(1, (rows_total + kWgradChunkTarget - 1) / kWgradChunkTarget);
            long chunks = (rows_total + rpc - 1) / rpc;
            max_partial = std::max(max_partial, sizeof(float) * (size_t)chunks * ly.p_len);
        }
    }
    if (r != H - net->patch + 1 || c != W - net->patch + 1) return false;
    if (training) {
        for (size_t l = 0; l < L; ++l) {
            const Layer& ly = net->layers[l];
            size_t elems = (size_t)B * g->rows[l] * g->cols[l] * ly.cout;
            g->act_off[l] = off;
            off = align_up(off + sizeof(float) * elems);
            if (ly.kind == MPCNN_MP) {
                g->code_off[l] = off;
                off = align_up(off + elems);
            }
        }
        g->delta_off[0] = off; off = align_up(off + max_act);
        g->delta_off[1] = off; off = align_up(off + max_act);
        g->partial_off = off; g->partial_bytes = max_partial; off = align_up(off + max_partial);
    } else {
        // forward only: layers alternate between two buffers, nothing is kept
        size_t buf[2];
        buf[0] = off; off = align_up(off + max_act);
        buf[1] = off; off = align_up(off + max_act);
        for (size_t l = 0; l < L; ++l) g->act_off[l] = buf[l & 1];
    }
    g->loss_partial_off = off; off = align_up(off + sizeof(double) * kLossBlocks);
    g->total = off;
    return true;
}

inline int grid_for(long total, int block = 256, int cap = 1 << 20)
{
    long g = (total + block - 1) / block;
    return (int)std::min<long>(std::max<long>(g, 1), cap);
}

// Forward through every layer; in training mode everything is kept for the backward.
mpcnn_status run_forward(mpcnn_net* net, const Geom& g, const float* image, char* ws,
                         const int32_t* labels, const float* pixw, float* probs, float* dZ,
                         double* loss_dev, hipStream_t st)
{
    using namespace mpcnn;
    const int B = g.B;
    const float* in = image;
    int Hi = g.H, Wi = g.W, Ci = net->in_ch;
    if (net->in_ch > 1) {
        float* staged = (float*)(ws + g.staged_off);
        long total = (long)B * Ci * Hi * Wi;
        stage_input_kernel<<<grid_for(total), 256, 0, st>>>(image, staged, B, Ci, Hi, Wi);
        in = staged;
    }
    const size_t L = net->layers.size();
    for (size_t l = 0; l < L; ++l) {
        const Layer& ly = net->layers[l];
        float* out = (float*)(ws + g.act_off[l]);
        const int Ho = g.rows[l], Wo = g.cols[l];
        if (ly.kind == MPCNN_MP) {
            uint8_t* code = g.training ? (uint8_t*)(ws + g.code_off[l]) : nullptr;
            long total = (long)B * Ho * Wo * ly.cout;
            maxfilter_fwd_direct_kernel<<<grid_for(total), 256, 0, st>>>(in, out, code, B, Hi, Wi,
                                                                        ly.cout, Ho, Wo, ly.k, ly.dil);
        } else {
            const float* Wk = net->d_params + ly.p_off;
            long total = (long)B * Ho * Wo * ly.cout;
            if (ly.tanh_out)
                conv_fwd_direct_kernel<true><<<grid_for(total), 256, 0, st>>>(
                    in, Wk, out, B, Hi, Wi, Ci, Ho, Wo, ly.cout, ly.k, ly.dil);
            else
                conv_fwd_direct_kernel<false><<<grid_for(total), 256, 0, st>>>(
                    in, Wk, out, B, Hi, Wi, Ci, Ho, Wo, ly.cout, ly.k, ly.dil);
        }
        in = out; Hi = Ho; Wi = Wo; Ci = ly.cout;
    }
    // class logits -> probabilities, deltas, loss
    double* lp = (double*)(ws + g.loss_partial_off);
    const bool want_loss = labels && loss_dev;
    long total = (long)B * Hi * Wi;
    int blocks = std::min<long>(kLossBlocks, (total + 255) / 256);
    softmax_ce_kernel<<<blocks, 256, 0, st>>>(in, probs, labels, pixw, dZ, want_loss ? lp : nullptr,
                                              B, Hi, Wi, g.H, g.W, (net->patch - 1) / 2, net->n_cls);
    if (want_loss) loss_reduce_kernel<<<1, 64, 0, st>>>(lp, blocks, loss_dev);
    HIP_TRY(hipGetLastError());
    return MPCNN_OK;
}

mpcnn_status run_backward(mpcnn_net* net, const Geom& g, const float* image, char* ws,
                          hipStream_t st)
{
    using namespace mpcnn;
    const int B = g.B;
    const size_t L = net->layers.size();
    const float* in0 = net->in_ch > 1 ? (const float*)(ws + g.staged_off) : image;
    float* dbuf[2] = {(float*)(ws + g.delta_off[0]), (float*)(ws + g.delta_off[1])};
    float* partial = (float*)(ws + g.partial_off);
    int cur = 0;  // dbuf[cur] holds dL/d(pre-activation) of layer l's output (dL/d(output) for MP)
    for (size_t li = L; li-- > 0;) {
        const Layer& ly = net->layers[li];
        const int Ho = g.rows[li], Wo = g.cols[li];
        const float* A = li == 0 ? in0 : (const float*)(ws + g.act_off[li - 1]);
        const int Hi = li == 0 ? g.H : g.rows[li - 1], Wi = li == 0 ? g.W : g.cols[li - 1];
        const int Ci = ly.cin;
        const bool below_tanh = li > 0 && net->layers[li - 1].tanh_out;
        const float* dY = dbuf[cur];
        float* dA = dbuf[cur ^ 1];
        if (ly.kind == MPCNN_MP) {
            if (li == 0) break;  // nothing below has parameters
            const uint8_t* code = (const uint8_t*)(ws + g.code_off[li]);
            long total = (long)B * Hi * Wi * Ci;
            if (below_tanh)
                maxfilter_bwd_direct_kernel<true><<<grid_for(total), 256, 0, st>>>(
                    dY, code, A, dA, B, Hi, Wi, Ci, Ho, Wo, ly.k, ly.dil);
            else
                maxfilter_bwd_direct_kernel<false><<<grid_for(total), 256, 0, st>>>(
                    dY, code, A, dA, B, Hi, Wi, Ci, Ho, Wo, ly.k, ly.dil);
        } else {
            // parameter gradient: split over output rows, then a fixed-order sum
            long rows_total = (long)B * Ho;
            long rpc = std::max<long>(1, (rows_total + kWgradChunkTarget - 1) / kWgradChunkTarget);
            int chunks = (int)((rows_total + rpc - 1) / rpc);
            dim3 grid((unsigned)((ly.p_len + 255) / 256), (unsigned)chunks);
            conv_wgrad_direct_kernel<<<grid, 256, 0, st>>>(A, dY, partial, B, Hi, Wi, Ci, Ho, Wo,
                                                           ly.cout, ly.k, ly.dil, (int)rpc);
            reduce_partials_kernel<<<(unsigned)((ly.p_len + 255) / 256), 256, 0, st>>>(
                partial, net->d_grads + ly.p_off, (long)ly.p_len, chunks);
            if (li == 0) break;  // the image needs no gradient
            const float* Wk = net->d_params + ly.p_off;
            long total = (long)B * Hi * Wi * Ci;
            if (below_tanh)
                conv_dgrad_direct_kernel<true><<<grid_for(total), 256, 0, st>>>(
                    dY, Wk, A, dA, B, Hi, Wi, Ci, Ho, Wo, ly.cout, ly.k, ly.dil);
            else
                conv_dgrad_direct_kernel<false><<<grid_for(total), 256, 0, st>>>(
                    dY, Wk, A, dA, B, Hi, Wi, Ci, Ho, Wo, ly.cout, ly.k, ly.dil);
        }
        cur ^= 1;
    }
    HIP_TRY(hipGetLastError());
    return MPCNN_OK;
}

// host parameter order W[o][c][u][v], b[o]  <->  device order W[u][v][c][o], b[o]
void to_device_order(const mpcnn_net* net, const float* host, float* dev_order)
{
    for (const Layer& ly : net->layers) {
        if (ly.kind == MPCNN_MP) continue;
        const int k = ly.k, ci = ly.cin, co = ly.cout;
        const float* src = host + ly.p_off;
        float* dst = dev_order + ly.p_off;
        for (int o = 0; o < co; ++o)
            for (int c = 0; c < ci; ++c)
                for (int t = 0; t < k * k; ++t)
                    dst[((size_t)t * ci + c) * co + o] = src[((size_t)o * ci + c) * k * k + t];
        memcpy(dst + (size_t)k * k * ci * co, src + (size_t)k * k * ci * co, sizeof(float) * co);
    }
}

void to_host_order(const mpcnn_net* net, const float* dev_order, float* host)
{
    for (const Layer& ly : net->layers) {
        if (ly.kind == MPCNN_MP) continue;
        const int k = ly.k, ci = ly.cin, co = ly.cout;
        const float* src = dev_order + ly.p_off;
        float* dst = host + ly.p_off;
        for (int o = 0; o < co; ++o)
            for (int c = 0; c < ci; ++c)
                for (int t = 0; t < k * k; ++t)
                    dst[((size_t)o * ci + c) * k * k + t] = src[((size_t)t * ci + c) * co + o];
        memcpy(dst + (size_t)k * k * ci * co, src + (size_t)k * k * ci * co, sizeof(float) * co);
    }
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

}  // namespace

extern "C" {

const char* mpcnn_last_error(void) { return g_err; }

mpcnn_status mpcnn_net_create(const mpcnn_layer_desc* layers, int n_layers, int in_channels,
                              int patch, mpcnn_dtype dtype, mpcnn_net** out)
{
    if (!layers || !out) return fail(MPCNN_EINVAL, "null argument");
    *out = nullptr;
    if (n_layers < 1 || n_layers > 64 || in_channels < 1 || patch < 1)
        return fail(MPCNN_EINVAL, "n_layers=%d in_channels=%d patch=%d", n_layers, in_channels, patch);
    if (dtype != MPCNN_F32) {
        if (dtype == MPCNN_BF16) return fail(MPCNN_EUNSUPPORTED, "bf16 storage is not built yet");
        return fail(MPCNN_EINVAL, "unknown dtype %d", (int)dtype);
    }
    mpcnn_net* net = new (std::nothrow) mpcnn_net;
    if (!net) return fail(MPCNN_ENOMEM, "out of host memory");
    net->in_ch = in_channels; net->patch = patch;
    int side = patch, ch = in_channels, dil = 1;
    bool seen_fc = false;
    size_t off = 0;
    mpcnn_status st = MPCNN_OK;
    for (int l = 0; l < n_layers && st == MPCNN_OK; ++l) {
        const mpcnn_layer_desc& d = layers[l];
        Layer ly{};
        ly.kind = d.kind; ly.cin = ch; ly.dil = dil;
        if (d.kind == MPCNN_C) {
            if (d.maps < 1 || d.k < 1) st = fail(MPCNN_EINVAL, "layer %d: C needs maps >= 1, k >= 1", l);
            else if (seen_fc) st = fail(MPCNN_ESHAPE, "layer %d: C after FC", l);
            else if (side - d.k + 1 < 1) st = fail(MPCNN_ESHAPE, "layer %d: %dx%d filter on a %dx%d map", l, d.k, d.k, side, side);
            else { ly.k = d.k; ly.cout = d.maps; ly.tanh_out = true; side -= d.k - 1; }
        } else if (d.kind == MPCNN_MP) {
            if (d.k < 1) st = fail(MPCNN_EINVAL, "layer %d: MP needs k >= 1", l);
            else if (seen_fc) st = fail(MPCNN_ESHAPE, "layer %d: MP after FC", l);
            else if (side / d.k < 1) st = fail(MPCNN_ESHAPE, "layer %d: %dx%d pooling on a %dx%d map", l, d.k, d.k, side, side);
            else if (side % d.k != 0) st = fail(MPCNN_EUNSUPPORTED, "layer %d: map side %d is not a multiple of the pooling side %d", l, side, d.k);
            else if (d.k * d.k > 255) st = fail(MPCNN_EUNSUPPORTED, "layer %d: pooling window too large for byte tap codes", l);
            else { ly.k = d.k; ly.cout = ch; ly.tanh_out = false; side /= d.k; dil *= d.k; }
        } else if (d.kind == MPCNN_FC) {
            if (d.maps < 1) st = fail(MPCNN_EINVAL, "layer %d: FC needs maps >= 1", l);
            else { ly.k = seen_fc ? 1 : side; ly.cout = d.maps; ly.tanh_out = (l != n_layers - 1); side = 1; seen_fc = true; }
        } else st = fail(MPCNN_EINVAL, "layer %d: unknown kind %d", l, d.kind);
        if (st != MPCNN_OK) break;
        if (ly.kind != MPCNN_MP) {
            ly.p_off = off;
            ly.p_len = ((size_t)ly.k * ly.k * ly.cin + 1) * ly.cout;
            off += ly.p_len;
        }
        ch = ly.cout;
        net->layers.push_back(ly);
    }
    if (st == MPCNN_OK && layers[n_layers - 1].kind != MPCNN_FC)
        st = fail(MPCNN_ESHAPE, "the last layer must be FC");
    if (st == MPCNN_OK && ch > mpcnn::kMaxClasses)
        st = fail(MPCNN_EUNSUPPORTED, "%d classes, at most %d are built", ch, mpcnn::kMaxClasses);
    if (st != MPCNN_OK) { delete net; return st; }
    net->n_cls = ch; net->n_params = off;
    *out = net;
    return MPCNN_OK;
}

void mpcnn_net_destroy(mpcnn_net* net)
{
    if (!net) return;
    if (net->d_params || net->d_grads) {
        (void)hipSetDevice(net->device);
        (void)hipFree(net->d_params);
        (void)hipFree(net->d_grads);
    }
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
    Geom g;
    if (!make_geom(net, 1, H, W, false, &g)) return fail(MPCNN_ESHAPE, "image %dx%d smaller than the %d patch", H, W, net->patch);
    const Layer& ly = net->layers[layer];
    if (rows) *rows = g.rows[layer];
    if (cols) *cols = g.cols[layer];
    if (channels) *channels = ly.cout;
    if (spacing) *spacing = ly.kind == MPCNN_MP ? ly.dil * ly.k : ly.dil;
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
    }
    std::vector<float> tmp(n);
    to_device_order(net, params_host, tmp.data());
    HIP_TRY(hipSetDevice(net->device));
    HIP_TRY(hipDeviceSynchronize());
    HIP_TRY(hipMemcpy(net->d_params, tmp.data(), sizeof(float) * n, hipMemcpyHostToDevice));
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
    if (!net) return 0;
    Geom g;
    if (!make_geom(net, B, H, W, training != 0, &g)) return 0;
    return g.total;
}

static mpcnn_status check_call(mpcnn_net* net, const float* image, int B, int H, int W, void* ws,
                               size_t ws_bytes, bool training, Geom* g)
{
    if (!net || !image || !ws) return fail(MPCNN_EINVAL, "null argument");
    if (!net->d_params) return fail(MPCNN_EINVAL, "parameters were never set");
    if (B < 1) return fail(MPCNN_EINVAL, "B = %d", B);
    if (H < net->patch || W < net->patch)
        return fail(MPCNN_ESHAPE, "image %dx%d smaller than the %dx%d patch", H, W, net->patch, net->patch);
    if (!make_geom(net, B, H, W, training, g)) return fail(MPCNN_ESHAPE, "layer plan does not fit a %dx%d image", H, W);
    if (ws_bytes < g->total) return fail(MPCNN_EWORKSPACE, "workspace %zu bytes, need %zu", ws_bytes, g->total);
    if (((uintptr_t)ws & 255u) != 0) return fail(MPCNN_EINVAL, "workspace must be 256-byte aligned");
    return MPCNN_OK;
}

mpcnn_status mpcnn_seg_forward(mpcnn_net* net, const float* image_dev, int B, int H, int W,
                               float* probs_dev, void* ws_dev, size_t ws_bytes, void* hip_stream)
{
    Geom g;
    mpcnn_status st = check_call(net, image_dev, B, H, W, ws_dev, ws_bytes, false, &g);
    if (st != MPCNN_OK) return st;
    if (!probs_dev) return fail(MPCNN_EINVAL, "null probs_dev");
    st = run_forward(net, g, image_dev, (char*)ws_dev, nullptr, nullptr, probs_dev, nullptr, nullptr,
                     (hipStream_t)hip_stream);
    net->last = g; net->last_ws = ws_dev;
    return st;
}

mpcnn_status mpcnn_seg_backward(mpcnn_net* net, const float* image_dev, const int32_t* labels_dev,
                                const float* pixw_dev, int B, int H, int W, float* probs_dev,
                                double* loss_dev, void* ws_dev, size_t ws_bytes, void* hip_stream)
{
    Geom g;
    mpcnn_status st = check_call(net, image_dev, B, H, W, ws_dev, ws_bytes, true, &g);
    if (st != MPCNN_OK) return st;
    if (!labels_dev) return fail(MPCNN_EINVAL, "null labels_dev");
    hipStream_t stream = (hipStream_t)hip_stream;
    char* ws = (char*)ws_dev;
    float* dZ = (float*)(ws + g.delta_off[0]);
    st = run_forward(net, g, image_dev, ws, labels_dev, pixw_dev, probs_dev, dZ, loss_dev, stream);
    net->last = g; net->last_ws = ws_dev;
    if (st != MPCNN_OK) return st;
    return run_backward(net, g, image_dev, ws, stream);
}

mpcnn_status mpcnn_sgd_step(mpcnn_net* net, float lr, float grad_scale, void* hip_stream)
{
    if (!net) return fail(MPCNN_EINVAL, "null net");
    if (!net->d_params) return fail(MPCNN_EINVAL, "parameters were never set");
    long n = (long)net->n_params;
    mpcnn::sgd_kernel<<<(unsigned)((n + 255) / 256), 256, 0, (hipStream_t)hip_stream>>>(
        net->d_params, net->d_grads, lr * grad_scale, n);
    HIP_TRY(hipGetLastError());
    return MPCNN_OK;
}

mpcnn_status mpcnn_get_activation(const mpcnn_net* net, int layer, float* host, size_t n)
{
    if (!net || !host) return fail(MPCNN_EINVAL, "null argument");
    if (!net->last_ws || !net->last.training) return fail(MPCNN_EINVAL, "no backward call has been made");
    if (layer < 0 || layer >= (int)net->layers.size()) return fail(MPCNN_EINVAL, "layer %d out of range", layer);
    const Geom& g = net->last;
    size_t elems = (size_t)g.B * g.rows[layer] * g.cols[layer] * net->layers[layer].cout;
    if (n != elems) return fail(MPCNN_EINVAL, "n = %zu, layer holds %zu elements", n, elems);
    HIP_TRY(hipSetDevice(net->device));
    HIP_TRY(hipDeviceSynchronize());
    HIP_TRY(hipMemcpy(host, (char*)net->last_ws + g.act_off[layer], sizeof(float) * elems, hipMemcpyDeviceToHost));
    return MPCNN_OK;
}

mpcnn_status mpcnn_get_argmax(const mpcnn_net* net, int layer, uint8_t* host, size_t n)
{
    if (!net || !host) return fail(MPCNN_EINVAL, "null argument");
    if (!net->last_ws || !net->last.training) return fail(MPCNN_EINVAL, "no backward call has been made");
    if (layer < 0 || layer >= (int)net->layers.size() || net->layers[layer].kind != MPCNN_MP)
        return fail(MPCNN_EINVAL, "layer %d is not an MP layer", layer);
    const Geom& g = net->last;
    size_t elems = (size_t)g.B * g.rows[layer] * g.cols[layer] * net->layers[layer].cout;
    if (n != elems) return fail(MPCNN_EINVAL, "n = %zu, layer holds %zu elements", n, elems);
    HIP_TRY(hipSetDevice(net->device));
    HIP_TRY(hipDeviceSynchronize());
    HIP_TRY(hipMemcpy(host, (char*)net->last_ws + g.code_off[layer], elems, hipMemcpyDeviceToHost));
    return MPCNN_OK;
}

}  // extern "C"
