/*
 * mpcnn.h - C ABI of libmpcnn: whole-image forward / backward of a MaxPooling
 * Convolutional Network (MPCNN) for per-pixel classification on one MI355X.
 *
 * What the library computes (Masci, Giusti, Ciresan, Fricout, Schmidhuber,
 * "A Fast Learning Algorithm for Image Segmentation with Max-Pooling
 * Convolutional Networks"):  a net made of C / MP / FC layers (Background) is
 * defined on a P x P patch and labels the patch's centre pixel.  Instead of
 * running it on every patch, the whole image is pushed through once (Method,
 * "The MaxPoolingFragment (MPF) layer", Alg. 1 and 3) and the per-pixel errors
 * are pushed back once (Method, "Back-propagation through an MPF layer",
 * Alg. 2 and 4).  Outputs equal, up to floating-point rounding, what the patch
 * net gives on the patch around every pixel, and the parameter gradient equals
 * the sum over all patches.
 *
 * Conventions
 *   - "host" / "dev" in a parameter name says where the pointer must live.
 *     All device memory except parameters and gradients belongs to the caller.
 *   - Image layout [B][C0][H][W] fp32 (planar).  Output pixel (i,j) of image b is
 *     the patch whose top-left corner is (i,j); there are (H-P+1) x (W-P+1) of
 *     them.  Its label and loss weight are read at image pixel (i+c, j+c),
 *     c = (P-1)/2 rounded down.
 *   - Parameter vectors on the host are flat fp32, layer by layer
 *     W[o][c][u][v] then b[o]; MP layers have none.  The first FC layer sees the
 *     remaining q x q maps flattened [c][r][s], i.e. its W is [o][c][q][q];
 *     later FC layers have 1 x 1 kernels.  Filtering is correlation (no flip).
 *   - C layers and all FC layers but the last apply tanh; the last FC layer
 *     feeds a softmax; the loss is the cross-entropy SUMMED over pixels
 *     (Results: multi-class cross-entropy, each pixel on its own).
 *   - Every call returns a status; nothing throws or aborts.  After an error,
 *     outputs are unspecified but nothing is written out of bounds.
 *     mpcnn_last_error() gives the calling thread's last message.
 *   - Calls that take a stream only enqueue work on it (they do not wait).
 *     One net must not be used from two streams at once.
 */
#ifndef MPCNN_H
#define MPCNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct mpcnn_net mpcnn_net; /* opaque: layer plan, parameters, gradients */

typedef enum {
    MPCNN_OK = 0,
    MPCNN_EINVAL = 1,       /* null pointer, bad count, bad enum */
    MPCNN_ESHAPE = 2,       /* layer list does not fit the patch, or image smaller than the patch */
    MPCNN_EWORKSPACE = 3,   /* workspace smaller than mpcnn_workspace_bytes() */
    MPCNN_EUNSUPPORTED = 4, /* valid per the paper but not built (see each call) */
    MPCNN_EHIP = 5,         /* a HIP runtime call failed */
    MPCNN_ENOMEM = 6
} mpcnn_status;

typedef enum { MPCNN_C = 0, MPCNN_MP = 1, MPCNN_FC = 2 } mpcnn_kind;

/* Storage type of activations, deltas and (as read by the kernels) weights; all arithmetic,
 * sums, the softmax, the loss and the parameter gradients are fp32 or wider.  MPCNN_BF16:
 * every activation and delta tensor (the channels-last copy of the image included) is rounded
 * to bf16, nearest-even, when it is stored; the kernels read the parameters rounded to bf16
 * while the fp32 originals remain what mpcnn_sgd_step updates and mpcnn_get_params returns.
 * Images, labels, weights, probabilities and gradients cross the boundary in fp32 either way. */
typedef enum { MPCNN_F32 = 0, MPCNN_BF16 = 1 } mpcnn_dtype;

/* One layer (Background, layer kinds).  C: `maps` output maps, k x k filters.
 * MP: non-overlapping k x k max-pooling (maps ignored), or k rows x k2 columns ("p_row x p_col
 * sub-regions"); windows start at the top left of the map, rows / columns left over when a side
 * is not a multiple of the window's are dropped.  After a rectangular pool the maps of a patch
 * are no longer square and rows and columns of the whole-image maps are spaced differently; such
 * layers run on the plain (not the matrix-core) kernels.  FC: `maps` units
 * (k ignored); the last layer must be FC and its `maps` is the class count. */
typedef struct {
    int kind; /* mpcnn_kind */
    int maps;
    int k;
    int k2;   /* MP only: columns of the pooling window, 0 = k (square); k is then its rows */
} mpcnn_layer_desc;

/*
 * Build the layer plan for a net that sees a `patch` x `patch` window of an
 * image with `in_channels` channels.  Host-only: allocates no device memory
 * (parameters are allocated on the current device by mpcnn_set_params).
 * Errors: EINVAL (null / counts / kinds), ESHAPE (a layer does not fit; no FC
 * at the end; C or MP after an FC), EUNSUPPORTED (a pool with k*k > 255; more than 16 classes).
 * Every legal net is accepted with either storage type; layers whose shape the matrix-core and
 * fused kernels do not take (channel counts that are not multiples of 4, fewer than 8 channels,
 * class layers with more than 4 classes or 256 inputs) run on plain kernels; layers behind a
 * rectangular pool multiply on the fp32 matrix instruction with either storage type.
 */
mpcnn_status mpcnn_net_create(const mpcnn_layer_desc* layers_host, int n_layers, int in_channels,
                              int patch, mpcnn_dtype dtype, mpcnn_net** out);
void mpcnn_net_destroy(mpcnn_net* net); /* frees parameters and gradients; NULL is allowed */

int mpcnn_net_patch(const mpcnn_net* net);      /* P */
int mpcnn_net_classes(const mpcnn_net* net);    /* maps of the last FC */
size_t mpcnn_param_count(const mpcnn_net* net); /* length of the flat parameter vector */

/*
 * Shape of the whole-image ("dense") map that layer `layer` produces for an
 * H x W image: rows, columns, channels, and the spacing in image pixels
 * between elements that are neighbours inside one patch (the product of the
 * pooling factors so far; the MPF offsets of Alg. 3 are the residues modulo
 * this spacing; behind a rectangular pool it is the spacing of the rows, the
 * columns' being the product of the windows' column counts).  Host-only.
 */
mpcnn_status mpcnn_layer_shape(const mpcnn_net* net, int H, int W, int layer, int* rows, int* cols,
                               int* channels, int* spacing);

/* Diagnostic: which kernel, tiling and launch shape the library would use for every layer of a
 * call with these sizes (the tiling rule is the paper's fragment: a workgroup's tile is a
 * rectangle of one residue class of the whole-image map), as NUL-terminated text of at most
 * `cap` bytes in text_host (cut off if longer).  Host-only.  Errors: EINVAL, ESHAPE. */
mpcnn_status mpcnn_plan_describe(const mpcnn_net* net, int B, int H, int W, int training, char* text_host,
                                 size_t cap);

/* Copy the flat fp32 parameter vector from / to the host (synchronous).
 * n must equal mpcnn_param_count().  The first mpcnn_set_params allocates the
 * parameter and gradient buffers on the current device. */
mpcnn_status mpcnn_set_params(mpcnn_net* net, const float* params_host, size_t n);
mpcnn_status mpcnn_get_params(const mpcnn_net* net, float* params_host, size_t n);
/* Gradient of the summed loss left by the last mpcnn_seg_backward, same order
 * as the parameters (Alg. 2: the sum over all fragments / pixels). */
mpcnn_status mpcnn_get_grads(const mpcnn_net* net, float* grads_host, size_t n);

/* What follows the last FC layer.  MCCE (default): softmax, L = sum w * -log p[t]
 * (Results: multi-class cross-entropy, every pixel on its own).  MSE: linear outputs,
 * L = sum w * 1/2 * sum_o (x^[o] - [o == t])^2, whose derivative w.r.t. the output image
 * is x^ - t (Method, first step of back-propagation); `probs_dev` of the forward and
 * backward calls then receives the linear outputs.  EINVAL on an unknown kind. */
typedef enum { MPCNN_LOSS_MCCE = 0, MPCNN_LOSS_MSE = 1 } mpcnn_loss;
mpcnn_status mpcnn_set_loss(mpcnn_net* net, mpcnn_loss kind);

/* The squashing function of C and hidden FC layers (Background, layer C: "e.g. tanh or
 * logistic").  TANH (default), or LOGISTIC: y = 1 / (1 + exp(-a)), derivative y (1 - y).
 * Takes effect at the next forward / backward call.  EINVAL on an unknown kind. */
typedef enum { MPCNN_TANH = 0, MPCNN_LOGISTIC = 1 } mpcnn_activation;
mpcnn_status mpcnn_set_activation(mpcnn_net* net, mpcnn_activation kind);

/* Tuning knob for the matrix-core convolution kernel of fp32-arithmetic layers (forward and
 * data gradient; Method, forward and backward of layer C): a workgroup computes 32 *
 * position_tiles positions of one residue class (16 * position_tiles where a layer's 16 or fewer
 * outputs put it on 16-wide tiles) and each of its waves owns tiles_per_wave of them for one
 * channel tile.  0 leaves either choice to the library's
 * planner (the default), which weighs matrix-instruction time against staging per layer and
 * image size.  A pair that no kernel instance serves for a layer's channel count (the waves of
 * a workgroup, channel tiles * position_tiles / tiles_per_wave, must be 4 or 8) leaves that
 * layer on the planner's fallback kernel.  Results do not depend on the tiling: every output
 * element is the same sum in the same order.  Takes effect at the next forward / backward
 * call.  EINVAL unless position_tiles is 0, 2, 4, 8 or 16 and tiles_per_wave 0, 1, 2 or 4. */
mpcnn_status mpcnn_set_conv_tiling(mpcnn_net* net, int position_tiles, int tiles_per_wave);

/* Per-class balanced pixel weights (Experiments, steel defects: the loss is minimised per
 * class because the data set is unbalanced):  pixw_dev[b][y][x] = 1 / N_k where the pixel is
 * the centre of a patch (an output pixel) with label k in [0, n_classes), N_k = number of
 * such pixels in the batch; 0 everywhere else.  Passed as pixw_dev to mpcnn_seg_backward it
 * makes L the sum over classes of each class's mean loss.
 *   labels_dev [B][H][W] int32, pixw_dev [B][H][W] fp32 (written),
 *   counts_dev: 64 bytes of device scratch (the N_k, 16 uint32, left there).
 * Errors: EINVAL, ESHAPE (H or W < P), EHIP. */
mpcnn_status mpcnn_class_balance_weights(const mpcnn_net* net, const int32_t* labels_dev, int B, int H,
                                         int W, float* pixw_dev, void* counts_dev, void* hip_stream);

/* Bytes of caller-owned device workspace a call with these sizes needs
 * (training != 0: mpcnn_seg_backward; 0: mpcnn_seg_forward).  0 on bad input. */
size_t mpcnn_workspace_bytes(const mpcnn_net* net, int B, int H, int W, int training);

/*
 * Whole-image forward (Alg. 1 / Alg. 3 over all layers):
 *   image_dev [B][C0][H][W] fp32  ->  probs_dev [B][n_classes][H-P+1][W-P+1] fp32,
 * the softmax output of the patch net for every pixel.  ws_dev: 256-byte
 * aligned scratch of at least mpcnn_workspace_bytes(net,B,H,W,0).
 * Errors: EINVAL, ESHAPE (H or W < P), EWORKSPACE, EHIP.
 */
mpcnn_status mpcnn_seg_forward(mpcnn_net* net, const float* image_dev, int B, int H, int W,
                               float* probs_dev, void* ws_dev, size_t ws_bytes, void* hip_stream);

/*
 * mpcnn_seg_forward for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  The caller passes the image
 * and the output only; the workspace is a fixed array of MPCNN_STATIC_WORKSPACE_BYTES inside the
 * library's device image (each GPU the library runs on holds its own copy until the process
 * ends; its address on the net's device is looked up when mpcnn_set_params first touches that
 * device).  The call allocates nothing and frees nothing, on the device or through the HIP
 * runtime; per-launch timing (mpcnn_profile_enable) is off during it.  Results are those of
 * mpcnn_seg_forward, bit for bit.
 *   - The net's device must be the current device.
 *   - Sizes with mpcnn_workspace_bytes(net, B, H, W, 0) > MPCNN_STATIC_WORKSPACE_BYTES are
 *     refused with MPCNN_EWORKSPACE (the message names both figures).
 *   - All calls on one GPU share that GPU's array (every net, every stream): calls that overlap
 *     in time race.  Nothing in it has to start at zero: each call writes what it reads.
 * Errors: EINVAL (null pointer, parameters never set, another device current), ESHAPE,
 * EWORKSPACE, EHIP.
 */
#define MPCNN_STATIC_WORKSPACE_BYTES (64u * 1024u * 1024u)
mpcnn_status mpcnn_seg_forward_static(mpcnn_net* net, const float* image_dev, int B, int H, int W,
                                      float* probs_dev, void* hip_stream);

/*
 * Deployment forward that keeps the image size (Experiments, membrane segmentation:
 * pixels outside the boundary of a test image are synthesised by mirroring, which
 * preserves the size of the output):
 *   image_dev [B][C0][H][W] fp32  ->  probs_dev [B][n_classes][H][W] fp32,
 * output pixel (i,j) being the patch centred on input pixel (i,j) (c = (P-1)/2
 * rounded down rows / columns above and to the left of it, P-1-c below and to the
 * right).  The mirror repeats the edge pixel: index -1-i stands for i < 0 and
 * 2n-1-i for i >= n.  Nothing is kept for a backward.  ws_dev: 256-byte aligned
 * scratch of at least mpcnn_workspace_bytes_same(net,B,H,W) (0 on bad input).
 * Errors: EINVAL, ESHAPE (H or W smaller than the widest border, P-1-c), EWORKSPACE, EHIP.
 */
size_t mpcnn_workspace_bytes_same(const mpcnn_net* net, int B, int H, int W);
mpcnn_status mpcnn_seg_forward_same(mpcnn_net* net, const float* image_dev, int B, int H, int W,
                                    float* probs_dev, void* ws_dev, size_t ws_bytes, void* hip_stream);

/*
 * Whole-image forward + backward (Alg. 1-4): computes the loss
 *   L = sum over b,i,j of w * -log p[b, t, i, j],  t = labels[b][i+c][j+c],
 *   w = pixw[b][i+c][j+c] (1 if pixw_dev is NULL); pixels with t < 0 or
 *   t >= n_classes add nothing;
 * and leaves dL/dW, dL/db of every layer in the net (read with mpcnn_get_grads,
 * consumed by mpcnn_sgd_step).
 *   labels_dev [B][H][W] int32, pixw_dev [B][H][W] fp32 or NULL,
 *   probs_dev  as in mpcnn_seg_forward, or NULL,
 *   loss_dev   one fp64 on the device, or NULL,
 *   ws_dev     at least mpcnn_workspace_bytes(net,B,H,W,1); it holds every
 *              layer's activations and argmax maps until the next call.
 * The result does not depend on launch timing: no floating-point atomics are
 * used, reductions have a fixed order.
 */
mpcnn_status mpcnn_seg_backward(mpcnn_net* net, const float* image_dev, const int32_t* labels_dev,
                                const float* pixw_dev, int B, int H, int W, float* probs_dev,
                                double* loss_dev, void* ws_dev, size_t ws_bytes, void* hip_stream);

/*
 * The same pass with the image taken in bands of `band_rows` output rows (the last band may be
 * shorter): an output pixel depends on its own patch only (Method: every pixel is the output of
 * the net on the patch around it), so a band of r output rows needs r + P - 1 image rows and
 * nothing else; gradients and loss are summed over the bands, in order.  For images whose
 * activations do not fit in memory at once: the workspace is that of one band,
 * mpcnn_workspace_bytes_banded(net, B, W, band_rows), which is enough for every shorter band
 * as well (the size never shrinks when band_rows grows).  Arguments and results as
 * mpcnn_seg_backward (probs_dev, if given, receives all H-P+1 rows); the test hooks afterwards
 * see the last band only.  Errors as mpcnn_seg_backward; EINVAL for band_rows < 1.
 */
size_t mpcnn_workspace_bytes_banded(const mpcnn_net* net, int B, int W, int band_rows);
mpcnn_status mpcnn_seg_backward_banded(mpcnn_net* net, const float* image_dev, const int32_t* labels_dev,
                                       const float* pixw_dev, int B, int H, int W, int band_rows,
                                       float* probs_dev, double* loss_dev, void* ws_dev, size_t ws_bytes,
                                       void* hip_stream);

/* Plain gradient step on every parameter: theta -= lr * grad_scale * g
 * (Results, "Membrane Segmentation": weights updated after every image). */
mpcnn_status mpcnn_sgd_step(mpcnn_net* net, float lr, float grad_scale, void* hip_stream);

/*
 * The loss alone, L as in mpcnn_seg_backward for the current parameters: a forward pass that
 * keeps nothing and computes no gradient (the evaluations of a line search).
 *   loss_dev: one fp64 on the device.  ws_dev: at least mpcnn_workspace_bytes(net,B,H,W,0).
 */
mpcnn_status mpcnn_seg_loss(mpcnn_net* net, const float* image_dev, const int32_t* labels_dev,
                            const float* pixw_dev, int B, int H, int W, double* loss_dev,
                            void* ws_dev, size_t ws_bytes, void* hip_stream);

/*
 * One gradient step safeguarded by the Armijo rule (Experiments, membrane segmentation:
 * stochastic gradient descent safeguarded by the Armijo rule, the weights updated after every
 * image).  To be called after mpcnn_seg_backward on the same inputs, whose gradient g the net
 * holds and whose loss the caller passes as f0.  Tries alpha = alpha0, beta*alpha0, ... (at most
 * max_trials values) and keeps the first for which
 *     L(theta - alpha*grad_scale*g) <= f0 - c * alpha * grad_scale * |g|^2 ;
 * each trial costs one loss-only forward.  If none passes the parameters are left as they were
 * and *alpha_host = 0.  Synchronous on hip_stream (every trial's loss is read back).
 *   alpha_host, loss_host, trials_host: results on the host (accepted alpha, loss at the new
 *   parameters, trials made); any may be NULL.  ws_dev as for mpcnn_seg_loss.
 * Errors: EINVAL (also: alpha0 <= 0, beta outside (0,1), c outside [0,1), max_trials < 1), ESHAPE,
 * EWORKSPACE, EHIP.
 */
mpcnn_status mpcnn_armijo_step(mpcnn_net* net, const float* image_dev, const int32_t* labels_dev,
                               const float* pixw_dev, int B, int H, int W, double f0, float alpha0,
                               float grad_scale, float c, float beta, int max_trials, void* ws_dev,
                               size_t ws_bytes, void* hip_stream, float* alpha_host, double* loss_host,
                               int* trials_host);

/*
 * One iteration of limited-memory BFGS with a back-tracking line search (Results, the steel
 * data set: LBFGS is the optimiser used there; the paper gives no details, so this is the
 * method's standard form).  To be called after mpcnn_seg_backward on the same inputs, whose
 * gradient g the net holds and whose loss the caller passes as f0; the objective is the summed
 * loss of that batch.
 *   1. If the call before this one accepted a step: s = theta - theta_prev, y = g - g_prev; the
 *      pair is stored (the oldest dropped beyond `history`, 1..64) iff s.y > 1e-10 |s| |y|.
 *   2. p = -H g by the two-loop recursion over the stored pairs, H_0 = (s.y / y.y) I of the
 *      newest pair (p = -g without pairs); if g.p >= 0 the pairs are dropped and p = -g.
 *   3. alpha = alpha0, beta*alpha0, ... (at most max_trials values): the first with
 *      L(theta + alpha p) <= f0 + c alpha g.p is accepted; each trial costs one loss-only forward.
 *   4. If none passes the parameters are left as they were, *alpha_host = 0, and the history is
 *      dropped.
 * Dot products are fp64 sums in a fixed order, the pairs and the direction are fp32 vectors
 * (2 (history + 1) + 3 parameter-sized device buffers, allocated at the first call; changing
 * `history` starts afresh).  mpcnn_set_params and mpcnn_lbfgs_reset drop the history.
 * Synchronous on hip_stream.
 *   alpha_host, loss_host, trials_host, pairs_host: results on the host (accepted alpha, loss at
 *   the new parameters, trials made, pairs the direction used); any may be NULL.  ws_dev as for
 *   mpcnn_seg_loss.
 * Errors: EINVAL (also: alpha0 <= 0, beta outside (0,1), c outside [0,1), max_trials < 1,
 * history outside 1..64), ESHAPE, EWORKSPACE, EHIP.
 */
mpcnn_status mpcnn_lbfgs_step(mpcnn_net* net, const float* image_dev, const int32_t* labels_dev,
                              const float* pixw_dev, int B, int H, int W, double f0, int history,
                              float alpha0, float c, float beta, int max_trials, void* ws_dev,
                              size_t ws_bytes, void* hip_stream, float* alpha_host, double* loss_host,
                              int* trials_host, int* pairs_host);
mpcnn_status mpcnn_lbfgs_reset(mpcnn_net* net);

/*
 * Test hooks: read back what the last forward/backward left in the workspace
 * (which must still be alive).  Synchronous.
 *   mpcnn_get_activation: output of layer `layer`, [B][rows][cols][channels] fp32.
 *   mpcnn_get_argmax:     for MP layer `layer`, the tap code u*k+v of the first
 *                         maximum in row-major (u,v) order of every pooled
 *                         element (the mpIDXS of Alg. 3), [B][rows][cols][channels].
 * n = number of elements the host buffer holds; must match.
 */
mpcnn_status mpcnn_get_activation(const mpcnn_net* net, int layer, float* host, size_t n);
mpcnn_status mpcnn_get_argmax(const mpcnn_net* net, int layer, uint8_t* host, size_t n);

/*
 * Per-kernel timing for the bench.  While enabled, every kernel launch of
 * mpcnn_seg_forward / mpcnn_seg_backward / mpcnn_sgd_step is bracketed by HIP
 * events recorded on the call's stream.  mpcnn_profile_read waits for them and
 * returns one record per launch site (kernel x layer), summed since the last
 * read: kernel name (ending in _mfma: fp32 matrix instruction, _bm: bf16 matrix
 * instruction), layer index, step of the path (1 = conv fwd, 2 = max filter,
 * 3 = class layer + softmax-CE, 4 = class layer backward, 5 = wgrad, 6 = dgrad,
 * 7 = routing, 8 = SGD, 0 = staging / reductions), launches, total milliseconds,
 * and the ALGORITHMIC work of one launch: flops = 2*M*N*K of the contraction
 * with the real N and K, bytes = each tensor the step must read or write
 * counted once.  Writes at most `cap` records, *n = number of sites.
 */
typedef struct {
    char name[48];
    int layer;
    int step;
    int launches;
    double ms_total;
    double flops;
    double bytes;
} mpcnn_kernel_stat;

mpcnn_status mpcnn_profile_enable(mpcnn_net* net, int on);
mpcnn_status mpcnn_profile_read(mpcnn_net* net, mpcnn_kernel_stat* out_host, int cap, int* n);

const char* mpcnn_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* MPCNN_H */
