/*
 * mpcnn_oracle.c - patch-by-patch MaxPooling-CNN forward / backward in fp64.
 *
 * TEST INFRASTRUCTURE ONLY.  This is the slow, plain definition that the fast
 * whole-image path is checked against: the network is evaluated, and
 * back-propagated, separately on the patch that belongs to every output pixel
 * (Background, "Image Segmentation with MPCNN": evaluate the net on every
 * patch), and the parameter gradient is the plain sum over patches.  Only the
 * tests, the smoke check and the bench's cpu_baseline leg may call it; it
 * shares no code with the HIP library and includes none of its headers.
 *
 * Layer definitions (Background, layers C / MP / FC):
 *   C   y[o][r][s] = tanh(b[o] + sum_{c,u,v} W[o][c][u][v] * x[c][r+u][s+v])
 *       valid, stride 1, no kernel flip, every input map feeds every output map
 *   MP  y[c][r][s] = max_{u<p_row, v<p_col} x[c][p_row*r+u][p_col*s+v], non-overlapping
 *       p_row x p_col windows (square unless the description says otherwise),
 *       trailing rows/columns that do not fill a window are dropped; the
 *       recorded argmax is the FIRST maximum met in (u,v) row-major order,
 *       coded u*p_col + v
 *   FC  the first FC sees the remaining maps flattened [c][r][s] row-major,
 *       i.e. it is a C layer whose kernel covers the whole map; later FCs are
 *       matrix * vector.  Hidden FCs apply tanh; the last FC feeds a softmax.
 *   The squashing function of C and hidden FC layers is tanh or, on request, the logistic
 *   function 1 / (1 + exp(-a)) (Background, layer C: "e.g. tanh or logistic").
 * Loss (Results, first paragraph): multi-class cross-entropy, each pixel on its
 * own, here summed over pixels: L = sum_pix w_pix * -log p_pix[t_pix].
 * Alternative (Method, before the MPF back-propagation): mean squared error with
 * linear outputs, whose derivative w.r.t. the output image is x^ - t; here
 * L = sum_pix w_pix * 1/2 * sum_o (x^_pix[o] - [o == t_pix])^2, the outputs being the
 * last FC's values without the softmax.
 * Back-propagation is the textbook one the paper defers to (Background, end).
 *
 * Pins: see tests/test_oracle_pins.py (autograd in fp64 on single patches,
 * central finite differences, scipy correlate2d, hand-worked pooling cases,
 * softmax closed forms).  No function here is "parity unpinned".
 *
 * Parameter order: layer by layer, W[o][c][u][v] then b[o]; MP has none.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_MAXL 32
enum { ORC_C = 0, ORC_MP = 1, ORC_FC = 2 };
enum { ORC_LOSS_MCCE = 0, ORC_LOSS_MSE = 1 };
enum { ORC_ACT_TANH = 0, ORC_ACT_LOGISTIC = 1 };

typedef struct {
    int n_layers, in_ch, patch, n_classes;
    int kind[ORC_MAXL];
    int kr[ORC_MAXL], kc[ORC_MAXL];           /* kernel rows x columns (C: k x k, first FC: the map) or p_row x p_col (MP) */
    int ch_in[ORC_MAXL], ch_out[ORC_MAXL];
    int rows_in[ORC_MAXL], cols_in[ORC_MAXL]; /* maps are square until a rectangular pool */
    int rows_out[ORC_MAXL], cols_out[ORC_MAXL];
    int stride_r[ORC_MAXL], stride_c[ORC_MAXL]; /* image pixels between neighbours of layer l's output */
    int reach_r[ORC_MAXL], reach_c[ORC_MAXL];   /* (rows_out-1)*stride_r, (cols_out-1)*stride_c: for dense maps */
    int tanh_after[ORC_MAXL];
    long w_off[ORC_MAXL], b_off[ORC_MAXL];
    long act_off[ORC_MAXL + 1];               /* act 0 = the patch itself, act l+1 = output of layer l */
    long idx_off[ORC_MAXL];
    long act_total, idx_total, n_params;
    int loss_kind;                            /* ORC_LOSS_*: what follows the last FC */
    int act_kind;                             /* ORC_ACT_*: the squashing function of C and hidden FC layers */
} orc_plan;

/* Shape inference.  Returns 0, or a negative code naming the first problem. */
static int orc_make_plan(orc_plan *pl, const int *kinds, const int *maps, const int *ks,
                         const int *ks2, int n_layers, int in_ch, int patch)
{
    if (n_layers < 1 || n_layers > ORC_MAXL || in_ch < 1 || patch < 1) return -1;
    memset(pl, 0, sizeof *pl);
    pl->n_layers = n_layers; pl->in_ch = in_ch; pl->patch = patch;
    int rows = patch, cols = patch, ch = in_ch, sr = 1, sc = 1, seen_fc = 0;
    long act = (long)in_ch * patch * patch, idx = 0, par = 0;
    pl->act_off[0] = 0;
    for (int l = 0; l < n_layers; ++l) {
        pl->kind[l] = kinds[l]; pl->ch_in[l] = ch; pl->rows_in[l] = rows; pl->cols_in[l] = cols;
        if (kinds[l] == ORC_C) {
            if (seen_fc || ks[l] < 1 || maps[l] < 1 || rows - ks[l] + 1 < 1 || cols - ks[l] + 1 < 1) return -2;
            pl->kr[l] = pl->kc[l] = ks[l]; pl->ch_out[l] = maps[l];
            pl->rows_out[l] = rows - ks[l] + 1; pl->cols_out[l] = cols - ks[l] + 1;
            pl->tanh_after[l] = 1;
        } else if (kinds[l] == ORC_MP) {
            /* p_row x p_col sub-regions (Background, layer MP); ks2 = 0 or absent: square */
            const int pr = ks[l], pc = (ks2 && ks2[l] > 0) ? ks2[l] : ks[l];
            if (seen_fc || pr < 1 || pc < 1 || rows / pr < 1 || cols / pc < 1 || pr * pc > 255) return -3;
            pl->kr[l] = pr; pl->kc[l] = pc; pl->ch_out[l] = ch;
            pl->rows_out[l] = rows / pr; pl->cols_out[l] = cols / pc;
            sr *= pr; sc *= pc;
        } else if (kinds[l] == ORC_FC) {
            if (maps[l] < 1) return -4;
            pl->kr[l] = seen_fc ? 1 : rows; pl->kc[l] = seen_fc ? 1 : cols;
            pl->ch_out[l] = maps[l]; pl->rows_out[l] = pl->cols_out[l] = 1;
            pl->tanh_after[l] = (l != n_layers - 1);
            seen_fc = 1;
        } else return -5;
        pl->stride_r[l] = sr; pl->stride_c[l] = sc;
        if (kinds[l] != ORC_MP) {
            pl->w_off[l] = par; par += (long)pl->ch_out[l] * ch * pl->kr[l] * pl->kc[l];
            pl->b_off[l] = par; par += pl->ch_out[l];
        } else {
            pl->idx_off[l] = idx; idx += (long)pl->ch_out[l] * pl->rows_out[l] * pl->cols_out[l];
        }
        rows = pl->rows_out[l]; cols = pl->cols_out[l]; ch = pl->ch_out[l];
        pl->reach_r[l] = (rows - 1) * sr; pl->reach_c[l] = (cols - 1) * sc;
        pl->act_off[l + 1] = act; act += (long)ch * rows * cols;
    }
    if (kinds[n_layers - 1] != ORC_FC) return -6;
    pl->n_classes = ch; pl->act_total = act; pl->idx_total = idx; pl->n_params = par;
    return 0;
}

/*
 * Near-ties.  The argmax of a pooling window is an integer decided by floating
 * point; a path that computes the same map in another precision can rank two
 * candidates closer than its rounding error the other way round, and both
 * rankings are then valid sub-gradients of the max.  So that such a result can
 * be checked exactly, the oracle can (a) report every window whose two largest
 * values are within `tau` of each other, with the tap it chose and the
 * runner-up tap, and (b) re-run with a list `alt` of (window, tap) pairs: in a
 * listed window the named tap receives the back-propagated value instead,
 * PROVIDED its value is within `tau` of the window's maximum (with coarse
 * storage more than two taps can be that close); a pair that names a tap
 * further away is counted in *rejected and ignored.  The forward value stays
 * the true maximum.  A window is named by its position in the whole-image map
 * of that MP layer: key = layer * 2^48 + ((b*C + c)*ny + y)*nx + x.
 * With tau = 0 and no list this is the plain first-maximum rule.
 */
typedef struct {
    double tau;
    const int64_t *alt; const uint8_t *alt_tap; long n_alt;   /* sorted keys and their taps */
    int64_t *amb; long amb_cap; long *amb_n; /* records of 4: key, chosen tap, runner-up tap, layer */
    long *rejected;                          /* listed pairs whose tap is not within tau of the maximum */
    int B, H, W;                             /* image batch and size, for the keys */
} orc_ties;

static long orc_key_listed(const orc_ties *t, int64_t key)   /* index in alt, or -1 */
{
    long lo = 0, hi = t->n_alt - 1;
    while (lo <= hi) {
        long mid = (lo + hi) / 2;
        if (t->alt[mid] == key) return mid;
        if (t->alt[mid] < key) lo = mid + 1; else hi = mid - 1;
    }
    return -1;
}

/* Forward of ONE patch.  act: all layer outputs; idx: argmax codes u*p+v of
 * every pooled element; gap (optional): largest minus second largest value of
 * every pooling window (0 on an exact tie).  probs: softmax of the last FC.
 * ties (optional) with the patch's image index b and corner (pi,pj): see above. */
static void orc_patch_forward(const orc_plan *pl, const double *par, double *act,
                              uint8_t *idx, double *gap, double *probs,
                              const orc_ties *ties, int pb, int pi, int pj)
{
    for (int l = 0; l < pl->n_layers; ++l) {
        const double *x = act + pl->act_off[l];
        double *y = act + pl->act_off[l + 1];
        const int nr = pl->rows_in[l], nc = pl->cols_in[l], mr = pl->rows_out[l], mc = pl->cols_out[l];
        const int kr = pl->kr[l], kc = pl->kc[l];
        const int ci = pl->ch_in[l], co = pl->ch_out[l];
        if (pl->kind[l] == ORC_MP) {
            for (int c = 0; c < co; ++c)
                for (int r = 0; r < mr; ++r)
                    for (int s = 0; s < mc; ++s) {
                        double best = 0, second = 0; int code = -1, code2 = -1;
                        for (int u = 0; u < kr; ++u)
                            for (int v = 0; v < kc; ++v) {
                                double a = x[((long)c * nr + (kr * r + u)) * nc + (kc * s + v)];
                                if (code < 0) { best = a; code = 0; second = -INFINITY; }
                                else if (a > best) { second = best; code2 = code; best = a; code = u * kc + v; }
                                else if (a > second) { second = a; code2 = u * kc + v; }
                            }
                        long e = ((long)c * mr + r) * mc + s;
                        y[e] = best;
                        if (ties && code2 >= 0 && (best - second <= ties->tau || ties->n_alt > 0)) {
                            const int str = pl->stride_r[l], stc = pl->stride_c[l];
                            const long ny = ties->H - pl->patch + pl->reach_r[l] + 1;
                            const long nx = ties->W - pl->patch + pl->reach_c[l] + 1;
                            int64_t key = ((int64_t)l << 48) +
                                          (((int64_t)pb * co + c) * ny + (pi + r * str)) * nx + (pj + s * stc);
                            if (ties->amb && best - second <= ties->tau) {
#pragma omp critical(orc_amb)
                                {
                                    long q = (*ties->amb_n)++;
                                    if (q < ties->amb_cap) {
                                        ties->amb[4 * q] = key; ties->amb[4 * q + 1] = code;
                                        ties->amb[4 * q + 2] = code2; ties->amb[4 * q + 3] = l;
                                    }
                                }
                            }
                            const long at = ties->n_alt > 0 ? orc_key_listed(ties, key) : -1;
                            if (at >= 0) {
                                const int tap = ties->alt_tap[at];
                                const int tu = tap / kc, tv = tap % kc;
                                if (tap < kr * kc &&
                                    best - x[((long)c * nr + (kr * r + tu)) * nc + (kc * s + tv)] <= ties->tau)
                                    code = tap;
                                else {
#pragma omp atomic
                                    (*ties->rejected)++;
                                }
                            }
                        }
                        idx[pl->idx_off[l] + e] = (uint8_t)code;
                        if (gap) gap[pl->idx_off[l] + e] = (kr * kc > 1) ? best - second : INFINITY;
                    }
        } else {
            const double *W = par + pl->w_off[l], *b = par + pl->b_off[l];
            for (int o = 0; o < co; ++o)
                for (int r = 0; r < mr; ++r)
                    for (int s = 0; s < mc; ++s) {
                        double acc = b[o];
                        for (int c = 0; c < ci; ++c)
                            for (int u = 0; u < kr; ++u)
                                for (int v = 0; v < kc; ++v)
                                    acc += W[(((long)o * ci + c) * kr + u) * kc + v] *
                                           x[((long)c * nr + (r + u)) * nc + (s + v)];
                        y[((long)o * mr + r) * mc + s] = !pl->tanh_after[l] ? acc
                            : pl->act_kind == ORC_ACT_LOGISTIC ? 1.0 / (1.0 + exp(-acc)) : tanh(acc);
                    }
        }
    }
    const double *z = act + pl->act_off[pl->n_layers];
    if (pl->loss_kind == ORC_LOSS_MSE) {   /* linear outputs */
        for (int o = 0; o < pl->n_classes; ++o) probs[o] = z[o];
        return;
    }
    double zmax = z[0], sum = 0;
    for (int o = 1; o < pl->n_classes; ++o) if (z[o] > zmax) zmax = z[o];
    for (int o = 0; o < pl->n_classes; ++o) { probs[o] = exp(z[o] - zmax); sum += probs[o]; }
    for (int o = 0; o < pl->n_classes; ++o) probs[o] /= sum;
}

/* Backward of ONE patch: adds this patch's dL/dparams into g.  dlt has the
 * layout of act; on return dlt[act 0] holds dL/d(patch) if want_dx. */
static void orc_patch_backward(const orc_plan *pl, const double *par, const double *act,
                               const uint8_t *idx, const double *probs, int label, double w,
                               double *dlt, double *g, int want_dx)
{
    const int L = pl->n_layers;
    double *dz = dlt + pl->act_off[L];
    for (int o = 0; o < pl->n_classes; ++o) dz[o] = w * (probs[o] - (o == label ? 1.0 : 0.0));
    for (int l = L - 1; l >= 0; --l) {
        const double *x = act + pl->act_off[l];
        const double *y = act + pl->act_off[l + 1];
        double *dy = dlt + pl->act_off[l + 1];
        double *dx = dlt + pl->act_off[l];
        const int nr = pl->rows_in[l], nc = pl->cols_in[l], mr = pl->rows_out[l], mc = pl->cols_out[l];
        const int kr = pl->kr[l], kc = pl->kc[l];
        const int ci = pl->ch_in[l], co = pl->ch_out[l];
        const int need_dx = (l > 0) || want_dx;
        if (need_dx) memset(dx, 0, sizeof(double) * (size_t)ci * nr * nc);
        if (pl->kind[l] == ORC_MP) {
            if (!need_dx) continue;
            for (int c = 0; c < co; ++c)
                for (int r = 0; r < mr; ++r)
                    for (int s = 0; s < mc; ++s) {
                        long e = ((long)c * mr + r) * mc + s;
                        int code = idx[pl->idx_off[l] + e];
                        int u = code / kc, v = code % kc;
                        dx[((long)c * nr + (kr * r + u)) * nc + (kc * s + v)] += dy[e];
                    }
        } else {
            const double *W = par + pl->w_off[l];
            double *gW = g + pl->w_off[l], *gb = g + pl->b_off[l];
            for (int o = 0; o < co; ++o)
                for (int r = 0; r < mr; ++r)
                    for (int s = 0; s < mc; ++s) {
                        long e = ((long)o * mr + r) * mc + s;
                        double d = dy[e];
                        if (pl->tanh_after[l])   /* derivative of the squashing function, from its output */
                            d *= pl->act_kind == ORC_ACT_LOGISTIC ? y[e] * (1.0 - y[e]) : 1.0 - y[e] * y[e];
                        gb[o] += d;
                        for (int c = 0; c < ci; ++c)
                            for (int u = 0; u < kr; ++u)
                                for (int v = 0; v < kc; ++v) {
                                    long wi = (((long)o * ci + c) * kr + u) * kc + v;
                                    long xi = ((long)c * nr + (r + u)) * nc + (s + v);
                                    gW[wi] += d * x[xi];
                                    if (need_dx) dx[xi] += W[wi] * d;
                                }
                    }
        }
    }
}

static void orc_crop(const orc_plan *pl, const double *image, int H, int W, int b, int i, int j,
                     double *dst)
{
    const int P = pl->patch;
    for (int c = 0; c < pl->in_ch; ++c)
        for (int r = 0; r < P; ++r)
            memcpy(dst + ((long)c * P + r) * P,
                   image + (((long)b * pl->in_ch + c) * H + (i + r)) * W + j, sizeof(double) * P);
}

/* ------------------------------------------------------------------ C ABI */

long orc_param_count(const int *kinds, const int *maps, const int *ks, const int *ks2, int n_layers,
                     int in_ch, int patch)
{
    orc_plan pl;
    int rc = orc_make_plan(&pl, kinds, maps, ks, ks2, n_layers, in_ch, patch);
    return rc < 0 ? rc : pl.n_params;
}

int orc_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Evaluate (and, if grads != NULL, back-propagate) the net on the patch of
 * every selected output pixel.
 *   image   [B][in_ch][H][W]
 *   labels  [B][H][W] or NULL (forward only); label < 0: pixel contributes no loss
 *   pixw    [B][H][W] per-pixel loss weight, or NULL = 1
 *   sel     n_sel flat indices into [B][H-P+1][W-P+1], or NULL = every pixel
 *   probs   sel==NULL: [B][n_cls][Ho][Wo]; else [n_sel][n_cls]   (may be NULL)
 *   loss    scalar sum (may be NULL)
 *   grads   [n_params] sum over patches (may be NULL)
 *   dimage  [B][in_ch][H][W] dL/d(image), sum over patches (may be NULL; small inputs)
 * Output pixel (i,j) is the patch with top-left corner (i,j); its label and
 * weight are read at image pixel (i+c, j+c), c = (P-1)/2 rounded down.
 *   tie_tau, alt + alt_tap, amb, rejected: near-tie reporting / alternative routing (see
 *   orc_ties); amb receives up to amb_cap records of 4 int64, *amb_n the number met, and
 *   *rejected the number of refused pairs (a window is met once per patch that contains it).
 *   loss_kind  ORC_LOSS_MCCE: probs = softmax; ORC_LOSS_MSE: probs = the linear outputs.
 *   (the delta at the outputs is w * (probs - onehot) in both cases)
 */
int orc_run(const int *kinds, const int *maps, const int *ks, const int *ks2, int n_layers, int in_ch, int patch,
            const double *params, const double *image, int B, int H, int W,
            const int32_t *labels, const double *pixw, const int64_t *sel, long n_sel,
            double *probs, double *loss, double *grads, double *dimage,
            double tie_tau, const int64_t *alt, const uint8_t *alt_tap, long n_alt,
            int64_t *amb, long amb_cap, long *amb_n, long *rejected, int loss_kind, int act_kind)
{
    orc_plan pl;
    int rc = orc_make_plan(&pl, kinds, maps, ks, ks2, n_layers, in_ch, patch);
    if (rc < 0) return rc;
    if (loss_kind != ORC_LOSS_MCCE && loss_kind != ORC_LOSS_MSE) return -12;
    if (act_kind != ORC_ACT_TANH && act_kind != ORC_ACT_LOGISTIC) return -13;
    pl.loss_kind = loss_kind; pl.act_kind = act_kind;
    const int P = patch, Ho = H - P + 1, Wo = W - P + 1, ctr = (P - 1) / 2, nc = pl.n_classes;
    if (Ho < 1 || Wo < 1 || B < 1) return -10;
    if ((grads || loss) && !labels) return -11;
    const long n_pix = sel ? n_sel : (long)B * Ho * Wo;
    const long n_img = (long)B * in_ch * H * W;
    int nt = orc_threads();
    double *g_all = grads ? calloc((size_t)nt * pl.n_params, sizeof(double)) : NULL;
    double *di_all = dimage ? calloc((size_t)nt * n_img, sizeof(double)) : NULL;
    double *loss_all = calloc((size_t)nt, sizeof(double));
    int fail = 0;
    long amb_dummy = 0, rej_dummy = 0;
    orc_ties ties = { tie_tau, alt, alt_tap, (alt && alt_tap) ? n_alt : 0, amb, amb_cap,
                      amb_n ? amb_n : &amb_dummy, rejected ? rejected : &rej_dummy, B, H, W };
    if (rejected) *rejected = 0;
    const orc_ties *tp = (tie_tau > 0 || ties.n_alt > 0) ? &ties : NULL;
    if (amb_n) *amb_n = 0;
#pragma omp parallel num_threads(nt)
    {
#ifdef _OPENMP
        const int t = omp_get_thread_num();
#else
        const int t = 0;
#endif
        double *act = malloc(sizeof(double) * pl.act_total);
        double *dlt = malloc(sizeof(double) * pl.act_total);
        uint8_t *idx = malloc(pl.idx_total + 1);
        double *pr = malloc(sizeof(double) * nc);
        if (!act || !dlt || !idx || !pr) {
#pragma omp atomic write
            fail = 1;
        } else {
#pragma omp for schedule(static)
            for (long q = 0; q < n_pix; ++q) {
                long f = sel ? sel[q] : q;
                int b = (int)(f / ((long)Ho * Wo));
                int i = (int)((f / Wo) % Ho), j = (int)(f % Wo);
                orc_crop(&pl, image, H, W, b, i, j, act);
                orc_patch_forward(&pl, params, act, idx, NULL, pr, tp, b, i, j);
                if (probs) {
                    for (int o = 0; o < nc; ++o) {
                        if (sel) probs[q * nc + o] = pr[o];
                        else probs[(((long)b * nc + o) * Ho + i) * Wo + j] = pr[o];
                    }
                }
                if (!labels) continue;
                long lp = ((long)b * H + (i + ctr)) * W + (j + ctr);
                int t_lab = labels[lp];
                double w = pixw ? pixw[lp] : 1.0;
                if (t_lab < 0 || t_lab >= nc) continue;
                if (pl.loss_kind == ORC_LOSS_MSE) {
                    double sq = 0;
                    for (int o = 0; o < nc; ++o) { double e = pr[o] - (o == t_lab ? 1.0 : 0.0); sq += e * e; }
                    loss_all[t] += w * 0.5 * sq;
                } else {
                    loss_all[t] += w * -log(pr[t_lab]);
                }
                if (!grads && !dimage) continue;
                double *g = grads ? g_all + (size_t)t * pl.n_params : NULL;
                double *gtmp = g;
                if (!gtmp) gtmp = calloc((size_t)pl.n_params, sizeof(double));
                orc_patch_backward(&pl, params, act, idx, pr, t_lab, w, dlt, gtmp, dimage != NULL);
                if (!g) free(gtmp);
                if (dimage) {
                    double *di = di_all + (size_t)t * n_img;
                    for (int c = 0; c < in_ch; ++c)
                        for (int r = 0; r < P; ++r)
                            for (int s = 0; s < P; ++s)
                                di[(((long)b * in_ch + c) * H + (i + r)) * W + (j + s)] +=
                                    dlt[((long)c * P + r) * P + s];
                }
            }
        }
        free(act); free(dlt); free(idx); free(pr);
    }
    /* fixed thread order: the sum is reproducible for a given thread count */
    if (grads) {
        memset(grads, 0, sizeof(double) * pl.n_params);
        for (int t = 0; t < nt; ++t)
            for (long e = 0; e < pl.n_params; ++e) grads[e] += g_all[(size_t)t * pl.n_params + e];
    }
    if (dimage) {
        memset(dimage, 0, sizeof(double) * n_img);
        for (int t = 0; t < nt; ++t)
            for (long e = 0; e < n_img; ++e) dimage[e] += di_all[(size_t)t * n_img + e];
    }
    if (loss) { *loss = 0; for (int t = 0; t < nt; ++t) *loss += loss_all[t]; }
    free(g_all); free(di_all); free(loss_all);
    return fail ? -12 : 0;
}

/* Side of the whole-image ("dense") map that layer `layer`'s outputs form when
 * all patches are laid over the image: element (r,s) of patch (i,j) sits at
 * (i + r*stride, j + s*stride).  Returns rows in *ny, columns in *nx. */
int orc_dense_shape(const int *kinds, const int *maps, const int *ks, const int *ks2, int n_layers, int in_ch,
                    int patch, int H, int W, int layer, int *ny, int *nx, int *ch, int *stride, int *stride_cols)
{
    orc_plan pl;
    int rc = orc_make_plan(&pl, kinds, maps, ks, ks2, n_layers, in_ch, patch);
    if (rc < 0) return rc;
    if (layer < 0 || layer >= n_layers || H < patch || W < patch) return -10;
    *ny = (H - patch) + pl.reach_r[layer] + 1;
    *nx = (W - patch) + pl.reach_c[layer] + 1;
    *ch = pl.ch_out[layer]; *stride = pl.stride_r[layer];
    if (stride_cols) *stride_cols = pl.stride_c[layer];
    return 0;
}

/*
 * Lay the per-patch outputs of one layer over the image.  Every patch is run
 * forward; each dense position is written by exactly one patch (the one with
 * the largest in-patch index that reaches it), so no two threads write the
 * same element.  Patches that share a dense position compute it from the same
 * inputs with the same operations, hence identically.
 *   act     [B][ch][ny][nx]  layer output (after tanh for C / hidden FC)
 *   codes   same shape, MP layers only: argmax tap u*p+v   (may be NULL)
 *   gap     same shape, MP layers only: top-1 minus top-2 of the window (may be NULL)
 *   covered same shape as one channel [B][ny][nx]: 1 where some patch reaches
 */
int orc_dense_layer(const int *kinds, const int *maps, const int *ks, const int *ks2, int n_layers, int in_ch,
                    int patch, const double *params, const double *image, int B, int H, int W,
                    int layer, double *act_out, uint8_t *codes, double *gap, uint8_t *covered, int act_kind)
{
    orc_plan pl;
    int rc = orc_make_plan(&pl, kinds, maps, ks, ks2, n_layers, in_ch, patch);
    if (rc < 0) return rc;
    if (act_kind != ORC_ACT_TANH && act_kind != ORC_ACT_LOGISTIC) return -13;
    pl.act_kind = act_kind;
    if (layer < 0 || layer >= n_layers || H < patch || W < patch) return -10;
    const int P = patch, Ho = H - P + 1, Wo = W - P + 1;
    const int str = pl.stride_r[layer], stc = pl.stride_c[layer];
    const int mr = pl.rows_out[layer], mc = pl.cols_out[layer], ch = pl.ch_out[layer];
    const int ny = Ho - 1 + pl.reach_r[layer] + 1, nx = Wo - 1 + pl.reach_c[layer] + 1;
    const int is_mp = pl.kind[layer] == ORC_MP;
    if (covered) memset(covered, 0, (size_t)B * ny * nx);
    int fail = 0;
#pragma omp parallel
    {
        double *act = malloc(sizeof(double) * pl.act_total);
        uint8_t *idx = malloc(pl.idx_total + 1);
        double *gp = malloc(sizeof(double) * (pl.idx_total + 1));
        double *pr = malloc(sizeof(double) * pl.n_classes);
        if (!act || !idx || !gp || !pr) {
#pragma omp atomic write
            fail = 1;
        } else {
#pragma omp for schedule(static)
            for (long q = 0; q < (long)B * Ho * Wo; ++q) {
                int b = (int)(q / ((long)Ho * Wo));
                int i = (int)((q / Wo) % Ho), j = (int)(q % Wo);
                orc_crop(&pl, image, H, W, b, i, j, act);
                orc_patch_forward(&pl, params, act, idx, gp, pr, NULL, b, i, j);
                const double *y = act + pl.act_off[layer + 1];
                for (int r = 0; r < mr; ++r) {
                    if (!(r == mr - 1 || i < str)) continue;
                    for (int s = 0; s < mc; ++s) {
                        if (!(s == mc - 1 || j < stc)) continue;
                        int yy = i + r * str, xx = j + s * stc;
                        for (int c = 0; c < ch; ++c) {
                            long e = ((long)c * mr + r) * mc + s;
                            long d = (((long)b * ch + c) * ny + yy) * nx + xx;
                            if (act_out) act_out[d] = y[e];
                            if (is_mp && codes) codes[d] = idx[pl.idx_off[layer] + e];
                            if (is_mp && gap) gap[d] = gp[pl.idx_off[layer] + e];
                        }
                        if (covered) covered[((long)b * ny + yy) * nx + xx] = 1;
                    }
                }
            }
        }
        free(act); free(idx); free(gp); free(pr);
    }
    return fail ? -12 : 0;
}
