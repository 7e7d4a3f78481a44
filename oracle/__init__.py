"""ctypes front end of the fp64 patch-by-patch oracle (`mpcnn_oracle.c`).

TEST INFRASTRUCTURE ONLY: imported by `tests/`, by the smoke check and by the
bench's cpu_baseline leg.  It imports nothing from the HIP package, and the HIP
package imports nothing from here.

Network description: a list of (kind, maps, k) integer triples, kind 0 = C
(maps, kernel side), 1 = MP (k = pooling side; a fourth entry k2 > 0 makes the
window k rows x k2 columns), 2 = FC (maps); plus the number of input channels
and the patch side P.  Parameters are one flat fp64 vector,
layer by layer W[o][c][u][v] then b[o] (Background, layer definitions).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mpcnn_oracle.c")
_LIB = os.path.join(_HERE, "liborc.so")
_lib = None


def _host_tag() -> str:
    """What `-march=native` means on this machine (the CPU's model and flag list): a library
    built elsewhere must not be loaded here."""
    model, flags = "", ""
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name") and not model:
                model = line.split(":", 1)[1].strip()
            elif line.startswith("flags") and not flags:
                flags = " ".join(sorted(line.split(":", 1)[1].split()))
            if model and flags:
                break
    except OSError:
        pass
    import hashlib
    return hashlib.sha1((model + "|" + flags).encode()).hexdigest()[:16]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc -O3 -march=native (OpenMP over patches).  ISO C mode keeps
    floating-point contraction off and nothing allows re-association, so the arithmetic is the
    source's, operation by operation.  The library is rebuilt when the source is newer or when
    it was built for another CPU (it travels with the tree)."""
    tag_file = _LIB + ".host"
    tag = _host_tag()
    try:
        same_host = open(tag_file).read().strip() == tag
    except OSError:
        same_host = False
    if force or not same_host or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O3", "-march=native", "-std=c11", "-fopenmp", "-fPIC", "-shared",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
        with open(tag_file + ".tmp%d" % os.getpid(), "w") as f:
            f.write(tag + "\n")
        os.replace(tag_file + ".tmp%d" % os.getpid(), tag_file)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_param_count.restype = C.c_long
    return _lib


def _desc(layers):
    arr = np.asarray([tuple(l) + (0,) * (4 - len(l)) for l in layers], dtype=np.int32).reshape(-1, 4)
    kinds = np.ascontiguousarray(arr[:, 0])
    maps = np.ascontiguousarray(arr[:, 1])
    ks = np.ascontiguousarray(arr[:, 2])
    ks2 = np.ascontiguousarray(arr[:, 3])
    return kinds, maps, (ks, ks2), len(arr)


def _p(a, ct):
    return None if a is None else a.ctypes.data_as(C.POINTER(ct))


def threads() -> int:
    return int(_load().orc_threads())


def param_count(layers, in_ch: int, patch: int) -> int:
    kinds, maps, ks, n = _desc(layers)
    r = _load().orc_param_count(_p(kinds, C.c_int), _p(maps, C.c_int), _p(ks[0], C.c_int), _p(ks[1], C.c_int), n,
                                in_ch, patch)
    if r < 0:
        raise ValueError("bad network description (code %d)" % r)
    return int(r)


def run(layers, in_ch, patch, params, image, labels=None, pixw=None, sel=None,
        want_probs=True, want_grads=False, want_dimage=False, tie_tau=0.0, alt=None, loss_fn="mcce",
        squash="tanh"):
    """Patch-by-patch forward (and backward).  Returns a dict with probs, loss,
    grads, dimage (those asked for).  probs is [B,n_cls,Ho,Wo], or [n_sel,n_cls]
    when `sel` (flat indices into [B,Ho,Wo]) is given.

    loss_fn: "mcce" (softmax + cross-entropy) or "mse" (linear outputs, half the squared
    error against the one-hot target; `probs` then holds the linear outputs).
    squash: "tanh" or "logistic", the squashing function of C and hidden FC layers.

    tie_tau > 0: also returns `near_ties`, an int64 array [n,4] of (window key,
    chosen tap, runner-up tap, layer) for every pooling window whose two largest
    values are within tie_tau; `alt`: (window key, tap) pairs - in those windows
    the named tap is to receive the gradient instead, which the oracle accepts only
    if that tap's value is within tie_tau of the maximum; `alt_rejected` counts the
    refusals, once per patch that contains the window (see orc_ties in the C source)."""
    lib = _load()
    kinds, maps, ks, n = _desc(layers)
    params = np.ascontiguousarray(params, dtype=np.float64)
    image = np.ascontiguousarray(image, dtype=np.float64)
    B, Cc, H, W = image.shape
    assert Cc == in_ch
    npar = param_count(layers, in_ch, patch)
    assert params.size == npar, (params.size, npar)
    n_cls = int(maps[-1])
    Ho, Wo = H - patch + 1, W - patch + 1
    if labels is not None:
        labels = np.ascontiguousarray(labels, dtype=np.int32)
        assert labels.shape == (B, H, W)
    if pixw is not None:
        pixw = np.ascontiguousarray(pixw, dtype=np.float64)
        assert pixw.shape == (B, H, W)
    n_sel = 0
    if sel is not None:
        sel = np.ascontiguousarray(sel, dtype=np.int64)
        n_sel = sel.size
        assert sel.min() >= 0 and sel.max() < B * Ho * Wo
    probs = None
    if want_probs:
        probs = np.zeros((n_sel, n_cls) if sel is not None else (B, n_cls, Ho, Wo))
    grads = np.zeros(npar) if want_grads else None
    dimage = np.zeros_like(image) if want_dimage else None
    n_alt = 0
    alt_key = alt_tap = None
    if alt is not None and len(alt):
        pairs = np.unique(np.asarray(alt, dtype=np.int64).reshape(-1, 2), axis=0)
        assert np.unique(pairs[:, 0]).size == pairs.shape[0], "a window is listed with two taps"
        alt_key = np.ascontiguousarray(pairs[:, 0])
        alt_tap = np.ascontiguousarray(pairs[:, 1].astype(np.uint8))
        n_alt = alt_key.size
    amb_cap = 1 << 20
    while True:
        amb = np.zeros((amb_cap, 4), dtype=np.int64) if tie_tau > 0 else None
        amb_n = C.c_long(0)
        rejected = C.c_long(0)
        loss = C.c_double(0.0)
        for out in (probs, grads, dimage):
            if out is not None:
                out[...] = 0.0
        rc = lib.orc_run(_p(kinds, C.c_int), _p(maps, C.c_int), _p(ks[0], C.c_int), _p(ks[1], C.c_int), n, in_ch, patch,
                         _p(params, C.c_double), _p(image, C.c_double), B, H, W,
                         _p(labels, C.c_int32), _p(pixw, C.c_double), _p(sel, C.c_int64),
                         C.c_long(n_sel), _p(probs, C.c_double),
                         C.byref(loss) if labels is not None else None,
                         _p(grads, C.c_double), _p(dimage, C.c_double),
                         C.c_double(tie_tau), _p(alt_key, C.c_int64), _p(alt_tap, C.c_uint8), C.c_long(n_alt),
                         _p(amb, C.c_int64), C.c_long(amb_cap if amb is not None else 0),
                         C.byref(amb_n), C.byref(rejected), {"mcce": 0, "mse": 1}[loss_fn],
                         {"tanh": 0, "logistic": 1}[squash])
        if rc != 0:
            raise ValueError("orc_run failed (code %d)" % rc)
        if amb is None or amb_n.value <= amb_cap:
            break
        amb_cap = amb_n.value   # the record buffer was too small (a window is met once per patch): again
    near = None
    if amb is not None:
        near = np.unique(amb[:amb_n.value], axis=0)
    return {"probs": probs, "loss": loss.value if labels is not None else None,
            "grads": grads, "dimage": dimage, "near_ties": near, "alt_rejected": rejected.value}


def mirror_pad(image, patch):
    """The image extended so that the patch net's output keeps the image size (Experiments,
    membrane segmentation: pixels outside the boundary of a test image are synthesised by
    mirroring).  c = (patch-1)//2 rows / columns are added above and to the left, patch-1-c
    below and to the right; the mirror repeats the edge pixel (index -1-i stands for i < 0,
    2n-1-i for i >= n), numpy's 'symmetric' mode."""
    c = (patch - 1) // 2
    image = np.asarray(image)
    return np.pad(image, ((0, 0), (0, 0), (c, patch - 1 - c), (c, patch - 1 - c)), mode="symmetric")


def class_balance_weights(labels, n_classes, patch):
    """Per-pixel weights that make the summed loss the sum over classes of each class's MEAN
    loss (Experiments, steel defects: the loss is minimised per class because the data set is
    unbalanced): w = 1 / N_k at a pixel of class k, N_k = number of output pixels of class k
    in the batch (labels are read at the patch centres, (i+c, j+c)); 0 elsewhere."""
    labels = np.asarray(labels)
    B, H, W = labels.shape
    c = (patch - 1) // 2
    Ho, Wo = H - patch + 1, W - patch + 1
    w = np.zeros(labels.shape, dtype=np.float64)
    centre = labels[:, c:c + Ho, c:c + Wo]
    for k in range(n_classes):
        n_k = int((centre == k).sum())
        if n_k:
            w[:, c:c + Ho, c:c + Wo][centre == k] = 1.0 / n_k
    return w


def armijo_step(f, theta, g, f0, alpha0, scale=1.0, c=1e-4, beta=0.5, max_trials=20):
    """Gradient step safeguarded by the Armijo rule (Experiments, membrane segmentation: SGD
    safeguarded by the Armijo rule, the weights updated after every image).  With the step
    direction -scale*g the first alpha in alpha0, beta*alpha0, beta^2*alpha0, ... (at most
    max_trials of them) is accepted for which
        f(theta - alpha*scale*g) <= f0 - c * alpha * scale * |g|^2 ,
    f0 = f(theta), f the summed loss.  Returns (new theta, alpha, f(new theta), trials);
    if no trial passes the parameters stay as they are and alpha = 0."""
    theta = np.asarray(theta, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64)
    gg = float(np.dot(g, g))
    alpha = float(alpha0)
    for trial in range(1, max_trials + 1):
        cand = theta - alpha * scale * g
        fc = float(f(cand))
        if fc <= f0 - c * alpha * scale * gg:
            return cand, alpha, fc, trial
        alpha *= beta
    return theta.copy(), 0.0, float(f0), max_trials


def lbfgs_direction(g, pairs):
    """Search direction p = -H g of the limited-memory BFGS method (Results, the steel data set:
    LBFGS is the optimiser used there; the paper gives no details, this is the method's
    standard two-loop recursion).  pairs = [(s_0, y_0), ...], oldest first, s = difference of
    two successive parameter vectors, y = difference of their gradients.  H is the inverse
    Hessian estimate the BFGS update builds from the pairs, starting from
    H_0 = (s.y / y.y) I of the newest pair; without pairs p = -g."""
    q = np.array(g, dtype=np.float64)
    if not pairs:
        return -q
    rho = [1.0 / float(np.dot(s, y)) for s, y in pairs]
    a = [0.0] * len(pairs)
    for i in range(len(pairs) - 1, -1, -1):           # newest to oldest
        s, y = pairs[i]
        a[i] = rho[i] * float(np.dot(s, q))
        q = q - a[i] * np.asarray(y, dtype=np.float64)
    s, y = pairs[-1]
    r = (float(np.dot(s, y)) / float(np.dot(y, y))) * q
    for i in range(len(pairs)):                       # oldest to newest
        s, y = pairs[i]
        b = rho[i] * float(np.dot(y, r))
        r = r + np.asarray(s, dtype=np.float64) * (a[i] - b)
    return -r


def lbfgs_step(f, theta, g, f0, state, alpha0=1.0, c=1e-4, beta=0.5, max_trials=20, history=8,
               curvature=1e-10):
    """One iteration of limited-memory BFGS with a back-tracking line search (same rule as
    armijo_step, along p instead of -g).  state is a dict the caller keeps between calls
    (start with {}): the previous parameters and gradient and the stored pairs.
      1. If there is a previous iterate: s = theta - theta_prev, y = g - g_prev; the pair is
         stored (the oldest dropped beyond `history`) iff s.y > curvature * |s| |y|.
      2. p = lbfgs_direction(g, pairs); if g.p >= 0 the pairs are dropped and p = -g.
      3. alpha = alpha0, beta*alpha0, ...: the first with f(theta + alpha p) <= f0 + c alpha g.p
         is accepted; theta and g become the previous iterate.
      4. If no trial passes: parameters unchanged, alpha = 0, history and previous iterate dropped.
    Returns (new theta, alpha, f(new theta), trials, pairs in use)."""
    theta = np.asarray(theta, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64)
    pairs = state.setdefault("pairs", [])
    if state.get("theta_prev") is not None:
        s, y = theta - state["theta_prev"], g - state["g_prev"]
        if float(np.dot(s, y)) > curvature * np.sqrt(float(np.dot(s, s)) * float(np.dot(y, y))):
            pairs.append((s, y))
            del pairs[:max(0, len(pairs) - history)]
    p = lbfgs_direction(g, pairs)
    slope = float(np.dot(g, p))
    if slope >= 0.0:
        del pairs[:]
        p, slope = -g, -float(np.dot(g, g))
    used = len(pairs)
    alpha = float(alpha0)
    for trial in range(1, max_trials + 1):
        cand = theta + alpha * p
        fc = float(f(cand))
        if fc <= f0 + c * alpha * slope:
            state["theta_prev"], state["g_prev"] = theta.copy(), g.copy()
            return cand, alpha, fc, trial, used
        alpha *= beta
    del pairs[:]
    state["theta_prev"] = state["g_prev"] = None
    return theta.copy(), 0.0, float(f0), max_trials, used


def window_key(layers, in_ch, patch, B, H, W, layer, b, c, y, x):
    """Key of a pooling window in the whole-image map of MP layer `layer` (see orc_ties)."""
    _, ch, ny, nx = dense_shape(layers, in_ch, patch, B, H, W, layer)[:4]
    return (layer << 48) + ((b * ch + c) * ny + y) * nx + x


def dense_shape(layers, in_ch, patch, B, H, W, layer):
    """(B, channels, rows, cols, stride) of layer `layer`'s whole-image map."""
    lib = _load()
    kinds, maps, ks, n = _desc(layers)
    ny, nx, ch, st = C.c_int(), C.c_int(), C.c_int(), C.c_int()
    rc = lib.orc_dense_shape(_p(kinds, C.c_int), _p(maps, C.c_int), _p(ks[0], C.c_int), _p(ks[1], C.c_int), n, in_ch,
                             patch, H, W, layer, C.byref(ny), C.byref(nx), C.byref(ch),
                             C.byref(st), None)
    if rc != 0:
        raise ValueError("orc_dense_shape failed (code %d)" % rc)
    return B, ch.value, ny.value, nx.value, st.value


def dense_layer(layers, in_ch, patch, params, image, layer, squash="tanh"):
    """Outputs of layer `layer` of every patch laid over the image.  Returns
    dict(act [B,ch,ny,nx], codes, gap (MP layers, else None), covered [B,ny,nx],
    stride (rows), stride_cols)."""
    lib = _load()
    kinds, maps, ks, n = _desc(layers)
    params = np.ascontiguousarray(params, dtype=np.float64)
    image = np.ascontiguousarray(image, dtype=np.float64)
    B, Cc, H, W = image.shape
    ny, nx, ch, st, stc = C.c_int(), C.c_int(), C.c_int(), C.c_int(), C.c_int()
    rc = lib.orc_dense_shape(_p(kinds, C.c_int), _p(maps, C.c_int), _p(ks[0], C.c_int), _p(ks[1], C.c_int), n, in_ch,
                             patch, H, W, layer, C.byref(ny), C.byref(nx), C.byref(ch),
                             C.byref(st), C.byref(stc))
    if rc != 0:
        raise ValueError("orc_dense_shape failed (code %d)" % rc)
    shape = (B, ch.value, ny.value, nx.value)
    is_mp = int(kinds[layer]) == 1
    act = np.zeros(shape)
    codes = np.zeros(shape, dtype=np.uint8) if is_mp else None
    gap = np.zeros(shape) if is_mp else None
    covered = np.zeros((B, ny.value, nx.value), dtype=np.uint8)
    rc = lib.orc_dense_layer(_p(kinds, C.c_int), _p(maps, C.c_int), _p(ks[0], C.c_int), _p(ks[1], C.c_int), n, in_ch,
                             patch, _p(params, C.c_double), _p(image, C.c_double), B, H, W,
                             layer, _p(act, C.c_double), _p(codes, C.c_uint8),
                             _p(gap, C.c_double), _p(covered, C.c_uint8), {"tanh": 0, "logistic": 1}[squash])
    if rc != 0:
        raise ValueError("orc_dense_layer failed (code %d)" % rc)
    return {"act": act, "codes": codes, "gap": gap, "covered": covered.astype(bool),
            "stride": st.value, "stride_cols": stc.value}
