"""Pins of the fp64 patch-by-patch oracle to things other than itself.

Each test names the passage of the paper it leans on.  None needs a GPU and
none touches the HIP library.  What is pinned:
  * one patch == the textbook MPCNN (Background, layers C/MP/FC) as written
    with fp64 library ops + autograd (conv2d, max_pool2d, linear, CE);
  * many patches == plain sum over crops (Method, "every pixel is replaced by
    the output of the corresponding MPCNN applied to every patch");
  * gradients == central finite differences;
  * C layer == scipy correlate2d; MP layer and its tie rule == hand-worked maps;
  * softmax / cross-entropy closed forms;
  * MPF bookkeeping (k^2 offsets, fragment sizes) and the whole-image
    equivalence that the fast path relies on, via dilated library ops.
"""
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F
from scipy.signal import correlate2d

import oracle
from paper_1302_1690_amd import workloads as wl

C, MP, FC = 0, 1, 2
TINY = wl.CONFIGS[0].layers
NETS = {
    "tiny18": (TINY, 1, 18),
    "rgb_p3": (((C, 3, 2), (MP, 0, 3), (C, 4, 2), (FC, 5, 0), (FC, 3, 0)), 3, 11),      # 11->10->3->2
    "cc_floor": (((C, 2, 3), (C, 3, 2), (MP, 0, 2), (FC, 4, 0), (FC, 6, 0), (FC, 2, 0)), 2, 10),  # 10->8->7->3 (floor)
    "fc_only": (((FC, 3, 0),), 2, 4),
    # rectangular pooling windows (Background, layer MP: p_row x p_col): 12 -> 11x11 -> (2x3, floor) 5x3 -> 4x2 -> FC
    "rect_2x3": (((C, 3, 2), (MP, 0, 2, 3), (C, 4, 2), (FC, 5, 0), (FC, 2, 0)), 2, 12),
}


def _four(layer):
    """(kind, maps, k, k2): k2 = columns of a pooling window, k if the description has none."""
    kind, maps, k = layer[:3]
    return kind, maps, k, (layer[3] if len(layer) > 3 and layer[3] else k)


def rand_params(layers, in_ch, patch, seed, amp=0.5):
    n = oracle.param_count(layers, in_ch, patch)
    return np.random.default_rng(seed).uniform(-amp, amp, n)


def split_params(layers, in_ch, patch, params):
    """(W[o,c,k,k], b[o]) per parametrised layer, in the documented order."""
    out, rows, cols, ch, off, seen_fc = [], patch, patch, in_ch, 0, False
    for kind, maps, k, k2 in (_four(l) for l in layers):
        if kind == MP:
            out.append(None)
            rows //= k
            cols //= k2
            continue
        kr, kc = (k, k) if kind == C else ((1, 1) if seen_fc else (rows, cols))
        nw = maps * ch * kr * kc
        W = params[off:off + nw].reshape(maps, ch, kr, kc)
        b = params[off + nw:off + nw + maps]
        off += nw + maps
        out.append((W, b))
        rows, cols = rows - kr + 1, cols - kc + 1
        ch = maps
        seen_fc = seen_fc or kind == FC
    assert off == params.size
    return out


def torch_patch_net(layers, in_ch, patch, params_t, x, squash=torch.tanh):
    """Textbook net on patches x [N,C,P,P] with library ops; returns logits [N,n_cls]."""
    rows, cols, ch, off, seen_fc = patch, patch, in_ch, 0, False
    h = x
    L = len(layers)
    for li, (kind, maps, k, k2) in enumerate(_four(l) for l in layers):
        if kind == MP:
            h = F.max_pool2d(h, (k, k2))    # floor semantics, non-overlapping
            rows //= k
            cols //= k2
            continue
        kr, kc = (k, k) if kind == C else ((1, 1) if seen_fc else (rows, cols))
        nw = maps * ch * kr * kc
        W = params_t[off:off + nw].reshape(maps, ch, kr, kc)
        b = params_t[off + nw:off + nw + maps]
        off += nw + maps
        if kind == C:
            h = squash(F.conv2d(h, W, b))
        else:
            h = F.linear(h.reshape(h.shape[0], -1), W.reshape(maps, -1), b)
            if li != L - 1:
                h = squash(h)
            h = h.reshape(h.shape[0], maps, 1, 1)
        rows, cols = rows - kr + 1, cols - kc + 1
        ch = maps
        seen_fc = seen_fc or kind == FC
    return h.reshape(h.shape[0], -1)


@pytest.mark.parametrize("name", list(NETS))
def test_single_patch_matches_autograd(name):
    """One P x P image is one patch: probs, loss, dL/dparams and dL/dimage must
    equal the textbook net written with fp64 library ops (Background)."""
    layers, in_ch, P = NETS[name]
    rng = np.random.default_rng(7)
    params = rand_params(layers, in_ch, P, 11)
    img = rng.uniform(0, 1, (2, in_ch, P, P))
    n_cls = layers[-1][1]
    lab = rng.integers(0, n_cls, (2, P, P)).astype(np.int32)
    pw = rng.uniform(0.5, 2.0, (2, P, P))
    r = oracle.run(layers, in_ch, P, params, img, lab, pw, want_grads=True, want_dimage=True)

    pt = torch.tensor(params, dtype=torch.float64, requires_grad=True)
    xt = torch.tensor(img, dtype=torch.float64, requires_grad=True)
    z = torch_patch_net(layers, in_ch, P, pt, xt)
    c = (P - 1) // 2
    t = torch.tensor(lab[:, c, c].astype(np.int64))
    w = torch.tensor(pw[:, c, c])
    loss = (F.cross_entropy(z, t, reduction="none") * w).sum()
    loss.backward()
    np.testing.assert_allclose(r["probs"].reshape(2, n_cls), torch.softmax(z, 1).detach().numpy(),
                               rtol=1e-12, atol=1e-14)
    assert abs(r["loss"] - loss.item()) <= 1e-12 * abs(loss.item())
    np.testing.assert_allclose(r["grads"], pt.grad.numpy(), rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(r["dimage"], xt.grad.numpy(), rtol=1e-10, atol=1e-13)


@pytest.mark.parametrize("name", ["tiny18", "rgb_p3", "cc_floor", "rect_2x3"])
def test_image_is_sum_over_crops(name):
    """An H x W image is (H-P+1)(W-P+1) patches; label and weight sit at the
    patch centre (P-1)//2; gradients add up (Alg. 2: gradients are accumulated)."""
    layers, in_ch, P = NETS[name]
    rng = np.random.default_rng(3)
    H, W, B = P + 3, P + 2, 2
    params = rand_params(layers, in_ch, P, 5)
    img = rng.uniform(0, 1, (B, in_ch, H, W))
    n_cls = layers[-1][1]
    lab = rng.integers(-1, n_cls, (B, H, W)).astype(np.int32)   # -1 = ignored pixel
    pw = rng.uniform(0.5, 2.0, (B, H, W))
    r = oracle.run(layers, in_ch, P, params, img, lab, pw, want_grads=True, want_dimage=True)

    pt = torch.tensor(params, dtype=torch.float64, requires_grad=True)
    xt = torch.tensor(img, dtype=torch.float64, requires_grad=True)
    c = (P - 1) // 2
    total = 0.0
    probs = np.zeros((B, n_cls, H - P + 1, W - P + 1))
    for b in range(B):
        for i in range(H - P + 1):
            for j in range(W - P + 1):
                z = torch_patch_net(layers, in_ch, P, pt, xt[b:b + 1, :, i:i + P, j:j + P])
                probs[b, :, i, j] = torch.softmax(z, 1).detach().numpy()[0]
                t = int(lab[b, i + c, j + c])
                if t >= 0:
                    total = total + pw[b, i + c, j + c] * F.cross_entropy(
                        z, torch.tensor([t]), reduction="sum")
    total.backward()
    np.testing.assert_allclose(r["probs"], probs, rtol=1e-12, atol=1e-14)
    assert abs(r["loss"] - total.item()) <= 1e-12 * abs(total.item())
    np.testing.assert_allclose(r["grads"], pt.grad.numpy(), rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(r["dimage"], xt.grad.numpy(), rtol=1e-9, atol=1e-12)


def test_pixel_subset_and_weight_mask_agree():
    """Evaluating a subset `sel` == weighting the loss by its indicator; and the
    gradient is linear in the per-pixel weights (Alg. 2)."""
    cfg = wl.crop(wl.CONFIGS[0], 2, 24, 25)
    img, lab = wl.make_inputs(cfg)
    params = wl.make_params(cfg).astype(np.float64)
    sel = wl.sample_pixels(cfg, 12, 9)
    full = oracle.run(cfg.layers, 1, cfg.patch, params, img, lab, want_grads=True)
    sub = oracle.run(cfg.layers, 1, cfg.patch, params, img, lab, sel=sel, want_grads=True)
    mask = np.zeros((cfg.batch, cfg.height, cfg.width))
    c = (cfg.patch - 1) // 2
    b, rem = np.divmod(sel, cfg.out_h * cfg.out_w)
    i, j = np.divmod(rem, cfg.out_w)
    mask[b, i + c, j + c] = 1.0
    msk = oracle.run(cfg.layers, 1, cfg.patch, params, img, lab, pixw=mask, want_grads=True)
    np.testing.assert_allclose(sub["grads"], msk["grads"], rtol=1e-11, atol=1e-14)
    assert abs(sub["loss"] - msk["loss"]) < 1e-11 * abs(sub["loss"])
    np.testing.assert_allclose(sub["probs"], full["probs"][b, :, i, j], rtol=0, atol=0)
    rest = oracle.run(cfg.layers, 1, cfg.patch, params, img, lab, pixw=1.0 - mask, want_grads=True)
    np.testing.assert_allclose(msk["grads"] + rest["grads"], full["grads"], rtol=1e-10, atol=1e-12)


@pytest.mark.parametrize("name", ["tiny18", "rgb_p3"])
def test_gradient_matches_central_differences(name):
    """dL/dparams against (L(theta+e) - L(theta-e)) / 2e on a small image."""
    layers, in_ch, P = NETS[name]
    rng = np.random.default_rng(17)
    H = W = P + 2
    params = rand_params(layers, in_ch, P, 23, amp=0.3)
    img = rng.uniform(0, 1, (1, in_ch, H, W))
    lab = rng.integers(0, layers[-1][1], (1, H, W)).astype(np.int32)
    r = oracle.run(layers, in_ch, P, params, img, lab, want_grads=True)
    g = r["grads"]
    eps = 1e-5
    idx = rng.choice(params.size, size=min(params.size, 120), replace=False)
    worst = 0.0
    for e in idx:
        p1, p2 = params.copy(), params.copy()
        p1[e] += eps
        p2[e] -= eps
        l1 = oracle.run(layers, in_ch, P, p1, img, lab, want_probs=False)["loss"]
        l2 = oracle.run(layers, in_ch, P, p2, img, lab, want_probs=False)["loss"]
        fd = (l1 - l2) / (2 * eps)
        worst = max(worst, abs(fd - g[e]) / (1e-2 + abs(g[e])))
    assert worst < 2e-7, worst


def test_conv_layer_is_valid_correlation():
    """C layer = valid 2-D filtering, no flip, all input maps summed, then tanh."""
    layers = ((C, 3, 3), (FC, 2, 0))
    in_ch, P = 2, 6
    rng = np.random.default_rng(1)
    params = rand_params(layers, in_ch, P, 2)
    img = rng.uniform(-1, 1, (1, in_ch, P, P))
    d = oracle.dense_layer(layers, in_ch, P, params, img, 0)
    (W, b), _ = split_params(layers, in_ch, P, params)
    for o in range(3):
        ref = b[o] + sum(correlate2d(img[0, c], W[o, c], mode="valid") for c in range(in_ch))
        np.testing.assert_allclose(d["act"][0, o], np.tanh(ref), rtol=1e-13, atol=1e-15)
    # hand-worked: x = [[1,2,3],[4,5,6],[7,8,9]], w = [[1,0],[0,-1]], b = 0.5 (no flip):
    # y[r][s] = x[r][s] - x[r+1][s+1] + 0.5 = -4 + 0.5 for every (r,s)
    layers = ((C, 1, 2), (FC, 2, 0))
    params = np.zeros(oracle.param_count(layers, 1, 3))
    params[:5] = [1, 0, 0, -1, 0.5]
    x = np.arange(1, 10, dtype=float).reshape(1, 1, 3, 3)
    d = oracle.dense_layer(layers, 1, 3, params, x, 0)
    np.testing.assert_allclose(d["act"][0, 0], np.tanh(np.full((2, 2), -3.5)), rtol=1e-15)
    # an asymmetric kernel tells correlation from convolution:
    # w = [[0,1],[0,0]] picks x[r][s+1]
    params[:5] = [0, 1, 0, 0, 0]
    d = oracle.dense_layer(layers, 1, 3, params, x, 0)
    np.testing.assert_allclose(d["act"][0, 0], np.tanh(np.array([[2., 3.], [5., 6.]])), rtol=1e-15)


def _pool_net_codes(x, p):
    """Pool directly on the image: net MP p, FC 2; patch = p (one window)."""
    layers = ((MP, 0, p), (FC, 2, 0))
    params = np.zeros(oracle.param_count(layers, 1, p))
    return oracle.dense_layer(layers, 1, p, params, x[None, None], 0)


def test_max_pool_values_and_tie_rule_hand_cases():
    """MP keeps the maximum of each window; ties go to the first element in
    row-major (u,v) order.  With patch = p the whole-image map is the stride-1
    max filter, i.e. the union of the p*p offset fragments of Alg. 3."""
    ramp = np.arange(16, dtype=float).reshape(4, 4)            # strictly increasing
    d = _pool_net_codes(ramp, 2)
    assert d["act"].shape == (1, 1, 3, 3)
    np.testing.assert_array_equal(d["act"][0, 0], ramp[1:, 1:])  # max = bottom-right
    assert (d["codes"] == 3).all()                               # last tap, 1*2+1
    np.testing.assert_array_equal(d["gap"][0, 0], np.ones((3, 3)))  # 2nd best is 1 below
    const = np.full((4, 4), 0.25)
    d = _pool_net_codes(const, 2)
    assert (d["codes"] == 0).all() and (d["gap"] == 0).all()     # tie -> first tap
    # -0.0 and +0.0 compare equal: still the first tap
    z = np.array([[0.0, -0.0], [-0.0, 0.0]])
    assert _pool_net_codes(z, 2)["codes"].item() == 0
    # tie between taps 1 and 2 only -> tap 1
    x = np.array([[0.0, 1.0], [1.0, 0.5]])
    assert _pool_net_codes(x, 2)["codes"].item() == 1
    # 3x3 window, maximum at (u,v)=(2,0) -> code 6; decreasing ramp -> code 0
    x = np.zeros((3, 3)); x[2, 0] = 1.0
    assert _pool_net_codes(x, 3)["codes"].item() == 6
    assert _pool_net_codes(-np.arange(9.).reshape(3, 3), 3)["codes"].item() == 0


def test_shared_maximum_receives_sum_of_deltas():
    """Fig. 2 situation: one element is the maximum for several pooling offsets;
    its back-propagated value is the SUM over those fragments, all others get 0
    (Alg. 4: contributions need to be accumulated)."""
    layers = ((MP, 0, 2), (FC, 2, 0))
    P = 2
    x = np.array([[0.1, 0.2, 0.3], [0.4, 1.0, 0.5], [0.6, 0.7, 0.8]])[None, None]
    params = np.array([0.7, -0.3, 0.0, 0.0])        # W[o][0][0][0] for o=0,1 ; b = 0
    lab = np.zeros((1, 3, 3), dtype=np.int32)
    lab[0, 0, 1] = 1                                 # centre of patch (0,1) is pixel (0,1)
    r = oracle.run(layers, 1, P, params, x, lab, want_grads=True, want_dimage=True)
    # all four 2x2 windows pick the centre 1.0 -> z = (0.7, -0.3) everywhere
    p = np.exp([0.7, -0.3]); p /= p.sum()
    np.testing.assert_allclose(r["probs"][0, :, 0, 0], p, rtol=1e-14)
    dz = np.array([[p[0] - 1, p[1]], [p[0], p[1] - 1], [p[0] - 1, p[1]], [p[0] - 1, p[1]]])
    expect = np.zeros((3, 3))
    expect[1, 1] = (dz @ np.array([0.7, -0.3])).sum()
    np.testing.assert_allclose(r["dimage"][0, 0], expect, rtol=1e-13, atol=1e-16)
    np.testing.assert_allclose(r["grads"][:2], dz.sum(0) * 1.0, rtol=1e-13)   # dW = sum dz * max
    np.testing.assert_allclose(r["grads"][2:], dz.sum(0), rtol=1e-13)          # db = sum dz
    assert abs(r["loss"] - (-3 * np.log(p[0]) - np.log(p[1]))) < 1e-13


def test_near_tie_report_and_alternative_routing():
    """A window whose two largest values are within tau is reported with both taps;
    listing it with a tap within tau of the maximum sends the back-propagated value
    there instead, and nothing else changes (valid sub-gradients of the max); a tap
    further from the maximum is refused and counted."""
    layers = ((MP, 0, 2), (FC, 2, 0))
    x = np.array([[1.0, 1.0 - 1e-9, 0.2], [0.1, 0.3, 0.4]])[None, None]   # two 2x2 windows
    params = np.array([0.7, -0.3, 0.1, 0.0])
    lab = np.ones((1, 2, 3), dtype=np.int32)
    r0 = oracle.run(layers, 1, 2, params, x, lab, want_grads=True, want_dimage=True, tie_tau=1e-6)
    assert r0["near_ties"].tolist() == [[oracle.window_key(layers, 1, 2, 1, 2, 3, 0, 0, 0, 0, 0), 0, 1, 0]]
    assert r0["dimage"][0, 0, 0, 0] != 0 and r0["dimage"][0, 0, 0, 1] != 0   # window 2 picks x[0][1]
    plain = oracle.run(layers, 1, 2, params, x, lab, want_grads=True, want_dimage=True)
    np.testing.assert_array_equal(plain["dimage"], r0["dimage"])              # reporting changes nothing
    r1 = oracle.run(layers, 1, 2, params, x, lab, want_grads=True, want_dimage=True, tie_tau=1e-6,
                    alt=r0["near_ties"][:, [0, 2]])
    assert r1["alt_rejected"] == 0
    d0, d1 = r0["dimage"][0, 0], r1["dimage"][0, 0]
    assert d1[0, 0] == 0.0 and abs(d1[0, 1] - (d0[0, 0] + d0[0, 1])) < 1e-15   # moved to the runner-up
    np.testing.assert_array_equal(r1["probs"], r0["probs"])                   # forward value unchanged
    np.testing.assert_array_equal(r1["grads"], r0["grads"])                   # FC sees the same maximum
    # a window that is not a near-tie cannot be rerouted, nor a near-tie to a distant tap
    for key, tap in ((oracle.window_key(layers, 1, 2, 1, 2, 3, 0, 0, 0, 0, 1), 2),
                     (oracle.window_key(layers, 1, 2, 1, 2, 3, 0, 0, 0, 0, 0), 3)):
        r2 = oracle.run(layers, 1, 2, params, x, lab, want_dimage=True, tie_tau=1e-6, alt=[(key, tap)])
        np.testing.assert_array_equal(r2["dimage"], r0["dimage"])
        assert r2["alt_rejected"] == 1
    # with a wide tau the third-best tap of a window qualifies too
    r3 = oracle.run(layers, 1, 2, params, x, lab, want_dimage=True, tie_tau=0.75,
                    alt=[(oracle.window_key(layers, 1, 2, 1, 2, 3, 0, 0, 0, 0, 0), 3)])
    assert r3["alt_rejected"] == 0
    d3 = r3["dimage"][0, 0]
    assert d3[0, 0] == 0.0 and abs(d3[1, 1] - d0[0, 0]) < 1e-15


def test_softmax_cross_entropy_closed_forms():
    """Zero last layer -> p = 1/n, L = N log n, delta = 1/n - onehot; deltas sum
    to zero over classes; db_last = sum of deltas (Results: MCCE, per pixel)."""
    layers, in_ch, P = NETS["rgb_p3"]
    rng = np.random.default_rng(4)
    params = rand_params(layers, in_ch, P, 8)
    n_last = 3 * 5 + 3
    params[-n_last:] = 0.0
    H = W = P + 4
    img = rng.uniform(0, 1, (1, in_ch, H, W))
    lab = rng.integers(0, 3, (1, H, W)).astype(np.int32)
    r = oracle.run(layers, in_ch, P, params, img, lab, want_grads=True)
    N = 25
    np.testing.assert_allclose(r["probs"], 1.0 / 3, rtol=1e-15)
    assert abs(r["loss"] - N * np.log(3.0)) < 1e-12
    c = (P - 1) // 2
    t = lab[0, c:c + 5, c:c + 5].ravel()
    db = np.array([(1.0 / 3 - (t == o)).sum() for o in range(3)])
    np.testing.assert_allclose(r["grads"][-3:], db, rtol=1e-13, atol=1e-14)
    # upstream gradients vanish because W_last = 0
    assert np.abs(r["grads"][:-n_last]).max() == 0.0
    # generic parameters: db_last sums to zero over classes, probs sum to one
    params = rand_params(layers, in_ch, P, 9)
    r = oracle.run(layers, in_ch, P, params, img, lab, want_grads=True)
    assert abs(r["grads"][-3:].sum()) < 1e-12
    np.testing.assert_allclose(r["probs"].sum(1), 1.0, rtol=1e-14)


def test_fragment_bookkeeping():
    """An MPF layer with k x k pooling has k^2 offsets; the fragment of offset
    (r,c) has floor((n-r)/k) rows; laid side by side they fill the stride-1 map
    of side n-(k-1) (Method, MPF layer)."""
    for n, k in [(62, 2), (57, 2), (31, 3), (10, 3)]:
        assert sum((n - r) // k for r in range(k)) == n - (k - 1)
    cfg = wl.CONFIGS[0]
    img, _ = wl.make_inputs(cfg)
    params = wl.make_params(cfg).astype(np.float64)
    sides = []
    for layer in range(len(cfg.layers)):
        d = oracle.dense_layer(cfg.layers, 1, cfg.patch, params, img[:, :, :40, :40], layer)
        sides.append((d["act"].shape[2], d["stride"], bool(d["covered"].all())))
    # 40 -> C3: 38 -> MP2: 37 (stride 2) -> C3 dilated 2: 33 -> MP2: 31 (stride 4) -> FC 3x3 dilated 4: 23 -> 23
    assert sides == [(38, 1, True), (37, 2, True), (33, 2, True), (31, 4, True), (23, 4, True),
                     (23, 4, True)]


def _dense_forward_torch(layers, in_ch, patch, params_t, x):
    """Whole-image evaluation with dilated library ops: MP -> stride-1 max
    filter with taps `d` apart, later kernels dilated by the pooling factors."""
    dr, dc, rows, cols, ch, off, seen_fc = 1, 1, patch, patch, in_ch, 0, False
    h = x
    L = len(layers)
    for li, (kind, maps, k, k2) in enumerate(_four(l) for l in layers):
        if kind == MP:
            h = F.max_pool2d(h, (k, k2), stride=1, dilation=(dr, dc))
            dr *= k
            dc *= k2
            rows //= k
            cols //= k2
            continue
        kr, kc = (k, k) if kind == C else ((1, 1) if seen_fc else (rows, cols))
        nw = maps * ch * kr * kc
        W = params_t[off:off + nw].reshape(maps, ch, kr, kc)
        b = params_t[off + nw:off + nw + maps]
        off += nw + maps
        h = F.conv2d(h, W, b, dilation=(dr, dc))
        if li != L - 1:
            h = torch.tanh(h)
        rows, cols = rows - kr + 1, cols - kc + 1
        ch = maps
        seen_fc = seen_fc or kind == FC
    return h


@pytest.mark.parametrize("name", ["tiny18", "rgb_p3", "rect_2x3"])
def test_whole_image_equivalence(name):
    """The invariant of the method: one dilated whole-image pass gives, at every
    pixel, the patch net's output, and its gradient is the sum over patches."""
    layers, in_ch, P = NETS[name]
    rng = np.random.default_rng(31)
    H, W = P + 9, P + 7
    params = rand_params(layers, in_ch, P, 13)
    img = rng.uniform(0, 1, (1, in_ch, H, W))
    n_cls = layers[-1][1]
    lab = rng.integers(0, n_cls, (1, H, W)).astype(np.int32)
    r = oracle.run(layers, in_ch, P, params, img, lab, want_grads=True)
    pt = torch.tensor(params, dtype=torch.float64, requires_grad=True)
    z = _dense_forward_torch(layers, in_ch, P, pt, torch.tensor(img))
    # a pool that drops a trailing row (floor) leaves the dense map one larger than the
    # number of patches; the valid outputs are the leading (H-P+1) x (W-P+1)
    assert z.shape[2] >= H - P + 1 and z.shape[3] >= W - P + 1
    z = z[:, :, :H - P + 1, :W - P + 1]
    np.testing.assert_allclose(r["probs"], torch.softmax(z, 1).detach().numpy(), rtol=1e-11,
                               atol=1e-14)
    c = (P - 1) // 2
    t = torch.tensor(lab[:, c:c + H - P + 1, c:c + W - P + 1].astype(np.int64))
    loss = F.cross_entropy(z, t, reduction="sum")
    loss.backward()
    assert abs(loss.item() - r["loss"]) < 1e-11 * r["loss"]
    np.testing.assert_allclose(r["grads"], pt.grad.numpy(), rtol=1e-9, atol=1e-11)


def test_translation_structure():
    """Shifting the image by one pixel shifts the output map by one pixel."""
    cfg = wl.crop(wl.CONFIGS[0], 1, 30, 30)
    img, _ = wl.make_inputs(cfg)
    params = wl.make_params(cfg).astype(np.float64)
    a = oracle.run(cfg.layers, 1, cfg.patch, params, img[:, :, :-1, :-1])["probs"]
    b = oracle.run(cfg.layers, 1, cfg.patch, params, img[:, :, 1:, 1:])["probs"]
    np.testing.assert_array_equal(a[:, :, 1:, 1:], b[:, :, :-1, :-1])


@pytest.mark.parametrize("name", ["tiny18", "rgb_p3"])
def test_mse_linear_outputs_vs_autograd_and_by_hand(name):
    """Mean squared error with linear outputs: the derivative w.r.t. the output image is
    x^ - t (Method, the first step of back-propagation).  Outputs = last FC without the
    softmax; L = sum w/2 |x^ - onehot|^2; everything below the outputs as for the other loss."""
    layers, in_ch, P = NETS[name]
    rng = np.random.default_rng(31)
    params = rand_params(layers, in_ch, P, 32)
    img = rng.uniform(0, 1, (2, in_ch, P, P))
    n_cls = layers[-1][1]
    lab = rng.integers(0, n_cls, (2, P, P)).astype(np.int32)
    pw = rng.uniform(0.5, 2.0, (2, P, P))
    r = oracle.run(layers, in_ch, P, params, img, lab, pw, want_grads=True, want_dimage=True, loss_fn="mse")
    pt = torch.tensor(params, dtype=torch.float64, requires_grad=True)
    xt = torch.tensor(img, dtype=torch.float64, requires_grad=True)
    z = torch_patch_net(layers, in_ch, P, pt, xt)
    c = (P - 1) // 2
    t = F.one_hot(torch.tensor(lab[:, c, c].astype(np.int64)), n_cls).to(torch.float64)
    loss = (0.5 * ((z - t) ** 2).sum(1) * torch.tensor(pw[:, c, c])).sum()
    loss.backward()
    np.testing.assert_allclose(r["probs"].reshape(2, n_cls), z.detach().numpy(), rtol=1e-12, atol=1e-14)
    assert abs(r["loss"] - loss.item()) <= 1e-12 * abs(loss.item())
    np.testing.assert_allclose(r["grads"], pt.grad.numpy(), rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(r["dimage"], xt.grad.numpy(), rtol=1e-10, atol=1e-13)
    # by hand, one FC on a 1x1 patch: z = W x + b = (0.25, 0.3), t = (0, 1)
    r1 = oracle.run(((FC, 2, 0),), 1, 1, np.array([0.3, -0.2, 0.1, 0.4]), np.array([[[[0.5]]]]),
                    np.array([[[1]]], dtype=np.int32), want_grads=True, loss_fn="mse")
    np.testing.assert_allclose(r1["probs"].ravel(), [0.25, 0.3], rtol=0, atol=1e-15)
    assert abs(r1["loss"] - 0.5 * (0.25 ** 2 + 0.7 ** 2)) < 1e-15
    np.testing.assert_allclose(r1["grads"], [0.125, -0.35, 0.25, -0.7], rtol=0, atol=1e-15)


def test_class_balance_weights_by_hand():
    """Loss minimised per class: w = 1/N_k over the OUTPUT pixels (labels at patch centres),
    so that each class contributes its mean loss (Experiments, steel defects)."""
    lab = np.array([[[0, 0, 0, 0],
                     [0, 1, 0, 9],
                     [0, 0, 0, 0],
                     [1, 1, 1, 1]]], dtype=np.int32)
    w = oracle.class_balance_weights(lab, 2, 3)       # P = 3: outputs are the 2x2 centres (1..2, 1..2)
    want = np.zeros((1, 4, 4))
    want[0, 1, 1] = 1.0                                # the only class-1 centre
    want[0, 1, 2] = want[0, 2, 1] = want[0, 2, 2] = 1.0 / 3
    np.testing.assert_array_equal(w, want)
    # with these weights the loss is the sum of the per-class mean losses
    layers, in_ch, P = ((FC, 2, 0),), 1, 3
    rng = np.random.default_rng(5)
    params = rng.uniform(-0.5, 0.5, oracle.param_count(layers, in_ch, P))
    img = rng.uniform(0, 1, (1, 1, 4, 4))
    r = oracle.run(layers, in_ch, P, params, img, lab, w)
    nll = -np.log(r["probs"][0])                       # [class][i][j]
    centre = lab[0, 1:3, 1:3]
    per_class = sum(nll[k][centre == k].mean() for k in (0, 1))
    assert abs(r["loss"] - per_class) < 1e-13


def test_armijo_rule_by_hand():
    """f = theta^2/2 at theta = 1 (g = 1, f0 = 1/2), c = 1e-4, halving: alpha = 4 gives f = 4.5 (too
    large), alpha = 2 gives f = 1/2 > 1/2 - 2e-4 (no sufficient decrease), alpha = 1 gives f = 0."""
    f = lambda th: 0.5 * float(th[0]) ** 2
    th, alpha, fv, trials = oracle.armijo_step(f, [1.0], [1.0], 0.5, 4.0)
    assert (th.tolist(), alpha, fv, trials) == ([0.0], 1.0, 0.0, 3)
    # the accepted point satisfies the inequality, the one before does not (here with a scale)
    th, alpha, fv, trials = oracle.armijo_step(f, [1.0], [2.0], 0.5, 4.0, scale=0.5)
    assert (th.tolist(), alpha, trials) == ([0.0], 1.0, 3)
    # nothing acceptable: parameters untouched, alpha = 0
    up = lambda th: 1.0 + abs(float(th[0]) - 1.0)
    th, alpha, fv, trials = oracle.armijo_step(up, [1.0], [1.0], 1.0, 1.0, max_trials=5)
    assert (th.tolist(), alpha, fv, trials) == ([1.0], 0.0, 1.0, 5)
    # on the real loss: the accepted step decreases it by at least c*alpha*|g|^2
    layers, in_ch, P = NETS["tiny18"]
    rng = np.random.default_rng(41)
    params = rand_params(layers, in_ch, P, 42)
    img = rng.uniform(0, 1, (1, in_ch, P + 2, P + 1))
    lab = rng.integers(0, 2, (1, P + 2, P + 1)).astype(np.int32)
    r = oracle.run(layers, in_ch, P, params, img, lab, want_grads=True)
    loss = lambda th: oracle.run(layers, in_ch, P, th, img, lab, want_probs=False)["loss"]
    th, alpha, fv, trials = oracle.armijo_step(loss, params, r["grads"], r["loss"], 64.0)
    assert trials > 1 and alpha == 64.0 * 0.5 ** (trials - 1)
    assert fv <= r["loss"] - 1e-4 * alpha * np.dot(r["grads"], r["grads"])
    assert loss(params - 2 * alpha * r["grads"]) > r["loss"] - 1e-4 * 2 * alpha * np.dot(r["grads"], r["grads"])


def _dense_bfgs_inverse(pairs, n):
    """Textbook BFGS update of the inverse Hessian estimate, written with dense matrices:
    H <- (I - rho s y^T) H (I - rho y s^T) + rho s s^T for each pair, oldest first, from
    H_0 = (s.y / y.y) I of the newest pair."""
    s, y = pairs[-1]
    H = (np.dot(s, y) / np.dot(y, y)) * np.eye(n)
    for s, y in pairs:
        rho = 1.0 / np.dot(s, y)
        V = np.eye(n) - rho * np.outer(y, s)
        H = V.T @ H @ V + rho * np.outer(s, s)
    return H


def test_logistic_activation_matches_autograd():
    """The logistic function as the squashing function of C and hidden FC layers (Background,
    layer C: tanh or logistic): probs, loss and all gradients of a two-patch batch equal the
    textbook net with torch.sigmoid; and by hand, sigma(0) = 1/2 with derivative 1/4."""
    for name in ("tiny18", "rgb_p3"):
        layers, in_ch, P = NETS[name]
        rng = np.random.default_rng(17)
        params = rand_params(layers, in_ch, P, 19) * 2.0
        img = rng.uniform(0, 1, (2, in_ch, P, P))
        n_cls = layers[-1][1]
        lab = rng.integers(0, n_cls, (2, P, P)).astype(np.int32)
        r = oracle.run(layers, in_ch, P, params, img, lab, want_grads=True, want_dimage=True, squash="logistic")
        pt = torch.tensor(params, dtype=torch.float64, requires_grad=True)
        xt = torch.tensor(img, dtype=torch.float64, requires_grad=True)
        z = torch_patch_net(layers, in_ch, P, pt, xt, squash=torch.sigmoid)
        c = (P - 1) // 2
        loss = F.cross_entropy(z, torch.tensor(lab[:, c, c].astype(np.int64)), reduction="sum")
        loss.backward()
        np.testing.assert_allclose(r["probs"].reshape(2, n_cls), torch.softmax(z, 1).detach().numpy(), rtol=1e-12, atol=1e-14)
        assert abs(r["loss"] - loss.item()) <= 1e-12 * abs(loss.item())
        np.testing.assert_allclose(r["grads"], pt.grad.numpy(), rtol=1e-10, atol=1e-13)
        np.testing.assert_allclose(r["dimage"], xt.grad.numpy(), rtol=1e-10, atol=1e-13)
        # not the tanh net
        r_t = oracle.run(layers, in_ch, P, params, img, lab, want_grads=True)
        assert np.abs(r_t["grads"] - r["grads"]).max() > 1e-3
    # by hand: one hidden unit h = sigma(w x + b) on a 1x1 patch, then a linear layer to 2 outputs with
    # weights (1, 0), MSE against class 0: x = 2, w = b = 0 -> h = 1/2, outputs (1/2, 0), L = 1/8,
    # x^ - t = (-1/2, 0), dL/dh = -1/2, through sigma' = h(1-h) = 1/4: dL/db = -1/8, dL/dw = -1/4
    layers = ((FC, 1, 0), (FC, 2, 0))
    params = np.array([0.0, 0.0, 1.0, 0.0, 0.0, 0.0])        # w, b | v0, v1, c0, c1
    r = oracle.run(layers, 1, 1, params, np.array([[[[2.0]]]]), np.array([[[0]]], dtype=np.int32), want_grads=True,
                   loss_fn="mse", squash="logistic")
    np.testing.assert_allclose(r["probs"].ravel(), [0.5, 0.0], atol=1e-15)
    assert abs(r["loss"] - 0.125) < 1e-15
    np.testing.assert_allclose(r["grads"], [-0.25, -0.125, -0.25, 0.0, -0.5, 0.0], atol=1e-15)


def test_lbfgs_direction_against_dense_bfgs_and_by_hand():
    """The two-loop recursion must apply exactly the matrix the BFGS update formula builds
    (Results, the steel data set: LBFGS)."""
    # one pair by hand: s = (1,0), y = (2,0): rho = 1/2, H0 = I/2, H = diag(1/2, 1/2); g = (4,6) -> p = -(2,3)
    p = oracle.lbfgs_direction([4.0, 6.0], [(np.array([1.0, 0.0]), np.array([2.0, 0.0]))])
    np.testing.assert_allclose(p, [-2.0, -3.0], rtol=0, atol=1e-15)
    # no pairs: steepest descent
    np.testing.assert_array_equal(oracle.lbfgs_direction([1.0, -2.0, 3.0], []), [-1.0, 2.0, -3.0])
    rng = np.random.default_rng(7)
    n = 9
    A = rng.normal(size=(n, n)); A = A @ A.T + n * np.eye(n)          # pairs of a convex quadratic: y = A s
    for m in (1, 2, 5, 9):
        pairs = []
        for _ in range(m):
            s = rng.normal(size=n)
            pairs.append((s, A @ s))
        g = rng.normal(size=n)
        H = _dense_bfgs_inverse(pairs, n)
        np.testing.assert_allclose(oracle.lbfgs_direction(g, pairs), -H @ g, rtol=1e-11, atol=1e-13)
        # secant equation of the newest pair: H y = s
        s, y = pairs[-1]
        np.testing.assert_allclose(oracle.lbfgs_direction(y, pairs), -s, rtol=1e-10, atol=1e-12)
    # the order of the pairs matters (a reversed history is another matrix)
    assert np.abs(oracle.lbfgs_direction(g, pairs[::-1]) + _dense_bfgs_inverse(pairs, n) @ g).max() > 1e-6


def test_lbfgs_step_rules_and_convergence():
    """History bookkeeping, the line-search inequality and the fallback, on functions with known
    minimisers."""
    rng = np.random.default_rng(8)
    n = 6
    A = rng.normal(size=(n, n)); A = A @ A.T + np.eye(n)
    b = rng.normal(size=n)
    f = lambda x: 0.5 * x @ A @ x - b @ x
    grad = lambda x: A @ x - b
    x, st = np.zeros(n), {}
    for it in range(40):
        g = grad(x)
        if np.linalg.norm(g) < 1e-8:     # below this the decrease is lost in f's rounding
            break
        x_new, alpha, fv, trials, used = oracle.lbfgs_step(f, x, g, f(x), st, history=4)
        assert used == min(it, 4) and alpha == 0.5 ** (trials - 1)
        # accepted point satisfies the inequality with the direction actually used
        p = (x_new - x) / alpha
        assert fv <= f(x) + 1e-4 * alpha * (g @ p) + 1e-15
        if trials > 1:   # and the step before it did not
            assert f(x + 2 * alpha * p) > f(x) + 1e-4 * 2 * alpha * (g @ p)
        x = x_new
    np.testing.assert_allclose(x, np.linalg.solve(A, b), rtol=0, atol=1e-9)
    assert it < 30                                         # far fewer steps than steepest descent needs
    # history: pairs are (theta_k+1 - theta_k, g_k+1 - g_k), newest last, at most `history`
    assert len(st["pairs"]) == 4
    # a pair without positive curvature is not stored
    st = {"theta_prev": np.array([0.0, 0.0]), "g_prev": np.array([1.0, 0.0]), "pairs": []}
    q = lambda x: 0.5 * float(x @ x)
    _, _, _, _, used = oracle.lbfgs_step(q, np.array([1.0, 0.0]), np.array([0.5, 0.0]), 0.5, st)
    assert used == 0 and st["pairs"] == []                 # s.y = -0.5
    # nothing acceptable: parameters untouched, alpha = 0, history dropped
    up = lambda x: 1.0 + float(np.abs(x - 1.0).sum())
    st = {}
    th, alpha, fv, trials, used = oracle.lbfgs_step(up, np.array([1.0]), np.array([1.0]), 1.0, st, max_trials=4)
    assert (th.tolist(), alpha, fv, trials) == ([1.0], 0.0, 1.0, 4) and st["theta_prev"] is None
    # on the real loss: three iterations decrease it monotonically
    layers, in_ch, P = NETS["tiny18"]
    params = rand_params(layers, in_ch, P, 52)
    img = rng.uniform(0, 1, (1, in_ch, P + 2, P + 1))
    lab = rng.integers(0, 2, (1, P + 2, P + 1)).astype(np.int32)
    loss = lambda th: oracle.run(layers, in_ch, P, th, img, lab, want_probs=False)["loss"]
    st, th, hist = {}, params, []
    for it in range(3):
        r = oracle.run(layers, in_ch, P, th, img, lab, want_grads=True)
        th, alpha, fv, trials, used = oracle.lbfgs_step(loss, th, r["grads"], r["loss"], st, alpha0=1.0)
        assert alpha > 0 and fv < r["loss"] and used == it
        hist.append(fv)
    assert hist[0] > hist[1] > hist[2]


GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _golden_rows(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [ln.strip() for ln in f if ln.strip() and not ln.startswith("#")]


def test_fragment_counts_printed_in_the_paper():
    """|F_out| = |F_in| k^2 and the 4 fragments of the 2 x 2 illustration (Method, MPF layer;
    tests/golden/paper_fragment_counts.txt): the spacing of the oracle's whole-image maps after
    the pools, squared, is the number of fragments (tests/test_abi_host.py holds the library's
    plan to the same file)."""
    for row in _golden_rows("paper_fragment_counts.txt"):
        pools, want = row.split("|")
        pools, want = [int(t) for t in pools.split()], int(want)
        layers, side = [], 1
        for p in reversed(pools):              # build backwards from a 1 x 1 output: C 2x2 then MPF p
            side = side * p + 1
        patch = side
        for p in pools:
            layers += [(C, 2, 2), (MP, 0, p)]
        layers += [(FC, 2, 0)]
        layers = tuple(layers)
        img = np.zeros((1, 1, patch + 3, patch + 2))
        params = np.zeros(oracle.param_count(layers, 1, patch))
        last_pool = 2 * len(pools) - 1
        d = oracle.dense_layer(layers, 1, patch, params, img, last_pool)
        assert d["stride"] ** 2 == want, (pools, d["stride"])


def test_patches_per_image_printed_in_the_paper():
    """With mirrored borders every pixel of the image gets its patch: the steel images, 550 x 240
    down-sampled by 4, hold "roughly 8.2K patches" (Results; tests/golden/paper_patch_counts.txt)."""
    for row in _golden_rows("paper_patch_counts.txt"):
        h, w, down, window, want, tol = [int(t) for t in row.split("|")]
        H, W = h // down, w // down
        ext = oracle.mirror_pad(np.zeros((1, 1, H, W)), window)
        patches = (ext.shape[2] - window + 1) * (ext.shape[3] - window + 1)
        assert patches == H * W and abs(patches - want) <= tol, patches


def test_oracle_values_on_file():
    """The oracle still computes the values stored by tests/golden/make_oracle_values.py (its own,
    written once: a guard against silent changes of its arithmetic, not a pin)."""
    import importlib.util
    spec = importlib.util.spec_from_file_location("make_oracle_values", os.path.join(GOLDEN, "make_oracle_values.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    now = mod.values()
    stored = dict((k, float(v)) for k, v in (r.split() for r in _golden_rows("oracle_values_tiny.txt")))
    assert set(now) == set(stored)
    for k, v in stored.items():
        assert abs(now[k] - v) <= 1e-12 * max(1.0, abs(v)), (k, now[k], v)


def test_rectangular_pool_by_hand():
    """A 2 x 3 window over a 4 x 6 map (Background, layer MP: p_row x p_col sub-regions): the
    maxima, the tap codes u * p_col + v of the FIRST maximum, and where the deltas go; the
    whole-image map of the pooled layer is p_row apart in rows and p_col apart in columns, i.e.
    p_row * p_col fragments (Method, MPF layer: one fragment per offset of the pooling kernel)."""
    x = np.array([[1., 5., 2., 0., 0., 0.],
                  [3., 5., 4., 0., 7., 0.],
                  [9., 1., 1., 2., 2., 2.],
                  [1., 1., 9., 2., 2., 2.]])
    layers = ((MP, 0, 2, 3), (FC, 2, 0))                 # patch 4... needs a square patch: 6 x 6, two rows unused
    img = np.zeros((1, 1, 6, 6)); img[0, 0, :4] = x
    # FC over the 3 x 2 pooled map [[5, 7], [9, 2], [0, 0]]; weights pick each entry in turn
    pooled = np.array([[5., 7.], [9., 2.], [0., 0.]])
    n = oracle.param_count(layers, 1, 6)
    assert n == 2 * 6 + 2
    for e in range(4):
        params = np.zeros(n); params[e] = 1.0            # class-0 logit = pooled entry e (row-major)
        r = oracle.run(layers, 1, 6, params, img, np.zeros((1, 6, 6), dtype=np.int32), want_grads=True,
                       want_dimage=True, loss_fn="mse")
        assert abs(r["probs"][0, 0, 0, 0] - pooled.ravel()[e]) < 1e-15
        # the delta of class 0 (output - 1) lands on the FIRST maximum of window e
        want = np.zeros((6, 6))
        where = {0: (0, 1), 1: (1, 4), 2: (2, 0), 3: (2, 3)}[e]
        want[where] = pooled.ravel()[e] - 1.0
        np.testing.assert_allclose(r["dimage"][0, 0], want, atol=1e-15)
    d = oracle.dense_layer(layers, 1, 6, np.zeros(n), np.zeros((1, 1, 9, 8)), 0)
    assert (d["stride"], d["stride_cols"]) == (2, 3)
    assert d["act"].shape == (1, 1, 9 - 6 + (3 - 1) * 2 + 1, 8 - 6 + (2 - 1) * 3 + 1)
    codes = oracle.dense_layer(layers, 1, 6, np.zeros(n), img, 0)["codes"][0, 0]
    assert codes[0, 0] == 0 * 3 + 1 and codes[0, 3] == 1 * 3 + 1 and codes[2, 0] == 0 and codes[2, 3] == 0


def test_mirror_pad_by_hand():
    """Borders synthesised by mirroring, edge pixel repeated; c = (P-1)//2 above/left and
    P-1-c below/right, so that output (i,j) is the patch centred on input (i,j)
    (Experiments, membrane segmentation).  Written out for a 2x3 image and P = 4."""
    x = np.array([[1., 2., 3.], [4., 5., 6.]])[None, None]
    got = oracle.mirror_pad(x, 4)[0, 0]          # c = 1: one row/col before, two after
    want = np.array([[1., 1., 2., 3., 3., 2.],
                     [1., 1., 2., 3., 3., 2.],
                     [4., 4., 5., 6., 6., 5.],
                     [4., 4., 5., 6., 6., 5.],
                     [1., 1., 2., 3., 3., 2.]])
    np.testing.assert_array_equal(got, want)
    # the patch net on the extended image gives one output per input pixel, and an interior
    # output equals the plain valid-region output of the same patch
    layers, in_ch, P = NETS["tiny18"]
    rng = np.random.default_rng(21)
    params = rand_params(layers, in_ch, P, 22)
    img = rng.uniform(0, 1, (1, in_ch, 22, 25))
    same = oracle.run(layers, in_ch, P, params, oracle.mirror_pad(img, P))["probs"]
    valid = oracle.run(layers, in_ch, P, params, img)["probs"]
    assert same.shape[2:] == img.shape[2:]
    c = (P - 1) // 2
    np.testing.assert_array_equal(same[:, :, c:c + valid.shape[2], c:c + valid.shape[3]], valid)


def test_bad_descriptions_are_rejected():
    with pytest.raises(ValueError):
        oracle.param_count(((C, 2, 3), (MP, 0, 2)), 1, 8)          # must end with FC
    with pytest.raises(ValueError):
        oracle.param_count(((C, 2, 9), (FC, 2, 0)), 1, 8)          # kernel larger than patch
    with pytest.raises(ValueError):
        oracle.param_count(((FC, 4, 0), (C, 2, 1), (FC, 2, 0)), 1, 8)  # C after FC
    assert oracle.param_count(wl.CONFIGS[1].layers, 1, 44) == 89646
    assert oracle.param_count(wl.CONFIGS[3].layers, 1, 78) == 332186
    assert oracle.param_count(wl.CONFIGS[4].layers, 3, 78) == 335523
