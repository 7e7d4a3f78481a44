"""Seeded synthetic inputs for the five benchmark configurations.

This module only *generates inputs* (images, per-pixel labels, parameter
vectors, pixel subsets).  It holds none of the network's arithmetic and is the
one module that both the CPU oracle's tests and the HIP path's tests/bench may
import; it depends on numpy alone.

The images stand in for the paper's two data sets (Results, "Membrane
Segmentation" and "Steel Defect Detection"): grayscale frames in which sparse
elongated defects cover part of the image and every pixel carries a class
label.  Neither data set is reproduced here; shapes and statistics follow the
benchmark configuration list, the generator details are this build's own.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Tuple

import numpy as np

# layer kinds, shared numbering with the C ABI and the oracle (plain integers)
C, MP, FC = 0, 1, 2


@dataclass(frozen=True)
class Workload:
    """One benchmark configuration: network, input shape, seeds."""
    name: str
    layers: Tuple[Tuple[int, int, int], ...]   # (kind, maps, k): C maps,k ; MP -,p ; FC maps,-
    patch: int                                 # side of the patch one output pixel sees
    in_channels: int
    n_classes: int
    batch: int
    height: int
    width: int
    weight_amp: float                          # parameters ~ U[-a, a]
    shapes: str                                # "bernoulli" | "rects" | "ellipses"
    dtype: str = "f32"                         # storage type asked of the HIP path
    lr: float = 0.0
    sgd_steps: int = 0
    seed_image: int = 0
    seed_label: int = 0
    seed_param: int = 0

    @property
    def out_h(self) -> int:
        return self.height - self.patch + 1

    @property
    def out_w(self) -> int:
        return self.width - self.patch + 1

    @property
    def valid_pixels(self) -> int:
        return self.batch * self.out_h * self.out_w


def _net(*spec):
    out = []
    for s in spec:
        if s[0] == "C":
            out.append((C, s[1], s[2]))
        elif s[0] == "MP":
            out.append((MP, 0, s[1]))
        else:
            out.append((FC, s[1], 0))
    return tuple(out)


_NET_TINY = _net(("C", 2, 3), ("MP", 2), ("C", 3, 3), ("MP", 2), ("FC", 8), ("FC", 2))
_NET_44 = _net(("C", 16, 5), ("MP", 2), ("C", 32, 5), ("MP", 2), ("C", 64, 3), ("MP", 2),
               ("FC", 100), ("FC", 2))
_NET_78 = _net(("C", 32, 7), ("MP", 2), ("C", 64, 5), ("MP", 2), ("C", 64, 5), ("MP", 2),
               ("C", 128, 3), ("MP", 2), ("FC", 200), ("FC", 2))
_NET_78_3 = _NET_78[:-1] + ((FC, 3, 0),)

CONFIGS: List[Workload] = [
    Workload("cfg0_tiny_64", _NET_TINY, 18, 1, 2, 1, 64, 64, 0.1, "bernoulli",
             seed_image=1000, seed_label=2000, seed_param=3000),
    Workload("cfg1_steel44_256", _NET_44, 44, 1, 2, 1, 256, 256, 0.05, "rects",
             seed_image=1001, seed_label=2001, seed_param=3001),
    Workload("cfg2_steel44_8x512_sgd", _NET_44, 44, 1, 2, 8, 512, 512, 0.05, "rects",
             lr=1e-3, sgd_steps=10, seed_image=1002, seed_label=2002, seed_param=3002),
    Workload("cfg3_deep78_1024", _NET_78, 78, 1, 2, 1, 1024, 1024, 0.05, "rects",
             seed_image=1003, seed_label=2003, seed_param=3003),
    Workload("cfg4_deep78_rgb_2x2048_bf16", _NET_78_3, 78, 3, 3, 2, 2048, 2048, 0.05, "ellipses",
             dtype="bf16", seed_image=1004, seed_label=2004, seed_param=3004),
]


def param_count(layers, in_channels: int, patch: int) -> int:
    """Number of parameters (all W then b, layer by layer) - bookkeeping only."""
    rows, cols, ch, total, seen_fc = patch, patch, in_channels, 0, False
    for layer in layers:
        kind, maps, k = layer[:3]
        k2 = layer[3] if len(layer) > 3 and layer[3] else k     # columns of a pooling window
        if kind == C:
            total += maps * ch * k * k + maps
            rows, cols, ch = rows - k + 1, cols - k + 1, maps
        elif kind == MP:
            rows, cols = rows // k, cols // k2
        else:
            kk = 1 if seen_fc else rows * cols
            total += maps * ch * kk + maps
            rows, cols, ch, seen_fc = 1, 1, maps, True
    return total


def round_bf16(x: np.ndarray) -> np.ndarray:
    """fp32 values rounded to the nearest bf16 (ties to even), returned as fp32.  Inputs of a
    bf16-storage workload are generated representable, so that rounding the stored weights and
    image is not a source of difference between the two sides."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(np.shape(x))


def make_params(wl: Workload, dtype=np.float32) -> np.ndarray:
    """Flat parameter vector, per layer W[o][c][u][v] then b[o], all ~ U[-a, a]."""
    n = param_count(wl.layers, wl.in_channels, wl.patch)
    rng = np.random.default_rng(wl.seed_param)
    p = rng.uniform(-wl.weight_amp, wl.weight_amp, size=n).astype(np.float32)
    if wl.dtype == "bf16":
        p = round_bf16(p)
    return p.astype(dtype)


def _rects(rng, img, lab):
    """Axis-aligned elongated bright/dark rectangles, long side 5..40 px."""
    _, H, W = img.shape
    n = max(1, int(round(H * W / 8192.0)))
    for _ in range(n):
        long_side = int(rng.integers(5, 41))
        short_side = int(rng.integers(5, max(5, long_side // 3) + 1))
        if rng.random() < 0.5:
            h, w = long_side, short_side
        else:
            h, w = short_side, long_side
        y0 = int(rng.integers(0, max(1, H - h + 1)))
        x0 = int(rng.integers(0, max(1, W - w + 1)))
        amp = rng.uniform(0.3, 0.5)
        if rng.random() < 0.5:
            amp = -amp
        img[:, y0:y0 + h, x0:x0 + w] += amp
        lab[y0:y0 + h, x0:x0 + w] = 1
    np.clip(img, 0.0, 1.0, out=img)


def _ellipses(rng, img, lab):
    """Rotated ellipses, diameters 10..80 px, class 1 or 2, later shapes overwrite."""
    Cc, H, W = img.shape
    n = max(1, int(round(H * W / 32768.0)))
    for _ in range(n):
        a = rng.integers(10, 81) / 2.0
        b = rng.integers(10, 81) / 2.0
        cy, cx = rng.uniform(0, H), rng.uniform(0, W)
        th = rng.uniform(0, np.pi)
        cls = 1 if rng.random() < 0.5 else 2
        shift = rng.uniform(-0.4, 0.4, size=Cc)
        r = int(np.ceil(max(a, b))) + 1
        y0, y1 = max(0, int(cy) - r), min(H, int(cy) + r + 1)
        x0, x1 = max(0, int(cx) - r), min(W, int(cx) + r + 1)
        if y0 >= y1 or x0 >= x1:
            continue
        yy, xx = np.mgrid[y0:y1, x0:x1]
        dy, dx = yy - cy, xx - cx
        ct, st = np.cos(th), np.sin(th)
        inside = ((dx * ct + dy * st) / a) ** 2 + ((-dx * st + dy * ct) / b) ** 2 <= 1.0
        for c in range(Cc):
            img[c, y0:y1, x0:x1][inside] += shift[c]
        lab[y0:y1, x0:x1][inside] = cls
    np.clip(img, 0.0, 1.0, out=img)


def make_inputs(wl: Workload, dtype=np.float32):
    """Returns (image [B,C,H,W] in [0,1], labels int32 [B,H,W])."""
    rng_i = np.random.default_rng(wl.seed_image)
    rng_l = np.random.default_rng(wl.seed_label)
    img = rng_i.uniform(0.0, 1.0, size=(wl.batch, wl.in_channels, wl.height, wl.width))
    lab = np.zeros((wl.batch, wl.height, wl.width), dtype=np.int32)
    for b in range(wl.batch):
        if wl.shapes == "bernoulli":
            lab[b] = (rng_l.random((wl.height, wl.width)) < 0.2).astype(np.int32)
        elif wl.shapes == "rects":
            _rects(rng_l, img[b], lab[b])
        elif wl.shapes == "ellipses":
            _ellipses(rng_l, img[b], lab[b])
        else:
            raise ValueError(wl.shapes)
    img = img.astype(np.float32)
    if wl.dtype == "bf16":
        img = round_bf16(img)
    return img.astype(dtype), lab


def crop(wl: Workload, batch: int, height: int, width: int, name_suffix="_crop") -> Workload:
    """Same network on a smaller input (for full-oracle parity at real layer shapes)."""
    from dataclasses import replace
    return replace(wl, name=wl.name + name_suffix, batch=batch, height=height, width=width)


def sample_pixels(wl: Workload, n: int, seed: int) -> np.ndarray:
    """Seeded subset of output pixels as flat indices into [B, out_h, out_w].

    Always holds the four corners of image 0 and a few pixels of the first and
    last output row/column; the rest is uniform without replacement.
    """
    B, oh, ow = wl.batch, wl.out_h, wl.out_w
    must = {0, ow - 1, (oh - 1) * ow, oh * ow - 1,
            ow // 2, (oh - 1) * ow + ow // 3, (oh // 2) * ow, (oh // 3) * ow + ow - 1,
            (B - 1) * oh * ow + oh * ow - 1}
    rng = np.random.default_rng(seed)
    total = B * oh * ow
    n = min(n, total)
    picked = set(int(v) for v in must if 0 <= v < total)
    while len(picked) < n:
        for v in rng.integers(0, total, size=n - len(picked)):
            picked.add(int(v))
    return np.array(sorted(picked), dtype=np.int64)


def sample_pixels_stratified(wl: Workload, n: int, seed: int, modulus: int = 16, blocks: int = 4) -> np.ndarray:
    """Seeded subset of about n output pixels, as flat indices into [B, out_h, out_w], laid out so
    that a fault confined to one part of a kernel's index space cannot hide between samples:

    * every residue class (i mod modulus, j mod modulus) gets the same number of pixels
      (modulus 16 = the largest tap spacing of the benchmark nets: every fragment of every layer),
    * the pixels of a class are dealt round-robin over a blocks x blocks grid of image regions and
      over the images of the batch (so every tile row / tile column of a launch, whatever its
      tiling, has samples in several classes),
    * the first and last output row and column of every image carry extra pixels, corners included.
    """
    B, oh, ow = wl.batch, wl.out_h, wl.out_w
    rng = np.random.default_rng(seed)
    picked = set()
    m = min(modulus, oh, ow)
    per = max(1, n // (m * m))
    turn = 0
    for ri in range(m):
        for rj in range(m):
            for _ in range(per):
                b = turn % B
                bi, bj = (turn // B) % blocks, (turn // (B * blocks)) % blocks
                turn += 1
                # rows of region bi with residue ri
                lo_i, hi_i = bi * oh // blocks, (bi + 1) * oh // blocks
                lo_j, hi_j = bj * ow // blocks, (bj + 1) * ow // blocks
                rows = np.arange(ri, oh, m)
                cols = np.arange(rj, ow, m)
                rows_in = rows[(rows >= lo_i) & (rows < hi_i)]
                cols_in = cols[(cols >= lo_j) & (cols < hi_j)]
                i = int(rng.choice(rows_in if rows_in.size else rows))
                j = int(rng.choice(cols_in if cols_in.size else cols))
                picked.add((b * oh + i) * ow + j)
    edge = max(4, n // 64)
    for b in range(B):
        base = b * oh * ow
        for i, j in ((0, 0), (0, ow - 1), (oh - 1, 0), (oh - 1, ow - 1)):
            picked.add(base + i * ow + j)
        for j in rng.integers(0, ow, size=edge):
            picked.add(base + int(j))
            picked.add(base + (oh - 1) * ow + int(j))
        for i in rng.integers(0, oh, size=edge):
            picked.add(base + int(i) * ow)
            picked.add(base + int(i) * ow + ow - 1)
    return np.array(sorted(picked), dtype=np.int64)
