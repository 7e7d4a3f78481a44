"""Host-side checks of libmpcnn that need no GPU: the library loads, exports every
symbol include/mpcnn.h declares, and its layer plan (shapes, parameter counts,
errors) agrees with the paper's definitions and with the oracle's bookkeeping."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
from paper_1302_1690_amd import mpcnn, workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
C, MP, FC = 0, 1, 2


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "mpcnn.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(mpcnn_[a-z_]+)\s*\(", hdr))
    assert declared == set(mpcnn.SYMBOLS), declared ^ set(mpcnn.SYMBOLS)
    lib = ctypes.CDLL(mpcnn.LIB_PATH)
    for name in sorted(declared):
        assert hasattr(lib, name), name


@pytest.mark.parametrize("cfg", wl.CONFIGS[:4], ids=lambda c: c.name)
def test_plan_matches_configs(cfg):
    net = mpcnn.Net(cfg.layers, cfg.in_channels, cfg.patch)
    assert net.patch == cfg.patch
    assert net.n_classes == cfg.n_classes
    assert net.param_count == wl.param_count(cfg.layers, cfg.in_channels, cfg.patch)
    assert net.param_count == oracle.param_count(cfg.layers, cfg.in_channels, cfg.patch)
    last = len(cfg.layers) - 1
    r, c, ch, sp = net.layer_shape(cfg.height, cfg.width, last)
    assert (r, c, ch) == (cfg.out_h, cfg.out_w, cfg.n_classes)
    assert net.workspace_bytes(cfg.batch, cfg.height, cfg.width, True) > \
        net.workspace_bytes(cfg.batch, cfg.height, cfg.width, False) > 0
    net.close()


def test_dense_shapes_follow_fragment_rule():
    """Each MPF layer multiplies the spacing by k (k^2 fragments, Method, MPF layer);
    the dense map of a layer is what the oracle gets by laying all patches out."""
    cfg = wl.CONFIGS[0]
    net = mpcnn.Net(cfg.layers, 1, cfg.patch)
    img = np.zeros((1, 1, 40, 36))
    params = np.zeros(net.param_count)
    for layer in range(len(cfg.layers)):
        d = oracle.dense_layer(cfg.layers, 1, cfg.patch, params, img, layer)
        r, c, ch, sp = net.layer_shape(40, 36, layer)
        assert d["act"].shape == (1, ch, r, c)
        assert d["stride"] == sp
    spacings = [net.layer_shape(40, 36, l)[3] for l in range(len(cfg.layers))]
    assert spacings == [1, 2, 2, 4, 4, 4]


def test_dense_shapes_with_dropped_rows():
    """Pools on sides that are not multiples of the pooling side (floor): the whole-image maps
    have the sizes the oracle gets by laying all patches out."""
    layers = ((C, 8, 3), (MP, 0, 3), (C, 8, 3), (MP, 0, 2), (FC, 12, 0), (FC, 2, 0))   # 18 -> 16 -> 5 -> 3 -> 1
    net = mpcnn.Net(layers, 1, 18)
    img = np.zeros((1, 1, 31, 27))
    params = np.zeros(net.param_count)
    for layer in range(len(layers)):
        d = oracle.dense_layer(layers, 1, 18, params, img, layer)
        r, c, ch, sp = net.layer_shape(31, 27, layer)
        assert d["act"].shape == (1, ch, r, c), layer
        assert d["stride"] == sp
    assert net.layer_shape(31, 27, len(layers) - 1)[:2] == (31 - 17, 27 - 17)
    net.close()


def test_fragment_counts_printed_in_the_paper():
    """|F_out| = |F_in| k^2 (Method, MPF layer; tests/golden/paper_fragment_counts.txt): the
    spacing the library plans after the pools, squared, is the number of fragments."""
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "paper_fragment_counts.txt")
    rows = [ln.strip() for ln in open(path) if ln.strip() and not ln.startswith("#")]
    assert rows
    for row in rows:
        pools, want = row.split("|")
        pools, want = [int(t) for t in pools.split()], int(want)
        side = 1
        for p in reversed(pools):              # backwards from a 1 x 1 output: C 2x2 then MPF p
            side = side * p + 1
        layers = []
        for p in pools:
            layers += [(C, 2, 2), (MP, 0, p)]
        layers = tuple(layers + [(FC, 2, 0)])
        net = mpcnn.Net(layers, 1, side)
        assert net.layer_shape(side + 3, side + 2, 2 * len(pools) - 1)[3] ** 2 == want
        net.close()


def test_dense_shapes_with_rectangular_pools():
    """p_row x p_col pooling windows: the library's whole-image maps have the sizes and the row
    spacing of the oracle's (Background, layer MP)."""
    layers = ((C, 4, 3), (MP, 0, 3, 2), (C, 6, 2), (MP, 0, 2, 3), (FC, 10, 0), (FC, 3, 0))   # 20 -> 18 -> 6x9 -> 5x8 -> 2x2
    net = mpcnn.Net(layers, 1, 20)
    assert net.param_count == oracle.param_count(layers, 1, 20) == wl.param_count(layers, 1, 20)
    img = np.zeros((1, 1, 29, 33))
    params = np.zeros(net.param_count)
    for layer in range(len(layers)):
        d = oracle.dense_layer(layers, 1, 20, params, img, layer)
        r, c, ch, sp = net.layer_shape(29, 33, layer)
        assert d["act"].shape == (1, ch, r, c), layer
        assert d["stride"] == sp
    net.close()


def test_errors():
    with pytest.raises(mpcnn.MpcnnError) as e:
        mpcnn.Net(((C, 2, 3), (MP, 0, 2)), 1, 8)
    assert e.value.status == 2                       # must end with FC
    with pytest.raises(mpcnn.MpcnnError) as e:
        mpcnn.Net(((C, 2, 9), (FC, 2, 0)), 1, 8)
    assert e.value.status == 2                       # filter larger than the map
    mpcnn.Net(((C, 2, 2), (MP, 0, 2), (FC, 2, 0)), 1, 8).close()   # 7 is not a multiple of 2: a row is dropped
    with pytest.raises(mpcnn.MpcnnError) as e:
        mpcnn.Net(((FC, 4, 0), (C, 2, 1), (FC, 2, 0)), 1, 8)
    assert e.value.status == 2
    with pytest.raises(mpcnn.MpcnnError) as e:
        mpcnn.Net(((FC, 2, 0),), 1, 8, dtype=7)
    assert e.value.status == 1
    with pytest.raises(mpcnn.MpcnnError) as e:
        mpcnn.Net(((FC, 2, 0),), 0, 8)
    assert e.value.status == 1
    net = mpcnn.Net(wl.CONFIGS[0].layers, 1, 18)
    assert net.workspace_bytes(1, 17, 64, True) == 0  # image smaller than the patch
    with pytest.raises(mpcnn.MpcnnError):
        net.layer_shape(64, 64, 99)
    with pytest.raises(mpcnn.MpcnnError):
        net.get_params()                              # never set
    assert "never set" in mpcnn.lib().mpcnn_last_error().decode()


def test_banded_workspace_grows_with_the_band():
    """A pass over bands sizes its workspace by the tallest band; the last band is shorter, so
    the size must not shrink when the band grows (host logic only: no device is touched)."""
    from paper_1302_1690_amd import mpcnn, workloads as wl
    L = mpcnn.lib()
    C, MP, FC = 0, 1, 2
    nets = [(wl.CONFIGS[1].layers, wl.CONFIGS[1].in_channels, wl.CONFIGS[1].patch, 1, 300),
            (wl.CONFIGS[3].layers, wl.CONFIGS[3].in_channels, wl.CONFIGS[3].patch, 1, 200),
            (((C, 8, 7), (MP, 0, 2), (C, 48, 2), (FC, 100, 0), (FC, 3, 0)), 1, 14, 3, 39)]
    for layers, cin, patch, B, W in nets:
        net = mpcnn.Net(layers, cin, patch)
        prev = 0
        for band in range(1, 120):
            n = L.mpcnn_workspace_bytes_banded(net._h, B, W, band)
            assert n >= prev > -1, (layers, band, n, prev)
            prev = n
        net.close()
