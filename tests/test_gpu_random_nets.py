"""Seeded random nets through the HIP path against the fp64 oracle, full image, every output
pixel: two or three convolution / pooling levels, 4-128 maps, 2x2-5x5 filters, pools of side
2-4 (also ones that drop trailing rows), 1 or 3 image channels, 2-4 classes, batches of 1-2,
ragged image sizes, both losses, both squashing functions, pixel weights and ignored labels
mixed in.  A bounded sample of the space the committed cases do not enumerate; the run stops at
its first failure, whose case line names the net."""
import numpy as np
import pytest

import test_gpu_parity as T
from paper_1302_1690_amd import workloads as wl

pytestmark = pytest.mark.gpu

C, MP, FC = 0, 1, 2


def random_case(rng, idx, dtype):
    """One net and input size; None if the draw is too large for a full-oracle check."""
    bf = dtype == "bf16"
    chans = [8, 12, 16, 20, 32, 36, 48, 64, 100, 128] if bf else [4, 8, 12, 16, 20, 32, 36, 48, 64, 100, 128]
    k1, p1, k2 = int(rng.choice([2, 3, 5])), int(rng.choice([2, 3, 4])), int(rng.choice([2, 3, 5]))
    c1, c2 = int(rng.choice(chans[:7])), int(rng.choice(chans))
    hidden = int(rng.choice([8, 16, 32, 40, 100]))
    n_cls, c_in = int(rng.choice([2, 3, 4])), int(rng.choice([1, 1, 3]))
    two = rng.random() < 0.6
    p2 = int(rng.choice([2, 3])) if two else 1
    m_fc = int(rng.integers(1, 4))                     # side of the map the first FC sees
    drop2 = int(rng.integers(0, p2)) if two else 0     # rows a floor pool drops
    drop1 = int(rng.integers(0, p1))
    side2 = m_fc * p2 + drop2 + (k2 - 1)               # before the second convolution
    patch = side2 * p1 + drop1 + (k1 - 1)
    if patch > 34:
        return None
    layers = [(C, c1, k1), (MP, 0, p1), (C, c2, k2)] + ([(MP, 0, p2)] if two else []) + [(FC, hidden, 0), (FC, n_cls, 0)]
    batch = int(rng.choice([1, 1, 2]))
    height, width = patch + int(rng.integers(0, 130)), patch + int(rng.integers(0, 130))
    work = batch * (height - patch + 1) * (width - patch + 1) * (
        c1 * k1 * k1 * c_in * patch ** 2 + c2 * c1 * k2 * k2 * side2 ** 2 + hidden * c2 * m_fc * m_fc)
    if work > 1.5e11:                                  # oracle flops: keeps a case to about a second
        return None
    amp = float(rng.choice([0.05, 0.1, 0.2] if bf else [0.15, 0.3]))
    cfg = wl.Workload("random_%s_%d" % (dtype, idx), tuple(layers), patch, c_in, n_cls, batch, height, width, amp,
                      "ellipses", dtype=dtype, seed_image=int(rng.integers(1, 10 ** 6)),
                      seed_label=int(rng.integers(1, 10 ** 6)), seed_param=int(rng.integers(1, 10 ** 6)))
    opts = dict(with_pixw=bool(rng.random() < 0.5), check_layers=bool(rng.random() < 0.5),
                squash="logistic" if rng.random() < 0.4 else "tanh", loss_fn="mse" if rng.random() < 0.5 else "mcce",
                ignore_some=bool(rng.random() < 0.3))
    return cfg, opts


def run_cases(seed, n_cases, dtype):
    rng = np.random.default_rng(seed)
    done = 0
    while done < n_cases:
        case = random_case(rng, done, dtype)
        if case is None:
            continue
        cfg, opts = case
        T.say("%s: layers %s, %d channels, %s" % (cfg.name, list(cfg.layers), cfg.in_channels, opts))
        T.full_parity(cfg, **opts)
        done += 1


def test_random_nets_fp32_storage():
    run_cases(20261, 20, "f32")


def test_random_nets_bf16_storage():
    run_cases(20262, 10, "bf16")


def test_bf16_long_reduction_behind_large_weights():
    """A second hidden layer that sums 1200 products of bf16-rounded inputs with weights of
    amplitude 0.3: its stored outputs differ from the oracle's by up to 0.027, which is the
    rounding of the layer below carried through the sum (`bf16_sigma`: rms 0.007), not a kernel
    fault - the bar on stored activations follows the arithmetic, the 2e-2 on probabilities
    and gradients is met."""
    layers = ((C, 48, 3), (MP, 0, 2), (C, 48, 5), (FC, 32, 0), (FC, 4, 0))   # 16 -> 14 -> 7 -> 3 -> FC over 3x3
    cfg = wl.Workload("bf16_long_sum", layers, 16, 1, 4, 1, 47, 110, 0.3, "ellipses", dtype="bf16",
                      seed_image=1121, seed_label=2121, seed_param=3121)
    assert T.act_bar(cfg, 2) > 2e-2 and T.tau_of(cfg) >= 2.0 ** -7
    T.full_parity(cfg)
