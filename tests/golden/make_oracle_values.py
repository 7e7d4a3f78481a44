"""Writes tests/golden/oracle_values_tiny.txt: loss, probabilities and gradient sums of the fp64
oracle on a small seeded case.  Calls nothing but `oracle/` and numpy; the stored values guard the
oracle's arithmetic against silent changes (they are the oracle's own, so they pin nothing by
themselves - the pins are in tests/test_oracle_pins.py).

    python tests/golden/make_oracle_values.py
"""
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))
import oracle  # noqa: E402

C, MP, FC = 0, 1, 2
LAYERS = ((C, 2, 3), (MP, 0, 2), (C, 3, 3), (MP, 0, 2), (FC, 8, 0), (FC, 2, 0))   # patch 18 -> 16 -> 8 -> 6 -> 3
IN_CH, PATCH, H, W = 1, 18, 21, 20


def case():
    rng = np.random.default_rng(20130207)
    params = rng.uniform(-0.5, 0.5, oracle.param_count(LAYERS, IN_CH, PATCH))
    img = rng.uniform(0, 1, (1, IN_CH, H, W))
    lab = rng.integers(0, 2, (1, H, W)).astype(np.int32)
    return params, img, lab


def values():
    params, img, lab = case()
    out = {}
    for squash in ("tanh", "logistic"):
        for loss_fn in ("mcce", "mse"):
            r = oracle.run(LAYERS, IN_CH, PATCH, params, img, lab, want_grads=True, loss_fn=loss_fn, squash=squash)
            key = "%s_%s" % (squash, loss_fn)
            out[key + "_loss"] = r["loss"]
            out[key + "_probs_sum_class0"] = float(r["probs"][0, 0].sum())
            out[key + "_probs_first"] = float(r["probs"][0, 0, 0, 0])
            out[key + "_grads_sum"] = float(r["grads"].sum())
            out[key + "_grads_abs_sum"] = float(np.abs(r["grads"]).sum())
            out[key + "_grads_last"] = float(r["grads"][-1])
    return out


if __name__ == "__main__":
    with open(os.path.join(HERE, "oracle_values_tiny.txt"), "w") as f:
        f.write("# written by tests/golden/make_oracle_values.py (fp64 oracle, seed 20130207); name value\n")
        for k, v in values().items():
            f.write("%s %.17g\n" % (k, v))
    print("wrote oracle_values_tiny.txt")
