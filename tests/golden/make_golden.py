"""Writes tests/golden/tiny_layer_step.txt from the CPU oracle alone.

The paper prints no worked numeric example for the layer step (Sec. 2.3 gives
Eq. 3-5 only), so this fixture is not a paper value: it freezes what the pinned
oracle returns on the tiny workload, so that a later change to the oracle's
arithmetic cannot pass unnoticed.  Run: python tests/golden/make_golden.py
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import relserve_oracle  # noqa: E402
from paper_2601_11546_amd import workloads as W  # noqa: E402

SAMPLES = [(0, 0), (0, 255), (17, 3), (63, 128), (64, 1), (127, 200), (128, 0), (129, 77), (133, 255), (131, 31)]


def compute():
    wl = W.workload_tiny()
    weights = W.make_weights(wl.shape, wl.seed)
    x = W.make_activations(wl.batch.T, wl.shape.hidden, wl.seed)
    kp, vp = W.make_cache(wl.shape, wl.batch.num_pages, wl.seed)
    res = relserve_oracle.load("f32").layer_step(wl.shape, wl.batch, weights, x, kp, vp)
    return res, kp, vp


def main():
    res, kp, vp = compute()
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_layer_step.txt")
    with open(path, "w") as f:
        f.write("# oracle output on workload_tiny(seed=1000): y[row, col] fp32 as hex, then cache checksums\n")
        f.write("# source: oracle/relserve_oracle.c via tests/golden/make_golden.py (no paper value exists for this path)\n")
        for r, c in SAMPLES:
            f.write(f"y {r} {c} {float(res.y_f32[r, c]).hex()}\n")
        f.write(f"sum_y_bf16 {int(res.y_bf16.astype(np.uint64).sum())}\n")
        f.write(f"sum_k_pages {int(kp.astype(np.uint64).sum())}\n")
        f.write(f"sum_v_pages {int(vp.astype(np.uint64).sum())}\n")
    print("wrote", path)


if __name__ == "__main__":
    main()
