"""Chooses the sharpening factor alpha of the skewed-routing workload and records the realised load histogram.

Rule: the smallest alpha in {1.0, 1.25, 1.5, ...} for which, on the DeepSeek-MoE-16B-shaped layer with
bias[e] = -alpha * 1.2 * ln(rank_e), the busiest expert receives at least 9x the mean number of rows AND at
least one expert receives none.  (A token picks an expert at most once, so max/mean <= E/k = 10.67.)

Calls only the CPU oracle and the input generator.  Run from the repository root:
    python tests/golden/make_skew_alpha.py
It prints the chosen alpha (to be set as skew_alpha of config "dsmoe16b_skew" in xmoe_inputs.py) and writes
tests/golden/skew_histogram.txt.
"""
import dataclasses
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
import xmoe_inputs as xi  # noqa: E402


def main():
    base = xi.CONFIGS["dsmoe16b_skew"]
    x, w = xi.make_x(base), xi.make_w_router(base)
    logits0 = oracle.gate_logits_contract(x, w, None)
    alpha = 1.0
    while True:
        cfg = dataclasses.replace(base, skew_alpha=alpha)
        bias = xi.make_gate_bias(cfg)
        # the contract adds the bias last, in float32
        logits = (logits0 + bias[None, :]).astype(np.float32)
        idx, _, _ = oracle.route(logits, cfg.k)
        tpe = np.bincount(idx.reshape(-1), minlength=cfg.E)
        ratio = tpe.max() / tpe.mean()
        print(f"alpha={alpha:.2f} max/mean={ratio:.3f} empty={int((tpe == 0).sum())}")
        if ratio >= 9.0 and (tpe == 0).any():
            break
        alpha += 0.25
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "skew_histogram.txt")
    with open(out, "w") as fh:
        fh.write("# tokens_per_expert of config dsmoe16b_skew (T=8192, E=64, k=6), written by make_skew_alpha.py\n")
        fh.write(f"# alpha={alpha} max/mean={ratio:.4f} empty_experts={int((tpe == 0).sum())}\n")
        fh.write(" ".join(str(int(v)) for v in tpe) + "\n")
    print("chosen alpha:", alpha)


if __name__ == "__main__":
    main()
