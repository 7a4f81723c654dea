"""Writes tests/golden/zipf_bias_<config>.txt: the additive router-logit bias
that skews a config's routing toward Zipf(s) expert shares.  The bias is an
INPUT of the skewed-routing stress case; it is found with the CPU oracle's own
router on the seeded synthetic x and W_gate, and calls nothing but oracle/ and
the input generator.

    python -m oracle.make_zipf_bias C2
"""
import os
import sys

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
import workloads as wl  # noqa: E402
from oracle import modse_oracle as orc  # noqa: E402


def main(name):
    cfg = wl.CONFIGS[name]
    T, d, N = cfg.n_tokens, cfg.d_model, cfg.n_experts
    x = wl._normal(cfg.seed, "x", (T, d), 1.0, cfg.dtype)
    Wg = wl._normal(cfg.seed, "W_gate", (d, N), 0.02, cfg.dtype)
    target = wl.zipf_target_shares(cfg.d_ff, cfg.zipf_s)
    bias, share = orc.calibrate_logit_bias(x, Wg, N, cfg.top_k, target)
    bias = bias.astype(np.float32)
    r = orc.route(x, Wg, N, cfg.top_k, bias)
    share = r.counts / r.counts.sum()
    out = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "tests", "golden",
                       f"zipf_bias_{name}.txt")
    with open(out, "w") as fh:
        fh.write(f"# Router logit bias for config {name}: expert shares of the T*k assignments follow\n")
        fh.write(f"# Zipf(s={cfg.zipf_s}) by descending expert width.  Written by oracle/make_zipf_bias.py\n")
        fh.write("# from the CPU oracle's router on the seeded synthetic inputs (T=%d, seed %d).\n" % (T, cfg.seed))
        fh.write("# target shares:   " + " ".join(f"{v:.4f}" for v in target) + "\n")
        fh.write("# realised shares: " + " ".join(f"{v:.4f}" for v in share) + "\n")
        fh.write("# realised counts: " + " ".join(str(int(v)) for v in r.counts) + "\n")
        for v in bias:
            fh.write(repr(float(v)) + "\n")
    print(out, share, np.abs(share - target).max())


if __name__ == "__main__":
    main(sys.argv[1] if len(sys.argv) > 1 else "C2")
