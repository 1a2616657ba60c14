"""Writes tests/golden/zipf_alpha.json: the scale alpha of the Zipf(1.2) router bias
b_e = alpha * (-1.2 ln rank_e) for which, on the 'qwen_zipf_b2s2048' workload, the hottest
expert receives about 8x the mean number of routed rows.  Calls only the oracle (never the
HIP path).  Run:  python tests/golden/calibrate_zipf.py
The value is then copied into synth/workloads.py (ZIPF_ALPHA) by hand, with this file as
its provenance."""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import synth  # noqa: E402
from oracle import revffn_oracle as O  # noqa: E402


def main():
    wl = synth.WORKLOADS["qwen_zipf_b2s2048"]
    cfg = O.Config(wl.d_model, wl.n_heads, wl.head_dim, wl.n_experts, wl.top_k, wl.d_expert, wl.d_shared)
    W = synth.make_weights(wl, alpha=0.0, f64=False)
    small = {k: W[k] for k in ("norm_a1", "norm_a2", "norm_m", "pup_a", "pdn_a", "pup_m", "wq", "wk", "wv", "wo",
                               "bq", "bk", "bv", "w_router")}
    small = O.as_f64(small)
    x1, x2, _, _ = synth.make_inputs(wl)
    A, _ = O.attn_half_forward(x1, x2, small, cfg, wl.B, wl.S, keep_probs=False)
    y1 = x1 + A
    Um = O.rmsnorm(y1, small["norm_m"], cfg.rms_eps) @ small["pup_m"].T
    z0 = Um @ small["w_router"].T
    unit = synth.zipf_router_bias(wl, wl.seed, alpha=1.0)

    def ratio(alpha):
        b = np.float32(alpha * unit).astype(np.float64)          # b_router is float32 at the boundary
        idx, _, _ = O.route(z0 + b, cfg)
        counts = np.bincount(idx.reshape(-1), minlength=cfg.n_experts)
        return counts.max() / (wl.T * wl.top_k / cfg.n_experts), counts

    lo, hi = 0.0, 1.0
    for _ in range(30):
        mid = 0.5 * (lo + hi)
        if ratio(mid)[0] < 8.0:
            lo = mid
        else:
            hi = mid
    alpha = round(0.5 * (lo + hi), 4)
    r, counts = ratio(alpha)
    out = {"workload": wl.name, "alpha": alpha, "hottest_over_mean": float(r),
           "counts_sorted": sorted(int(c) for c in counts)[::-1],
           "logit_std_without_bias": float(z0.std())}
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "zipf_alpha.json"), "w") as f:
        json.dump(out, f, indent=1)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
