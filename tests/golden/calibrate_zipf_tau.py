"""Calibrate the gate-bias scale tau of the skewed workload (calls only the oracle).

The bias is tau * ln(p_e) with p_e ~ (e+1)^-1.2.  Logit noise is Gaussian, not
Gumbel, so tau = 1 does not reproduce p_e; tau is bisected until expert 0
receives 36.5 % (+-0.5 %) of first choices on the seed-0 inputs.  The result is
snapped to a multiple of 2^-7 and written to zipf_tau.txt with the realised
histograms; paper_2506_22175_amd/synth.py carries the same constant.

Run from the repository root:  python tests/golden/calibrate_zipf_tau.py
"""
import dataclasses
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import moe_oracle as O          # noqa: E402
from paper_2506_22175_amd import synth      # noqa: E402


def share(tau):
    s = dataclasses.replace(synth.WORKLOADS["skewed"], zipf_tau=tau)
    d = synth.make_inputs(s, seed=0)
    logits, p, idx, w = O.route(d["x"], d["Wg"], s.k, d["gate_bias"])
    return s, idx


def main():
    lo, hi = 0.0, 4.0
    for _ in range(20):
        mid = 0.5 * (lo + hi)
        _, idx = share(mid)
        if np.mean(idx[:, 0] == 0) < 0.365:
            lo = mid
        else:
            hi = mid
    tau = round(0.5 * (lo + hi) * 128) / 128
    s, idx = share(tau)
    n = 4
    C_p = O.capacity(s.T, s.E, s.k, s.capacity_factor, n)
    slot, counts = O.assign_slots(idx, s.E, C_p, n)
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "zipf_tau.txt")
    with open(out, "w") as f:
        f.write("# written by tests/golden/calibrate_zipf_tau.py (oracle router, seed 0, skewed workload)\n")
        f.write(f"tau {tau!r}\n")
        f.write("top1_share " + " ".join(f"{np.mean(idx[:, 0] == e):.4f}" for e in range(s.E)) + "\n")
        f.write("top2_share " + " ".join(f"{np.mean(idx[:, 1] == e):.4f}" for e in range(s.E)) + "\n")
        f.write(f"capacity_per_partition {C_p}\n")
        f.write(f"kept_rows {int(counts.sum())}\n")
        f.write(f"drop_rate {float(np.mean(slot < 0)):.4f}\n")
    print(open(out).read())


if __name__ == "__main__":
    main()
