"""Timing helpers shared by bench.py and the GPU tests: how fast the expert GEMMs and the
permutation kernels run alone and side by side (the slowdown factors of Section II-C), per number
of compute units the GEMMs leave free.  Device-memory plumbing and HIP-event bookkeeping only; all
kernels are the library's."""
from __future__ import annotations

import time
from typing import Dict, Sequence

import torch

from . import binding as B
from . import runner

GEMM_KINDS = ("gemm_fwd1_gelu", "gemm_nn_store", "gemm_dgelu", "gemm_dgrad", "gemm_wgrad")
PERM_KINDS = ("dispatch", "combine", "dispatch_bwd")


def timed_steps(st: "runner.LayerState", steps: int, warmup: int = 2) -> Dict[str, float]:
    """ms per step (host clock between synchronisations) and, per kernel kind, the summed duration per
    step between HIP events recorded around each launch on the stream it runs on."""
    for _ in range(warmup):
        st.step()
    torch.cuda.synchronize()
    B.moe_profile_enable(True)
    t0 = time.perf_counter()
    for _ in range(steps):
        st.step()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) * 1e3 / steps
    B.moe_profile_enable(False)
    prof = B.moe_profile_read()
    out = {"step_ms": wall}
    out["gemm_ms"] = sum(prof[k][1] for k in GEMM_KINDS) / steps
    out["perm_ms"] = sum(prof[k][1] for k in PERM_KINDS) / steps
    out["side_ms"] = out["perm_ms"] + sum(prof[k][1] for k in ("route", "slots", "gate_bwd")) / steps
    out["gemm_launches"] = sum(prof[k][0] for k in GEMM_KINDS) // steps
    out["perm_launches"] = sum(prof[k][0] for k in PERM_KINDS) // steps
    return out


def interference(shape, inp, n: int, reuse: int, free_cus: Sequence[int] = (0, 8, 16, 32), steps: int = 5,
                 wgrad_group: int = 0) -> Dict:
    """Section II-C on this layer: the GEMMs and the permutation kernels alone (whole schedule on one
    stream, GEMMs on every compute unit) and side by side on two streams with r compute units left
    free by the GEMMs.  sigma(r) = GEMM time alone / GEMM time in the two-stream step, mu(r) likewise
    for the permutations (both are relative speeds, at most 1 up to timing noise).  With r = 0 a
    permutation kernel queued beside a GEMM mostly waits for a compute unit, so mu(0) measures that
    wait; with r > 0 it runs on the free units while the GEMM runs."""
    def state(r, two_streams):
        st = runner.LayerState(shape.T, shape.M, shape.H, shape.E, shape.k, shape.capacity_factor, n, shape.dtype,
                               reuse, second_stream=two_streams, grad_overwrite=1, wgrad_group=wgrad_group,
                               gemm_free_cus=r)
        st.upload(inp)
        return st

    st = state(0, False)
    alone = timed_steps(st, steps)
    del st
    rows = []
    for r in free_cus:
        st = state(r, True)
        t = timed_steps(st, steps)
        del st
        rows.append({"free_cus": r, "step_ms": t["step_ms"], "gemm_ms": t["gemm_ms"], "perm_ms": t["perm_ms"],
                     "sigma": alone["gemm_ms"] / t["gemm_ms"], "mu": alone["perm_ms"] / t["perm_ms"],
                     "exposed_ms": t["step_ms"] - t["gemm_ms"]})
    torch.cuda.empty_cache()
    best = min(rows, key=lambda x: x["step_ms"])
    return {"alone": alone, "side_by_side": rows, "best_free_cus": best["free_cus"]}


def pcie_elements_per_s(es: int, device="cuda:0", mib: int = 256) -> float:
    """Elements of es bytes per second through pinned host memory, both directions at once."""
    hb = torch.empty((mib << 20,), dtype=torch.uint8, pin_memory=True)
    db = torch.empty((mib << 20,), dtype=torch.uint8, device=device)
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    hb.copy_(db, non_blocking=True)
    torch.cuda.synchronize()
    c0.record()
    hb.copy_(db, non_blocking=True)
    db.copy_(hb, non_blocking=True)
    c1.record()
    torch.cuda.synchronize()
    return 2.0 * (mib << 20) / es / (c0.elapsed_time(c1) * 1e-3)


def strategy_model(shape, n: int, kept_rows: int, gemm_units_per_step: float, itf: Dict, free_cus: int) -> Dict:
    """Eq. 10 with measured speeds (Section III-E): W_comp, W_comm from the kernels alone, sigma and mu
    from the two-stream step with `free_cus` compute units left to the permutations, W_mem over PCIe.
    Returns the speeds, the model's cost of the five strategies of Table II per micro-batch and step, and
    the strategy it selects among all five and among the memory-saving four."""
    es = 2 if shape.dtype == "bf16" else 4
    rows_pp = kept_rows / n
    alone = itf["alone"]
    row = next(r for r in itf["side_by_side"] if r["free_cus"] == free_cus)
    sp = B.MoESpeeds(W_comp=gemm_units_per_step * rows_pp * shape.M * shape.H / (alone["gemm_ms"] * 1e-3),
                     W_comm=alone["perm_launches"] * rows_pp * shape.M / (alone["perm_ms"] * 1e-3),
                     W_mem=pcie_elements_per_s(es), sigma=min(1.0, row["sigma"]), mu_comp=min(1.0, row["mu"]),
                     mu_all=min(1.0, row["mu"]), eta_all=1.0)
    model = {}
    for name, num in (("none", 0), ("S1", 1), ("S2", 2), ("S3", 3), ("S4", 4)):
        fw, bw = B.moe_strategy_cost(num, int(round(rows_pp)), shape.M, shape.H, sp)
        model[name] = {"fw_ms_per_microbatch": fw * 1e3, "bw_ms_per_microbatch": bw * 1e3, "step_ms": n * (fw + bw) * 1e3}
    pick_all, _ = B.moe_select_strategy(0b11111, int(round(rows_pp)), shape.M, shape.H, sp)
    pick_saving, _ = B.moe_select_strategy(0b11110, int(round(rows_pp)), shape.M, shape.H, sp)
    return {"speeds": {"W_comp_TMAC_per_s": sp.W_comp / 1e12, "W_comm_Gelem_per_s": sp.W_comm / 1e9,
                       "W_mem_Gelem_per_s": sp.W_mem / 1e9, "sigma": sp.sigma, "mu": sp.mu_comp,
                       "free_cus_of_sigma_mu": free_cus},
            "eq10": model, "selected": B.STRATEGIES[pick_all], "selected_memory_saving": B.STRATEGIES[pick_saving],
            "_speeds_struct": sp}
