"""Section II-C's slowdown factors measured as real co-runs (the expert GEMMs leave compute units free for
the permutation kernels of the other stream), and Section III-E's selector on the measured speeds against the
measured step times of the strategies of Table II."""
import numpy as np
import pytest
import torch

from paper_2506_22175_amd import binding as B
from paper_2506_22175_amd import measure, runner, synth

pytestmark = pytest.mark.gpu


def test_free_compute_units_change_timing_not_results():
    s = synth.WORKLOADS["small"]
    d = synth.make_inputs(s, seed=9)
    base = runner.run_layer_step(s, d, 4, 2)
    for r in (8, 16, 250, 1000):                       # the last two leave the GEMMs eight units
        g = runner.run_layer_step(s, d, 4, 2, gemm_free_cus=r)
        for k_ in ("y", "dx", "dWg", "dW1", "dW2", "slot", "idx", "counts"):
            assert np.array_equal(g[k_], base[k_]), (r, k_)
    with pytest.raises(B.MoEError) as e:
        runner.run_layer_step(s, d, 4, 2, gemm_free_cus=-1)
    assert e.value.status == 3


def test_measured_slowdown_factors_and_strategy_selection():
    assert torch.cuda.is_available()
    s = synth.WORKLOADS["gpt"]
    d = synth.make_inputs(s, seed=0)
    n = 4
    itf = measure.interference(s, d, n, 2, free_cus=(0, 8, 16), steps=4)
    rows = {r["free_cus"]: r for r in itf["side_by_side"]}
    for r in (8, 16):
        # relative speeds: positive, and at most 1 up to timing noise
        assert 0.0 < rows[r]["sigma"] <= 1.05, rows[r]
        assert 0.0 < rows[r]["mu"] <= 1.05, rows[r]
        # fewer units for the GEMMs cannot make them faster than on the whole chip alone
        assert rows[r]["gemm_ms"] >= 0.97 * itf["alone"]["gemm_ms"]
    # the step of every strategy, measured
    measured = {}
    for name, mode in (("none", 0), ("S1", 3), ("S2", 4), ("S3", 5), ("S4", 2)):
        st = runner.LayerState(s.T, s.M, s.H, s.E, s.k, s.capacity_factor, n, s.dtype, mode, grad_overwrite=1)
        st.upload(d)
        measured[name] = measure.timed_steps(st, 3, warmup=1)["step_ms"]
        del st
    kept = int(runner.run_layer_step(s, d, n, 2)["counts"].sum())
    model = measure.strategy_model(s, n, kept, n * 7, itf, 8)
    assert model["selected"] == min(measured, key=measured.get), (model["selected"], measured)
    saving = {k_: v for k_, v in measured.items() if k_ != "none"}
    assert model["selected_memory_saving"] == min(saving, key=saving.get), (model["selected_memory_saving"], measured)
    # and the model orders the strategies as the measurement does where they differ by more than a tenth
    order = sorted(measured, key=measured.get)
    for a, b in zip(order, order[1:]):
        if measured[b] > 1.1 * measured[a]:
            assert model["eq10"][a]["step_ms"] < model["eq10"][b]["step_ms"], (a, b, measured, model["eq10"])
