"""Parity of the HIP path with the CPU oracle, through the C ABI, on an MI355X.

Integer results (chosen experts, slots, drop masks, counts) and the float32 gate
logits must match bit for bit; values must agree within
    max|gpu - ref| / max|ref|  <=  1e-4 (float32)   2e-2 (bf16 storage, float accumulation)
per tensor.  Every run starts from NaN-poisoned outputs and workspace, so a
result that was never written, or padding that leaked into a sum, shows up.
"""
import dataclasses

import numpy as np
import pytest
import torch

from paper_2506_22175_amd import synth

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}


def relerr(a, ref):
    ref = np.asarray(ref, dtype=np.float64)
    a = np.asarray(a, dtype=np.float64)
    assert a.shape == ref.shape
    assert np.all(np.isfinite(a)), "non-finite values in the GPU result"
    d = np.abs(a - ref).max()
    s = np.abs(ref).max()
    return d / s if s > 0 else d


@pytest.fixture(scope="module")
def runner():
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2506_22175_amd import runner as R
    return R


def _oracle(oracle, s, d, n):
    return oracle.layer_step(d["x"], d["Wg"], d["W1"], d["W2"], d["dy"], s.k, s.capacity_factor, n,
                             gate_bias=d.get("gate_bias"))


def _check_routing(g, r):
    assert np.array_equal(g["logits"].view(np.uint32), r["logits"].view(np.uint32)), "gate logits differ in bits"
    assert np.array_equal(g["idx"], r["idx"])
    assert np.array_equal(g["slot"], r["slot"])
    assert np.array_equal(g["counts"], r["counts"])
    assert g["C_p"] == r["C_p"]
    assert relerr(g["w"], r["w"]) <= 1e-5


def _check_values(g, r, tol, names=("y", "dx", "dWg", "dW1", "dW2")):
    errs = {k: relerr(g[k], r[k]) for k in names}
    bad = {k: v for k, v in errs.items() if v > tol}
    assert not bad, f"beyond tolerance {tol}: {bad} (all: {errs})"
    return errs


# ---------------------------------------------------------------------------------
# whole step, full tensors
# ---------------------------------------------------------------------------------

def test_tiny_f32_full_parity(oracle, runner):
    s = synth.WORKLOADS["tiny"]
    d = synth.make_inputs(s, seed=0)
    r = _oracle(oracle, s, d, 1)
    for mode in (0, 1, 2):
        g = runner.run_layer_step(s, d, 1, mode)
        _check_routing(g, r)
        _check_values(g, r, TOL["f32"])


@pytest.mark.parametrize("n", [1, 2, 4])
@pytest.mark.parametrize("mode", [0, 1, 2])
def test_small_bf16_full_parity(oracle, runner, n, mode):
    s = synth.WORKLOADS["small"]
    d = synth.make_inputs(s, seed=0)
    r = _oracle(oracle, s, d, n)
    g = runner.run_layer_step(s, d, n, mode)
    _check_routing(g, r)
    _check_values(g, r, TOL["bf16"])


CASES = [
    # name, T, M, H, E, k, cf, dtype, n, zipf
    ("ragged_f32", 200, 72, 88, 5, 2, 1.0, "f32", 2, None),
    ("ragged_bf16", 328, 264, 328, 6, 3, 0.9, "bf16", 2, None),
    ("dense_f32", 96, 64, 128, 1, 1, 1.0, "f32", 1, None),
    ("dense_bf16", 300, 256, 512, 1, 1, 1.0, "bf16", 1, None),
    ("k_equals_E_f32", 64, 32, 40, 4, 4, 1.0, "f32", 1, None),
    ("heavy_drops_bf16", 1024, 128, 256, 4, 2, 0.25, "bf16", 4, None),
    ("heavy_drops_f32", 512, 64, 64, 4, 2, 0.3, "f32", 2, None),
    ("many_experts_bf16", 2048, 128, 192, 64, 2, 1.5, "bf16", 2, None),
    ("many_experts_f32", 512, 64, 64, 33, 8, 1.5, "f32", 1, None),
    ("skew_empty_experts_bf16", 2048, 256, 256, 16, 2, 2.0, "bf16", 4, 4.0),
    ("min_dims_f32", 16, 8, 8, 2, 1, 1.0, "f32", 1, None),
    ("min_dims_bf16", 24, 8, 8, 3, 2, 1.0, "bf16", 3, None),
    ("one_token_per_partition", 4, 64, 64, 4, 2, 2.0, "f32", 4, None),
    ("wide_bf16", 512, 1536, 640, 8, 2, 1.25, "bf16", 2, None),
    # gate matrix too large for LDS: streamed in pieces by the gate, register-held in dispatch backward
    ("big_gate_bf16", 256, 2560, 64, 32, 2, 1.0, "bf16", 2, None),
    ("big_gate_f32", 128, 1088, 32, 33, 3, 1.0, "f32", 1, None),
    # rows wider than the 2048 columns one workgroup of the dispatch-backward kernel covers, four
    # choices per token, a last round of two tokens; then an expert count that is no multiple of four
    ("wide_rows_k4_bf16", 102, 2304, 64, 16, 4, 1.0, "bf16", 1, None),
    ("wide_rows_odd_experts_bf16", 90, 2056, 40, 7, 3, 1.5, "bf16", 3, None),
    # gate backward on the matrix cores: two blocks of sixteen experts with a ragged second block, columns
    # that end inside a wavefront's 64, partitions that end inside a block of 64 tokens
    ("gate_blocks_bf16", 260, 200, 64, 18, 2, 1.25, "bf16", 2, None),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
@pytest.mark.parametrize("mode", [0, 2])
def test_edge_cases_full_parity(oracle, runner, case, mode):
    name, T, M, H, E, k, cf, dt, n, zipf = case
    kw = dict(zipf_s=1.2, zipf_tau=zipf) if zipf else {}
    s = synth.custom_shape(T, M, H, E, k, cf, dtype=dt, x_std=1.0, w_std=0.05, name=name, **kw)
    d = synth.make_inputs(s, seed=3)
    r = _oracle(oracle, s, d, n)
    g = runner.run_layer_step(s, d, n, mode)
    _check_routing(g, r)
    _check_values(g, r, TOL[dt])
    dropped = (r["slot"] < 0).all(axis=1)
    if dropped.any():                       # fully dropped tokens pass through as exact zeros
        assert np.all(g["y"][dropped] == 0.0) and np.all(g["dx"][dropped] == 0.0)
    if name.startswith("heavy_drops") or name.startswith("skew"):
        assert (r["slot"] < 0).any()
    if name.startswith("skew"):
        assert (r["counts"] == 0).any(), "case is meant to leave some expert without rows"


@pytest.mark.parametrize("case,mode", [("small", 2), ("small", 0), ("tiny", 0), ("k3", 2)])
def test_renormalised_gate_variant(oracle, runner, case, mode):
    """Combine weights divided by their sum over the token's k choices (gate_renormalize)."""
    if case == "k3":
        s, n = synth.custom_shape(328, 264, 328, 6, 3, 0.9, dtype="bf16", x_std=1.0, w_std=0.05, name="k3"), 2
    else:
        s, n = synth.WORKLOADS[case], (2 if case == "small" else 1)
    d = synth.make_inputs(s, seed=6)
    r = oracle.layer_step(d["x"], d["Wg"], d["W1"], d["W2"], d["dy"], s.k, s.capacity_factor, n,
                          gate_bias=d.get("gate_bias"), renormalize=True)
    g = runner.run_layer_step(s, d, n, mode, gate_renormalize=1)
    _check_routing(g, r)
    if s.k > 1:
        _check_values(g, r, TOL[s.dtype])
        assert np.abs(g["w"].sum(axis=1) - 1.0).max() <= 1e-6
    else:
        # one choice: its weight is exactly 1 and the gate gets no gradient at all
        _check_values(g, r, TOL[s.dtype], names=("y", "dx", "dW1", "dW2"))
        assert np.all(g["w"] == 1.0)
        assert np.abs(g["dWg"]).max() <= 1e-6 * np.abs(g["dW1"]).max()


@pytest.mark.parametrize("mode", [3, 4, 5])
@pytest.mark.parametrize("n", [1, 2, 4])
def test_offloading_strategies_give_the_same_step(oracle, runner, mode, n):
    """S1, S2, S3 of Table II: T_DI and/or T_M travel to pinned host memory in forward and back in
    backward on a third stream.  Copies change no value: S1/S2 equal mode 1 bit for bit (T_M kept,
    here on the host), S3 equals mode 2 (T_M recomputed); and the oracle agrees as for any mode."""
    s = synth.WORKLOADS["small"]
    d = synth.make_inputs(s, seed=7)
    g = runner.run_layer_step(s, d, n, mode)
    same = runner.run_layer_step(s, d, n, 2 if mode == 5 else 1)
    for k_ in ("y", "dx", "dWg", "dW1", "dW2", "idx", "slot", "counts", "w"):
        assert np.array_equal(g[k_], same[k_]), k_
    r = _oracle(oracle, s, d, n)
    _check_routing(g, r)
    _check_values(g, r, TOL[s.dtype])


def test_offloading_needs_its_own_entry_point_and_pinned_memory(runner):
    import torch
    from paper_2506_22175_amd import binding as B
    s = synth.WORKLOADS["tiny"]
    d = synth.make_inputs(s, seed=0)
    st = runner.LayerState(s.T, s.M, s.H, s.E, s.k, s.capacity_factor, 1, s.dtype, 3)
    st.upload(d)
    i = st.inputs
    args = (st.cfg, i["x"], i["dy"], i["Wg"], i["gate_bias"], i["W1"], i["W2"], st.y, st.dx, st.dWg, st.dW1, st.dW2,
            st.logits, st.topk_idx, st.topk_w, st.slot, st.counts, st.workspace)
    with pytest.raises(B.MoEError) as e:                      # the plain entry point refuses the mode
        B.moe_layer_step(*args, [st.s0, st.s1])
    assert e.value.status == 3
    pageable = torch.empty((B.moe_offload_bytes(st.cfg),), dtype=torch.uint8)
    with pytest.raises(B.MoEError) as e:
        B.moe_layer_step_offload(*args, pageable, [st.s0, st.s1, st.s2])
    assert e.value.status == 3
    with pytest.raises(B.MoEError) as e:                      # two streams are not enough
        B.moe_layer_step_offload(*args, st.host_buffer, [st.s0, st.s1])
    assert e.value.status == 2
    small = torch.empty((16,), dtype=torch.uint8, pin_memory=True)
    with pytest.raises(B.MoEError) as e:
        B.moe_layer_step_offload(*args, small, [st.s0, st.s1, st.s2])
    assert e.value.status == 4
    st.step()                                                 # and the right call works
    torch.cuda.synchronize()
    assert np.isfinite(runner.to_host(st.y)).all()


def _random_case(i):
    rng = np.random.default_rng(1000 + i)
    dt = "bf16" if i % 2 == 0 else "f32"
    n = int(rng.choice([1, 2, 3, 4]))
    T = n * int(rng.integers(8, 160))
    M = 8 * int(rng.integers(1, 41))
    H = 8 * int(rng.integers(1, 51))
    E = int(rng.integers(1, 21))
    k = int(rng.integers(1, min(4, E) + 1))
    cf = float(rng.choice([0.3, 0.75, 1.0, 1.25, 2.5]))
    mode = int(rng.integers(0, 6))
    renorm = int(rng.integers(0, 2))
    fuse = int(rng.integers(0, 2)) if mode not in (3, 5) else 0
    return dict(T=T, M=M, H=H, E=E, k=k, cf=cf, dt=dt, n=n, mode=mode, renorm=renorm, fuse=fuse)


@pytest.mark.parametrize("i", range(16))
def test_random_configurations_full_parity(oracle, runner, i):
    """Seeded random shapes, partition counts, memory modes (offloading included) and gate variants."""
    c = _random_case(i)
    s = synth.custom_shape(c["T"], c["M"], c["H"], c["E"], c["k"], c["cf"], dtype=c["dt"], x_std=1.0, w_std=0.05,
                           name=f"random{i}")
    d = synth.make_inputs(s, seed=i)
    r = oracle.layer_step(d["x"], d["Wg"], d["W1"], d["W2"], d["dy"], s.k, s.capacity_factor, c["n"],
                          gate_bias=d.get("gate_bias"), renormalize=bool(c["renorm"]))
    g = runner.run_layer_step(s, d, c["n"], c["mode"], gate_renormalize=c["renorm"], fuse_gather=c["fuse"])
    _check_routing(g, r)
    names = ["y", "dx", "dW1", "dW2"]
    if np.abs(r["dWg"]).max() > 1e-12:        # one choice renormalised, or one expert: the gate gets no gradient
        names.append("dWg")
    else:
        assert np.abs(g["dWg"]).max() <= 1e-6 * max(np.abs(g["dW1"]).max(), 1e-30)
    _check_values(g, r, TOL[c["dt"]], names=tuple(names))


def _random_larger_case(i):
    rng = np.random.default_rng(5000 + i)
    dt = "bf16" if i % 4 else "f32"
    n = int(rng.choice([1, 2, 3, 4, 8]))
    T = n * int(rng.integers(100, 700))
    M = 8 * int(rng.integers(16, 330 if dt == "bf16" else 80))
    H = 8 * int(rng.integers(16, 200 if dt == "bf16" else 60))
    E = int(rng.integers(1, 17))
    k = int(rng.integers(1, min(4, E) + 1))
    cf = float(rng.choice([0.5, 1.0, 1.25, 2.0]))
    mode = int(rng.integers(0, 6))
    renorm = int(rng.integers(0, 2))
    fuse = int(rng.integers(0, 2)) if mode not in (3, 5) else 0
    return dict(T=T, M=M, H=H, E=E, k=k, cf=cf, dt=dt, n=n, mode=mode, renorm=renorm, fuse=fuse)


@pytest.mark.parametrize("i", range(10))
def test_random_larger_configurations_full_parity(oracle, runner, i):
    """As above with shapes that span several 256-wide tiles in every dimension, ragged tails included."""
    c = _random_larger_case(i)
    s = synth.custom_shape(c["T"], c["M"], c["H"], c["E"], c["k"], c["cf"], dtype=c["dt"], x_std=1.0, w_std=0.05,
                           name=f"larger{i}")
    d = synth.make_inputs(s, seed=i)
    r = oracle.layer_step(d["x"], d["Wg"], d["W1"], d["W2"], d["dy"], s.k, s.capacity_factor, c["n"],
                          gate_bias=d.get("gate_bias"), renormalize=bool(c["renorm"]))
    g = runner.run_layer_step(s, d, c["n"], c["mode"], gate_renormalize=c["renorm"], fuse_gather=c["fuse"])
    _check_routing(g, r)
    names = ["y", "dx", "dW1", "dW2"]
    if np.abs(r["dWg"]).max() > 1e-12:
        names.append("dWg")
    _check_values(g, r, TOL[c["dt"]], names=tuple(names))


def test_results_do_not_depend_on_streams_or_reuse_mode(runner):
    """Same kernels, same order of accumulation: one stream or two, and the three
    memory modes, give identical routing and values that agree to rounding."""
    s = synth.WORKLOADS["small"]
    d = synth.make_inputs(s, seed=1)
    base = runner.run_layer_step(s, d, 4, 0, second_stream=False)
    for mode, two in ((0, True), (1, True), (2, True), (2, False)):
        g = runner.run_layer_step(s, d, 4, mode, second_stream=two)
        for k_ in ("idx", "slot", "counts"):
            assert np.array_equal(g[k_], base[k_])
        assert np.array_equal(g["y"], base["y"])                 # forward never differs
        for k_ in ("dx", "dWg", "dW1", "dW2"):
            assert relerr(g[k_], base[k_]) <= 1e-2
    # recomputed T_M is the stored T_M: modes 1 and 2 agree exactly
    g1 = runner.run_layer_step(s, d, 4, 1)
    g2 = runner.run_layer_step(s, d, 4, 2)
    for k_ in ("dx", "dWg", "dW1", "dW2"):
        assert np.array_equal(g1[k_], g2[k_]), k_


def test_repeated_steps_reuse_the_workspace_cleanly(oracle, runner):
    """Second step on a workspace holding the first step's leftovers; weight
    gradients accumulate (the caller zeroes them)."""
    s = synth.WORKLOADS["small"]
    d = synth.make_inputs(s, seed=2)
    st = runner.LayerState(s.T, s.M, s.H, s.E, s.k, s.capacity_factor, 4, s.dtype, 2)
    st.upload(d)
    st.poison()
    st.zero_grads()
    st.step()
    a = st.results()
    st.step()
    b = st.results()
    assert np.array_equal(a["y"], b["y"]) and np.array_equal(a["dx"], b["dx"])
    assert relerr(b["dW1"], 2.0 * a["dW1"]) <= 1e-6
    assert relerr(b["dWg"], 2.0 * a["dWg"]) <= 1e-6


@pytest.mark.parametrize("case", ["small", "skew_empty_experts_bf16", "ragged_f32", "min_dims_bf16"])
def test_grad_overwrite_equals_accumulation_from_zero(runner, case):
    """With grad_overwrite the first partition stores the weight gradients, so buffers
    full of NaN give what accumulation into zeroed buffers gives, bit for bit; an
    expert without rows in partition 0 still gets its zeros written."""
    if case == "small":
        s, n = synth.WORKLOADS["small"], 4
    else:
        name, T, M, H, E, k, cf, dt, n, zipf = next(c for c in CASES if c[0] == case)
        kw = dict(zipf_s=1.2, zipf_tau=zipf) if zipf else {}
        s = synth.custom_shape(T, M, H, E, k, cf, dtype=dt, x_std=1.0, w_std=0.05, name=name, **kw)
    d = synth.make_inputs(s, seed=3)
    base = runner.run_layer_step(s, d, n, 2)
    st = runner.LayerState(s.T, s.M, s.H, s.E, s.k, s.capacity_factor, n, s.dtype, 2, grad_overwrite=1)
    st.upload(d)
    st.poison()
    for t in (st.dWg, st.dW1, st.dW2):
        t.fill_(float("nan"))
    for _ in range(2):                        # the second step overwrites the first one's result
        st.step()
        g = st.results()
        for k_ in ("y", "dx", "dWg", "dW1", "dW2"):
            assert np.array_equal(g[k_], base[k_]), k_
    if case.startswith("skew"):
        assert (base["counts"][0] == 0).any(), "case is meant to leave an expert empty in partition 0"


# ---------------------------------------------------------------------------------
# the large workloads: routing on everything, values on samples
# ---------------------------------------------------------------------------------

def _sampled_check(oracle, runner, s, n, mode, seed=0, n_tokens=256, n_experts=4, n_cols=16, grad_overwrite=0,
                   fuse_gather=0):
    """Routing on the whole input; y and dx of n_tokens sampled tokens (plus some with dropped choices) and
    n_experts x n_cols (expert, column) slices of each weight gradient, each computed by the oracle one by
    one from the definition."""
    d = synth.make_inputs(s, seed=seed)
    logits, p, idx, w = oracle.route(d["x"], d["Wg"], s.k, d.get("gate_bias"))
    C_p = oracle.capacity(s.T, s.E, s.k, s.capacity_factor, n)
    slot, counts = oracle.assign_slots(idx, s.E, C_p, n)
    r = dict(logits=logits, idx=idx, w=w, slot=slot, counts=counts, C_p=C_p)
    g = runner.run_layer_step(s, d, n, mode, grad_overwrite=grad_overwrite, fuse_gather=fuse_gather)
    _check_routing(g, r)
    rng = np.random.default_rng(seed + 100)
    toks = rng.choice(s.T, size=n_tokens, replace=False)
    dropped = np.nonzero((slot < 0).any(axis=1))[0]
    if len(dropped):
        toks = np.concatenate([toks, dropped[:8]])
    sm = oracle.sampled_tokens(d["x"], d["Wg"], d["W1"], d["W2"], d["dy"], r, toks)
    tol = TOL[s.dtype]
    ys, dxs = np.abs(sm["y"]).max(), np.abs(sm["dx"]).max()
    assert np.abs(g["y"][toks] - sm["y"]).max() / ys <= tol
    assert np.abs(g["dx"][toks] - sm["dx"]).max() / dxs <= tol
    full = (slot < 0).all(axis=1)
    if full.any():
        assert np.all(g["y"][full] == 0.0) and np.all(g["dx"][full] == 0.0)
    for e in rng.choice(s.E, size=n_experts, replace=False):
        hc = rng.choice(s.H, size=n_cols, replace=False)
        mc = rng.choice(s.M, size=n_cols, replace=False)
        a, b = oracle.sampled_weight_grads(d["x"], d["W1"], d["W2"], d["dy"], r, n, C_p, int(e), hc, mc)
        assert relerr(g["dW1"][e][:, hc], a) <= tol
        assert relerr(g["dW2"][e][:, mc], b) <= tol
    assert np.all(np.isfinite(g["dWg"])) and np.all(np.isfinite(g["dW1"])) and np.all(np.isfinite(g["dW2"]))
    return g, r


_LAST_ORACLE = {}


def _oracle_once(oracle, name, n, seed=0):
    """The whole oracle step of a named workload; the last result is kept, so tests that differ only in the
    memory mode (which the oracle does not know) share one evaluation."""
    key = (name, n, seed)
    if key not in _LAST_ORACLE:
        _LAST_ORACLE.clear()
        s = synth.WORKLOADS[name]
        d = synth.make_inputs(s, seed=seed)
        _LAST_ORACLE[key] = (d, _oracle(oracle, s, d, n))
    return _LAST_ORACLE[key]


def test_gpt_workload_sampled(oracle, runner):
    _sampled_check(oracle, runner, synth.WORKLOADS["gpt"], 4, 2)


@pytest.mark.parametrize("mode", [0, 1, 2])
@pytest.mark.parametrize("n", [1, 2, 4, 8])
def test_gpt_workload_every_partitioning_and_memory_mode_full_oracle(oracle, runner, n, mode):
    """The three memory modes (keep everything; share T_DI / T_DO; share and recompute T_M) at every
    partition count the workload names, every tensor compared in full."""
    s = synth.WORKLOADS["gpt"]
    d, r = _oracle_once(oracle, "gpt", n)
    g = runner.run_layer_step(s, d, n, mode)
    _check_routing(g, r)
    _check_values(g, r, TOL["bf16"])


def test_skewed_workload_sampled(oracle, runner):
    s = synth.WORKLOADS["skewed"]
    g, r = _sampled_check(oracle, runner, s, 4, 2)
    assert (r["slot"] < 0).mean() > 0.1          # the skew really drops tokens
    assert r["counts"].max() == r["C_p"]         # and fills the popular experts to capacity


def test_skewed_workload_full_oracle(oracle, runner):
    """Zipf-biased gate, heavy drops, experts from full to nearly empty: every tensor in full, the
    gate-weight gradient (which sees the bias and the drops) included."""
    s = synth.WORKLOADS["skewed"]
    d, r = _oracle_once(oracle, "skewed", 4)
    assert (r["slot"] < 0).mean() > 0.1 and r["counts"].max() == r["C_p"]
    for overwrite in (0, 1):
        g = runner.run_layer_step(s, d, 4, 2, grad_overwrite=overwrite)
        _check_routing(g, r)
        _check_values(g, r, TOL["bf16"])
        full = (r["slot"] < 0).all(axis=1)
        assert full.any() and np.all(g["y"][full] == 0.0) and np.all(g["dx"][full] == 0.0)


@pytest.mark.parametrize("n,fuse", [(2, 0), (4, 1), (8, 0)])
def test_large_workload_full_oracle_in_bench_configuration(oracle, runner, n, fuse):
    """The shape and launch configuration bench.py times (n = 2: two streams, buffers shared and T_M
    recomputed, weight gradients stored by the first partition), and the workload's other partition
    counts, one of them with the first GEMM gathering its rows from the token-major input.  Every output
    tensor is compared in full with the oracle's."""
    s = synth.WORKLOADS["large"]
    d, r = _oracle_once(oracle, "large", n)
    g = runner.run_layer_step(s, d, n, 2, grad_overwrite=1, fuse_gather=fuse)
    _check_routing(g, r)
    _check_values(g, r, TOL["bf16"])


def test_large_workload_sampled(oracle, runner):
    """Outputs the oracle computes one by one from the definition, at the full size."""
    _sampled_check(oracle, runner, synth.WORKLOADS["large"], 2, 2, grad_overwrite=1)


# ---------------------------------------------------------------------------------
# one choice per token (the paper's own gate): the combine fused into the second expert GEMM
# ---------------------------------------------------------------------------------

K1_CASES = [
    ("tiny", None, 1),
    ("k1_bf16", (1024, 256, 512, 8, 1, 1.0, "bf16"), 2),
    ("k1_bf16_heavy_drops", (1536, 264, 328, 6, 1, 0.5, "bf16"), 3),
    ("k1_f32_ragged", (200, 72, 88, 5, 1, 0.8, "f32"), 2),
    ("k1_dense_bf16", (300, 256, 512, 1, 1, 1.0, "bf16"), 1),
]


def _k1_shape(case):
    name, dims, n = case
    if dims is None:
        return synth.WORKLOADS[name], n
    T, M, H, E, k, cf, dt = dims
    return synth.custom_shape(T, M, H, E, k, cf, dtype=dt, x_std=1.0, w_std=0.05, name=name), n


@pytest.mark.parametrize("case", K1_CASES, ids=[c[0] for c in K1_CASES])
@pytest.mark.parametrize("mode", [0, 1, 2])
@pytest.mark.parametrize("gather", [0, 1])
def test_fused_combine_full_parity(oracle, runner, case, mode, gather):
    """k = 1: y[t] = w * (row of the second GEMM) written by that GEMM's epilogue, zeros for dropped tokens,
    no T_DO anywhere; backward takes the combine-weight gradient from the GeLU-backward GEMM in every mode."""
    s, n = _k1_shape(case)
    d = synth.make_inputs(s, seed=12)
    r = _oracle(oracle, s, d, n)
    g = runner.run_layer_step(s, d, n, mode, fuse_combine=1, fuse_gather=gather)
    _check_routing(g, r)
    names = ["y", "dx", "dW1", "dW2"] + (["dWg"] if np.abs(r["dWg"]).max() > 1e-12 else [])
    _check_values(g, r, TOL[s.dtype], names=tuple(names))
    dropped = (r["slot"] < 0).all(axis=1)
    if dropped.any():
        assert np.all(g["y"][dropped] == 0.0) and np.all(g["dx"][dropped] == 0.0)
    if "drops" in case[0]:
        assert dropped.mean() > 0.2
    plain = runner.run_layer_step(s, d, n, mode, fuse_gather=gather)
    if s.dtype == "f32":
        assert np.array_equal(g["y"], plain["y"])        # w * row in float either way
    else:
        assert relerr(g["y"], plain["y"]) <= 1e-2         # one rounding to bfloat16 fewer


def test_fused_combine_runs_no_permutation_in_forward_and_keeps_no_T_DO(runner):
    from paper_2506_22175_amd import binding as B
    s, n = _k1_shape(K1_CASES[1])
    d = synth.make_inputs(s, seed=0)
    for mode in (0, 2):
        st = runner.LayerState(s.T, s.M, s.H, s.E, s.k, s.capacity_factor, n, s.dtype, mode, fuse_gather=1, fuse_combine=1)
        base = runner.LayerState(s.T, s.M, s.H, s.E, s.k, s.capacity_factor, n, s.dtype, mode, fuse_gather=1)
        st.upload(d)
        st.zero_grads()
        B.moe_launch_counts(reset=True)
        st.forward()
        torch.cuda.synchronize()
        gemms, perms, _ = B.moe_launch_counts(reset=True)
        assert (gemms, perms) == (2 * n, 0)
        st.backward()
        torch.cuda.synchronize()
        gemms, perms, _ = B.moe_launch_counts(reset=True)
        assert (gemms, perms) == ((5 if mode == 2 else 4) * n, 3 * n)
        if mode == 0:
            # T_DO of every partition is gone from what forward keeps for backward
            Rp = st.C_p * s.E
            assert base.ws_saved - st.ws_saved == n * Rp * s.M * 2
    with pytest.raises(B.MoEError) as e:                  # two choices per token: a row is not the whole output
        s2 = synth.WORKLOADS["small"]
        runner.LayerState(s2.T, s2.M, s2.H, s2.E, s2.k, s2.capacity_factor, 2, s2.dtype, 2, fuse_combine=1)
    assert e.value.status == 3


# ---------------------------------------------------------------------------------
# weight gradients of several partitions in one GEMM (wgrad_group)
# ---------------------------------------------------------------------------------

@pytest.mark.parametrize("case", ["small", "ragged_bf16", "heavy_drops_bf16", "skew_empty_experts_bf16", "ragged_f32",
                                  "one_token_per_partition"])
@pytest.mark.parametrize("mode", [0, 1, 2])
def test_grouped_weight_gradients_full_parity(oracle, runner, case, mode):
    """The reduction over the rows of G partitions as one GEMM (float32: G GEMMs in a row) gives the
    oracle's gradients for every memory mode, with groups that do and do not divide n, experts without
    rows in some partitions, and gradients stored by the first group or accumulated."""
    if case == "small":
        s, n = synth.WORKLOADS["small"], 4
    else:
        name, T, M, H, E, k, cf, dt, n, zipf = next(c for c in CASES if c[0] == case)
        kw = dict(zipf_s=1.2, zipf_tau=zipf) if zipf else {}
        s = synth.custom_shape(T, M, H, E, k, cf, dtype=dt, x_std=1.0, w_std=0.05, name=name, **kw)
    d = synth.make_inputs(s, seed=3)
    r = _oracle(oracle, s, d, n)
    for G, overwrite in ((2, 0), (3, 1), (8, 0)):
        g = runner.run_layer_step(s, d, n, mode, wgrad_group=G, grad_overwrite=overwrite)
        _check_routing(g, r)
        _check_values(g, r, TOL[s.dtype])


@pytest.mark.parametrize("n,G", [(4, 2), (8, 4), (8, 8)])
def test_large_workload_grouped_weight_gradients_full_oracle(oracle, runner, n, G):
    s = synth.WORKLOADS["large"]
    d, r = _oracle_once(oracle, "large", n)
    g = runner.run_layer_step(s, d, n, 2, grad_overwrite=1, wgrad_group=G)
    _check_routing(g, r)
    _check_values(g, r, TOL["bf16"])


def test_launch_counts_with_grouped_weight_gradients(runner):
    """Per partition backward still runs Table II's GEMM units other than the two weight-gradient
    ones (2, or 3 with recomputation); those two run once per group."""
    from paper_2506_22175_amd import binding as B
    s = synth.WORKLOADS["small"]
    d = synth.make_inputs(s, seed=0)
    n = 4
    for mode, per_part in ((0, 2), (2, 3)):
        for G, groups in ((1, 4), (2, 2), (3, 2), (4, 1)):
            st = runner.LayerState(s.T, s.M, s.H, s.E, s.k, s.capacity_factor, n, s.dtype, mode, wgrad_group=G)
            st.upload(d)
            st.zero_grads()
            st.forward()
            torch.cuda.synchronize()
            B.moe_launch_counts(reset=True)
            st.backward()
            torch.cuda.synchronize()
            g, p, _ = B.moe_launch_counts(reset=True)
            assert g == per_part * n + 2 * groups, (mode, G, g)


# ---------------------------------------------------------------------------------
# schedule: op counts of Table II, and the entry points one by one
# ---------------------------------------------------------------------------------

@pytest.mark.parametrize("mode,gemm_bwd,perm_bwd", [(0, 4, 2), (1, 4, 3), (2, 5, 3)])
def test_launch_counts_match_table_two(runner, mode, gemm_bwd, perm_bwd):
    """Per partition: forward 2 GEMMs and 2 permutations; backward 4 GEMMs and 2
    permutations, 3 permutations when T_DI is dispatched again, 5 GEMMs when T_M is
    recomputed (the paper's Q vectors [2,2,0] and [4,2,0] / [5,3,0])."""
    from paper_2506_22175_amd import binding as B
    s = synth.WORKLOADS["small"]
    d = synth.make_inputs(s, seed=0)
    n = 4
    st = runner.LayerState(s.T, s.M, s.H, s.E, s.k, s.capacity_factor, n, s.dtype, mode)
    st.upload(d)
    st.zero_grads()
    B.moe_launch_counts(reset=True)
    st.forward()
    torch.cuda.synchronize()
    g, p, _ = B.moe_launch_counts(reset=True)
    assert (g, p) == (2 * n, 2 * n)
    st.backward()
    torch.cuda.synchronize()
    g, p, _ = B.moe_launch_counts(reset=True)
    assert (g, p) == (gemm_bwd * n, perm_bwd * n)


def test_entry_points_one_by_one_equal_the_layer_step(oracle, runner):
    """Route, slots, dispatch, FFN forward, combine, and the backward pieces called
    through the C ABI one at a time give what moe_layer_step gives."""
    from paper_2506_22175_amd import binding as B
    s = synth.custom_shape(640, 256, 384, 6, 2, 0.8, dtype="bf16", w_std=0.05)
    d = synth.make_inputs(s, seed=5)
    n = 2
    ref = runner.run_layer_step(s, d, n, 2)
    orc = _oracle(oracle, s, d, n)
    st = runner.LayerState(s.T, s.M, s.H, s.E, s.k, s.capacity_factor, n, s.dtype, 2)
    st.upload(d)
    st.poison()
    st.zero_grads()
    cfg, i = st.cfg, st.inputs
    dev, bf = "cuda:0", torch.bfloat16
    Rp = st.C_p * s.E
    parts = B.moe_dw_parts(cfg)
    slot_w = torch.full((n * Rp,), float("nan"), device=dev)
    sscr = torch.empty(B.moe_slot_scratch_bytes(cfg), dtype=torch.uint8, device=dev)
    gscr = torch.empty(B.moe_gate_scratch_bytes(cfg), dtype=torch.uint8, device=dev)
    B.moe_route(cfg, i["x"], i["Wg"], None, st.logits, st.topk_idx, st.topk_w)
    B.moe_assign_slots(cfg, st.topk_idx, st.topk_w, st.slot, st.counts, slot_w, sscr)
    assert np.array_equal(st.slot.cpu().numpy(), orc["slot"])
    dL = torch.full((s.T, s.E), float("nan"), device=dev)
    for p in range(n):
        nan = float("nan")
        DI = torch.full((Rp, s.M), nan, dtype=bf, device=dev)
        A = torch.full((Rp, s.H), nan, dtype=bf, device=dev)
        DO = torch.full((Rp, s.M), nan, dtype=bf, device=dev)
        B.moe_dispatch(cfg, p, i["x"], st.slot, DI)
        B.moe_expert_ffn_fwd(cfg, p, DI, st.counts, i["W1"], i["W2"], None, A, DO)
        B.moe_combine(cfg, p, DO, st.slot, st.topk_w, st.y)
        dDO = torch.full((Rp, s.M), nan, dtype=bf, device=dev)
        Z = torch.full((Rp, s.H), nan, dtype=bf, device=dev)
        dZ = torch.full((Rp, s.H), nan, dtype=bf, device=dev)
        dDI = torch.full((Rp, s.M), nan, dtype=bf, device=dev)
        dwp = torch.full((Rp, parts), nan, device=dev)
        B.moe_dispatch(cfg, p, i["dy"], st.slot, dDO)
        B.moe_expert_ffn_bwd(cfg, p, 1, DI, Z, dDO, st.counts, slot_w, i["W1"], i["W2"], dZ, dDI, st.dW1, st.dW2, dwp)
        B.moe_gate_bwd(cfg, p, i["x"], st.logits, st.topk_idx, st.slot, None, dwp, dL, st.dWg, gscr)
        B.moe_dispatch_bwd(cfg, p, dDI, st.slot, dL, i["Wg"], st.dx)
    got = st.results()
    for k_ in ("y", "dx", "dWg", "dW1", "dW2"):
        assert np.array_equal(got[k_], ref[k_]), k_
    _check_values(got, orc, TOL["bf16"])



# ---------------------------------------------------------------------------------
# the first expert GEMM reading its rows straight from the token-major input
# ---------------------------------------------------------------------------------

@pytest.mark.parametrize("dt", ["bf16", "f32"])
def test_gathered_first_gemm_equals_dispatch_then_gemm_bit_for_bit(oracle, runner, dt):
    """moe_slot_rows inverts the oracle's slot map exactly, and moe_expert_ffn_fwd_gather gives, on every
    valid row, the bits that moe_dispatch followed by moe_expert_ffn_fwd gives."""
    from paper_2506_22175_amd import binding as B
    s = synth.custom_shape(602, 264, 328, 7, 3, 0.9, dtype=dt, x_std=1.0, w_std=0.05, name="gather")
    d = synth.make_inputs(s, seed=11)
    n = 2
    orc = _oracle(oracle, s, d, n)
    st = runner.LayerState(s.T, s.M, s.H, s.E, s.k, s.capacity_factor, n, s.dtype, 0)
    st.upload(d)
    cfg, i = st.cfg, st.inputs
    dev, td = "cuda:0", (torch.bfloat16 if dt == "bf16" else torch.float32)
    Rp = st.C_p * s.E
    sscr = torch.empty(B.moe_slot_scratch_bytes(cfg), dtype=torch.uint8, device=dev)
    B.moe_route(cfg, i["x"], i["Wg"], None, st.logits, st.topk_idx, st.topk_w)
    B.moe_assign_slots(cfg, st.topk_idx, st.topk_w, st.slot, st.counts, None, sscr)
    rows = torch.full((n, Rp), -7, dtype=torch.int32, device=dev)
    B.moe_slot_rows(cfg, st.slot, rows)
    torch.cuda.synchronize()
    # the inverse map, entry by entry, from the oracle's slots
    want = np.full((n, Rp), -7, dtype=np.int32)
    Tp = s.T // n
    for t in range(s.T):
        for j in range(s.k):
            sl = orc["slot"][t, j]
            if sl >= 0:
                want[t // Tp, sl] = t
    assert np.array_equal(rows.cpu().numpy(), want)
    assert (want >= 0).sum() == orc["counts"].sum()
    for p in range(n):
        out = {}
        for kind in ("dispatched", "gathered"):
            Z = torch.zeros((Rp, s.H), dtype=td, device=dev)
            A = torch.zeros((Rp, s.H), dtype=td, device=dev)
            DO = torch.zeros((Rp, s.M), dtype=td, device=dev)
            if kind == "dispatched":
                DI = torch.zeros((Rp, s.M), dtype=td, device=dev)
                B.moe_dispatch(cfg, p, i["x"], st.slot, DI)
                B.moe_expert_ffn_fwd(cfg, p, DI, st.counts, i["W1"], i["W2"], Z, A, DO)
            else:
                B.moe_expert_ffn_fwd_gather(cfg, p, i["x"], rows, st.counts, i["W1"], i["W2"], Z, A, DO)
            torch.cuda.synchronize()
            out[kind] = [runner.to_host(t_) for t_ in (Z, A, DO)]
        valid = np.zeros(Rp, dtype=bool)
        for e in range(s.E):
            valid[e * st.C_p: e * st.C_p + orc["counts"][p, e]] = True
        for a, b in zip(out["dispatched"], out["gathered"]):
            assert np.array_equal(a[valid], b[valid])
        assert np.abs(out["gathered"][2][valid]).max() > 0


@pytest.mark.parametrize("mode,n", [(0, 1), (0, 4), (1, 4), (2, 2), (2, 4), (4, 4)])
def test_layer_step_with_the_gathered_first_gemm(oracle, runner, mode, n):
    """fuse_gather changes where the first GEMM reads from, not one bit of any result."""
    s = synth.WORKLOADS["small"]
    d = synth.make_inputs(s, seed=2)
    r = _oracle(oracle, s, d, n)
    plain = runner.run_layer_step(s, d, n, mode)
    fused = runner.run_layer_step(s, d, n, mode, fuse_gather=1)
    _check_routing(fused, r)
    _check_values(fused, r, TOL[s.dtype])
    for k_ in ("y", "dx", "dWg", "dW1", "dW2"):
        assert np.array_equal(fused[k_], plain[k_]), k_


@pytest.mark.parametrize("mode", [0, 1, 2])
def test_launch_counts_with_the_gathered_first_gemm(runner, mode):
    """Forward: two GEMMs and one permutation (the combine) per partition; backward dispatches dy and
    T_I and runs dispatch-backward in every mode."""
    from paper_2506_22175_amd import binding as B
    s = synth.WORKLOADS["small"]
    d = synth.make_inputs(s, seed=0)
    n = 4
    st = runner.LayerState(s.T, s.M, s.H, s.E, s.k, s.capacity_factor, n, s.dtype, mode, fuse_gather=1)
    st.upload(d)
    st.zero_grads()
    B.moe_launch_counts(reset=True)
    st.forward()
    torch.cuda.synchronize()
    g, p, _ = B.moe_launch_counts(reset=True)
    assert (g, p) == (2 * n, n)
    st.backward()
    torch.cuda.synchronize()
    g, p, _ = B.moe_launch_counts(reset=True)
    assert (g, p) == ((5 if mode == 2 else 4) * n, 3 * n)


def test_kernel_timing_hooks_see_every_gemm(runner):
    from paper_2506_22175_amd import binding as B
    s = synth.WORKLOADS["small"]
    d = synth.make_inputs(s, seed=0)
    st = runner.LayerState(s.T, s.M, s.H, s.E, s.k, s.capacity_factor, 2, s.dtype, 2)
    st.upload(d)
    st.zero_grads()
    B.moe_profile_enable(True)
    st.step()
    torch.cuda.synchronize()
    B.moe_profile_enable(False)
    prof = B.moe_profile_read()
    assert prof["gemm_fwd1_gelu"][0] == 2 and prof["gemm_nn_store"][0] == 4 and prof["gemm_wgrad"][0] == 4
    # dispatches: x forward and dy backward per partition; with two partitions no T_DI buffer is
    # shared, so backward finds T_DI where forward left it and does not dispatch x again
    assert prof["gemm_dgelu"][0] == 2 and prof["gemm_dgrad"][0] == 2 and prof["dispatch"][0] == 4
    assert all(ms > 0 for cnt, ms in prof.values() if cnt)


def test_graph_replay_equals_eager_every_time(runner):
    """A captured step replayed several times, with eager steps and synchronisations
    between the replays, gives the eager result each time."""
    s = synth.WORKLOADS["small"]
    d = synth.make_inputs(s, seed=4)
    st = runner.LayerState(s.T, s.M, s.H, s.E, s.k, s.capacity_factor, 4, s.dtype, 2)
    st.upload(d)
    st.zero_grads()
    st.step()
    eager = st.results()
    graph = st.capture()
    for rep in range(4):
        st.poison()
        st.zero_grads()
        graph.replay()
        got = st.results()
        for k_ in ("y", "dx", "dWg", "dW1", "dW2", "slot", "idx", "counts"):
            assert np.array_equal(got[k_], eager[k_]), (rep, k_)
        st.zero_grads()
        st.step()                      # eager work between replays
        torch.cuda.synchronize()


def test_granularity_search_by_trials_and_algorithm_one_on_the_gpu(oracle, runner):
    """searchBestGran (Algorithm 1, Section III-C) times the real step for each candidate n;
    the whole algorithm then answers a repeated batch size from its table, and a step with the
    chosen n matches the oracle like any other."""
    from paper_2506_22175_amd import binding as B
    s = synth.WORKLOADS["small"]
    d = synth.make_inputs(s, seed=4)
    cands = [1, 2, 3, 4, 8]                                  # 3 does not divide T: skipped
    st = runner.LayerState(s.T, s.M, s.H, s.E, s.k, s.capacity_factor, 1, s.dtype, 2, size_for_partitions=cands)
    st.upload(d)
    st.poison()
    best, ms = st.search_best_gran(cands, warmup=1, iters=3)
    assert ms[2] == -1.0 and all(m > 0 for i, m in enumerate(ms) if i != 2)
    assert best == cands[min((m, i) for i, m in enumerate(ms) if m > 0)[1]]
    g = B.GranHandle()
    n1, searched1 = st.gran_get(g, cands)
    n2, searched2 = st.gran_get(g, cands)
    assert searched1 and not searched2 and n1 == n2 and n1 in (1, 2, 4, 8)
    assert B.moe_gran_ranges(g) == [(s.T, s.T, n1)]
    g.close()
    # the chosen n is an ordinary configuration: parity as usual
    r = _oracle(oracle, s, d, n1)
    out = runner.run_layer_step(s, d, n1, 2)
    _check_routing(out, r)
    _check_values(out, r, TOL[s.dtype])
