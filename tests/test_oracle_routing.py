"""Pins for the oracle's gate, top-k and slot assignment (CPU only).

Each check is independent of the oracle's own code path: exact rational
arithmetic for the float32 summation order, full sorts and O(N^2) counting for
routing and slot ranking, and the invariants the method states.
"""
from fractions import Fraction

import numpy as np
import pytest

from paper_2506_22175_amd import synth


# ---------- exact emulation of float32 fused multiply-add ----------------------

def _round_f32(fr: Fraction) -> np.float32:
    """Correctly rounded (nearest, ties to even) float32 of an exact rational."""
    if fr == 0:
        return np.float32(0.0)
    c = np.float32(float(fr))            # within one ulp of the answer
    cands = {c, np.nextafter(c, np.float32(np.inf)), np.nextafter(c, np.float32(-np.inf))}
    best = None
    for v in cands:
        if not np.isfinite(v):
            continue
        err = abs(Fraction(float(v)) - fr)
        even = (np.array(v, dtype=np.float32).view(np.uint32) & 1) == 0
        key = (err, 0 if even else 1)
        if best is None or key < best[0]:
            best = (key, v)
    return best[1]


def _logit_exact_order(xrow, wcol, bias=None):
    acc = [np.float32(0.0)] * 64
    for d in range(len(xrow)):
        l = (d // 8) % 64
        acc[l] = _round_f32(Fraction(float(xrow[d])) * Fraction(float(wcol[d])) + Fraction(float(acc[l])))
    off = 32
    while off >= 1:
        for l in range(off):
            acc[l] = np.float32(acc[l] + acc[l + off])
        off //= 2
    v = acc[0]
    if bias is not None:
        v = np.float32(v + np.float32(bias))
    return v


@pytest.mark.parametrize("M,E,seed,scale", [(64, 3, 0, 1.0), (8, 2, 1, 1.0), (520, 2, 2, 1e3), (1032, 1, 3, 1e-3)])
def test_gate_logits_follow_the_written_order_bit_for_bit(oracle, M, E, seed, scale):
    g = np.random.default_rng(seed)
    x = (g.standard_normal((3, M)) * scale).astype(np.float32)
    W = g.standard_normal((M, E)).astype(np.float32)
    b = g.standard_normal(E).astype(np.float32)
    got = oracle.gate_logits(x, W, b)
    for t in range(3):
        for e in range(E):
            want = _logit_exact_order(x[t], W[:, e], b[e])
            assert got[t, e].view(np.uint32) == np.float32(want).view(np.uint32), (t, e)


def test_gate_logits_order_matters_and_is_detected(oracle):
    """A different (plain left-to-right) order gives different bits somewhere:
    the pin above would catch an oracle that summed in the wrong order."""
    g = np.random.default_rng(5)
    x = g.standard_normal((64, 1024)).astype(np.float32)
    W = g.standard_normal((1024, 4)).astype(np.float32)
    got = oracle.gate_logits(x, W)
    seq = np.zeros((64, 4), dtype=np.float32)
    for d in range(1024):
        seq = (seq + x[:, d:d + 1] * W[d:d + 1, :]).astype(np.float32)
    assert np.any(got.view(np.uint32) != seq.view(np.uint32))
    np.testing.assert_allclose(got, x.astype(np.float64) @ W.astype(np.float64), rtol=0, atol=2e-4)


def test_gate_logits_close_to_float64_matmul(oracle):
    s = synth.WORKLOADS["small"]
    d = synth.make_inputs(s, seed=3)
    L = oracle.gate_logits(d["x"][:512], d["Wg"])
    ref = d["x"][:512].astype(np.float64) @ d["Wg"].astype(np.float64)
    assert np.abs(L - ref).max() <= 1e-5 * np.abs(ref).max() + 1e-6


# ---------- top-k ---------------------------------------------------------------

def _topk_bruteforce(row, k):
    items = [(-(float("-inf") if np.isnan(v) else float(v)), e) for e, v in enumerate(row)]
    items.sort()                          # descending value, then ascending index
    return [e for _, e in items[:k]]


def test_topk_matches_full_sort_with_ties_and_nan(oracle):
    g = np.random.default_rng(0)
    L = g.integers(-3, 4, size=(200, 7)).astype(np.float32)     # many exact ties
    L[5, 2] = np.nan
    L[6, :] = 1.0                                               # all equal -> 0,1,2
    L[7, 3] = -0.0
    L[7, 4] = 0.0
    for k in (1, 2, 3, 7):
        got = oracle.top_k(L, k)
        for t in range(L.shape[0]):
            assert list(got[t]) == _topk_bruteforce(L[t], k), (t, k)
    assert list(oracle.top_k(L, 3)[6]) == [0, 1, 2]


def test_route_weights_are_the_chosen_softmax_probabilities(oracle):
    g = np.random.default_rng(1)
    x = g.standard_normal((50, 64)).astype(np.float32)
    W = g.standard_normal((64, 6)).astype(np.float32)
    for k in (1, 2, 6):
        logits, p, idx, w = oracle.route(x, W, k)
        assert idx.shape == (50, k)
        for t in range(50):
            assert len(set(idx[t])) == k                        # k distinct experts
            vals = logits[t, idx[t]]
            assert np.all(np.diff(vals) <= 0)                   # descending logits
            ex = [np.exp(float(v) - float(logits[t].max())) for v in logits[t]]
            for j in range(k):
                assert abs(w[t, j] - ex[idx[t, j]] / sum(ex)) < 1e-14
        s = w.sum(axis=1)
        assert np.all(s <= 1 + 1e-12)
        if k == 6:
            np.testing.assert_allclose(s, 1.0, atol=1e-12)     # k = E: weights sum to 1
    _, _, idx1, w1 = oracle.route(x, W[:, :1], 1)               # E = 1: weight is exactly 1
    assert np.all(idx1 == 0) and np.all(w1 == 1.0)


# ---------- slots ---------------------------------------------------------------

def _slots_bruteforce(idx, E, C_p, n):
    T, k = idx.shape
    T_p = T // n
    slot = -np.ones((T, k), dtype=np.int64)
    counts = np.zeros((n, E), dtype=np.int64)
    for t in range(T):
        for j in range(k):
            p = t // T_p
            pos = 0
            for t2 in range(p * T_p, (p + 1) * T_p):
                for j2 in range(k):
                    if idx[t2, j2] == idx[t, j] and (j2, t2) < (j, t):
                        pos += 1
            if pos < C_p:
                slot[t, j] = idx[t, j] * C_p + pos
                counts[p, idx[t, j]] += 1
    return slot, counts


@pytest.mark.parametrize("T,E,k,cf,n", [(24, 4, 2, 1.0, 1), (24, 4, 2, 0.5, 2), (30, 3, 1, 1.25, 3),
                                         (16, 2, 2, 2.0, 1), (32, 5, 3, 0.7, 4)])
def test_slots_match_quadratic_definition(oracle, T, E, k, cf, n):
    g = np.random.default_rng(T + E)
    idx = np.stack([g.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    C_p = oracle.capacity(T, E, k, cf, n)
    slot, counts = oracle.assign_slots(idx, E, C_p, n)
    s2, c2 = _slots_bruteforce(idx, E, C_p, n)
    assert np.array_equal(slot, s2)
    assert np.array_equal(counts, c2)


def test_slot_invariants_on_a_skewed_batch(oracle):
    s = synth.custom_shape(2048, 64, 64, 16, 2, 2.0, zipf_s=1.2, zipf_tau=1.0)
    d = synth.make_inputs(s, seed=7)
    n = 4
    _, _, idx, _ = oracle.route(d["x"], d["Wg"], s.k, d["gate_bias"])
    C_p = oracle.capacity(s.T, s.E, s.k, s.capacity_factor, n)
    slot, counts = oracle.assign_slots(idx, s.E, C_p, n)
    T_p = s.T // n
    assert (slot < 0).any(), "the skew is meant to overflow expert 0"
    for p in range(n):
        sp = slot[p * T_p:(p + 1) * T_p]
        ip = idx[p * T_p:(p + 1) * T_p]
        assert np.all(counts[p] <= C_p)
        kept = sp[sp >= 0]
        assert len(np.unique(kept)) == len(kept)                       # injective
        for e in range(s.E):
            pos = np.sort(kept[(kept // C_p) == e] % C_p)
            assert np.array_equal(pos, np.arange(counts[p, e]))        # 0..count-1, once each
            # kept slots belong to the expert that was chosen
            assert np.all(ip[(sp >= 0) & (sp // C_p == e)] == e)
            # first choices come before second choices; within a choice, token order
            first = sp[:, 0][(ip[:, 0] == e) & (sp[:, 0] >= 0)] % C_p
            second = sp[:, 1][(ip[:, 1] == e) & (sp[:, 1] >= 0)] % C_p
            assert np.all(np.diff(first) > 0) and np.all(np.diff(second) > 0)
            if len(first) and len(second):
                assert first.max() < second.min()
            # a dropped first choice means no second choice of that expert was kept
            if ((ip[:, 0] == e) & (sp[:, 0] < 0)).any():
                assert len(second) == 0


def test_capacity_formula(oracle):
    assert oracle.capacity(256, 4, 1, 1.25, 1) == 80
    assert oracle.capacity(4096, 8, 2, 1.25, 4) == 320
    assert oracle.capacity(32768, 16, 2, 1.0, 8) == 512
    assert oracle.capacity(16384, 16, 2, 2.0, 4) == 1024
    assert oracle.capacity(10, 3, 1, 1.0, 1) == 4          # ceil(10/3)
    with pytest.raises(ValueError):
        oracle.capacity(10, 3, 1, 1.0, 3)


def test_skewed_workload_uses_the_calibrated_tau():
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "zipf_tau.txt")
    vals = dict(l.split(None, 1) for l in open(path) if not l.startswith("#"))
    assert float(vals["tau"]) == synth.WORKLOADS["skewed"].zipf_tau
    top1 = [float(v) for v in vals["top1_share"].split()]
    assert abs(top1[0] - 0.365) <= 0.005 and top1[0] > top1[1] > top1[2]
