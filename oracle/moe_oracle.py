"""CPU oracle for one GPU's share of an MoE layer's training step.

TEST INFRASTRUCTURE ONLY.  Nothing on the product path may import this file;
only tests, the smoke check and the benchmark's cpu_baseline leg use it.  It
shares no code with the HIP path and never receives values computed there.

What it computes is the plain definition of the layer, written out in float64
with numpy (matmul, sort and erf are library steps), with no blocking, fusion
or reordering:

  gate (linear map with E*M parameters, top-k; Sections II-B2 and IV-A)
  -> dispatch T_I into the expert-contiguous T_DI           (Fig. 1, Section II-A)
  -> expert FFN: T_M = T_DI W1, activation, T_DO = act(T_M) W2, no biases
     (two linear layers and one activation, 2*H*M parameters; Section II-B2)
  -> combine T_DO into T_O weighted by the gate              (Fig. 1)
  and the backward pass of exactly these steps ("symmetric", Section III-B).

Micro-batch pipelining (Section III-B) and memory reuse (Section III-D) change
the schedule and the memory, not the result: partitions are independent
(Section III-B), and a recomputed T_M equals the stored one (Section III-D).
The number of partitions n therefore enters here only through the capacity,
which is applied per partition.

Readings where the paper is silent (each also listed in the design notes):
  * softmax over all E logits; the k largest *logits* are chosen, ties to the
    lower expert index; combine weights are the chosen probabilities, not
    renormalised;
  * capacity C_p = ceil(cf * k * (T/n) / E) rows per expert per partition;
    inside a partition, slots are granted choice-major (all first choices in
    token order, then all second choices, ...); an assignment whose position
    reaches C_p is dropped and contributes zero; surviving weights are not
    rescaled;
  * slot = e * C_p + position (padded, fixed stride);
  * the activation is exact GeLU, 0.5 z (1 + erf(z / sqrt 2)); the stored
    middle tensor T_M is the pre-activation;
  * top-k indices and drops carry no gradient.

Pins (see tests/test_oracle_*.py): brute-force routing and slot ranking on tiny
inputs, exact-rational emulation of the float32 logit order, the dense-FFN
special case against a textbook FFN, central finite differences for every
gradient, partition independence, permutation identities, the closed forms of
Eq. 1-6 and the memory-saving ratios they imply.
"""
from __future__ import annotations

import ctypes
import math
import os
from typing import Dict, Optional, Sequence

import numpy as np
from scipy.special import erf as _erf

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None


def _lib():
    """The small C helper holding the float32 logit summation order."""
    global _LIB
    if _LIB is None:
        path = os.path.join(_HERE, "_gate_logits.so")
        if not os.path.exists(path):
            from . import build as _build
            _build.build()
        _LIB = ctypes.CDLL(path)
        _LIB.oracle_gate_logits_f32.restype = None
        _LIB.oracle_gate_logits_f32.argtypes = [ctypes.c_void_p] * 3 + [ctypes.c_int64] * 3 + [ctypes.c_void_p]
    return _LIB


# --------------------------------------------------------------------------
# capacity and the paper's memory model
# --------------------------------------------------------------------------

def capacity(T: int, E: int, k: int, capacity_factor: float, n: int) -> int:
    """Rows per expert per partition: ceil(cf * k * (T/n) / E), cf taken as float32."""
    if T % n:
        raise ValueError("T must be divisible by n")
    cf = float(np.float32(capacity_factor))
    return int(math.ceil(cf * float(k * (T // n)) / float(E)))


def paper_memory_model(B: int, M: int, H: int, E: int, n: int) -> Dict[str, float]:
    """Eq. 1-6 in elements: model states, activations, temporary buffers, saving."""
    m_ms = 4 * (E * M + 2 * H * M)                      # Eq. 1
    m_act = 4 * B * M + B * H                            # Eq. 2
    m_buf_seq = B * M + B * H                            # Eq. 3
    m_pipe = 4 * B * M + B * H                           # Eq. 4 (act and buf alike)
    delta = B * (2 * M * (n - 2) / n + H * (n - 1) / n)  # Eq. 5
    phi = (2 * delta) / (m_ms + 2 * m_pipe)              # Eq. 6
    return dict(M_ms=m_ms, M_act=m_act, M_buf=m_buf_seq, M_act_pipe=m_pipe,
                M_buf_pipe=m_pipe, delta=delta, phi=phi)


def workspace_model(R_p: int, n: int, M: int, H: int, mode: int) -> int:
    """Activation elements kept for backward: T_DI + T_M + T_DO over R = n*R_p rows.

    mode 0 keeps all n partitions; mode 1 shares two T_DI and two T_DO partition
    buffers and keeps T_M whole; mode 2 also shares one T_M buffer (Section III-D:
    one buffer for T_M, two each for T_DI and T_DO)."""
    R = n * R_p
    if mode == 0:
        return R * (2 * M + H)
    if mode == 1:
        return 4 * R_p * M + R * H
    if mode == 2:
        return 4 * R_p * M + R_p * H
    raise ValueError(mode)


# --------------------------------------------------------------------------
# gate
# --------------------------------------------------------------------------

def gate_logits(x: np.ndarray, Wg: np.ndarray, bias: Optional[np.ndarray] = None) -> np.ndarray:
    """float32 logits in the fixed summation order documented in gate_logits.c."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    Wg = np.ascontiguousarray(Wg, dtype=np.float32)
    T, M = x.shape
    E = Wg.shape[1]
    assert Wg.shape[0] == M
    out = np.empty((T, E), dtype=np.float32)
    b = None
    if bias is not None:
        b = np.ascontiguousarray(bias, dtype=np.float32)
        assert b.shape == (E,)
    _lib().oracle_gate_logits_f32(x.ctypes.data, Wg.ctypes.data,
                                  None if b is None else b.ctypes.data,
                                  T, M, E, out.ctypes.data)
    return out


def softmax_rows(logits: np.ndarray) -> np.ndarray:
    L = logits.astype(np.float64)
    L = L - L.max(axis=1, keepdims=True)
    ex = np.exp(L)
    return ex / ex.sum(axis=1, keepdims=True)


def top_k(logits: np.ndarray, k: int) -> np.ndarray:
    """Indices of the k largest logits per row, descending, ties to the lower index.

    NaN logits are ordered as minus infinity."""
    L = np.where(np.isnan(logits), -np.inf, logits).astype(np.float64)
    order = np.argsort(-L, axis=1, kind="stable")
    return order[:, :k].astype(np.int32)


def route(x, Wg, k: int, bias=None, renormalize: bool = False):
    """logits (float32), probabilities (float64), chosen experts and their weights.

    renormalize (a gate variant the paper does not use: it runs k = 1, where this would
    make every weight 1): the chosen probabilities are divided by their sum over the k
    choices of the token, before any drop."""
    logits = gate_logits(x, Wg, bias)
    p = softmax_rows(logits)
    idx = top_k(logits, k)
    w = np.take_along_axis(p, idx.astype(np.int64), axis=1)
    if renormalize:
        w = w / w.sum(axis=1, keepdims=True)
    return logits, p, idx, w


# --------------------------------------------------------------------------
# capacity-bounded slot assignment
# --------------------------------------------------------------------------

def assign_slots(idx: np.ndarray, E: int, C_p: int, n: int):
    """slot[t, j] (partition-local, -1 = dropped) and counts[p, e] of kept rows."""
    T, k = idx.shape
    T_p = T // n
    slot = np.full((T, k), -1, dtype=np.int32)
    counts = np.zeros((n, E), dtype=np.int32)
    for p in range(n):
        sl = slice(p * T_p, (p + 1) * T_p)
        # choice-major sequence: j = 0 for all tokens, then j = 1, ...
        seq = idx[sl].T.reshape(-1).astype(np.int64)          # length k*T_p
        pos = np.empty_like(seq)
        for e in range(E):
            m = seq == e
            pos[m] = np.arange(int(m.sum()))
            counts[p, e] = min(C_p, int(m.sum()))
        s = np.where(pos < C_p, seq * C_p + pos, -1).astype(np.int32)
        slot[sl] = s.reshape(k, T_p).T
    return slot, counts


# --------------------------------------------------------------------------
# activation
# --------------------------------------------------------------------------

def gelu(z):
    return 0.5 * z * (1.0 + _erf(z / math.sqrt(2.0)))


def gelu_grad(z):
    return 0.5 * (1.0 + _erf(z / math.sqrt(2.0))) + z * np.exp(-0.5 * z * z) / math.sqrt(2.0 * math.pi)


# --------------------------------------------------------------------------
# the whole layer, forward and backward
# --------------------------------------------------------------------------

def layer_step(x, Wg, W1, W2, dy, k: int, capacity_factor: float, n: int = 1,
               gate_bias=None, keep_intermediates: bool = False, renormalize: bool = False) -> Dict[str, np.ndarray]:
    """Forward and backward of the MoE layer over T tokens split into n partitions.

    x [T,M], Wg [M,E], W1 [E,M,H], W2 [E,H,M], dy [T,M] (upstream gradient).
    Returns routing (logits, idx, w, slot, counts), y, and the gradients
    dx, dWg, dW1, dW2 (all float64), plus dw [T,k] (gradient of the combine
    weights)."""
    T, M = x.shape
    E, _, H = W1.shape
    C_p = capacity(T, E, k, capacity_factor, n)
    T_p = T // n
    logits, p, idx, w = route(x, Wg, k, gate_bias, renormalize)
    slot, counts = assign_slots(idx, E, C_p, n)

    X = x.astype(np.float64)
    dY = dy.astype(np.float64)
    W1d = W1.astype(np.float64)
    W2d = W2.astype(np.float64)
    Wgd = Wg.astype(np.float64)

    y = np.zeros((T, M))
    dx = np.zeros((T, M))
    dW1 = np.zeros((E, M, H))
    dW2 = np.zeros((E, H, M))
    dw = np.zeros((T, k))
    inter = {}

    for part in range(n):
        t0 = part * T_p
        for e in range(E):
            c = int(counts[part, e])
            if c == 0:
                continue
            # rows of this expert in slot order: row r holds the (t, j) with slot e*C_p + r
            tt, jj = np.nonzero((slot[t0:t0 + T_p] >= e * C_p) & (slot[t0:t0 + T_p] < (e + 1) * C_p))
            r = slot[t0 + tt, jj] - e * C_p
            order = np.argsort(r)
            tt, jj = tt[order] + t0, jj[order]
            assert np.array_equal(np.sort(r), np.arange(c))
            # forward
            DI = X[tt]                      # dispatch
            Z = DI @ W1d[e]                 # first linear layer  (T_M, pre-activation)
            A = gelu(Z)
            O = A @ W2d[e]                  # second linear layer (T_DO)
            wrow = w[tt, jj][:, None]
            np.add.at(y, tt, wrow * O)      # combine
            # backward
            dw[tt, jj] = np.einsum("rm,rm->r", dY[tt], O)
            dO = wrow * dY[tt]
            dA = dO @ W2d[e].T
            dW2[e] += A.T @ dO
            dZ = dA * gelu_grad(Z)
            dDI = dZ @ W1d[e].T
            dW1[e] += DI.T @ dZ
            np.add.at(dx, tt, dDI)
            if keep_intermediates:
                inter[(part, e)] = dict(tokens=tt, choice=jj, DI=DI, Z=Z, O=O, dO=dO, dZ=dZ, dDI=dDI)

    # gate backward: softmax Jacobian on the chosen probabilities
    dp_sel = dw
    if renormalize:
        # w_j = p_j / S with S the sum of the chosen probabilities: d/dp_j = dw_j / S - sum_j' dw_j' p_j' / S^2
        p_sel = np.take_along_axis(p, idx.astype(np.int64), axis=1)
        S = p_sel.sum(axis=1, keepdims=True)
        dp_sel = dw / S - (dw * p_sel).sum(axis=1, keepdims=True) / (S * S)
    dp = np.zeros((T, E))
    np.put_along_axis(dp, idx.astype(np.int64), dp_sel, axis=1)
    dL = p * (dp - (dp * p).sum(axis=1, keepdims=True))
    dWg = X.T @ dL
    dx += dL @ Wgd.T

    out = dict(logits=logits, p=p, idx=idx, w=w, slot=slot, counts=counts, C_p=C_p,
               y=y, dx=dx, dWg=dWg, dW1=dW1, dW2=dW2, dw=dw, dL=dL)
    if keep_intermediates:
        out["inter"] = inter
    return out


# --------------------------------------------------------------------------
# sampled evaluation for shapes too large to run whole
# --------------------------------------------------------------------------

def _rows_of_expert(slot_part: np.ndarray, e: int, C_p: int):
    tt, jj = np.nonzero((slot_part >= e * C_p) & (slot_part < (e + 1) * C_p))
    r = slot_part[tt, jj] - e * C_p
    order = np.argsort(r)
    return tt[order], jj[order]


def sampled_tokens(x, Wg, W1, W2, dy, routing: Dict[str, np.ndarray], tokens: Sequence[int]):
    """y[t], dw[t], and the expert-path part of dx[t] for chosen tokens, from the definition.

    `routing` holds w [T,k], idx [T,k], slot [T,k] from route()/assign_slots().
    The gate path of dx needs dL[t], which depends only on token t: it is added
    here too, so the returned dx rows are complete."""
    tokens = np.asarray(tokens, dtype=np.int64)
    T, M = x.shape
    k = routing["idx"].shape[1]
    p = softmax_rows(routing["logits"][tokens])
    y = np.zeros((len(tokens), M))
    dx = np.zeros((len(tokens), M))
    dw = np.zeros((len(tokens), k))
    cache = {}
    for i, t in enumerate(tokens):
        xt = x[t].astype(np.float64)
        dyt = dy[t].astype(np.float64)
        for j in range(k):
            if routing["slot"][t, j] < 0:
                continue
            e = int(routing["idx"][t, j])
            if e not in cache:
                if len(cache) >= 4:
                    cache.pop(next(iter(cache)))
                cache[e] = (W1[e].astype(np.float64), W2[e].astype(np.float64))
            W1e, W2e = cache[e]
            wt = float(routing["w"][t, j])
            z = xt @ W1e
            a = gelu(z)
            o = a @ W2e
            y[i] += wt * o
            dw[i, j] = dyt @ o
            dz = ((wt * dyt) @ W2e.T) * gelu_grad(z)
            dx[i] += dz @ W1e.T
        dp = np.zeros(p.shape[1])
        dp[routing["idx"][t].astype(np.int64)] = dw[i]
        dL = p[i] * (dp - (dp * p[i]).sum())
        dx[i] += dL @ Wg.astype(np.float64).T
    return dict(y=y, dx=dx, dw=dw)


def sampled_weight_grads(x, W1, W2, dy, routing, n: int, C_p: int, e: int,
                         h_cols: Sequence[int], m_cols: Sequence[int]):
    """dW1[e][:, h_cols] and dW2[e][:, m_cols] over all partitions, from the definition.

    dW1[e][:, h] = sum_s DI_s^T dZ_s[h] needs, per row, only column h of T_M and of
    its gradient; dW2[e][:, m] = sum_s A_s^T dO_s[m] needs the whole activation row,
    so T_M of expert e is formed once."""
    T, M = x.shape
    T_p = T // n
    W1e = W1[e].astype(np.float64)
    W2e = W2[e].astype(np.float64)
    h_cols = np.asarray(h_cols, dtype=np.int64)
    m_cols = np.asarray(m_cols, dtype=np.int64)
    dW1c = np.zeros((M, len(h_cols)))
    dW2c = np.zeros((W2e.shape[0], len(m_cols)))
    for part in range(n):
        t0 = part * T_p
        tt, jj = _rows_of_expert(routing["slot"][t0:t0 + T_p], e, C_p)
        if len(tt) == 0:
            continue
        tt = tt + t0
        DI = x[tt].astype(np.float64)
        dO = routing["w"][tt, jj][:, None] * dy[tt].astype(np.float64)
        Z = DI @ W1e
        A = gelu(Z)
        dW2c += A.T @ dO[:, m_cols]
        dA_c = dO @ W2e[h_cols].T
        dZ_c = dA_c * gelu_grad(Z[:, h_cols])
        dW1c += DI.T @ dZ_c
    return dW1c, dW2c
