"""CPU oracle for the performance model of the memory-reuse strategies
(Section III-E: Eq. 7-10 and Table II).

TEST INFRASTRUCTURE ONLY.  Nothing on the product path may import this file.
It shares no code with the C++ implementation behind the C ABI.

Per micro-batch of b tokens the three streams carry (Eq. 7-9)
    v0_comp = b * H * M      multiply-adds of one GEMM
    v0_comm = b * M          elements of one All-to-All (here: one local dispatch or combine)
    v0_mem  = b * M          elements of one copy of T_DI between device and host
and a strategy is described by how many such units each stream executes in the
forward and in the backward pass, Q = [q1, q2, q3] (Table II), and by which
slowdown factors apply to its streams.  The cost of a pass is the time of its
slowest stream (Eq. 10, first line):

    C = max( q1 v0_comp / (sigma W_comp), q2 v0_comm / (mu W_comm), q3 v0_mem / (eta W_mem) )

Readings (also in the design notes): the section's prose fixes sigma for
computation, mu for communication, eta for memory copies; the first line of
Eq. 10 prints mu in its third term, the second line eta - eta is taken.  The
second and third lines of Eq. 10 are the same expression divided through by
v0_comp / W_comp with alpha, beta absorbing the volume ratios; `cost_relative`
writes that form out and a test ties the two together.  The strategy chosen is
the one with the smallest forward + backward cost; ties go to the earlier row of
Table II.
"""
from __future__ import annotations

from typing import Dict, Iterable, Tuple

# Table II: how T_DI and T_M are restored in backward, which slowdown factors apply, Q_fw, Q_bw
TABLE_II: Dict[str, dict] = {
    "none": dict(T_DI="-", T_M="-", mu="mu_comp", eta=None, Q_fw=(2, 2, 0), Q_bw=(4, 2, 0)),
    "S1": dict(T_DI="offload", T_M="offload", mu="mu_all", eta="eta_all", Q_fw=(2, 2, 5), Q_bw=(4, 2, 5)),
    "S2": dict(T_DI="comm.", T_M="offload", mu="mu_all", eta="eta_all", Q_fw=(2, 2, 4), Q_bw=(4, 3, 4)),
    "S3": dict(T_DI="offload", T_M="recompute", mu="mu_all", eta="eta_all", Q_fw=(2, 2, 1), Q_bw=(5, 2, 1)),
    "S4": dict(T_DI="comm.", T_M="recompute", mu="mu_comp", eta=None, Q_fw=(2, 2, 0), Q_bw=(5, 3, 0)),
}
ORDER = ("none", "S1", "S2", "S3", "S4")


def v0(b: float, H: float, M: float) -> Tuple[float, float, float]:
    """Eq. 7-9."""
    return (b * H * M, b * M, b * M)


def cost(Q: Iterable[float], v: Tuple[float, float, float], W_comp: float, W_comm: float, W_mem: float,
         sigma: float, mu: float, eta: float) -> float:
    """Eq. 10, first line (eta in the third term)."""
    q1, q2, q3 = Q
    t_comp = q1 * v[0] / (sigma * W_comp)
    t_comm = q2 * v[1] / (mu * W_comm)
    t_mem = q3 * v[2] / (eta * W_mem) if q3 else 0.0
    return max(t_comp, t_comm, t_mem)


def cost_relative(Q: Iterable[float], alpha: float, beta: float, mu: float, eta: float) -> float:
    """Eq. 10, last line without the 1/W_comp factor: max(Q . [1, 1/mu, 1/eta] . [1, alpha, beta]),
    with alpha, beta the ratios of the time of one unit of communication / copying to the time of one
    unit of computation (sigma = 1 as the section sets it)."""
    q1, q2, q3 = Q
    return max(q1, q2 * alpha / mu, (q3 * beta / eta) if q3 else 0.0)


def strategy_cost(name: str, b: float, H: float, M: float, speeds: dict) -> Tuple[float, float]:
    """(forward, backward) cost of a row of Table II for micro-batches of b tokens.
    speeds: W_comp, W_comm, W_mem, sigma, mu_comp, mu_all, eta_all."""
    row = TABLE_II[name]
    v = v0(b, H, M)
    mu = speeds[row["mu"]]
    eta = speeds[row["eta"]] if row["eta"] else 1.0
    args = (speeds["W_comp"], speeds["W_comm"], speeds["W_mem"], speeds["sigma"], mu, eta)
    return cost(row["Q_fw"], v, *args), cost(row["Q_bw"], v, *args)


def select(allowed: Iterable[str], b: float, H: float, M: float, speeds: dict) -> Tuple[str, float]:
    """The allowed strategy with the smallest forward + backward cost; ties to the earlier row."""
    best, best_cost = None, None
    for name in ORDER:
        if name not in allowed:
            continue
        fw, bw = strategy_cost(name, b, H, M, speeds)
        if best is None or fw + bw < best_cost:
            best, best_cost = name, fw + bw
    return best, best_cost
