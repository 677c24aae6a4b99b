"""Thin ctypes binding of libmoe_hip.so: argument marshalling only.

Every function has the name and the argument order of its C entry point in
include/moe.h; tensors are torch tensors on the GPU (used here only as device
memory), streams are torch.cuda.Stream objects or raw integers.  A non-zero
status raises MoEError.  There is no CPU fallback: if the HIP library is not
built, importing this module's functions raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmoe_hip.so")

MOE_F32, MOE_BF16 = 0, 1
MOE_REUSE_NONE, MOE_REUSE_BUFFERS, MOE_REUSE_RECOMPUTE = 0, 1, 2
MOE_REUSE_S1, MOE_REUSE_S2, MOE_REUSE_S3 = 3, 4, 5

EXPORTS = [
    "moe_capacity", "moe_workspace_bytes", "moe_route", "moe_assign_slots", "moe_assign_slots_static", "moe_slot_scratch_bytes",
    "moe_dispatch", "moe_expert_ffn_fwd", "moe_expert_ffn_bwd", "moe_dw_parts", "moe_combine",
    "moe_slot_rows", "moe_expert_ffn_fwd_gather",
    "moe_gate_bwd", "moe_gate_scratch_bytes", "moe_dispatch_bwd", "moe_layer_step",
    "moe_layer_forward", "moe_layer_backward", "moe_launch_counts", "moe_status_string",
    "moe_last_error", "moe_profile_enable", "moe_profile_read",
    "moe_gran_create", "moe_gran_destroy", "moe_gran_lookup", "moe_gran_record", "moe_gran_ranges",
    "moe_search_best_gran", "moe_gran_get", "moe_strategy_cost", "moe_select_strategy",
    "moe_offload_bytes", "moe_layer_step_offload",
]


class MoEError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        detail = lib().moe_last_error().decode() if status == 5 else ""
        super().__init__(f"{where}: status {status} ({status_string(status)}) {detail}")


class MoEConfig(ctypes.Structure):
    _fields_ = [("T", ctypes.c_int32), ("M", ctypes.c_int32), ("H", ctypes.c_int32), ("E", ctypes.c_int32),
                ("k", ctypes.c_int32), ("capacity_factor", ctypes.c_float), ("n_partitions", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("reuse", ctypes.c_int32), ("grad_overwrite", ctypes.c_int32), ("gate_renormalize", ctypes.c_int32),
                ("fuse_gather", ctypes.c_int32), ("wgrad_group", ctypes.c_int32), ("gemm_free_cus", ctypes.c_int32),
                ("fuse_combine", ctypes.c_int32)]


def make_config(T, M, H, E, k, capacity_factor, n_partitions=1, dtype=MOE_BF16, reuse=MOE_REUSE_NONE,
                grad_overwrite=0, gate_renormalize=0, fuse_gather=0, wgrad_group=0, gemm_free_cus=0, fuse_combine=0) -> MoEConfig:
    return MoEConfig(int(T), int(M), int(H), int(E), int(k), float(capacity_factor), int(n_partitions),
                     int(dtype), int(reuse), int(grad_overwrite), int(gate_renormalize), int(fuse_gather),
                     int(wgrad_group), int(gemm_free_cus), int(fuse_combine))


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is not built; run `python -m paper_2506_22175_amd.build` "
                               "(there is no fallback path)")
        _lib = ctypes.CDLL(LIB_PATH)
        for name in EXPORTS:
            fn = getattr(_lib, name)
            fn.restype = ctypes.c_char_p if name in ("moe_status_string", "moe_last_error") else ctypes.c_int
    return _lib


def status_string(status: int) -> str:
    return lib().moe_status_string(ctypes.c_int(status)).decode()


def _p(t) -> ctypes.c_void_p:
    """Device (or host) pointer of a tensor, an int, or None."""
    if t is None:
        return ctypes.c_void_p(0)
    if isinstance(t, int):
        return ctypes.c_void_p(t)
    return ctypes.c_void_p(t.data_ptr())


def _s(stream) -> ctypes.c_void_p:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    if isinstance(stream, int):
        return ctypes.c_void_p(stream)
    return ctypes.c_void_p(stream.cuda_stream)


def _check(status: int, where: str):
    if status != 0:
        raise MoEError(status, where)


def _cfg(cfg: MoEConfig):
    return ctypes.byref(cfg)


# ---- host-only queries -----------------------------------------------------------

def moe_capacity(cfg: MoEConfig) -> int:
    out = ctypes.c_int32(0)
    _check(lib().moe_capacity(_cfg(cfg), ctypes.byref(out)), "moe_capacity")
    return out.value


def moe_workspace_bytes(cfg: MoEConfig):
    """(total, saved, temp, routing) bytes."""
    v = [ctypes.c_size_t(0) for _ in range(4)]
    _check(lib().moe_workspace_bytes(_cfg(cfg), *[ctypes.byref(x) for x in v]), "moe_workspace_bytes")
    return tuple(x.value for x in v)


def moe_slot_scratch_bytes(cfg: MoEConfig) -> int:
    v = ctypes.c_size_t(0)
    _check(lib().moe_slot_scratch_bytes(_cfg(cfg), ctypes.byref(v)), "moe_slot_scratch_bytes")
    return v.value


def moe_gate_scratch_bytes(cfg: MoEConfig) -> int:
    v = ctypes.c_size_t(0)
    _check(lib().moe_gate_scratch_bytes(_cfg(cfg), ctypes.byref(v)), "moe_gate_scratch_bytes")
    return v.value


def moe_dw_parts(cfg: MoEConfig) -> int:
    v = ctypes.c_int32(0)
    _check(lib().moe_dw_parts(_cfg(cfg), ctypes.byref(v)), "moe_dw_parts")
    return v.value


def moe_launch_counts(reset: bool = False):
    arr = (ctypes.c_int64 * 3)()
    _check(lib().moe_launch_counts(arr, ctypes.c_int32(1 if reset else 0)), "moe_launch_counts")
    return tuple(arr)


PROFILE_KINDS = ["gemm_fwd1_gelu", "gemm_nn_store", "gemm_dgelu", "gemm_dgrad", "gemm_wgrad", "dispatch",
                 "combine", "dispatch_bwd", "route", "slots", "gate_bwd"]


def moe_profile_enable(on: bool):
    _check(lib().moe_profile_enable(ctypes.c_int32(1 if on else 0)), "moe_profile_enable")


def moe_profile_read():
    """{kind: (launches, total_ms)} of the kernels timed since moe_profile_enable(True)."""
    n = len(PROFILE_KINDS)
    launches = (ctypes.c_int64 * n)()
    ms = (ctypes.c_double * n)()
    _check(lib().moe_profile_read(ctypes.c_int32(n), launches, ms), "moe_profile_read")
    return {PROFILE_KINDS[i]: (int(launches[i]), float(ms[i])) for i in range(n)}


# ---- device calls ----------------------------------------------------------------

def moe_route(cfg, x, Wg, gate_bias, logits, topk_idx, topk_w, stream=None):
    _check(lib().moe_route(_cfg(cfg), _p(x), _p(Wg), _p(gate_bias), _p(logits), _p(topk_idx), _p(topk_w),
                           _s(stream)), "moe_route")


def moe_assign_slots(cfg, topk_idx, topk_w, slot, counts, slot_w, scratch, stream=None):
    _check(lib().moe_assign_slots(_cfg(cfg), _p(topk_idx), _p(topk_w), _p(slot), _p(counts), _p(slot_w),
                                  _p(scratch), _s(stream)), "moe_assign_slots")


def moe_assign_slots_static(cfg, topk_idx, topk_w, slot, counts, slot_w, stream=None):
    _check(lib().moe_assign_slots_static(_cfg(cfg), _p(topk_idx), _p(topk_w), _p(slot), _p(counts), _p(slot_w),
                                         _s(stream)), "moe_assign_slots_static")


def moe_dispatch(cfg, part, src, slot, DI, dO_saved=None, dw=None, stream=None):
    _check(lib().moe_dispatch(_cfg(cfg), ctypes.c_int32(part), _p(src), _p(slot), _p(DI), _p(dO_saved), _p(dw),
                              _s(stream)), "moe_dispatch")


def moe_slot_rows(cfg, slot, rows, stream=None):
    _check(lib().moe_slot_rows(_cfg(cfg), _p(slot), _p(rows), _s(stream)), "moe_slot_rows")


def moe_expert_ffn_fwd_gather(cfg, part, x, rows, counts, W1, W2, Z, A, DO, stream=None):
    _check(lib().moe_expert_ffn_fwd_gather(_cfg(cfg), ctypes.c_int32(part), _p(x), _p(rows), _p(counts), _p(W1),
                                           _p(W2), _p(Z), _p(A), _p(DO), _s(stream)), "moe_expert_ffn_fwd_gather")


def moe_expert_ffn_fwd(cfg, part, DI, counts, W1, W2, Z, A, DO, stream=None):
    _check(lib().moe_expert_ffn_fwd(_cfg(cfg), ctypes.c_int32(part), _p(DI), _p(counts), _p(W1), _p(W2),
                                    _p(Z), _p(A), _p(DO), _s(stream)), "moe_expert_ffn_fwd")


def moe_expert_ffn_bwd(cfg, part, recompute, DI, Z, dDO, counts, slot_w, W1, W2, dZ, dDI, dW1, dW2, dw_part,
                       stream=None):
    _check(lib().moe_expert_ffn_bwd(_cfg(cfg), ctypes.c_int32(part), ctypes.c_int32(int(recompute)), _p(DI),
                                    _p(Z), _p(dDO), _p(counts), _p(slot_w), _p(W1), _p(W2), _p(dZ), _p(dDI),
                                    _p(dW1), _p(dW2), _p(dw_part), _s(stream)), "moe_expert_ffn_bwd")


def moe_combine(cfg, part, DO, slot, topk_w, y, stream=None):
    _check(lib().moe_combine(_cfg(cfg), ctypes.c_int32(part), _p(DO), _p(slot), _p(topk_w), _p(y), _s(stream)),
           "moe_combine")


def moe_gate_bwd(cfg, part, x, logits, topk_idx, slot, dw, dw_part, dL, dWg, scratch, stream=None):
    _check(lib().moe_gate_bwd(_cfg(cfg), ctypes.c_int32(part), _p(x), _p(logits), _p(topk_idx), _p(slot),
                              _p(dw), _p(dw_part), _p(dL), _p(dWg), _p(scratch), _s(stream)), "moe_gate_bwd")


def moe_dispatch_bwd(cfg, part, dDI, slot, dL, Wg, dx, stream=None):
    _check(lib().moe_dispatch_bwd(_cfg(cfg), ctypes.c_int32(part), _p(dDI), _p(slot), _p(dL), _p(Wg), _p(dx),
                                  _s(stream)), "moe_dispatch_bwd")


def _streams(streams: Optional[Sequence]):
    import torch
    if streams is None:
        cur = torch.cuda.current_stream()
        streams = [cur, cur]
    arr = (ctypes.c_void_p * len(streams))(*[_s(s).value for s in streams])
    return arr, ctypes.c_int32(len(streams))


def moe_layer_step(cfg, x, dy, Wg, gate_bias, W1, W2, y, dx, dWg, dW1, dW2, logits, topk_idx, topk_w, slot,
                   counts, workspace, streams=None):
    arr, n = _streams(streams)
    _check(lib().moe_layer_step(_cfg(cfg), _p(x), _p(dy), _p(Wg), _p(gate_bias), _p(W1), _p(W2), _p(y), _p(dx),
                                _p(dWg), _p(dW1), _p(dW2), _p(logits), _p(topk_idx), _p(topk_w), _p(slot),
                                _p(counts), _p(workspace), ctypes.c_size_t(workspace.numel() * workspace.element_size()),
                                arr, n), "moe_layer_step")


def moe_layer_forward(cfg, x, Wg, gate_bias, W1, W2, y, logits, topk_idx, topk_w, slot, counts, workspace,
                      streams=None):
    arr, n = _streams(streams)
    _check(lib().moe_layer_forward(_cfg(cfg), _p(x), _p(Wg), _p(gate_bias), _p(W1), _p(W2), _p(y), _p(logits),
                                   _p(topk_idx), _p(topk_w), _p(slot), _p(counts), _p(workspace),
                                   ctypes.c_size_t(workspace.numel() * workspace.element_size()), arr, n),
           "moe_layer_forward")


def moe_layer_backward(cfg, x, dy, Wg, W1, W2, dx, dWg, dW1, dW2, logits, topk_idx, topk_w, slot, counts,
                       workspace, streams=None):
    arr, n = _streams(streams)
    _check(lib().moe_layer_backward(_cfg(cfg), _p(x), _p(dy), _p(Wg), _p(W1), _p(W2), _p(dx), _p(dWg), _p(dW1),
                                    _p(dW2), _p(logits), _p(topk_idx), _p(topk_w), _p(slot), _p(counts),
                                    _p(workspace), ctypes.c_size_t(workspace.numel() * workspace.element_size()),
                                    arr, n), "moe_layer_backward")


# ---- adaptive pipeline granularity ---------------------------------------------------

class GranHandle:
    """Owner of a moe_gran handle (the table and the range set of the granularity search)."""

    def __init__(self):
        self._h = ctypes.c_void_p(0)
        _check(lib().moe_gran_create(ctypes.byref(self._h)), "moe_gran_create")

    def close(self):
        if self._h:
            lib().moe_gran_destroy(self._h)
            self._h = ctypes.c_void_p(0)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def moe_gran_lookup(g: GranHandle, B: int) -> int:
    n = ctypes.c_int32(0)
    _check(lib().moe_gran_lookup(g._h, ctypes.c_int64(B), ctypes.byref(n)), "moe_gran_lookup")
    return n.value


def moe_gran_record(g: GranHandle, B: int, n: int):
    _check(lib().moe_gran_record(g._h, ctypes.c_int64(B), ctypes.c_int32(n)), "moe_gran_record")


def moe_gran_ranges(g: GranHandle):
    """[(lower, upper, n), ...] ordered by lower bound."""
    count = ctypes.c_int32(0)
    _check(lib().moe_gran_ranges(g._h, ctypes.c_int32(0), None, None, None, ctypes.byref(count)), "moe_gran_ranges")
    c = count.value
    lo, up, nn = (ctypes.c_int64 * max(c, 1))(), (ctypes.c_int64 * max(c, 1))(), (ctypes.c_int32 * max(c, 1))()
    _check(lib().moe_gran_ranges(g._h, ctypes.c_int32(c), lo, up, nn, ctypes.byref(count)), "moe_gran_ranges")
    return [(int(lo[i]), int(up[i]), int(nn[i])) for i in range(c)]


def _layer_args(cfg, x, dy, Wg, gate_bias, W1, W2, y, dx, dWg, dW1, dW2, logits, topk_idx, topk_w, slot, counts,
                workspace, streams):
    arr, n = _streams(streams)
    return (_cfg(cfg), _p(x), _p(dy), _p(Wg), _p(gate_bias), _p(W1), _p(W2), _p(y), _p(dx), _p(dWg), _p(dW1),
            _p(dW2), _p(logits), _p(topk_idx), _p(topk_w), _p(slot), _p(counts), _p(workspace),
            ctypes.c_size_t(workspace.numel() * workspace.element_size()), arr, n), arr


def moe_search_best_gran(cfg, x, dy, Wg, gate_bias, W1, W2, y, dx, dWg, dW1, dW2, logits, topk_idx, topk_w, slot,
                         counts, workspace, streams, candidates, warmup=1, iters=3):
    """(best n, [ms per step per candidate, -1 = skipped])."""
    args, keep = _layer_args(cfg, x, dy, Wg, gate_bias, W1, W2, y, dx, dWg, dW1, dW2, logits, topk_idx, topk_w,
                             slot, counts, workspace, streams)
    cand = (ctypes.c_int32 * len(candidates))(*candidates)
    ms = (ctypes.c_float * len(candidates))()
    best = ctypes.c_int32(0)
    _check(lib().moe_search_best_gran(*args, cand, ctypes.c_int32(len(candidates)), ctypes.c_int32(warmup),
                                      ctypes.c_int32(iters), ctypes.byref(best), ms), "moe_search_best_gran")
    return best.value, [float(v) for v in ms]


def moe_gran_get(g: GranHandle, cfg, x, dy, Wg, gate_bias, W1, W2, y, dx, dWg, dW1, dW2, logits, topk_idx, topk_w,
                 slot, counts, workspace, streams, candidates, warmup=1, iters=3):
    """(n, searched) for B = cfg.T."""
    args, keep = _layer_args(cfg, x, dy, Wg, gate_bias, W1, W2, y, dx, dWg, dW1, dW2, logits, topk_idx, topk_w,
                             slot, counts, workspace, streams)
    cand = (ctypes.c_int32 * len(candidates))(*candidates)
    n = ctypes.c_int32(0)
    searched = ctypes.c_int32(0)
    _check(lib().moe_gran_get(g._h, *args, cand, ctypes.c_int32(len(candidates)), ctypes.c_int32(warmup),
                              ctypes.c_int32(iters), ctypes.byref(n), ctypes.byref(searched)), "moe_gran_get")
    return n.value, bool(searched.value)


# ---- performance model of the reuse strategies -----------------------------------------

class MoESpeeds(ctypes.Structure):
    _fields_ = [("W_comp", ctypes.c_double), ("W_comm", ctypes.c_double), ("W_mem", ctypes.c_double),
                ("sigma", ctypes.c_double), ("mu_comp", ctypes.c_double), ("mu_all", ctypes.c_double),
                ("eta_all", ctypes.c_double)]


STRATEGIES = ("none", "S1", "S2", "S3", "S4")


def moe_strategy_cost(strategy: int, b: int, M: int, H: int, speeds: MoESpeeds):
    """(forward, backward) seconds per micro-batch."""
    fw, bw = ctypes.c_double(0), ctypes.c_double(0)
    _check(lib().moe_strategy_cost(ctypes.c_int32(strategy), ctypes.c_int64(b), ctypes.c_int64(M), ctypes.c_int64(H),
                                   ctypes.byref(speeds), ctypes.byref(fw), ctypes.byref(bw)), "moe_strategy_cost")
    return fw.value, bw.value


def moe_select_strategy(allowed_mask: int, b: int, M: int, H: int, speeds: MoESpeeds):
    """(strategy number, forward + backward seconds)."""
    best, cost = ctypes.c_int32(0), ctypes.c_double(0)
    _check(lib().moe_select_strategy(ctypes.c_uint32(allowed_mask), ctypes.c_int64(b), ctypes.c_int64(M),
                                     ctypes.c_int64(H), ctypes.byref(speeds), ctypes.byref(best), ctypes.byref(cost)),
           "moe_select_strategy")
    return best.value, cost.value


# ---- offloading strategies ---------------------------------------------------------------

def moe_offload_bytes(cfg: MoEConfig) -> int:
    v = ctypes.c_size_t(0)
    _check(lib().moe_offload_bytes(_cfg(cfg), ctypes.byref(v)), "moe_offload_bytes")
    return v.value


def moe_layer_step_offload(cfg, x, dy, Wg, gate_bias, W1, W2, y, dx, dWg, dW1, dW2, logits, topk_idx, topk_w, slot,
                           counts, workspace, host_buffer, streams):
    """host_buffer: pinned host tensor (uint8); streams: three streams."""
    arr, n = _streams(streams)
    _check(lib().moe_layer_step_offload(_cfg(cfg), _p(x), _p(dy), _p(Wg), _p(gate_bias), _p(W1), _p(W2), _p(y),
                                        _p(dx), _p(dWg), _p(dW1), _p(dW2), _p(logits), _p(topk_idx), _p(topk_w),
                                        _p(slot), _p(counts), _p(workspace),
                                        ctypes.c_size_t(workspace.numel() * workspace.element_size()),
                                        _p(host_buffer), ctypes.c_size_t(host_buffer.numel() * host_buffer.element_size()),
                                        arr, n), "moe_layer_step_offload")
