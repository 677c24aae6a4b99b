"""Device-memory plumbing around the C ABI: upload inputs, allocate outputs and the
workspace with torch, call moe_layer_step, download results.  No arithmetic of the
layer happens here."""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np
import torch

from . import binding as B

_TORCH_DT = {"f32": torch.float32, "bf16": torch.bfloat16}
_MOE_DT = {"f32": B.MOE_F32, "bf16": B.MOE_BF16}


def to_device(a: np.ndarray, dtype: str, device="cuda:0") -> torch.Tensor:
    """float32 host array -> device tensor of the storage type (values must be representable)."""
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device).to(_TORCH_DT[dtype]).contiguous()


def to_host(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.bfloat16:
        t = t.float()
    return t.cpu().numpy()


class LayerState:
    """All device buffers of one layer step for a given configuration."""

    def __init__(self, T, M, H, E, k, capacity_factor, n_partitions=1, dtype="bf16", reuse=0, device="cuda:0",
                 second_stream: bool = True, grad_overwrite: int = 0, size_for_partitions=(),
                 gate_renormalize: int = 0, fuse_gather: int = 0, wgrad_group: int = 0, gemm_free_cus: int = 0, fuse_combine: int = 0):
        self.dtype = dtype
        self.device = device
        self.cfg = B.make_config(T, M, H, E, k, capacity_factor, n_partitions, _MOE_DT[dtype], reuse, grad_overwrite,
                                 gate_renormalize, fuse_gather, wgrad_group, gemm_free_cus, fuse_combine)
        self.C_p = B.moe_capacity(self.cfg)
        self.ws_total, self.ws_saved, self.ws_temp, self.ws_routing = B.moe_workspace_bytes(self.cfg)
        ws_alloc, n_max = self.ws_total, n_partitions
        for n_alt in size_for_partitions:      # buffers that also fit these partition counts (granularity search)
            if T % n_alt == 0:
                alt = B.make_config(T, M, H, E, k, capacity_factor, n_alt, _MOE_DT[dtype], reuse, grad_overwrite,
                                    gate_renormalize, fuse_gather, wgrad_group, gemm_free_cus, fuse_combine)
                ws_alloc = max(ws_alloc, B.moe_workspace_bytes(alt)[0])
                n_max = max(n_max, n_alt)
        td = _TORCH_DT[dtype]
        dev = device
        self.y = torch.empty((T, M), dtype=td, device=dev)
        self.dx = torch.empty((T, M), dtype=td, device=dev)
        self.dWg = torch.zeros((M, E), dtype=torch.float32, device=dev)
        self.dW1 = torch.zeros((E, M, H), dtype=torch.float32, device=dev)
        self.dW2 = torch.zeros((E, H, M), dtype=torch.float32, device=dev)
        self.logits = torch.empty((T, E), dtype=torch.float32, device=dev)
        self.topk_idx = torch.empty((T, k), dtype=torch.int32, device=dev)
        self.topk_w = torch.empty((T, k), dtype=torch.float32, device=dev)
        self.slot = torch.empty((T, k), dtype=torch.int32, device=dev)
        self.counts = torch.empty((n_max, E), dtype=torch.int32, device=dev)
        self.workspace = torch.empty((ws_alloc,), dtype=torch.uint8, device=dev)
        self.s0 = torch.cuda.current_stream(dev)
        self.s1 = torch.cuda.Stream(dev) if second_stream else self.s0
        # offloading strategies: pinned host buffer and a third stream for the copies
        self.host_buffer = None
        self.s2 = None
        if reuse >= B.MOE_REUSE_S1:
            self.host_buffer = torch.empty((max(B.moe_offload_bytes(self.cfg), 1),), dtype=torch.uint8, pin_memory=True)
            self.s2 = torch.cuda.Stream(dev) if second_stream else self.s0
        self.inputs: Dict[str, Optional[torch.Tensor]] = {}

    def upload(self, inp: Dict[str, np.ndarray]):
        for name in ("x", "Wg", "W1", "W2", "dy"):
            self.inputs[name] = to_device(inp[name], self.dtype, self.device)
        gb = inp.get("gate_bias")
        self.inputs["gate_bias"] = None if gb is None else torch.from_numpy(np.asarray(gb, dtype=np.float32)).to(self.device)

    def zero_grads(self):
        self.dWg.zero_()
        self.dW1.zero_()
        self.dW2.zero_()

    def poison(self):
        """Fill everything the step must overwrite with NaN / -2 so stale data shows."""
        self.workspace.fill_(0xFF)          # 0xFFFF bf16 and 0xFFFFFFFF float are NaN
        if self.host_buffer is not None:
            self.host_buffer.fill_(0xFF)
        for t in (self.y, self.dx, self.logits, self.topk_w):
            t.fill_(float("nan"))
        self.topk_idx.fill_(-2)
        self.slot.fill_(-2)
        self.counts.fill_(-2)

    def step(self):
        i = self.inputs
        if self.host_buffer is not None:
            B.moe_layer_step_offload(self.cfg, i["x"], i["dy"], i["Wg"], i["gate_bias"], i["W1"], i["W2"], self.y,
                                     self.dx, self.dWg, self.dW1, self.dW2, self.logits, self.topk_idx, self.topk_w,
                                     self.slot, self.counts, self.workspace, self.host_buffer,
                                     [self.s0, self.s1, self.s2])
            return
        B.moe_layer_step(self.cfg, i["x"], i["dy"], i["Wg"], i["gate_bias"], i["W1"], i["W2"], self.y, self.dx,
                         self.dWg, self.dW1, self.dW2, self.logits, self.topk_idx, self.topk_w, self.slot,
                         self.counts, self.workspace, [self.s0, self.s1])

    def forward(self):
        i = self.inputs
        B.moe_layer_forward(self.cfg, i["x"], i["Wg"], i["gate_bias"], i["W1"], i["W2"], self.y, self.logits,
                            self.topk_idx, self.topk_w, self.slot, self.counts, self.workspace, [self.s0, self.s1])

    def backward(self):
        i = self.inputs
        B.moe_layer_backward(self.cfg, i["x"], i["dy"], i["Wg"], i["W1"], i["W2"], self.dx, self.dWg, self.dW1,
                             self.dW2, self.logits, self.topk_idx, self.topk_w, self.slot, self.counts,
                             self.workspace, [self.s0, self.s1])

    def search_best_gran(self, candidates, warmup=1, iters=3):
        """Timed trials of the step over the candidate partition counts (this state's buffers
        must have been sized for the largest candidate).  Returns (best n, ms per candidate)."""
        i = self.inputs
        return B.moe_search_best_gran(self.cfg, i["x"], i["dy"], i["Wg"], i["gate_bias"], i["W1"], i["W2"], self.y,
                                      self.dx, self.dWg, self.dW1, self.dW2, self.logits, self.topk_idx,
                                      self.topk_w, self.slot, self.counts, self.workspace, [self.s0, self.s1],
                                      candidates, warmup, iters)

    def gran_get(self, handle, candidates, warmup=1, iters=3):
        """Algorithm 1 for this state's batch size: (n, searched)."""
        i = self.inputs
        return B.moe_gran_get(handle, self.cfg, i["x"], i["dy"], i["Wg"], i["gate_bias"], i["W1"], i["W2"], self.y,
                              self.dx, self.dWg, self.dW1, self.dW2, self.logits, self.topk_idx, self.topk_w,
                              self.slot, self.counts, self.workspace, [self.s0, self.s1], candidates, warmup, iters)

    def capture(self):
        """Record one step into a HIP graph (all launches and the cross-stream events of
        moe_layer_step are capturable; the library issues no memset nodes).  Returns the graph;
        call .replay() on it.  The step must have run eagerly once before (kernel attributes)."""
        torch.cuda.synchronize(self.device)
        side = torch.cuda.Stream(self.device)
        keep0 = self.s0
        g = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            self.s0 = side
            try:
                with torch.cuda.graph(g, stream=side):
                    self.step()
            finally:
                self.s0 = keep0
        torch.cuda.synchronize(self.device)
        return g

    def results(self) -> Dict[str, np.ndarray]:
        torch.cuda.synchronize(self.device)
        return dict(y=to_host(self.y), dx=to_host(self.dx), dWg=to_host(self.dWg), dW1=to_host(self.dW1),
                    dW2=to_host(self.dW2), logits=to_host(self.logits), idx=to_host(self.topk_idx),
                    w=to_host(self.topk_w), slot=to_host(self.slot), counts=to_host(self.counts))


def run_layer_step(shape, inp: Dict[str, np.ndarray], n_partitions=1, reuse=0, poison=True,
                   second_stream=True, device="cuda:0", gate_renormalize=0, grad_overwrite=0,
                   fuse_gather=0, wgrad_group=0, gemm_free_cus=0, fuse_combine=0) -> Dict[str, np.ndarray]:
    """One step of the HIP path on a synth.MoEShape-like object; returns host arrays.  With
    grad_overwrite the weight-gradient buffers start as NaN instead of zero: the step must store them."""
    st = LayerState(shape.T, shape.M, shape.H, shape.E, shape.k, shape.capacity_factor, n_partitions,
                    shape.dtype, reuse, device, second_stream, grad_overwrite=grad_overwrite,
                    gate_renormalize=gate_renormalize, fuse_gather=fuse_gather, wgrad_group=wgrad_group,
                    gemm_free_cus=gemm_free_cus, fuse_combine=fuse_combine)
    st.upload(inp)
    if poison:
        st.poison()
    st.zero_grads()
    if grad_overwrite:
        for t in (st.dWg, st.dW1, st.dW2):
            t.fill_(float("nan"))
    st.step()
    out = st.results()
    out["C_p"] = st.C_p
    return out
