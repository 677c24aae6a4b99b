"""Seeded synthetic inputs for one MoE layer step.

The paper trains on randomly generated tokens (Section V-A, "dummy dataset"),
so synthetic inputs are its workload.  This module only draws random numbers
and rounds them to the storage type; it contains none of the layer's
arithmetic.  Both the CPU oracle's tests and the HIP path's tests read the
arrays produced here, so the two sides always see identical bits.

Draw order (one ``numpy.random.Generator(PCG64(seed))``): x, W_g, W1, W2, dY,
all as float32 standard normals scaled by the configured standard deviation.
For bf16 workloads each array is then rounded once to bf16 (round to nearest,
ties to even) and kept as float32 holding exactly representable values.
"""
from __future__ import annotations

import dataclasses
from typing import Dict, Optional

import numpy as np


@dataclasses.dataclass(frozen=True)
class MoEShape:
    """Shape of one GPU's share of an MoE layer (Table I notation: B->T, M, H, E)."""
    name: str
    T: int                 # tokens in the batch
    M: int                 # model dimension
    H: int                 # expert hidden dimension
    E: int                 # local experts
    k: int                 # experts per token
    capacity_factor: float
    dtype: str             # "f32" or "bf16"
    x_std: float
    w_std: float
    n_partitions: tuple    # pipeline granularities the workload names
    zipf_s: Optional[float] = None   # gate-bias skew exponent, None = no bias
    zipf_tau: float = 0.0            # scale of the bias, see gate_bias()


# The five workloads.  Shapes 3 and 4 have the model/hidden dimensions of the
# paper's MoE-BERT-L and MoE-GPT3-XL layers (Table III); token counts lie in
# its 4k-32k range (Section V-C).
WORKLOADS: Dict[str, MoEShape] = {
    "tiny": MoEShape("tiny", 256, 64, 128, 4, 1, 1.25, "f32", 0.02, 0.02, (1,)),
    "small": MoEShape("small", 4096, 512, 2048, 8, 2, 1.25, "bf16", 1.0, 0.02, (1, 2, 4)),
    "gpt": MoEShape("gpt", 16384, 1024, 4096, 8, 2, 1.25, "bf16", 1.0, 0.02, (1, 2, 4, 8)),
    "large": MoEShape("large", 32768, 2048, 8192, 16, 2, 1.0, "bf16", 1.0, 0.02, (2, 4, 8)),
    # zipf_tau was calibrated with the oracle's router so that expert 0 takes
    # 36.5 % of first choices (tests/golden/calibrate_zipf_tau.py writes it).
    "skewed": MoEShape("skewed", 16384, 1024, 4096, 16, 2, 2.0, "bf16", 1.0, 0.02, (4,),
                       zipf_s=1.2, zipf_tau=0.390625),
}


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); result stays float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32).astype(np.uint64)
    lsb = (bits >> 16) & 1
    rounded = ((bits + 0x7FFF + lsb) >> 16) << 16
    return rounded.astype(np.uint32).view(np.float32).reshape(a.shape)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of float32 values that are already bf16-representable."""
    bits = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    assert not np.any(bits & 0xFFFF), "values are not bf16-representable"
    return (bits >> 16).astype(np.uint16)


def gate_bias(shape: MoEShape) -> Optional[np.ndarray]:
    """Fixed gate bias tau*ln(p_e), p_e ~ (e+1)^-s, giving Zipf-like expert popularity."""
    if shape.zipf_s is None:
        return None
    p = (np.arange(shape.E, dtype=np.float64) + 1.0) ** (-shape.zipf_s)
    p /= p.sum()
    return (shape.zipf_tau * np.log(p)).astype(np.float32)


def make_inputs(shape: MoEShape, seed: int = 0, dy_std: float = 1.0) -> Dict[str, np.ndarray]:
    """All tensors of one step as float32 arrays (bf16-representable for bf16 shapes)."""
    g = np.random.Generator(np.random.PCG64(seed))
    T, M, H, E = shape.T, shape.M, shape.H, shape.E

    def normal(dims, std):
        return (g.standard_normal(dims, dtype=np.float32) * np.float32(std)).astype(np.float32)

    out = {
        "x": normal((T, M), shape.x_std),
        "Wg": normal((M, E), shape.w_std),
        "W1": normal((E, M, H), shape.w_std),
        "W2": normal((E, H, M), shape.w_std),
        "dy": normal((T, M), dy_std),
    }
    if shape.dtype == "bf16":
        out = {k_: round_to_bf16(v) for k_, v in out.items()}
    b = gate_bias(shape)
    if b is not None:
        out["gate_bias"] = b
    return out


def custom_shape(T, M, H, E, k, capacity_factor, dtype="f32", x_std=1.0, w_std=0.02,
                 name="custom", zipf_s=None, zipf_tau=0.0) -> MoEShape:
    return MoEShape(name, T, M, H, E, k, capacity_factor, dtype, x_std, w_std, (1,),
                    zipf_s=zipf_s, zipf_tau=zipf_tau)
