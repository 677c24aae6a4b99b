"""moe_assign_slots_static (the entry point for callers that cannot allocate: its histograms live in an
array the library holds on the GPU) gives what moe_assign_slots gives, bit for bit, on two calls in a
row that share the array, the second on a smaller input."""
import numpy as np
import pytest
import torch

from paper_2506_22175_amd import binding as B

pytestmark = pytest.mark.gpu


def _both(T, E, k, cf, n, seed):
    dev = "cuda:0"
    cfg = B.make_config(T, 64, 64, E, k, cf, n, B.MOE_BF16, 0)
    rng = np.random.default_rng(seed)
    # k distinct experts per token, skewed so that some experts overflow their capacity
    p = (np.arange(E) + 1.0) ** -1.0
    idx = np.stack([rng.choice(E, size=k, replace=False, p=p / p.sum()) for _ in range(T)]).astype(np.int32)
    w = rng.random((T, k), dtype=np.float32)
    Rp = B.moe_capacity(cfg) * E
    d_idx, d_w = torch.from_numpy(idx).to(dev), torch.from_numpy(w).to(dev)
    out = []
    for static in (False, True):
        slot = torch.full((T, k), -2, dtype=torch.int32, device=dev)
        counts = torch.full((n, E), -2, dtype=torch.int32, device=dev)
        slot_w = torch.full((n * Rp,), -3.0, dtype=torch.float32, device=dev)
        if static:
            B.moe_assign_slots_static(cfg, d_idx, d_w, slot, counts, slot_w)
        else:
            scr = torch.full((B.moe_slot_scratch_bytes(cfg),), 0xFF, dtype=torch.uint8, device=dev)
            B.moe_assign_slots(cfg, d_idx, d_w, slot, counts, slot_w, scr)
        torch.cuda.synchronize()
        out.append((slot.cpu().numpy(), counts.cpu().numpy(), slot_w.cpu().numpy()))
    return out


def test_static_scratch_entry_point_equals_the_workspace_one_twice_in_a_row():
    assert torch.cuda.is_available()
    for T, E, k, cf, n, seed in ((8192, 16, 2, 1.0, 4, 0), (1000, 5, 3, 0.6, 2, 1)):   # the second is smaller
        (s0, c0, w0), (s1, c1, w1) = _both(T, E, k, cf, n, seed)
        assert np.array_equal(s0, s1) and np.array_equal(c0, c1) and np.array_equal(w0, w1)
        assert (s0 >= 0).any() and (s0 == -1).any() and c0.max() > 0


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    # n*k*ceil(T_p/1024)*E ints must fit 256 KiB: 64 partitions x 8 choices x 4 blocks x 64 experts do not
    cfg = B.make_config(64 * 4096, 64, 64, 64, 8, 1.0, 64, B.MOE_BF16, 0)
    assert B.moe_slot_scratch_bytes(cfg) > 256 * 1024
    t = torch.zeros((8,), dtype=torch.int32, device="cuda:0")
    with pytest.raises(B.MoEError) as e:
        B.moe_assign_slots_static(cfg, t, None, t, t, None)
    assert e.value.status == 4
