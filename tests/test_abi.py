"""The C-ABI library loads, exports every symbol include/moe.h declares, and its
host-only entry points (capacity, workspace sizes, argument checks) behave as the
header says.  No GPU is needed: none of these calls touches the device."""
import ctypes
import os
import re

import pytest

from paper_2506_22175_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "moe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared()
    assert len(names) >= 16 and "moe_layer_step" in names and "moe_route" in names
    lib = B.lib()
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(B.EXPORTS) == names


def test_capacity_matches_the_definition(oracle):
    for T, E, k, cf, n in [(256, 4, 1, 1.25, 1), (4096, 8, 2, 1.25, 4), (32768, 16, 2, 1.0, 8),
                           (16384, 16, 2, 2.0, 4), (10, 3, 1, 1.0, 1), (96, 5, 3, 0.7, 4), (64, 7, 2, 1.1, 2)]:
        cfg = B.make_config(T, 64, 64, E, k, cf, n)
        assert B.moe_capacity(cfg) == oracle.capacity(T, E, k, cf, n)


def test_argument_errors_are_status_codes():
    ok = B.make_config(256, 64, 128, 4, 1, 1.25, 1, B.MOE_F32)
    assert B.moe_capacity(ok) == 80
    bad = [
        (B.make_config(256, 64, 128, 4, 5, 1.25), 2),          # k > E
        (B.make_config(256, 64, 128, 4, 1, 1.25, 3), 2),       # T % n != 0
        (B.make_config(0, 64, 128, 4, 1, 1.25), 2),
        (B.make_config(256, 64, 128, 4, 1, 0.0), 2),
        (B.make_config(256, 64, 128, 65, 1, 1.0), 3),          # E > 64
        (B.make_config(256, 60, 128, 4, 1, 1.0), 3),           # M % 8
        (B.make_config(256, 64, 128, 4, 1, 1.0, 1, 7), 3),     # dtype
        (B.make_config(256, 64, 128, 4, 1, 1.0, fuse_gather=2), 3),
        # the strategies that copy forward's T_DI to the host need a T_DI in forward
        (B.make_config(256, 64, 128, 4, 1, 1.0, 2, B.MOE_BF16, B.MOE_REUSE_S1, fuse_gather=1), 3),
        (B.make_config(256, 64, 128, 4, 1, 1.0, 2, B.MOE_BF16, B.MOE_REUSE_S3, fuse_gather=1), 3),
        # grouped weight gradients: at most eight partitions, not with the offloading strategies
        (B.make_config(256, 64, 128, 4, 1, 1.0, 2, wgrad_group=9), 3),
        (B.make_config(256, 64, 128, 4, 1, 1.0, 2, wgrad_group=-1), 3),
        (B.make_config(256, 64, 128, 4, 1, 1.0, 2, B.MOE_BF16, B.MOE_REUSE_S2, wgrad_group=2), 3),
        # the fused combine needs one choice per token
        (B.make_config(256, 64, 128, 4, 2, 1.0, 2, fuse_combine=1), 3),
        (B.make_config(256, 64, 128, 4, 1, 1.0, 2, fuse_combine=2), 3),
        (B.make_config(256, 64, 128, 4, 1, 1.0, 2, B.MOE_BF16, B.MOE_REUSE_S1, fuse_combine=1), 3),
        (B.make_config(256, 64, 128, 4, 1, 1.0, 2, gemm_free_cus=-8), 3),
    ]
    for cfg, code in bad:
        with pytest.raises(B.MoEError) as ei:
            B.moe_capacity(cfg)
        assert ei.value.status == code
    # NULL pointers are reported before anything is launched
    lib = B.lib()
    assert lib.moe_capacity(ctypes.byref(ok), None) == 1
    assert lib.moe_route(ctypes.byref(ok), None, None, None, None, None, None, None) == 1
    assert lib.moe_layer_step(ctypes.byref(ok), *([None] * 18), ctypes.c_size_t(0), None, 2) == 1
    assert B.status_string(4) == "workspace too small"


def test_workspace_follows_the_memory_model(oracle):
    """saved bytes = the paper's shared-buffer bookkeeping (Section III-D) in elements
    times the element size, up to 256-byte alignment of each buffer."""
    T, M, H, E, k, cf = 16384, 1024, 4096, 8, 2, 1.25
    for n in (1, 2, 4, 8):
        C_p = oracle.capacity(T, E, k, cf, n)
        R_p = C_p * E
        sizes = {}
        for mode in (0, 1, 2):
            cfg = B.make_config(T, M, H, E, k, cf, n, B.MOE_BF16, mode)
            total, saved, temp, routing = B.moe_workspace_bytes(cfg)
            assert total == saved + temp + routing
            sizes[mode] = saved
        assert sizes[0] == 2 * oracle.workspace_model(R_p, n, M, H, 0)
        # sharing needs at least as many partitions as buffers (Eq. 5 is negative below that)
        if n >= 2:
            assert sizes[1] == 2 * oracle.workspace_model(R_p, n, M, H, 1)
            assert sizes[2] == 2 * oracle.workspace_model(R_p, n, M, H, 2)
            delta = oracle.paper_memory_model(R_p * n, M, H, E, n)["delta"]
            assert sizes[0] - sizes[2] == 2 * delta
        assert sizes[2] <= sizes[1] <= sizes[0] or n == 1
        # the gathered first GEMM: forward keeps no T_DI, backward dispatches into min(n, 2) buffers;
        # the shared-buffer modes had that many already, so only "keep everything" shrinks
        bufM = 2 * R_p * M
        for mode in (0, 1, 2):
            cfg = B.make_config(T, M, H, E, k, cf, n, B.MOE_BF16, mode, fuse_gather=1)
            saved_f = B.moe_workspace_bytes(cfg)[1]
            assert saved_f == sizes[mode] - (bufM * (n - 2) if (mode == 0 and n > 2) else 0)


def test_workspace_with_grouped_weight_gradients_and_fused_combine(oracle):
    """wgrad_group = G keeps G partition buffers of T_DI, dT_DO (which alias T_DO in the shared-buffer modes),
    T_M (with recomputation) and dT_M alive in backward; the fused combine keeps no T_DO.  In buffer counts:"""
    T, M, H, E, k, cf = 16384, 1024, 4096, 8, 2, 1.25
    for n in (2, 4, 8):
        R_p = oracle.capacity(T, E, k, cf, n) * E
        bufM, bufH = 2 * R_p * M, 2 * R_p * H
        for G in (1, 2, 4, 8):
            g = min(G, n)
            alive = max(2, g)
            cfg = B.make_config(T, M, H, E, k, cf, n, B.MOE_BF16, 2, wgrad_group=G)
            total, saved, temp, routing = B.moe_workspace_bytes(cfg)
            nbuf = alive if n > alive else n
            assert saved == 2 * nbuf * bufM + g * bufH              # T_DI and T_DO buffers, T_M buffers
            assert temp == g * bufH + 2 * bufM                      # dT_M buffers, two dT_DI (dT_DO aliases T_DO)
            plain = B.moe_workspace_bytes(B.make_config(T, M, H, E, k, cf, n, B.MOE_BF16, 2))
            assert total >= plain[0] and (G == 1) == (total == plain[0]) or g == 1
        # G larger than n counts as n
        assert B.moe_workspace_bytes(B.make_config(T, M, H, E, k, cf, n, B.MOE_BF16, 2, wgrad_group=8)) == \
            B.moe_workspace_bytes(B.make_config(T, M, H, E, k, cf, n, B.MOE_BF16, 2, wgrad_group=min(8, n)))
    # one choice per token
    k = 1
    for n in (1, 4):
        R_p = oracle.capacity(T, E, k, cf, n) * E
        bufM = 2 * R_p * M
        for mode in (0, 1, 2):
            a = B.moe_workspace_bytes(B.make_config(T, M, H, E, k, cf, n, B.MOE_BF16, mode))
            f = B.moe_workspace_bytes(B.make_config(T, M, H, E, k, cf, n, B.MOE_BF16, mode, fuse_combine=1))
            n_do = n if (mode == 0 or n <= 2) else 2
            assert a[1] - f[1] == n_do * bufM                       # no T_DO among what forward keeps
