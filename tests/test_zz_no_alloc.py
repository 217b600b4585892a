"""The allocation-free split-k entry point (static device scratch) against the entry point that takes a workspace.

Both run the same kernels, so the bar is bit-for-bit equality of Y -- on two calls in a row that share the GPU's
scratch array, the second on a smaller problem (the array then still holds the first call's partial sums beyond
what the second one writes)."""
import numpy as np
import pytest
import torch

from paper_2501_16103_amd import binding as mb
from paper_2501_16103_amd import workloads as wk

pytestmark = pytest.mark.gpu

POISON = 0x7FC1


def _both(dev, T, E, K, N, parts, seed):
    wl = wk.Workload("no_alloc_splitk", T, E, 1, K, N, "bf16", "gauss_topk", 256, 256)
    g = torch.Generator().manual_seed(seed)
    ids = torch.randint(0, E, (T, 1), generator=g, dtype=torch.int32)
    X = wk.make_x(wl).to(dev)
    W = wk.make_w(wl).to(dev)
    tmap = mb.alloc_task_map(T, 1, E, 256, 256, N)
    mb.moe_build_task_map(ids.to(dev), T, 1, E, 256, 256, N, tmap)
    desc = mb.GemmDesc(mb.MOE_DTYPE_BF16, T, 1, E, K, N, 256, 256)
    pad = 3
    out = []
    for static in (False, True):
        buf = torch.full((T + 2 * pad, N), POISON, dtype=torch.int16, device=dev)
        Y = buf[pad: pad + T]
        if static:
            print(f"moe_grouped_gemm_splitk_static T={T} E={E} K={K} N={N} parts={parts}", flush=True)
            mb.moe_grouped_gemm_splitk_static(X, W, tmap, Y, desc, parts)
        else:
            ws = torch.empty(mb.moe_splitk_workspace_bytes(T, 1, N, parts) // 4, dtype=torch.float32, device=dev)
            mb.moe_grouped_gemm_splitk(X, W, tmap, Y, desc, parts, ws)
        torch.cuda.synchronize()
        bits = buf.cpu().numpy().view(np.uint16)
        assert np.all(bits[:pad] == POISON) and np.all(bits[pad + T:] == POISON), "wrote outside Y"
        assert not np.any(bits[pad: pad + T] == POISON), "an output was never written"
        out.append(bits[pad: pad + T].copy())
    return out


def test_static_scratch_split_k_matches_the_workspace_entry_point():
    dev = torch.device("cuda:0")
    assert mb.moe_splitk_static_scratch_bytes() == 32 << 20
    # first a problem that fills a good part of the array (2 x 1100 x 1024 fp32 = 9 MB), then a smaller one
    for (T, E, K, N, parts, seed) in ((1100, 4, 2048, 1024, 2, 1), (300, 3, 1024, 512, 2, 2)):
        with_ws, with_static = _both(dev, T, E, K, N, parts, seed)
        np.testing.assert_array_equal(with_static, with_ws)


def test_static_scratch_rejects_what_does_not_fit():
    dev = torch.device("cuda:0")
    T, E, K, N = 4096, 8, 1024, 2048          # 2 x 4096 x 2048 fp32 = 64 MiB > 32 MiB
    assert mb.moe_splitk_workspace_bytes(T, 1, N, 2) > mb.moe_splitk_static_scratch_bytes()
    d = mb.GemmDesc(mb.MOE_DTYPE_BF16, T, 1, E, K, N, 256, 256)
    one = torch.zeros(64, dtype=torch.int32, device=dev)   # never read: the size check comes first
    rc = mb.moe_grouped_gemm_splitk_static(one, one, one, one, d, 2, check=False)
    assert rc == mb.MOE_ERR_TOO_LARGE
    assert "scratch" in mb.strerror(rc)
