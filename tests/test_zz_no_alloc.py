"""grp_spmm_static, the aggregation for callers that cannot allocate: its partial sums live in a scratch
array built into the library.  Its results must equal grp_spmm's bit for bit (same kernels), on two calls in
a row, the second on a smaller input, and a partition that needs more than the built-in scratch is refused."""
import numpy as np
import pytest
import torch

import synth

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _run(g, n, E, F, bf16, seed):
    s, d = synth.rmat_graph(13, E, seed=seed, n_nodes=n, device=DEV)
    part = g.grp_partition_from_local_coo(s, d, n)
    assert g.grp_spmm_workspace_bytes(part, False, F) > 0 and g.grp_spmm_workspace_bytes(part, True, F) > 0   # rows are split
    x = synth.normal_matrix(n, F, seed)
    x = (synth.to_bf16_rne(x) if bf16 else x).to(DEV)
    dt = g.DTYPE_BF16 if bf16 else g.DTYPE_FP32
    for transposed in (False, True):
        want = torch.full((n, F), float("nan"), device=DEV)
        got = torch.full((n, F), float("nan"), device=DEV)
        g.grp_spmm(part, transposed, g.SCALE_MEAN, False, F, x, F, dt, want, F)
        g.grp_spmm_static(part, transposed, g.SCALE_MEAN, False, F, x, F, dt, got, F)
        torch.cuda.synchronize()
        assert not torch.isnan(got).any()
        assert torch.equal(got, want), (n, E, F, transposed)
    part.destroy()


def test_static_scratch_aggregation_equals_the_workspace_one():
    import paper_2602_01872_amd as g
    g.load()
    print("[case] grp_spmm_static, two calls in a row, the second smaller", flush=True)
    _run(g, 6000, 500000, 64, True, 77)          # hub rows of several chunks in both directions
    _run(g, 2000, 90000, 16, False, 78)          # a smaller partition and a narrower row: the scratch holds stale sums


def test_static_scratch_refuses_what_does_not_fit():
    import paper_2602_01872_amd as g
    g.load()
    n, E, F = 3000, 6_000_000, 1024               # ~12,000 chunks of 4 KiB of partial sums each: more than 32 MiB
    s, d = synth.rmat_graph(12, E, seed=5, n_nodes=n, device=DEV)
    part = g.grp_partition_from_local_coo(s, d, n)
    assert g.grp_spmm_workspace_bytes(part, False, F) > (32 << 20)
    x = torch.zeros(n, F, device=DEV)
    y = torch.zeros(n, F, device=DEV)
    with pytest.raises(g.GrappaError) as ei:
        g.grp_spmm_static(part, False, g.SCALE_MEAN, False, F, x, F, g.DTYPE_FP32, y, F)
    assert ei.value.status == g.EWORKSPACE
    g.grp_spmm(part, False, g.SCALE_MEAN, False, F, x, F, g.DTYPE_FP32, y, F)      # the workspace call takes it
    torch.cuda.synchronize()
    part.destroy()
