"""sbi_gemm_static (the entry point that allocates nothing: its split-K workspace is a device
array inside the library) against sbi_gemm with a caller's workspace: same kernels, same plan,
so the same bits, and both within the parity bar of the CPU oracle.  Two calls in a row share the
library's array, the second with a smaller problem; then the first again."""
import numpy as np
import pytest

from oracle import oracle as orc
from paper_2207_00032_amd import workloads as wl

pytestmark = pytest.mark.gpu


def test_static_scratch_gemm_matches_the_workspace_call(gpu):
    import torch
    from paper_2207_00032_amd import binding as sb
    cases = [(8, 16384, 4096, "bias_residual"), (3, 4096, 1024, "bias_gelu"), (8, 16384, 4096, "bias_residual"),
             (64, 2048, 520, "bias"), (1, 4096, 12288, "none")]
    prepared = {}
    for B, K, N, epi in cases:
        if (B, K, N) in prepared:
            continue
        W, bias, X, R = wl.make_gemm_inputs(K, N, B, seed=21, config_id=107)
        dev = [torch.from_numpy(a).to(gpu) for a in (W, bias, X, R)]
        Wl = sb.layout_weights(dev[0])
        need = sb.workspace_bytes(B, K, N)
        assert need <= sb.STATIC_SCRATCH_BYTES
        ws = sb.new_workspace(need, gpu) if need else None
        want = sb.gemm(Wl, K, N, dev[2], dev[1] if "bias" in epi else None, dev[3] if "residual" in epi else None,
                       epi, workspace=ws)
        torch.cuda.synchronize()
        oracle = orc.gemm(X, W, bias if "bias" in epi else None, R if "residual" in epi else None,
                          epi={"none": 0, "bias": orc.EPI_BIAS, "bias_gelu": orc.EPI_BIAS | orc.EPI_GELU,
                               "bias_residual": orc.EPI_BIAS | orc.EPI_RES}[epi])
        ok, rep = orc.check_close(want.cpu().numpy(), oracle, ulps=2, abs_tol=1e-3)
        assert ok, rep
        prepared[(B, K, N)] = (Wl, dev, want, need)
    assert prepared[(8, 16384, 4096)][3] > 0 and prepared[(3, 4096, 1024)][3] > 0      # both use the scratch array
    # back to back on one stream, no synchronisation in between: the calls share the array
    outs = []
    for B, K, N, epi in cases:
        Wl, dev, want, _ = prepared[(B, K, N)]
        out = torch.full((B, N), float("nan"), dtype=torch.float16, device=gpu)
        sb.gemm_static(Wl, K, N, dev[2], dev[1] if "bias" in epi else None, dev[3] if "residual" in epi else None,
                       epi, out=out)
        outs.append(out)
    torch.cuda.synchronize()
    for (B, K, N, epi), out in zip(cases, outs):
        want = prepared[(B, K, N)][2]
        assert torch.equal(out.view(torch.int16), want.view(torch.int16)), f"B={B} K={K} N={N} {epi}"
