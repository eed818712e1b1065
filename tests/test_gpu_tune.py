"""Measured launch plans (sbi_layer_tune / sbi_gemm_tune): whatever candidate wins, the results stay
within the parity bar of the CPU oracle and bit-identical from call to call, the plan queries report
the winner, and other problems keep their plans."""
import numpy as np
import pytest

from oracle import oracle as orc
from paper_2207_00032_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _dev(a, gpu):
    import torch
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(gpu)


@pytest.mark.parametrize("B,K,N", [(1, 4096, 1024), (8, 2048, 4096), (33, 4096, 520)])
def test_tuned_single_gemm_matches_oracle(gpu, B, K, N):
    import torch
    from paper_2207_00032_amd import binding as sb
    W, bias, X, R = wl.make_gemm_inputs(K, N, B, seed=31, config_id=108)
    Wl = sb.layout_weights(_dev(W, gpu))
    copies = [Wl, Wl.clone(), Wl.clone()]
    Xd, bd, Rd = _dev(X, gpu), _dev(bias, gpu), _dev(R, gpu)
    other_before = sb.plan(B, K, N + 64)
    ws = sb.new_workspace(64 << 20, gpu)
    rep = sb.gemm_tune(copies, K, N, Xd, bd, Rd, "bias_residual", workspace=ws)
    assert rep["candidates"] >= 1 and 0 < rep["us_best"] <= rep["us_model"]
    pl = sb.plan(B, K, N)
    assert (pl["waves"], pl["depth"], pl["panels"]) == (rep["waves"], rep["depth"], rep["panels"])
    assert pl["workspace_bytes"] <= ws.numel()
    assert sb.plan(B, K, N + 64) == other_before                  # another problem keeps its plan
    want = orc.gemm(X, W, bias, R, epi=orc.EPI_BIAS | orc.EPI_RES)
    first = None
    for rep_i in range(3):
        Y = sb.gemm(copies[rep_i], K, N, Xd, bd, Rd, "bias_residual", workspace=ws)
        torch.cuda.synchronize()
        ok, r = orc.check_close(Y.cpu().numpy(), want, ulps=2, abs_tol=1e-3)
        assert ok, r
        first = Y.clone() if first is None else first
        assert torch.equal(Y.view(torch.int16), first.view(torch.int16))
    assert not ws[:256 * 1024].cpu().numpy().any()


@pytest.mark.parametrize("B,ln", [(1, False), (8, False), (4, True), (24, False)])
def test_tuned_layer_launch_matches_oracle(gpu, B, ln):
    import torch
    from paper_2207_00032_amd import binding as sb
    cfg = wl.CONFIGS[1]
    data = [wl.make_gemm_inputs(s.K, s.N, B, seed=2, config_id=109, gemm_id=i) for i, s in enumerate(cfg.gemms)]
    Wl0 = [sb.layout_weights(_dev(d[0], gpu)) for d in data]
    biases = [_dev(d[1], gpu) for d in data]
    g = cfg.gemms
    gamma, beta, _ = wl.make_layernorm_inputs(g[0].K, B, seed=2, config_id=109)
    lnp = (_dev(gamma, gpu), _dev(beta, gpu)) if ln else None
    sets = [Wl0, [w.clone() for w in Wl0]]          # make_layer keeps bare pointers: the tensors must outlive the layers
    layers = [sb.make_layer(*ws_, g[0].K, g[0].N, g[1].K, g[2].N, g[3].K,
                            bqkv=biases[0], bout=biases[1], bffn1=biases[2], bffn2=biases[3], ffn1_gelu=True,
                            ln1=lnp, ln2=lnp) for ws_ in sets]
    ws = sb.new_workspace(64 << 20, gpu)
    Xs = [_dev(d[2], gpu) for d in data]
    Rd = _dev(data[3][3], gpu)
    Ys = [torch.empty((B, s.N), dtype=torch.float16, device=gpu) for s in g]
    rep = sb.layer_tune(layers, B, Xs[0], Xs[1], Xs[2], Xs[3], Rd, Ys[0], Ys[1], Ys[2], Ys[3], ws)
    assert rep["candidates"] >= 1 and 0 < rep["us_best"] <= rep["us_model"]
    plans, grid = sb.layer_plan(layers[0], B)
    assert sb.layer_workspace_bytes(layers[0], B) <= ws.numel()
    first = None
    for it in range(2):
        sb.layer_gemms(layers[it], B, Xs[0], Xs[1], Xs[2], Xs[3], Rd, Ys[0], Ys[1], Ys[2], Ys[3], ws)
        torch.cuda.synchronize()
        Yh = [y.cpu().numpy() for y in Ys]
        for gi, (epi, r) in enumerate((("bias", None), ("bias", None), ("bias_gelu", None), ("bias_residual", data[3][3]))):
            xin = data[gi][2]
            if ln and gi in (0, 2):
                xin = orc.layernorm(xin, gamma, beta, 1e-5)
            want = orc.gemm(xin, data[gi][0], data[gi][1], r,
                            epi={"bias": orc.EPI_BIAS, "bias_gelu": orc.EPI_BIAS | orc.EPI_GELU,
                                 "bias_residual": orc.EPI_BIAS | orc.EPI_RES}[epi])
            ok, rr = orc.check_close(Yh[gi], want, ulps=2, abs_tol=1e-3)
            assert ok, f"tuned layer B={B} ln={ln} gemm {gi}: {rr}"
        first = [y.clone() for y in Ys] if first is None else first
        assert all(torch.equal(y.view(torch.int16), f.view(torch.int16)) for y, f in zip(Ys, first))
    assert not ws[:256 * 1024].cpu().numpy().any()


def test_occupancy_table_matches_the_compiled_kernels(gpu):
    """The dispatcher counts resident blocks per compute unit from a table of registers per lane; for
    every variant it can choose, the compiled kernel's allocation must give the same number of resident
    wavefronts (512 registers per lane and SIMD, allocated in eights, at most 8 wavefronts per SIMD)."""
    from paper_2207_00032_amd import binding as sb

    def waves(v):
        return min(8, 512 // ((v + 7) // 8 * 8))
    reachable = []
    for mb in (1, 2, 3, 4):
        for shp in ((4, 2, 1), (8, 4, 1), (4, 4, 1)):
            reachable += [(mb, shp, f) for f in ("fp16", "fp16_ln", "int8_codes")]
            if mb == 1:
                reachable.append((mb, shp, "int8"))
        reachable.append((mb, (8, 2, 1), "fp16"))
        if mb >= 2:
            reachable += [(mb, (8, 4, 2), "fp16"), (mb, (8, 2, 2), "fp16")]
        if mb >= 3:
            reachable += [(mb, (8, 4, 2), "int8_codes"), (mb, (8, 2, 2), "int8_codes")]
    bad = []
    for mb, (nw, depth, pw), flavour in reachable:
        got = sb.kernel_registers(16 * mb, nw, depth, pw, flavour)
        assert got is not None, (mb, nw, depth, pw, flavour)
        allocated, assumed = got
        assert 0 < allocated <= 512
        if waves(allocated) != waves(assumed):
            bad.append((mb, nw, depth, pw, flavour, allocated, assumed))
    assert not bad, bad
    assert sb.kernel_registers(16, 8, 8, 2, "fp16") is None          # no such variant


@pytest.mark.parametrize("B,ln", [(2, False), (8, True), (24, False), (40, True)])
def test_tuned_int8_layer_launch_matches_oracle(gpu, B, ln):
    """sbi_layer_tune on an INT8 layer (quantising in the blocks up to 8 rows, from codes above; with the
    layer-norms in front: always from codes): whichever plan wins, every GeMM stays within the bar of the
    INT8 oracle on the same weight codes, and the results are bit-identical from call to call."""
    import torch
    from paper_2207_00032_amd import binding as sb
    from test_gpu_int8 import prepare, check, check_ln
    cfg = wl.CONFIGS[1]
    g = cfg.gemms
    data = [wl.make_gemm_inputs(s.K, s.N, B, seed=4, config_id=110, gemm_id=i) for i, s in enumerate(g)]
    prep = [prepare(gpu, d[0]) for d in data]
    biases = [_dev(d[1], gpu) for d in data]
    lns = {gi: wl.make_layernorm_inputs(g[0].K, B, seed=4, config_id=110, gemm_id=gi) for gi in (0, 2)}
    ln_d = {gi: (_dev(lns[gi][0], gpu), _dev(lns[gi][1], gpu)) for gi in (0, 2)}    # kept alive: the struct holds pointers
    sets = [[p[0] for p in prep], [p[0].clone() for p in prep]]
    layers = [sb.make_layer(*ws_, g[0].K, g[0].N, g[1].K, g[2].N, g[3].K,
                            bqkv=biases[0], bout=biases[1], bffn1=biases[2], bffn2=biases[3], ffn1_gelu=True,
                            scales=[p[1] for p in prep], ln1=ln_d[0] if ln else None, ln2=ln_d[2] if ln else None)
              for ws_ in sets]
    ws = sb.new_workspace(64 << 20, gpu)
    Xh = [lns[0][2] if ln else data[0][2], data[1][2], lns[2][2] if ln else data[2][2], data[3][2]]
    Xs = [_dev(x, gpu) for x in Xh]
    Rd = _dev(data[3][3], gpu)
    Ys = [torch.empty((B, s.N), dtype=torch.float16, device=gpu) for s in g]
    rep = sb.layer_tune(layers, B, Xs[0], Xs[1], Xs[2], Xs[3], Rd, Ys[0], Ys[1], Ys[2], Ys[3], ws)
    assert rep["candidates"] >= 1 and 0 < rep["us_best"] <= rep["us_model"]
    assert sb.layer_workspace_bytes(layers[0], B) <= ws.numel()
    first = None
    for it in range(2):
        sb.layer_gemms(layers[it], B, Xs[0], Xs[1], Xs[2], Xs[3], Rd, Ys[0], Ys[1], Ys[2], Ys[3], ws)
        torch.cuda.synchronize()
        Yh = [y.cpu().numpy() for y in Ys]
        for gi, (epi, r) in enumerate((("bias", None), ("bias", None), ("bias_gelu", None), ("bias_residual", data[3][3]))):
            what = f"tuned INT8 layer B={B} ln={ln} gemm {gi}"
            if ln and gi in (0, 2):
                check_ln(Yh[gi], Xh[gi], lns[gi][0], lns[gi][1], prep[gi][2], prep[gi][3], data[gi][1], r, epi, what)
            else:
                check(Yh[gi], Xh[gi], prep[gi][2], prep[gi][3], data[gi][1], r, epi, what)
        first = [y.clone() for y in Ys] if first is None else first
        assert all(torch.equal(y.view(torch.int16), f.view(torch.int16)) for y, f in zip(Ys, first))
    assert not ws[:256 * 1024].cpu().numpy().any()
