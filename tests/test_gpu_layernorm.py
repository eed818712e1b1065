"""GPU parity of the layer-norm fused in front of the GeMM (sbi_gemm_ln, and the ln1/ln2 fields
of sbi_layer) against the oracle's  gemm(layernorm(X)).  Same acceptance as the plain GeMM:
|gpu - oracle| <= max(2 ulp16(oracle), 1e-3), bit-identical run to run.  With an identity
weight matrix the GeMM returns the normalised activations themselves, which must match the
oracle's fp16 layer-norm output to 1 ulp16 (fp32 statistics against fp64 ones can move a
value across a rounding boundary, never further)."""
import numpy as np
import pytest

from oracle import oracle as orc
from paper_2207_00032_amd import workloads as wl

pytestmark = pytest.mark.gpu

EPS = 1e-5
EPI_ORACLE = {"none": 0, "bias": orc.EPI_BIAS, "bias_gelu": orc.EPI_BIAS | orc.EPI_GELU,
              "bias_residual": orc.EPI_BIAS | orc.EPI_RES}


def _dev(a, gpu):
    import torch
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(gpu)


def ln_gemm(gpu, W, bias, X, R, gamma, beta, epi, Wl=None, eps=EPS, **tuning):
    import torch
    from paper_2207_00032_amd import binding as sb
    K, N = W.shape
    if Wl is None:
        Wl = sb.layout_weights(_dev(W, gpu))
    g, b = _dev(gamma, gpu), _dev(beta, gpu)
    Y = sb.gemm(Wl, K, N, _dev(X, gpu), _dev(bias, gpu) if "bias" in epi else None,
                _dev(R, gpu) if "residual" in epi else None, epi, layernorm=(g, b, eps), **tuning)
    torch.cuda.synchronize()
    return Y.cpu().numpy(), Wl


def check_ln(Y, W, bias, X, R, gamma, beta, epi, what, eps=EPS):
    Xn = orc.layernorm(X, gamma, beta, eps)
    want = orc.gemm(Xn, W, bias, R, epi=EPI_ORACLE[epi])
    ok, rep = orc.check_close(Y, want, ulps=2, abs_tol=1e-3)
    assert ok, f"{what}: {rep}"


@pytest.mark.parametrize("B,K,N", [(1, 8, 1), (1, 64, 64), (3, 264, 200), (8, 1000, 130), (8, 4096, 192),
                                   (5, 4104, 72), (16, 2048, 320), (17, 4096, 136), (33, 1024, 192),
                                   (64, 2048, 128), (2, 12288, 64), (48, 12288, 192), (64, 520, 72)])
def test_ln_gemm_shapes_and_epilogues(gpu, B, K, N):
    W, bias, _, R = wl.make_gemm_inputs(K, N, B, seed=B + K + N, config_id=200)
    gamma, beta, X = wl.make_layernorm_inputs(K, B, seed=B + K + N, config_id=200)
    Wl = None
    for epi in ("none", "bias", "bias_gelu", "bias_residual"):
        Y, Wl = ln_gemm(gpu, W, bias, X, R, gamma, beta, epi, Wl=Wl)
        check_ln(Y, W, bias, X, R, gamma, beta, epi, f"B={B} K={K} N={N} {epi}")


@pytest.mark.parametrize("B,K,N", [(1, 4096, 192), (8, 2048, 320), (16, 4096, 128), (40, 1024, 192),
                                   (64, 2048, 128)])
@pytest.mark.parametrize("waves,depth", [(4, 2), (4, 4), (8, 4)])
def test_ln_gemm_split_k_and_tuning_variants(gpu, B, K, N, waves, depth):
    from paper_2207_00032_amd import binding as sb
    W, bias, _, R = wl.make_gemm_inputs(K, N, B, seed=2, config_id=201)
    gamma, beta, X = wl.make_layernorm_inputs(K, B, seed=2, config_id=201)
    Wl = None
    for S in (1, 2, 3, 7, 16):
        try:
            sb.plan(B, K, N, sb.PATH_MFMA, S, waves, depth, layernorm=True)
        except sb.SbiError:
            continue          # this (waves, depth) cannot stage X for this batch size in LDS
        Y, Wl = ln_gemm(gpu, W, bias, X, R, gamma, beta, "bias_residual", Wl=Wl, path=sb.PATH_MFMA,
                        split_k=S, waves=waves, depth=depth)
        check_ln(Y, W, bias, X, R, gamma, beta, "bias_residual", f"B={B} K={K} N={N} S={S} w={waves} d={depth}")


@pytest.mark.parametrize("B,K", [(1, 64), (7, 520), (16, 1024), (33, 2048), (4, 4096), (3, 6144)])
def test_identity_weights_return_the_normalised_rows(gpu, B, K):
    gamma, beta, X = wl.make_layernorm_inputs(K, B, seed=K + B, config_id=202, row_shift=3.0, row_scale=8.0)
    W = np.eye(K, dtype=np.float16)
    Y, _ = ln_gemm(gpu, W, None, X, None, gamma, beta, "none")
    want = orc.layernorm(X, gamma, beta, EPS)
    ok, rep = orc.check_close(Y, want, ulps=1, abs_tol=0.0)
    assert ok, rep
    assert (Y.view(np.uint16) == want.view(np.uint16)).mean() > 0.99


def test_ln_special_rows(gpu):
    """A constant row (variance 0: the result is beta), a row far from zero with a small spread
    (cancellation in a one-pass variance), and eps large enough to matter."""
    K, N, B = 1024, 136, 4
    W, bias, _, R = wl.make_gemm_inputs(K, N, B, seed=5, config_id=203)
    gamma, beta, X = wl.make_layernorm_inputs(K, B, seed=5, config_id=203)
    X[0, :] = np.float16(3.25)
    rng = np.random.default_rng(11)
    X[1, :] = (200.0 + 0.25 * rng.integers(-4, 5, size=K)).astype(np.float16)     # exact in fp16
    X[2, :] = 0
    for eps in (1e-5, 1e-12, 0.5):
        Y, _ = ln_gemm(gpu, W, bias, X, R, gamma, beta, "bias", eps=eps)
        check_ln(Y, W, bias, X, R, gamma, beta, "bias", f"eps={eps}", eps=eps)


def test_ln_determinism_and_plain_gemm_unaffected(gpu):
    import torch
    from paper_2207_00032_amd import binding as sb
    K, N, B = 4096, 1024, 8
    W, bias, Xp, R = wl.make_gemm_inputs(K, N, B, seed=7, config_id=204)
    gamma, beta, X = wl.make_layernorm_inputs(K, B, seed=7, config_id=204)
    ws = sb.new_workspace(max(sb.ln_workspace_bytes(B, K, N), sb.workspace_bytes(B, K, N)), gpu)
    Wl = sb.layout_weights(_dev(W, gpu))
    g, b, Xd, Xpd, bd = (_dev(a, gpu) for a in (gamma, beta, X, Xp, bias))
    first = None
    for rep in range(3):
        Y = sb.gemm(Wl, K, N, Xd, bd, None, "bias", workspace=ws, layernorm=(g, b, EPS))
        Yp = sb.gemm(Wl, K, N, Xpd, bd, None, "bias", workspace=ws)          # same workspace, plain GeMM
        torch.cuda.synchronize()
        if first is None:
            first = (Y.clone(), Yp.clone())
        assert torch.equal(Y.view(torch.int16), first[0].view(torch.int16))
        assert torch.equal(Yp.view(torch.int16), first[1].view(torch.int16))
    check_ln(first[0].cpu().numpy(), W, bias, X, None, gamma, beta, "bias", "ln")
    want = orc.gemm(Xp, W, bias, None, epi=orc.EPI_BIAS)
    ok, rep = orc.check_close(first[1].cpu().numpy(), want, ulps=2, abs_tol=1e-3)
    assert ok, rep
    assert not ws[:256 * 1024].cpu().numpy().any()


@pytest.mark.parametrize("cfg_id,B,chained,which", [(1, 4, True, "both"), (1, 1, False, "ln1"),
                                                    (2, 8, False, "both"), (2, 3, True, "ln2")])
def test_layer_gemms_with_fused_layernorms(gpu, cfg_id, B, chained, which):
    """sbi_layer_gemms with ln1 (in front of QKV) and/or ln2 (in front of FFN1); the other GeMMs
    of the same grouped launch must be untouched by the layer-norm kernel variant."""
    import torch
    from paper_2207_00032_amd import binding as sb
    cfg = wl.CONFIGS[cfg_id]
    data = [wl.make_gemm_inputs(s.K, s.N, B, seed=3, config_id=cfg_id, gemm_id=i) for i, s in enumerate(cfg.gemms)]
    h = cfg.gemms[0].K
    ln = [wl.make_layernorm_inputs(h, B, seed=3, config_id=cfg_id, gemm_id=i) for i in (0, 2)]
    use1, use2 = which in ("both", "ln1"), which in ("both", "ln2")
    Wls = [sb.layout_weights(_dev(d[0], gpu)) for d in data]
    biases = [_dev(d[1], gpu) for d in data]
    lnd = [(_dev(g, gpu), _dev(b, gpu)) for g, b, _ in ln]
    L = sb.make_layer(*Wls, h, cfg.gemms[0].N, cfg.gemms[1].K, cfg.gemms[2].N, cfg.gemms[3].K,
                      bqkv=biases[0], bout=biases[1], bffn1=biases[2], bffn2=biases[3], ffn1_gelu=True,
                      ln1=lnd[0] if use1 else None, ln2=lnd[1] if use2 else None, ln_eps=EPS)
    ws = sb.new_workspace(sb.layer_workspace_bytes(L, B), gpu)
    Xh = [ln[0][2] if use1 else data[0][2], data[1][2], ln[1][2] if use2 else data[2][2], data[3][2]]
    Xs = [_dev(x, gpu) for x in Xh]
    Rd = _dev(data[3][3], gpu)
    Ys = [torch.empty((B, s.N), dtype=torch.float16, device=gpu) for s in cfg.gemms]
    for rep in range(2):
        sb.layer_gemms(L, B, Xs[0], Xs[1], Xs[2], None if chained else Xs[3], Rd,
                       Ys[0], Ys[1], Ys[2], Ys[3], ws)
        torch.cuda.synchronize()
        Yh = [y.cpu().numpy() for y in Ys]
        x0 = orc.layernorm(Xh[0], ln[0][0], ln[0][1], EPS) if use1 else Xh[0]
        x2 = orc.layernorm(Xh[2], ln[1][0], ln[1][1], EPS) if use2 else Xh[2]
        for y, d, x, r, e, name in ((Yh[0], data[0], x0, None, orc.EPI_BIAS, "qkv"),
                                    (Yh[1], data[1], Xh[1], None, orc.EPI_BIAS, "attn_out"),
                                    (Yh[2], data[2], x2, None, orc.EPI_BIAS | orc.EPI_GELU, "ffn1"),
                                    (Yh[3], data[3], Yh[2] if chained else Xh[3], data[3][3],
                                     orc.EPI_BIAS | orc.EPI_RES, "ffn2")):
            ok, report = orc.check_close(y, orc.gemm(x, d[0], d[1], r, epi=e), ulps=2, abs_tol=1e-3)
            assert ok, f"{name}: {report}"
    assert not ws[:256 * 1024].cpu().numpy().any()


def test_ln_layer_under_graph_replay(gpu):
    """The layer with both layer-norms fused, FFN2 chained, captured into a HIP graph: every replay
    reproduces the eager bits (the fused variant, too, enqueues nothing but kernels)."""
    import torch
    from paper_2207_00032_amd import binding as sb
    cfg = wl.CONFIGS[1]
    B = 2
    data = [wl.make_gemm_inputs(s.K, s.N, B, seed=4, config_id=1, gemm_id=i) for i, s in enumerate(cfg.gemms)]
    h = cfg.gemms[0].K
    ln = [wl.make_layernorm_inputs(h, B, seed=4, config_id=1, gemm_id=i) for i in (0, 2)]
    Wls = [sb.layout_weights(_dev(d[0], gpu)) for d in data]
    biases = [_dev(d[1], gpu) for d in data]
    lnd = [(_dev(g, gpu), _dev(b, gpu)) for g, b, _ in ln]
    L = sb.make_layer(*Wls, h, cfg.gemms[0].N, cfg.gemms[1].K, cfg.gemms[2].N, cfg.gemms[3].K,
                      bqkv=biases[0], bout=biases[1], bffn1=biases[2], bffn2=biases[3], ffn1_gelu=True,
                      ln1=lnd[0], ln2=lnd[1], ln_eps=EPS)
    ws = sb.new_workspace(sb.layer_workspace_bytes(L, B), gpu)
    Xs = [_dev(ln[0][2], gpu), _dev(data[1][2], gpu), _dev(ln[1][2], gpu)]
    Rd = _dev(data[3][3], gpu)
    Ys = [torch.empty((B, s.N), dtype=torch.float16, device=gpu) for s in cfg.gemms]

    def run():
        sb.layer_gemms(L, B, Xs[0], Xs[1], Xs[2], None, Rd, Ys[0], Ys[1], Ys[2], Ys[3], ws)

    run()
    torch.cuda.synchronize()
    eager = [y.clone() for y in Ys]
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            run()
    torch.cuda.synchronize()
    for rep in range(3):
        for y in Ys:
            y.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        for y, e in zip(Ys, eager):
            assert torch.equal(y.view(torch.int16), e.view(torch.int16)), f"replay {rep} differs"
        run()
        torch.cuda.synchronize()
    x2 = orc.layernorm(ln[1][2], ln[1][0], ln[1][1], EPS)
    ok, rep = orc.check_close(eager[2].cpu().numpy(),
                              orc.gemm(x2, data[2][0], data[2][1], None, epi=orc.EPI_BIAS | orc.EPI_GELU),
                              ulps=2, abs_tol=1e-3)
    assert ok, rep
    assert not ws[:256 * 1024].cpu().numpy().any()


@pytest.mark.parametrize("B,K,N,split", [(1, 256, 64, 0), (4, 1024, 200, 0), (8, 2048, 4096, 0), (17, 512, 136, 0),
                                         (5, 4096, 192, 4), (33, 1024, 72, 3), (64, 2048, 128, 2)])
def test_epilogue_emits_panel_moments_of_the_stored_outputs(gpu, B, K, N, split):
    """sbi_gemm_moments: per row and 64-column panel (mean, sum of squared deviations) of the fp16
    values the call stored, also for ragged last panels and for split-K launches (where the
    last-arriving block finishes the panel)."""
    import torch
    from paper_2207_00032_amd import binding as sb
    W, bias, X, R = wl.make_gemm_inputs(K, N, B, seed=B + N, config_id=205)
    Wl = sb.layout_weights(_dev(W, gpu))
    P = -(-N // 64)
    mom = torch.full((B, P, 2), float("nan"), dtype=torch.float32, device=gpu)
    tune = dict(path=sb.PATH_MFMA, split_k=split, waves=4, depth=4 if B <= 16 else 2) if split else {}
    Y = sb.gemm(Wl, K, N, _dev(X, gpu), _dev(bias, gpu), _dev(R, gpu), "bias_residual", moments_out=mom, **tune)
    torch.cuda.synchronize()
    Yh = Y.cpu().numpy()
    ok, rep = orc.check_close(Yh, orc.gemm(X, W, bias, R, epi=orc.EPI_BIAS | orc.EPI_RES), ulps=2, abs_tol=1e-3)
    assert ok, rep
    m = mom.cpu().numpy().astype(np.float64)
    Yd = Yh.astype(np.float64)
    for p in range(P):
        seg = Yd[:, 64 * p:min(64 * p + 64, N)]
        mean = seg.mean(axis=1)
        m2 = ((seg - mean[:, None]) ** 2).sum(axis=1)
        assert np.allclose(m[:, p, 0], mean, rtol=1e-5, atol=1e-6), (p, m[:, p, 0], mean)
        assert np.allclose(m[:, p, 1], m2, rtol=1e-4, atol=1e-5), (p, m[:, p, 1], m2)


@pytest.mark.parametrize("B,K1,H,N2", [(1, 512, 1024, 192), (4, 1024, 4096, 200), (8, 4096, 4096, 1024),
                                       (16, 256, 2048, 136), (40, 512, 1024, 72)])
def test_residual_path_feeds_the_next_layernorm(gpu, B, K1, H, N2):
    """A GeMM with bias + residual whose epilogue leaves the row moments of its output, and the
    next GeMM whose layer-norm takes its statistics from them instead of reading the rows:
    compared with the oracle (layer-norm of the fp16 rows the first call stored) and with the
    same second call computing its statistics itself."""
    import torch
    from paper_2207_00032_amd import binding as sb
    W1, b1, X, R = wl.make_gemm_inputs(K1, H, B, seed=B + H, config_id=206)
    W2, b2, _, _ = wl.make_gemm_inputs(H, N2, B, seed=B + H, config_id=207)
    gamma, beta, _ = wl.make_layernorm_inputs(H, B, seed=B, config_id=206)
    R = (R.astype(np.float32) * 3 + 0.7).astype(np.float16)          # a residual stream with its own mean and spread
    Wl1, Wl2 = sb.layout_weights(_dev(W1, gpu)), sb.layout_weights(_dev(W2, gpu))
    mom = torch.empty((B, H // 64, 2), dtype=torch.float32, device=gpu)
    g, be = _dev(gamma, gpu), _dev(beta, gpu)
    Y1 = sb.gemm(Wl1, K1, H, _dev(X, gpu), _dev(b1, gpu), _dev(R, gpu), "bias_residual", moments_out=mom)
    Y2 = sb.gemm(Wl2, H, N2, Y1, _dev(b2, gpu), None, "bias_gelu", layernorm=(g, be, EPS), moments_in=mom)
    Y2b = sb.gemm(Wl2, H, N2, Y1, _dev(b2, gpu), None, "bias_gelu", layernorm=(g, be, EPS))
    torch.cuda.synchronize()
    Y1h = Y1.cpu().numpy()
    want = orc.gemm(orc.layernorm(Y1h, gamma, beta, EPS), W2, b2, None, epi=orc.EPI_BIAS | orc.EPI_GELU)
    for y, name in ((Y2, "statistics from the moments"), (Y2b, "statistics from the rows")):
        ok, rep = orc.check_close(y.cpu().numpy(), want, ulps=2, abs_tol=1e-3)
        assert ok, f"{name}: {rep}"
    ok, rep = orc.check_close(Y2.cpu().numpy(), Y2b.cpu().numpy(), ulps=1, abs_tol=5e-4)
    assert ok, rep
