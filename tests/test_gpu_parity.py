"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs.  Acceptance per element: |gpu - oracle| <= max(2 ulp16(oracle), 1e-3), and the
GPU result is bit-identical from run to run.  Integer/byte work (the weight pre-layout) is
compared bit for bit."""
import numpy as np
import pytest

from oracle import oracle as orc
from paper_2207_00032_amd import workloads as wl

pytestmark = pytest.mark.gpu

EPI_ORACLE = {"none": 0, "bias": orc.EPI_BIAS, "bias_gelu": orc.EPI_BIAS | orc.EPI_GELU,
              "bias_residual": orc.EPI_BIAS | orc.EPI_RES, "gelu": orc.EPI_GELU, "residual": orc.EPI_RES}


def _dev(a, gpu):
    import torch
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(gpu)


def gpu_gemm(gpu, W, bias, X, R, epi, Wl=None, **tuning):
    """Lay W out (unless given), run the GeMM, return (Y as numpy fp16, laid-out tensor)."""
    import torch
    from paper_2207_00032_amd import binding as sb
    K, N = W.shape
    if Wl is None:
        Wl = sb.layout_weights(_dev(W, gpu))
    use_bias = "bias" in epi
    use_res = "residual" in epi
    Y = sb.gemm(Wl, K, N, _dev(X, gpu), _dev(bias, gpu) if use_bias else None,
                _dev(R, gpu) if use_res else None, epi, **tuning)
    torch.cuda.synchronize()
    return Y.cpu().numpy(), Wl


def check(Y, W, bias, X, R, epi, what):
    want = orc.gemm(X, W, bias, R, epi=EPI_ORACLE[epi])
    ok, rep = orc.check_close(Y, want, ulps=2, abs_tol=1e-3)
    assert ok, f"{what}: {rep}"
    return rep


# ------------------------------------------------------------------------------ layout (bit-exact)
@pytest.mark.parametrize("K,N", [(32, 64), (8, 1), (1, 1), (40, 24), (103, 71), (264, 200), (1000, 130),
                                 (512, 1024), (2056, 520)])
def test_layout_bit_exact_and_invertible(gpu, K, N):
    import torch
    from paper_2207_00032_amd import binding as sb
    rng = np.random.default_rng(K * 7919 + N)
    Wbits = rng.integers(1, 65536, size=(K, N), dtype=np.uint16)
    Wd = torch.from_numpy(Wbits.view(np.float16)).to(gpu)
    Wl = sb.layout_weights(Wd)
    torch.cuda.synchronize()
    raw = Wl.cpu().numpy()
    assert raw.size == sb.layout_bytes(K, N)
    assert np.array_equal(raw[256:].view(np.uint16), orc.layout_weights(Wbits))
    hdr = raw[:256]
    assert hdr[:4].tobytes() == b"SBIG" and not hdr[56:].any()
    assert tuple(hdr[8:40].view(np.int64)) == (K, N, orc.layout_dims(K, N)[0], -(-N // 64))
    back = sb.unlayout_weights(Wl, K, N)
    torch.cuda.synchronize()
    assert np.array_equal(back.cpu().numpy().view(np.uint16), Wbits)
    assert sb.layout_check(Wl, K, N) == 0
    assert sb.layout_check(Wl, K + 1, N) == 5 and sb.layout_check(Wl, K, N + 64) == 5
    assert sb.layout_check(torch.zeros_like(Wl), K, N) == 5


# ------------------------------------------------------------------------------ small / ragged shapes
@pytest.mark.parametrize("B,K,N", wl.ragged_shapes())
def test_ragged_shapes_all_epilogues_both_paths(gpu, B, K, N):
    from paper_2207_00032_amd import binding as sb
    W, bias, X, R = wl.make_gemm_inputs(K, N, B, seed=B + K + N, config_id=100)
    Wl = None
    paths = [sb.PATH_AUTO, sb.PATH_MFMA] + ([sb.PATH_STREAM] if B <= 8 else []) + \
        ([sb.PATH_STREAMK] if K % 8 == 0 else [])
    for epi in ("none", "bias", "bias_gelu", "bias_residual", "gelu", "residual"):
        for path in paths:
            Y, Wl = gpu_gemm(gpu, W, bias, X, R, epi, Wl=Wl, path=path)
            check(Y, W, bias, X, R, epi, f"B={B} K={K} N={N} {epi} path={path}")


@pytest.mark.parametrize("B,K,N", [(1, 4096, 192), (4, 4096, 192), (8, 2048, 320), (16, 4096, 128),
                                   (40, 1024, 192), (64, 2048, 128)])
@pytest.mark.parametrize("waves,depth", [(4, 2), (4, 4), (4, 8), (8, 4), (8, 8)])
def test_split_k_and_tuning_variants(gpu, B, K, N, waves, depth):
    from paper_2207_00032_amd import binding as sb
    W, bias, X, R = wl.make_gemm_inputs(K, N, B, seed=1, config_id=101)
    Wl = None
    for path in [sb.PATH_MFMA] + ([sb.PATH_STREAM] if B <= 8 else []):
        try:
            sb.plan(B, K, N, path, 1, waves, depth)
        except sb.SbiError:
            continue      # this (waves, depth) cannot stage X for this batch size in LDS
        if path == sb.PATH_STREAM and waves == 8 and depth == 8 and B >= 4:
            continue      # that instantiation spills registers; the dispatcher never selects it
        for S in (1, 2, 3, 7, 16):
            try:
                sb.plan(B, K, N, path, S, waves, depth)
            except sb.SbiError:
                continue
            Y, Wl = gpu_gemm(gpu, W, bias, X, R, "bias_residual", Wl=Wl, path=path,
                             split_k=S, waves=waves, depth=depth)
            check(Y, W, bias, X, R, "bias_residual", f"B={B} K={K} N={N} S={S} w={waves} d={depth} path={path}")


@pytest.mark.parametrize("B,K,N", [(1, 4096, 192), (5, 2048, 320), (8, 1032, 1000), (16, 520, 72),
                                   (17, 4096, 130), (40, 1024, 192), (64, 2048, 136)])
def test_streamk_range_cuts(gpu, B, K, N):
    """The work-balanced kernel with every kind of range cut: one wavefront for everything,
    ranges that end inside panels, ranges shorter than a panel (many slabs per panel)."""
    from paper_2207_00032_amd import binding as sb
    W, bias, X, R = wl.make_gemm_inputs(K, N, B, seed=3, config_id=104)
    Wl = None
    for waves, depth in ((4, 4), (4, 8), (8, 4), (8, 8)):
        if waves == 8 and depth == 8 and B > 16:
            continue
        for blocks in (1, 2, 3, 7, 64, 512):
            for epi in ("bias_gelu", "bias_residual"):
                Y, Wl = gpu_gemm(gpu, W, bias, X, R, epi, Wl=Wl, path=sb.PATH_STREAMK,
                                 waves=waves, depth=depth, blocks=blocks)
                check(Y, W, bias, X, R, epi, f"streamk B={B} K={K} N={N} w={waves} d={depth} blocks={blocks} {epi}")


@pytest.mark.parametrize("B,K,N", [(1, 1024, 192), (8, 2048, 320), (16, 520, 72), (17, 4096, 136),
                                   (33, 1024, 448), (48, 2048, 200), (64, 4096, 192), (40, 1100, 136), (64, 2500, 72)])
def test_two_panel_blocks(gpu, B, K, N):
    """Blocks that stream two adjacent panels (odd panel counts leave a lone last panel)."""
    from paper_2207_00032_amd import binding as sb
    W, bias, X, R = wl.make_gemm_inputs(K, N, B, seed=7, config_id=105)
    Wl = None
    ran = 0
    for waves, depth in ((4, 2), (4, 4), (8, 2), (8, 4)):      # (8, 4): two wave groups, one panel each (B > 16)
        for S in (1, 2, 5):
            try:
                sb.plan(B, K, N, sb.PATH_MFMA, S, waves, depth, panels=2)
            except sb.SbiError:
                continue
            for epi in ("bias_gelu", "bias_residual"):
                Y, Wl = gpu_gemm(gpu, W, bias, X, R, epi, Wl=Wl, path=sb.PATH_MFMA, split_k=S,
                                 waves=waves, depth=depth, panels=2)
                check(Y, W, bias, X, R, epi, f"2-panel B={B} K={K} N={N} S={S} w={waves} d={depth} {epi}")
                ran += 1
    assert ran > 0


def test_workspace_reuse_and_determinism(gpu):
    """One workspace serves calls of different shapes back to back (the counters return to
    zero), and repeated calls give identical bits."""
    import torch
    from paper_2207_00032_amd import binding as sb
    shapes = [(4, 2048, 256), (8, 4096, 64), (2, 1024, 16384), (4, 2048, 256), (3, 512, 40000)]
    for tune in (dict(path=sb.PATH_MFMA, split_k=8), dict(path=sb.PATH_STREAMK), dict(path=sb.PATH_STREAMK, blocks=37)):
        ws = sb.new_workspace(max(sb.plan(B, K, N, **tune)["workspace_bytes"] for B, K, N in shapes), gpu)
        for rep in range(2):
            for B, K, N in shapes:
                W, bias, X, R = wl.make_gemm_inputs(K, N, B, seed=5, config_id=102)
                Y1, Wl = gpu_gemm(gpu, W, bias, X, R, "bias_gelu", workspace=ws, **tune)
                Y2, _ = gpu_gemm(gpu, W, bias, X, R, "bias_gelu", Wl=Wl, workspace=ws, **tune)
                assert np.array_equal(Y1.view(np.uint16), Y2.view(np.uint16))
                check(Y1, W, bias, X, R, "bias_gelu", f"reuse rep={rep} {B}x{K}x{N} {tune}")
        torch.cuda.synchronize()
        assert not ws[:256 * 1024].cpu().numpy().any()   # every arrival counter is back to zero


def test_residual_may_alias_output(gpu):
    import torch
    from paper_2207_00032_amd import binding as sb
    B, K, N = 4, 1024, 384
    W, bias, X, R = wl.make_gemm_inputs(K, N, B, seed=9, config_id=103)
    Wl = sb.layout_weights(_dev(W, gpu))
    Rd = _dev(R, gpu)
    sb.gemm(Wl, K, N, _dev(X, gpu), _dev(bias, gpu), Rd, "bias_residual", out=Rd)
    torch.cuda.synchronize()
    check(Rd.cpu().numpy(), W, bias, X, R, "bias_residual", "in-place residual")


def test_subnormal_and_exact_inputs(gpu):
    """fp16 subnormal weights must not be flushed; identity / power-of-two data is exact."""
    from paper_2207_00032_amd import binding as sb
    rng = np.random.default_rng(2)
    B, K, N = 8, 512, 128
    Wsub = rng.integers(1, 0x400, size=(K, N)).astype(np.uint16)            # positive subnormals
    Wsub |= (rng.integers(0, 2, size=(K, N)).astype(np.uint16) << 15)
    W = Wsub.view(np.float16)
    X = (rng.standard_normal((B, K)) * 64).astype(np.float16)
    for path in (sb.PATH_MFMA, sb.PATH_STREAM, sb.PATH_STREAMK):
        Y, _ = gpu_gemm(gpu, W, None, X, None, "none", path=path)
        want = orc.gemm(X, W)
        assert np.abs(want.astype(np.float64)).max() > 0.05                  # the products do matter
        ok, rep = orc.check_close(Y, want, ulps=2, abs_tol=1e-4)
        assert ok, f"subnormal weights path={path}: {rep}"
    # identity weights: Y == X bit for bit
    K = N = 256
    X = rng.standard_normal((B, K)).astype(np.float16)
    for path in (sb.PATH_MFMA, sb.PATH_STREAM, sb.PATH_STREAMK):
        Y, _ = gpu_gemm(gpu, np.eye(K, dtype=np.float16), None, X, None, "none", path=path)
        assert np.array_equal(Y.view(np.uint16), X.view(np.uint16))
    # large magnitudes: an overflow to inf must match the oracle's
    Wbig = np.full((K, N), 16.0, np.float16)
    Xbig = np.full((2, K), 32.0, np.float16)
    Y, _ = gpu_gemm(gpu, Wbig, None, Xbig, None, "none")
    assert np.isinf(Y).all() and np.isinf(orc.gemm(Xbig, Wbig)).all()


# ------------------------------------------------------------------------------ benchmark configurations
def _config_case(gpu, cfg_id, gi, seed, batches, paths=None):
    from paper_2207_00032_amd import binding as sb
    cfg = wl.CONFIGS[cfg_id]
    spec, W, bias, X, R = wl.make_config_gemm(cfg_id, gi, seed)
    Wl = None
    worst = 0.0
    for B in batches:
        for path in (paths or [sb.PATH_AUTO]):
            if path == sb.PATH_STREAM and B > 8:
                continue
            Y, Wl = gpu_gemm(gpu, W, bias, X[:B], R[:B], spec.epilogue, Wl=Wl, path=path)
            rep = check(Y, W, bias, X[:B], R[:B], spec.epilogue,
                        f"config {cfg_id} {spec.name} seed={seed} B={B} path={path}")
            worst = max(worst, rep["max_ulp"] if rep["max_abs"] > 1e-3 else 0.0)
    return worst


@pytest.mark.parametrize("gi", [0, 1, 2, 3])
def test_config1_h1024_layer(gpu, gi):
    from paper_2207_00032_amd import binding as sb
    _config_case(gpu, 1, gi, 0, (1,), [sb.PATH_AUTO, sb.PATH_MFMA, sb.PATH_STREAM, sb.PATH_STREAMK])


@pytest.mark.parametrize("gi", [0, 1, 2, 3])
@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_config2_h4096_layer(gpu, gi, seed):
    from paper_2207_00032_amd import binding as sb
    paths = [sb.PATH_AUTO, sb.PATH_MFMA, sb.PATH_STREAM] if seed == 0 else [sb.PATH_AUTO]
    _config_case(gpu, 2, gi, seed, wl.CONFIGS[2].batches, paths)


@pytest.mark.parametrize("gi", [0, 1, 2, 3])
def test_config3_h12288_tp_slice(gpu, gi):
    _config_case(gpu, 3, gi, 0, wl.CONFIGS[3].batches)


@pytest.mark.parametrize("gi", [0, 1, 2, 3])
def test_config4_h12288_full_size(gpu, gi):
    """Full-size matrices of the unsliced h=12288 layer (QKV [12288,36864], attention output,
    FFN1 [12288,49152] + GeLU, FFN2 [49152,12288]), every output element compared."""
    _config_case(gpu, 4, gi, 0, wl.CONFIGS[4].batches)


def test_config5_crossover_sweep_with_outliers(gpu):
    """The h=8192 FFN1 over the whole batch sweep, 1 % of the input channels scaled by 50, on the
    dispatcher's own pick and on every forced path; then the literal reading of "1 % of rows" at
    B = 64 (one batch row of X scaled by 50) on the same weights."""
    from paper_2207_00032_amd import binding as sb
    _config_case(gpu, 5, 0, 0, wl.CONFIGS[5].batches, [sb.PATH_AUTO, sb.PATH_STREAMK, sb.PATH_MFMA, sb.PATH_STREAM])
    spec = wl.CONFIGS[5].gemms[0]
    W, bias, X, R = wl.make_gemm_inputs(spec.K, spec.N, 64, 0, 5, 0, outlier_rows=0.01, outlier_scale=50.0)
    assert (np.abs(X.astype(np.float32)).max(axis=1) > 60).sum() == 1      # exactly one scaled row
    Wl = None
    for path in (sb.PATH_AUTO, sb.PATH_MFMA):
        Y, Wl = gpu_gemm(gpu, W, bias, X, R, spec.epilogue, Wl=Wl, path=path)
        check(Y, W, bias, X, R, spec.epilogue, f"config 5, one row of 64 scaled by 50, path={path}")


EPI_NAME = {wl.NONE: "none", wl.BIAS: "bias", wl.BIAS_GELU: "bias_gelu", wl.BIAS_RESIDUAL: "bias_residual",
            wl.GELU: "gelu", wl.RESIDUAL: "residual"}


@pytest.mark.parametrize("cfg_id", [3, 4])
def test_layer_gemms_at_h12288_matches_oracle(gpu, cfg_id):
    """sbi_layer_gemms on the h=12288 configurations (one GPU's tensor-parallel slice at B = 1, 4, 16;
    the full 3.6 GB layer at B = 1, 8) with the configurations' own epilogues: the grouped launch
    and the plan the dispatcher picks for it, every output element of all four GeMMs compared."""
    import torch
    from paper_2207_00032_amd import binding as sb
    cfg = wl.CONFIGS[cfg_id]
    Bmax = max(cfg.batches)
    Wls, host = [], []
    for i, s in enumerate(cfg.gemms):
        W, bias, X, R = wl.make_gemm_inputs(s.K, s.N, Bmax, seed=0, config_id=cfg_id, gemm_id=i)
        Wls.append(sb.layout_weights(_dev(W, gpu)))
        torch.cuda.synchronize()
        host.append((W, bias, X, R))
    epis = [EPI_NAME[s.epilogue] for s in cfg.gemms]
    assert not any("residual" in e for e in epis)
    biases = [_dev(d[1], gpu) if "bias" in e else None for d, e in zip(host, epis)]
    g = cfg.gemms
    L = sb.make_layer(*Wls, g[0].K, g[0].N, g[1].K, g[2].N, g[3].K, bqkv=biases[0], bout=biases[1],
                      bffn1=biases[2], bffn2=biases[3], ffn1_gelu="gelu" in epis[2])
    for B in cfg.batches:
        ws = sb.new_workspace(sb.layer_workspace_bytes(L, B), gpu)
        Xs = [_dev(d[2][:B], gpu) for d in host]
        Ys = [torch.full((B, s.N), float("nan"), dtype=torch.float16, device=gpu) for s in g]
        sb.layer_gemms(L, B, Xs[0], Xs[1], Xs[2], Xs[3], None, Ys[0], Ys[1], Ys[2], Ys[3], ws)
        torch.cuda.synchronize()
        for i, s in enumerate(g):
            W, bias, X, _ = host[i]
            check(Ys[i].cpu().numpy(), W, bias, X[:B], None, epis[i], f"config {cfg_id} layer launch {s.name} B={B}")
        assert not ws[:256 * 1024].cpu().numpy().any()


@pytest.mark.parametrize("B", [1, 5, 8, 24, 64])
def test_split_k_hand_over_soak(gpu, B):
    """Many split panels in flight at once, several split factors, one workspace reused by every call
    (so a partial sum read before it was written would be the previous call's): every call must give
    the bits of the first call of its shape, which is compared with the oracle.  Stops at the first
    mismatch."""
    import torch
    from paper_2207_00032_amd import binding as sb
    K, N = 8192, 4096
    W, bias, X, R = wl.make_gemm_inputs(K, N, B, seed=11, config_id=106)
    Wd, Xd, bd, Rd = _dev(W, gpu), _dev(X, gpu), _dev(bias, gpu), _dev(R, gpu)
    Wl = sb.layout_weights(Wd)
    splits = [s for s in (2, 3, 4, 8, 16, 32) if _plan_ok(sb, B, K, N, s)]
    assert len(splits) >= 4
    ws = sb.new_workspace(max(sb.plan(B, K, N, sb.PATH_MFMA, s)["workspace_bytes"] for s in splits), gpu)
    first = {}
    for rep in range(12):
        # the activations change from call to call, so stale partial sums could not go unnoticed
        Xr = Xd if rep % 2 == 0 else (Xd * 0.5).contiguous()
        for s in splits:
            Y = sb.gemm(Wl, K, N, Xr, bd, Rd, "bias_residual", workspace=ws, path=sb.PATH_MFMA, split_k=s)
            key = (s, rep % 2)
            if key not in first:
                torch.cuda.synchronize()
                first[key] = Y.clone()
                check(Y.cpu().numpy(), W, bias, Xr.cpu().numpy(), R, "bias_residual", f"soak B={B} S={s} rep={rep}")
            else:
                assert torch.equal(Y.view(torch.int16), first[key].view(torch.int16)), f"B={B} S={s} rep={rep}"
    torch.cuda.synchronize()
    assert not ws[:256 * 1024].cpu().numpy().any()


def _plan_ok(sb, B, K, N, s):
    try:
        sb.plan(B, K, N, sb.PATH_MFMA, s)
        return True
    except sb.SbiError:
        return False


@pytest.mark.parametrize("cfg_id,B,chained", [(1, 4, True), (1, 1, False), (2, 8, False), (2, 3, True)])
def test_layer_gemms_matches_oracle(gpu, cfg_id, B, chained):
    """sbi_layer_gemms: the independent GeMMs go out as one grouped launch; with Xffn2 = NULL
    FFN2 is chained on FFN1's fp16 output."""
    import torch
    from paper_2207_00032_amd import binding as sb
    cfg = wl.CONFIGS[cfg_id]
    data = [wl.make_gemm_inputs(s.K, s.N, B, seed=0, config_id=cfg_id, gemm_id=i) for i, s in enumerate(cfg.gemms)]
    Wls = [sb.layout_weights(_dev(d[0], gpu)) for d in data]
    biases = [_dev(d[1], gpu) for d in data]
    h = cfg.gemms[0].K
    L = sb.make_layer(*Wls, h, cfg.gemms[0].N, cfg.gemms[1].K, cfg.gemms[2].N, cfg.gemms[3].K,
                      bqkv=biases[0], bout=None, bffn1=biases[2], bffn2=biases[3], ffn1_gelu=True)
    ws = sb.new_workspace(sb.layer_workspace_bytes(L, B), gpu)
    Xs = [_dev(d[2], gpu) for d in data]
    Rd = _dev(data[3][3], gpu)
    Ys = [torch.empty((B, s.N), dtype=torch.float16, device=gpu) for s in cfg.gemms]
    for rep in range(2):
        sb.layer_gemms(L, B, Xs[0], Xs[1], Xs[2], None if chained else Xs[3], Rd,
                       Ys[0], Ys[1], Ys[2], Ys[3], ws)
        torch.cuda.synchronize()
        Yh = [y.cpu().numpy() for y in Ys]
        check(Yh[0], data[0][0], data[0][1], data[0][2], None, "bias", "layer qkv")
        check(Yh[1], data[1][0], None, data[1][2], None, "none", "layer attn_out")
        check(Yh[2], data[2][0], data[2][1], data[2][2], None, "bias_gelu", "layer ffn1")
        # a chained FFN2 consumed the GPU's own fp16 FFN1 output
        xin = Yh[2] if chained else data[3][2]
        check(Yh[3], data[3][0], data[3][1], xin, data[3][3], "bias_residual", "layer ffn2")
    assert not ws[:256 * 1024].cpu().numpy().any()


def test_layer_gemms_under_graph_replay(gpu):
    """The library enqueues only kernels (no memset, no allocation, no synchronisation), so a
    layer can be captured into a HIP graph; every replay must reproduce the eager bits, also
    with eager launches on the same workspace in between."""
    import torch
    from paper_2207_00032_amd import binding as sb
    cfg = wl.CONFIGS[1]
    B = 2
    data = [wl.make_gemm_inputs(s.K, s.N, B, seed=1, config_id=1, gemm_id=i) for i, s in enumerate(cfg.gemms)]
    Wls = [sb.layout_weights(_dev(d[0], gpu)) for d in data]
    biases = [_dev(d[1], gpu) for d in data]
    h = cfg.gemms[0].K
    L = sb.make_layer(*Wls, h, cfg.gemms[0].N, cfg.gemms[1].K, cfg.gemms[2].N, cfg.gemms[3].K,
                      bqkv=biases[0], bout=biases[1], bffn1=biases[2], bffn2=biases[3], ffn1_gelu=True)
    ws = sb.new_workspace(sb.layer_workspace_bytes(L, B), gpu)
    Xs = [_dev(d[2], gpu) for d in data]
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
    for rep in range(4):
        for y in Ys:
            y.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        for y, e in zip(Ys, eager):
            assert torch.equal(y.view(torch.int16), e.view(torch.int16)), f"replay {rep} differs"
        run()                                   # eager work between replays
        torch.cuda.synchronize()
    assert not ws[:256 * 1024].cpu().numpy().any()
    check(eager[3].cpu().numpy(), data[3][0], data[3][1], eager[2].cpu().numpy(), data[3][3],
          "bias_residual", "graph layer ffn2")


def test_binding_rejects_tensors_smaller_than_the_call_reads(gpu):
    """The C ABI takes bare pointers, so the binding checks extents before it passes them on."""
    import torch
    from paper_2207_00032_amd import binding as sb
    K, N, B = 256, 256, 4
    W, bias, X, R = wl.make_gemm_inputs(K, N, B, seed=9, config_id=300)
    Wl = sb.layout_weights(_dev(W, gpu))
    Xd, bd, Rd = _dev(X, gpu), _dev(bias, gpu), _dev(R, gpu)
    with pytest.raises(ValueError):
        sb.gemm(Wl, K, N, Xd[:, :128].contiguous(), bd, None, "bias")          # fewer columns than K
    with pytest.raises(ValueError):
        sb.gemm(Wl, K, N, Xd, bd[:64].contiguous(), None, "bias")              # short bias
    with pytest.raises(ValueError):
        sb.gemm(Wl, K, N, Xd, bd, Rd[:2].contiguous(), "bias_residual")        # residual with fewer rows
    with pytest.raises(ValueError):
        sb.gemm(Wl[:1024], K, N, Xd, bd, None, "bias")                          # truncated weights
    L = sb.make_layer(Wl, Wl, Wl, Wl, K, N, K, N, K)
    Y = torch.empty((B, N), dtype=torch.float16, device=gpu)
    ws = sb.new_workspace(sb.layer_workspace_bytes(L, B), gpu)
    with pytest.raises(ValueError):
        sb.layer_gemms(L, B, Xd[:2].contiguous(), Xd, Xd, Xd, None, Y, Y.clone(), Y.clone(), Y.clone(), ws)
    with pytest.raises(ValueError):
        sb.make_layer(Wl, Wl[:4096], Wl, Wl, K, N, K, N, K)
