"""GPU parity of the INT8 path (sbi_gemm_i8 and its weight preparation) against the oracle.
Integer work is compared bit for bit: weight codes and scales from sbi_gemm_i8_quantize_weights,
the laid-out bytes from sbi_gemm_i8_layout_weights.  The GeMM is compared with the oracle's
gemm_i8_from_fp16 on the same codes: the activation codes are decided in binary32 on both sides,
so the integer sums agree exactly and only the fp32-vs-fp64 epilogue remains:
|gpu - oracle| <= max(2 ulp16(oracle), 1e-3), bit-identical run to run."""
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


def prepare(gpu, W):
    """Quantise and lay out W on the GPU; return (laid-out tensor, scales tensor, host codes, host scales)."""
    import torch
    from paper_2207_00032_amd import binding as sb
    Wq_d, sw_d = sb.i8_quantize_weights(_dev(W, gpu))
    Wl = sb.i8_layout_weights(Wq_d)
    torch.cuda.synchronize()
    return Wl, sw_d, Wq_d.cpu().numpy(), sw_d.cpu().numpy()


def check(Y, X, Wq, sw, bias, R, epi, what):
    want = orc.gemm_i8_from_fp16(X, Wq, sw, bias, R, EPI_ORACLE[epi])
    ok, rep = orc.check_close(Y, want, ulps=2, abs_tol=1e-3)
    assert ok, f"{what}: {rep}"


@pytest.mark.parametrize("K,N", [(16, 1), (64, 64), (200, 150), (1000, 130), (2048, 520), (4096, 192)])
def test_weight_quantisation_and_layout_bit_exact(gpu, K, N):
    import torch
    from paper_2207_00032_amd import binding as sb
    rng = np.random.default_rng(K * 31 + N)
    W = (rng.standard_normal((K, N)) * 0.02 * np.exp(rng.uniform(-2, 2, (1, N)))).astype(np.float16)
    if N > 3:
        W[:, 3] = 0                                        # an all-zero output channel
    Wl, sw_d, Wq, sw = prepare(gpu, W)
    Wq_ref, sw_ref = orc.quantize_columns(W)
    assert np.array_equal(Wq, Wq_ref)
    assert np.array_equal(sw.view(np.uint32), sw_ref.view(np.uint32))
    raw = Wl.cpu().numpy()
    assert raw.size == sb.i8_layout_bytes(K, N)
    assert np.array_equal(raw[256:].view(np.int8), orc.layout_weights_i8(Wq_ref))
    hdr = raw[:256]
    KS, P = orc.layout_dims_i8(K, N)
    assert hdr[:4].tobytes() == b"SBIG" and not hdr[56:].any()
    assert tuple(hdr[8:40].view(np.int64)) == (K, N, KS, P)
    assert tuple(hdr[40:56].view(np.int32)) == (16, 64, 4, 16)
    assert sb.i8_layout_check(Wl, K, N) == 0 and sb.layout_check(Wl, K, N) == 5
    assert sb.i8_layout_check(Wl, K + 16, N) == 5
    if K % 8 == 0:
        assert sb.i8_layout_check(sb.layout_weights(_dev(W, gpu)), K, N) == 5      # an fp16 layout is not an int8 one


@pytest.mark.parametrize("B,K,N", [(1, 16, 1), (1, 64, 64), (3, 272, 200), (8, 1008, 130), (8, 4096, 192),
                                   (5, 4112, 72), (16, 2048, 320), (17, 4096, 136), (33, 1024, 192),
                                   (64, 2048, 128), (2, 12288, 64), (48, 8192, 192), (64, 528, 72)])
def test_int8_gemm_shapes_and_epilogues(gpu, B, K, N):
    from paper_2207_00032_amd import binding as sb
    W, bias, X, R = wl.make_gemm_inputs(K, N, B, seed=B + K + N, config_id=400)
    Wl, sw_d, Wq, sw = prepare(gpu, W)
    Xd, bd, Rd = _dev(X, gpu), _dev(bias, gpu), _dev(R, gpu)
    for epi in ("none", "bias", "bias_gelu", "bias_residual", "gelu", "residual"):
        Y = sb.gemm_i8(Wl, sw_d, K, N, Xd, bd if "bias" in epi else None, Rd if "residual" in epi else None, epi)
        check(Y.cpu().numpy(), X, Wq, sw, bias, R, epi, f"B={B} K={K} N={N} {epi}")


@pytest.mark.parametrize("B,K,N", [(1, 4096, 192), (8, 2048, 320), (16, 4096, 128), (40, 1024, 192),
                                   (64, 2048, 128)])
@pytest.mark.parametrize("waves,depth", [(4, 2), (4, 4), (8, 4)])
def test_int8_gemm_split_k_and_tuning_variants(gpu, B, K, N, waves, depth):
    from paper_2207_00032_amd import binding as sb
    W, bias, X, R = wl.make_gemm_inputs(K, N, B, seed=3, config_id=401)
    Wl, sw_d, Wq, sw = prepare(gpu, W)
    Xd, bd, Rd = _dev(X, gpu), _dev(bias, gpu), _dev(R, gpu)
    for S in (1, 2, 3, 7, 16):
        try:
            sb.plan(B, K, N, sb.PATH_MFMA, S, waves, depth, int8=True)
        except sb.SbiError:
            continue
        Y = sb.gemm_i8(Wl, sw_d, K, N, Xd, bd, Rd, "bias_residual", path=sb.PATH_MFMA, split_k=S,
                       waves=waves, depth=depth)
        check(Y.cpu().numpy(), X, Wq, sw, bias, R, "bias_residual", f"B={B} K={K} N={N} S={S} w={waves} d={depth}")


@pytest.mark.parametrize("B,K,N", [(17, 4096, 136), (24, 1040, 72), (33, 8192, 200), (48, 2048, 448), (64, 4096, 192)])
def test_int8_two_panel_blocks(gpu, B, K, N):
    """Batches above 16: blocks that stream two adjacent panels of int8 weights against codes from
    the workspace (odd panel counts leave a lone last panel); automatic plan and forced splits."""
    from paper_2207_00032_amd import binding as sb
    W, bias, X, R = wl.make_gemm_inputs(K, N, B, seed=4, config_id=402)
    Wl, sw_d, Wq, sw = prepare(gpu, W)
    Xd, bd, Rd = _dev(X, gpu), _dev(bias, gpu), _dev(R, gpu)
    ran = 0
    for depth in (2, 4):                                   # 4: two wave groups, one panel each
        for S in (0, 1, 2, 5):
            try:
                sb.plan(B, K, N, sb.PATH_MFMA, S, 8, depth, panels=2, int8=True)
            except sb.SbiError:
                continue
            for epi in ("bias_gelu", "bias_residual"):
                Y = sb.gemm_i8(Wl, sw_d, K, N, Xd, bd, Rd, epi, path=sb.PATH_MFMA, split_k=S, waves=8, depth=depth, panels=2)
                check(Y.cpu().numpy(), X, Wq, sw, bias, R, epi, f"2-panel B={B} K={K} N={N} S={S} d={depth} {epi}")
                ran += 1
    assert ran > 0


def test_int8_special_rows_and_determinism(gpu):
    """An all-zero activation row (scale 0), a row dominated by one outlier (every other code 0 or
    +-1), exact ties in the code decision, a shared workspace across differently shaped calls."""
    import torch
    from paper_2207_00032_amd import binding as sb
    K, N, B = 2048, 200, 5
    W, bias, X, R = wl.make_gemm_inputs(K, N, B, seed=8, config_id=402)
    X[1, :] = 0
    X[2, :] = (np.random.default_rng(1).standard_normal(K) * 0.3).astype(np.float16)
    X[2, 77] = 300.0
    X[3, :] = np.tile(np.array([127, 0.5, 1.5, 2.5, -0.5, -1.5, 63.5, -2.5], np.float16), K // 8)   # inv = 1: ties
    Wl, sw_d, Wq, sw = prepare(gpu, W)
    Xd, bd = _dev(X, gpu), _dev(bias, gpu)
    ws = sb.new_workspace(max(sb.i8_workspace_bytes(B, K, N), sb.i8_workspace_bytes(2, K, N)), gpu)
    first = None
    for rep in range(3):
        Y = sb.gemm_i8(Wl, sw_d, K, N, Xd, bd, None, "bias", workspace=ws)
        Y2 = sb.gemm_i8(Wl, sw_d, K, N, Xd[:2].contiguous(), bd, None, "bias", workspace=ws)
        torch.cuda.synchronize()
        if first is None:
            first = Y.clone()
        assert torch.equal(Y.view(torch.int16), first.view(torch.int16))
        assert torch.equal(Y2.view(torch.int16), first[:2].view(torch.int16))
    check(first.cpu().numpy(), X, Wq, sw, bias, None, "bias", "special rows")
    assert not ws[:256 * 1024].cpu().numpy().any()


def test_int8_with_unit_scales_equals_the_fp16_path_bits(gpu):
    """Integer-valued operands with amax = 127: codes are the values, scales are 1, and the INT8
    kernel must give the same fp16 bits as the fp16 kernel (both exact before the one rounding)."""
    import torch
    from paper_2207_00032_amd import binding as sb
    rng = np.random.default_rng(4)
    B, K, N = 6, 1024, 136
    X = rng.integers(-20, 21, (B, K)).astype(np.float16)
    W = rng.integers(-3, 4, (K, N)).astype(np.float16)
    X[:, 0] = 127
    W[0, :] = -127
    bias = rng.standard_normal(N).astype(np.float16)
    Wl8, sw_d, Wq, sw = prepare(gpu, W)
    assert np.all(sw == 1)
    Y8 = sb.gemm_i8(Wl8, sw_d, K, N, _dev(X, gpu), _dev(bias, gpu), None, "bias")
    Y16 = sb.gemm(sb.layout_weights(_dev(W, gpu)), K, N, _dev(X, gpu), _dev(bias, gpu), None, "bias")
    torch.cuda.synchronize()
    assert torch.equal(Y8.view(torch.int16), Y16.view(torch.int16))
    assert np.array_equal(Y8.cpu().numpy().view(np.uint16), orc.gemm(X, W, bias, None, epi=orc.EPI_BIAS).view(np.uint16))


@pytest.mark.parametrize("gi", [0, 1, 2, 3])
@pytest.mark.parametrize("B", [1, 8])
def test_int8_config2_h4096_gemms(gpu, gi, B):
    from paper_2207_00032_amd import binding as sb
    spec, W, bias, X, R = wl.make_config_gemm(2, gi, seed=0, B=B)
    Wl, sw_d, Wq, sw = prepare(gpu, W)
    # the GPU's weight codes and scales are the oracle's, bit for bit, before they are handed to it
    Wq_ref, sw_ref = orc.quantize_columns(W)
    assert np.array_equal(Wq, Wq_ref) and np.array_equal(sw.view(np.uint32), sw_ref.view(np.uint32))
    assert np.array_equal(Wl.cpu().numpy()[256:].view(np.int8), orc.layout_weights_i8(Wq_ref))
    epi = {wl.NONE: "none", wl.BIAS: "bias", wl.BIAS_GELU: "bias_gelu", wl.BIAS_RESIDUAL: "bias_residual",
           wl.GELU: "gelu", wl.RESIDUAL: "residual"}[spec.epilogue]
    Y = sb.gemm_i8(Wl, sw_d, spec.K, spec.N, _dev(X, gpu), _dev(bias, gpu) if "bias" in epi else None,
                   _dev(R, gpu) if "residual" in epi else None, epi)
    check(Y.cpu().numpy(), X, Wq, sw, bias, R, epi, f"config2 {spec.name} B={B}")


@pytest.mark.parametrize("cfg_id,B,chained", [(1, 4, True), (1, 1, False), (2, 8, False), (2, 3, True)])
def test_int8_layer_gemms(gpu, cfg_id, B, chained):
    """sbi_layer_gemms with int8 weights and per-channel scales: the grouped launch runs the INT8
    kernel; a chained FFN2 quantises the GPU's own fp16 FFN1 output."""
    import torch
    from paper_2207_00032_amd import binding as sb
    cfg = wl.CONFIGS[cfg_id]
    data = [wl.make_gemm_inputs(s.K, s.N, B, seed=5, config_id=cfg_id, gemm_id=i) for i, s in enumerate(cfg.gemms)]
    prep = [prepare(gpu, d[0]) for d in data]
    biases = [_dev(d[1], gpu) for d in data]
    h = cfg.gemms[0].K
    L = sb.make_layer(*[p[0] for p in prep], h, cfg.gemms[0].N, cfg.gemms[1].K, cfg.gemms[2].N, cfg.gemms[3].K,
                      bqkv=biases[0], bout=biases[1], bffn1=biases[2], bffn2=biases[3], ffn1_gelu=True,
                      scales=[p[1] for p in prep])
    ws = sb.new_workspace(sb.layer_workspace_bytes(L, B), gpu)
    Xs = [_dev(d[2], gpu) for d in data]
    Rd = _dev(data[3][3], gpu)
    Ys = [torch.empty((B, s.N), dtype=torch.float16, device=gpu) for s in cfg.gemms]
    for rep in range(2):
        sb.layer_gemms(L, B, Xs[0], Xs[1], Xs[2], None if chained else Xs[3], Rd, Ys[0], Ys[1], Ys[2], Ys[3], ws)
        torch.cuda.synchronize()
        Yh = [y.cpu().numpy() for y in Ys]
        for g, (epi, r) in enumerate((("bias", None), ("bias", None), ("bias_gelu", None),
                                      ("bias_residual", data[3][3]))):
            xin = Yh[2] if (g == 3 and chained) else data[g][2]
            check(Yh[g], xin, prep[g][2], prep[g][3], data[g][1], r, epi, f"layer gemm {g}")
    assert not ws[:256 * 1024].cpu().numpy().any()


# ------------------------------------------------------------------------------ layer-norm in front
def check_ln(Y, X, gamma, beta, Wq, sw, bias, R, epi, what):
    want = orc.gemm_i8_ln_from_fp16(X, gamma, beta, 1e-5, Wq, sw, bias, R, EPI_ORACLE[epi])
    ok, rep = orc.check_close(Y, want, ulps=2, abs_tol=1e-3)
    assert ok, f"{what}: {rep}"


@pytest.mark.parametrize("B,K,N", [(1, 64, 64), (3, 272, 200), (8, 4096, 192), (5, 4112, 72), (16, 2048, 320),
                                   (33, 1024, 192), (64, 2048, 128), (2, 12288, 64), (48, 8192, 192)])
def test_int8_gemm_with_layernorm_in_front(gpu, B, K, N):
    """sbi_gemm_i8_ln against the oracle's composition layernorm -> quantize_rows -> gemm_i8."""
    from paper_2207_00032_amd import binding as sb
    W, bias, _, R = wl.make_gemm_inputs(K, N, B, seed=B + K + N, config_id=403)
    gamma, beta, X = wl.make_layernorm_inputs(K, B, seed=B + K, config_id=403)
    Wl, sw_d, Wq, sw = prepare(gpu, W)
    ln = (_dev(gamma, gpu), _dev(beta, gpu), 1e-5)
    Xd, bd, Rd = _dev(X, gpu), _dev(bias, gpu), _dev(R, gpu)
    for epi in ("none", "bias_gelu", "bias_residual"):
        Y = sb.gemm_i8(Wl, sw_d, K, N, Xd, bd if "bias" in epi else None, Rd if "residual" in epi else None, epi,
                       layernorm=ln)
        check_ln(Y.cpu().numpy(), X, gamma, beta, Wq, sw, bias, R, epi, f"LN+INT8 B={B} K={K} N={N} {epi}")


def test_int8_layernorm_codes_are_the_oracles(gpu):
    """Weights 127 * identity (codes 127 on the diagonal, column scales 1) make Y[b,n] = code[b,n] * amax_b:
    one activation code off by one would move an output by a whole amax, far beyond the tolerance.  Rows
    with very different means and spreads, a constant row (variance 0), 2048 features."""
    import torch
    from paper_2207_00032_amd import binding as sb
    K = N = 2048
    B = 9
    gamma, beta, X = wl.make_layernorm_inputs(K, B, seed=77, config_id=404, row_shift=3.0, row_scale=8.0)
    X[4, :] = np.float16(1.25)                                   # constant row: normalises to beta
    W = (127.0 * np.eye(K)).astype(np.float16)
    Wl, sw_d, Wq, sw = prepare(gpu, W)
    assert np.all(sw == 1) and np.array_equal(np.diag(Wq), np.full(K, 127, np.int8))
    Y = sb.gemm_i8(Wl, sw_d, K, N, _dev(X, gpu), None, None, "none", layernorm=(_dev(gamma, gpu), _dev(beta, gpu), 1e-5))
    torch.cuda.synchronize()
    want = orc.gemm_i8_ln_from_fp16(X, gamma, beta, 1e-5, Wq, sw)
    ok, rep = orc.check_close(Y.cpu().numpy(), want, ulps=2, abs_tol=1e-3)
    assert ok, rep
    Xq, sx = orc.quantize_rows(orc.layernorm(X, gamma, beta, 1e-5))
    assert np.abs(Xq).max() == 127 and len(np.unique(Xq)) > 200    # the case does exercise the code range
    # a code off by one moves an output by the row's amax = 127 * sx; the tolerance is far below that everywhere
    step = (127.0 * sx.astype(np.float64))[:, None]
    diff = np.abs(Y.cpu().numpy().astype(np.float64) - want.astype(np.float64))
    assert (diff < 0.25 * np.maximum(step, 1e-6)).all() or (step == 0).any()
    assert (diff[sx > 0] < 0.25 * step[sx > 0]).all()


@pytest.mark.parametrize("cfg_id,B,chained", [(1, 4, True), (1, 1, False), (2, 8, False), (1, 24, False)])
def test_int8_layer_gemms_with_layernorms(gpu, cfg_id, B, chained):
    """sbi_layer_gemms with int8 weights and ln1 / ln2: QKV and FFN1 see normalised rows, the attention
    output and FFN2 plain ones, all four in one INT8 launch behind one quantisation kernel."""
    import torch
    from paper_2207_00032_amd import binding as sb
    cfg = wl.CONFIGS[cfg_id]
    data = [wl.make_gemm_inputs(s.K, s.N, B, seed=6, config_id=cfg_id, gemm_id=i) for i, s in enumerate(cfg.gemms)]
    h = cfg.gemms[0].K
    lns = {gi: wl.make_layernorm_inputs(h, B, seed=6, config_id=cfg_id, gemm_id=gi) for gi in (0, 2)}
    prep = [prepare(gpu, d[0]) for d in data]
    biases = [_dev(d[1], gpu) for d in data]
    ln_d = {gi: (_dev(lns[gi][0], gpu), _dev(lns[gi][1], gpu)) for gi in (0, 2)}     # the layer struct holds bare pointers
    L = sb.make_layer(*[p[0] for p in prep], h, cfg.gemms[0].N, cfg.gemms[1].K, cfg.gemms[2].N, cfg.gemms[3].K,
                      bqkv=biases[0], bout=biases[1], bffn1=biases[2], bffn2=biases[3], ffn1_gelu=True,
                      scales=[p[1] for p in prep], ln1=ln_d[0], ln2=ln_d[2])
    ws = sb.new_workspace(sb.layer_workspace_bytes(L, B), gpu)
    Xh = [lns[0][2], data[1][2], lns[2][2], data[3][2]]
    Xs = [_dev(x, gpu) for x in Xh]
    Rd = _dev(data[3][3], gpu)
    Ys = [torch.empty((B, s.N), dtype=torch.float16, device=gpu) for s in cfg.gemms]
    for rep in range(2):
        sb.layer_gemms(L, B, Xs[0], Xs[1], Xs[2], None if chained else Xs[3], Rd, Ys[0], Ys[1], Ys[2], Ys[3], ws)
        torch.cuda.synchronize()
        Yh = [y.cpu().numpy() for y in Ys]
        for g, (epi, r) in enumerate((("bias", None), ("bias", None), ("bias_gelu", None), ("bias_residual", data[3][3]))):
            xin = Yh[2] if (g == 3 and chained) else Xh[g]
            if g in (0, 2):
                check_ln(Yh[g], xin, lns[g][0], lns[g][1], prep[g][2], prep[g][3], data[g][1], r, epi, f"LN INT8 layer gemm {g}")
            else:
                check(Yh[g], xin, prep[g][2], prep[g][3], data[g][1], r, epi, f"LN INT8 layer gemm {g}")
    assert not ws[:256 * 1024].cpu().numpy().any()
