"""The token-generation step of a whole layer (paper Sec. III-D: the four fused regions in sequence)
through paper_2207_00032_amd.decoder: every stage against the oracle fed with the GPU's own
previous stage (the per-call parity bar), the whole chain against the oracle's own chain (errors of
five roundings to fp16 compound: a looser, stated bound), and a HIP-graph replay against eager."""
import numpy as np
import pytest

from oracle import oracle as orc
from paper_2207_00032_amd import workloads as wl

pytestmark = pytest.mark.gpu
EPS = 1e-5


def _make(gpu, h, heads, f, B, S, seed):
    import torch
    from paper_2207_00032_amd import decoder
    host = {}
    for gi, (name, K, N) in enumerate((("qkv", h, 3 * h), ("out", h, h), ("ffn1", h, f), ("ffn2", f, h))):
        W, bias, _, _ = wl.make_gemm_inputs(K, N, 1, seed=seed, config_id=700, gemm_id=gi)
        host["W" + name], host["b" + name] = W, bias
    host["g1"], host["be1"], x = wl.make_layernorm_inputs(h, B, seed=seed, config_id=700, gemm_id=0)
    host["g2"], host["be2"], _ = wl.make_layernorm_inputs(h, B, seed=seed, config_id=700, gemm_id=2)
    _, Kc, Vc = wl.make_attention_inputs(B, heads, h // heads, S, seed=seed, config_id=700)
    d = {k: torch.from_numpy(v).to(gpu) for k, v in host.items()}
    layer = decoder.DecoderLayer(h, heads, d["Wqkv"], d["bqkv"], d["Wout"], d["bout"], d["Wffn1"], d["bffn1"],
                                 d["Wffn2"], d["bffn2"], d["g1"], d["be1"], d["g2"], d["be2"], EPS)
    return layer, host, x, Kc, Vc


def _oracle_step(hw, x, Kc, Vc, pos):
    qkv = orc.gemm(orc.layernorm(x, hw["g1"], hw["be1"], EPS), hw["Wqkv"], hw["bqkv"], None, epi=orc.EPI_BIAS)
    B = x.shape[0]
    H, d = Kc.shape[1], Kc.shape[3]
    ctx, K2, V2 = orc.attn_decode(qkv.reshape(B, 3, H, d), Kc, Vc, pos)
    x2 = orc.gemm(ctx, hw["Wout"], hw["bout"], x, epi=orc.EPI_BIAS | orc.EPI_RES)
    f = orc.gemm(orc.layernorm(x2, hw["g2"], hw["be2"], EPS), hw["Wffn1"], hw["bffn1"], None, epi=orc.EPI_BIAS | orc.EPI_GELU)
    y = orc.gemm(f, hw["Wffn2"], hw["bffn2"], x2, epi=orc.EPI_BIAS | orc.EPI_RES)
    return y, K2, V2


@pytest.mark.parametrize("h,heads,f,B,S,pos", [(512, 4, 2048, 3, 200, 150), (1024, 16, 4096, 8, 700, 640), (256, 2, 1024, 1, 8, 0)])
def test_decoder_step_stage_by_stage_and_end_to_end(gpu, h, heads, f, B, S, pos):
    import torch
    layer, hw, x, Kc, Vc = _make(gpu, h, heads, f, B, S, seed=h + B)
    d = h // heads
    st = layer.new_state(B, S, gpu, torch.from_numpy(Kc).to(gpu), torch.from_numpy(Vc).to(gpu))
    y = layer.step(torch.from_numpy(x).to(gpu), pos, st)
    torch.cuda.synchronize()
    g = {k: getattr(st, k).cpu().numpy() for k in ("qkv", "ctx", "x2", "f", "y")}
    stages = [
        ("qkv", g["qkv"].reshape(B, 3 * h), orc.gemm(orc.layernorm(x, hw["g1"], hw["be1"], EPS), hw["Wqkv"], hw["bqkv"], None, epi=orc.EPI_BIAS)),
        ("attention", g["ctx"], orc.attn_decode(g["qkv"], Kc, Vc, pos)[0]),
        ("attn-out", g["x2"], orc.gemm(g["ctx"], hw["Wout"], hw["bout"], x, epi=orc.EPI_BIAS | orc.EPI_RES)),
        ("ffn1", g["f"], orc.gemm(orc.layernorm(g["x2"], hw["g2"], hw["be2"], EPS), hw["Wffn1"], hw["bffn1"], None,
                                  epi=orc.EPI_BIAS | orc.EPI_GELU)),
        ("ffn2", g["y"], orc.gemm(g["f"], hw["Wffn2"], hw["bffn2"], g["x2"], epi=orc.EPI_BIAS | orc.EPI_RES)),
    ]
    for name, got, want in stages:
        ok, rep = orc.check_close(got, want, ulps=2, abs_tol=1e-3)
        assert ok, (name, rep)
    _, K2, V2 = orc.attn_decode(g["qkv"], Kc, Vc, pos)
    assert np.array_equal(st.k_cache.cpu().numpy().view(np.uint16), K2.view(np.uint16))
    assert np.array_equal(st.v_cache.cpu().numpy().view(np.uint16), V2.view(np.uint16))
    # the whole chain against the oracle's own chain: five fp16 roundings in sequence, each stage's
    # 1-ulp differences amplified by at most the next stage's gain
    want, _, _ = _oracle_step(hw, x, Kc, Vc, pos)
    ok, rep = orc.check_close(y.cpu().numpy(), want, ulps=8, abs_tol=8e-3)
    assert ok, ("end to end", rep)


def test_decoder_steps_under_graph_replay(gpu):
    """Three generated tokens, each step replayed from one captured graph per position, with eager
    work in between; every replay must give the eager bits."""
    import torch
    h, heads, f, B, S = 512, 4, 2048, 2, 64
    layer, hw, x, Kc, Vc = _make(gpu, h, heads, f, B, S, seed=9)
    xd = torch.from_numpy(x).to(gpu)
    st_e = layer.new_state(B, S, gpu, torch.from_numpy(Kc).to(gpu), torch.from_numpy(Vc).to(gpu))
    st_g = layer.new_state(B, S, gpu, torch.from_numpy(Kc).to(gpu), torch.from_numpy(Vc).to(gpu))
    for pos in (40, 41, 42):
        want = layer.step(xd, pos, st_e).clone()
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            layer.step(xd, pos, st_g)                      # warm-up outside the capture
            side.synchronize()
            with torch.cuda.graph(graph, stream=side):
                layer.step(xd, pos, st_g)
        for _ in range(3):
            st_g.y.zero_()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(st_g.y.view(torch.int16), want.view(torch.int16))
            (st_g.y.float() * 2).sum().item()              # unrelated eager work between replays
        assert torch.equal(st_g.k_cache.view(torch.int16), st_e.k_cache.view(torch.int16))
        xd = want                                          # the next token's input: this step's output


def test_ragged_decoder_steps_from_one_graph(gpu):
    """Sequences of different lengths (sbi_attn_decode_ragged inside the step).  The positions live on
    the device, so ONE captured graph serves consecutive tokens: between replays only the position
    array is advanced.  Every replay's attention stage is checked against the oracle sequence by
    sequence on the GPU's own QKV rows, the caches bit for bit, the output against an eager twin."""
    import torch
    h, heads, f, B, S, bound = 512, 4, 2048, 3, 80, 70
    d = h // heads
    layer, hw, x, Kc, Vc = _make(gpu, h, heads, f, B, S, seed=11)
    xd = torch.from_numpy(x).to(gpu)
    st_e = layer.new_state(B, S, gpu, torch.from_numpy(Kc).to(gpu), torch.from_numpy(Vc).to(gpu))
    st_g = layer.new_state(B, S, gpu, torch.from_numpy(Kc).to(gpu), torch.from_numpy(Vc).to(gpu))
    pos = [60, 0, 33]
    pos_g = torch.tensor(pos, dtype=torch.int32, device=gpu)
    x_g = xd.clone()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    warm = layer.new_state(B, S, gpu)                      # the warm-up and the capture run must not touch st_g's caches
    with torch.cuda.stream(side):
        layer.step(x_g, pos_g, warm, pos_bound=bound)
        side.synchronize()
    keep = {k: getattr(st_g, k) for k in ("k_cache", "v_cache")}
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            layer.step(x_g, pos_g, st_g, pos_bound=bound)
    Ko, Vo = Kc, Vc
    for token in range(3):
        want = layer.step(xd, torch.tensor(pos, dtype=torch.int32, device=gpu), st_e, pos_bound=bound).clone()
        x_g.copy_(xd)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(st_g.y.view(torch.int16), want.view(torch.int16)), token
        qkv = st_g.qkv.cpu().numpy()
        ctx = st_g.ctx.cpu().numpy()
        Kn, Vn = Ko.copy(), Vo.copy()
        for b in range(B):
            w, Kn[b:b + 1], Vn[b:b + 1] = orc.attn_decode(qkv[b:b + 1], Ko[b:b + 1], Vo[b:b + 1], pos[b])
            ok, rep = orc.check_close(ctx[b:b + 1], w, ulps=2, abs_tol=1e-3)
            assert ok, (token, b, rep)
        Ko, Vo = Kn, Vn
        assert np.array_equal(keep["k_cache"].cpu().numpy().view(np.uint16), Ko.view(np.uint16))
        assert np.array_equal(keep["v_cache"].cpu().numpy().view(np.uint16), Vo.view(np.uint16))
        pos = [p + 1 for p in pos]
        pos_g.add_(1)                                      # eager work between the replays
        xd = want


def test_two_layers_chained_through_the_output_moments(gpu):
    """Layer 2's input layer-norm takes its row statistics from the moments layer 1's FFN2 epilogue left
    (no second pass over the rows).  Its QKV stage is checked against the oracle fed with layer 1's
    GPU output, and the two-layer result against the same chain run with recomputed statistics."""
    import torch
    h, heads, f, B, S, pos = 1024, 8, 4096, 5, 96, 70
    layer, hw, x, Kc, Vc = _make(gpu, h, heads, f, B, S, seed=21)
    xd = torch.from_numpy(x).to(gpu)
    mk = lambda: layer.new_state(B, S, gpu, torch.from_numpy(Kc).to(gpu), torch.from_numpy(Vc).to(gpu))
    s1, s2, s2_ref = mk(), mk(), mk()
    y1 = layer.step(xd, pos, s1)
    y2 = layer.step(y1, pos, s2, x_moments=s1.y_moments)
    y2_ref = layer.step(y1, pos, s2_ref)
    torch.cuda.synchronize()
    y1h = y1.cpu().numpy()
    want_qkv = orc.gemm(orc.layernorm(y1h, hw["g1"], hw["be1"], EPS), hw["Wqkv"], hw["bqkv"], None, epi=orc.EPI_BIAS)
    ok, rep = orc.check_close(s2.qkv.cpu().numpy().reshape(B, 3 * h), want_qkv, ulps=2, abs_tol=1e-3)
    assert ok, rep
    # moments of y1 against their definition (per 64-feature panel: mean and sum of squared deviations)
    m = s1.y_moments.cpu().numpy().astype(np.float64)
    panels = y1h.astype(np.float64).reshape(B, h // 64, 64)
    assert np.allclose(m[..., 0], panels.mean(-1), rtol=0, atol=2e-3)
    assert np.allclose(m[..., 1], ((panels - panels.mean(-1, keepdims=True)) ** 2).sum(-1), rtol=2e-3, atol=1e-2)
    ok, rep = orc.check_close(y2.cpu().numpy(), y2_ref.cpu().numpy(), ulps=8, abs_tol=8e-3)
    assert ok, rep
