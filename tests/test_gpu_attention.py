"""GPU parity of the single-token attention with a KV cache (sbi_attn_decode) against the oracle:
outputs within max(2 ulp16(oracle), 1e-3), the cache update (the "transposition") bit for bit,
bit-identical run to run."""
import numpy as np
import pytest

from oracle import oracle as orc
from paper_2207_00032_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _dev(a, gpu):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).to(gpu)


@pytest.mark.parametrize("B,H,d,S,pos,ks", [
    (1, 1, 64, 8, 0, 1.0), (1, 1, 128, 1, 0, 1.0), (2, 4, 128, 136, 135, 1.0), (3, 5, 64, 70, 33, 2.0),
    (8, 32, 128, 136, 128, 1.0), (4, 16, 64, 2048, 2047, 1.0), (64, 8, 128, 300, 150, 1.0),
    (3, 5, 128, 1000, 777, 4.0), (1, 2, 128, 8192, 8000, 1.0), (2, 40, 128, 520, 511, 3.0), (1, 1, 64, 700, 256, 1.0),
])
def test_attention_decode_matches_oracle(gpu, B, H, d, S, pos, ks):
    import torch
    from paper_2207_00032_amd import binding as sb
    qkv, Kc, Vc = wl.make_attention_inputs(B, H, d, S, seed=B + H + S, config_id=500, key_scale=ks)
    want, K2, V2 = orc.attn_decode(qkv, Kc, Vc, pos)
    Kd, Vd = _dev(Kc, gpu), _dev(Vc, gpu)
    ws = sb.new_workspace(sb.attn_workspace_bytes(B, H, d, S), gpu)
    first = None
    for rep in range(2):
        out = sb.attn_decode(_dev(qkv, gpu), Kd, Vd, pos, workspace=ws)
        torch.cuda.synchronize()
        if first is None:
            first = out.clone()
        assert torch.equal(out.view(torch.int16), first.view(torch.int16))
    ok, rep = orc.check_close(first.cpu().numpy(), want, ulps=2, abs_tol=1e-3)
    assert ok, rep
    assert np.array_equal(Kd.cpu().numpy().view(np.uint16), K2.view(np.uint16))
    assert np.array_equal(Vd.cpu().numpy().view(np.uint16), V2.view(np.uint16))
    assert not ws[:256 * 1024].cpu().numpy().any()


def test_eight_generated_tokens_after_a_prompt_of_128(gpu):
    """The paper's latency workload shape (Sec. V: prompt of 128 tokens, 8 generated): eight
    consecutive calls, each appending to the cache the GPU itself maintains."""
    import torch
    from paper_2207_00032_amd import binding as sb
    B, H, d, S = 8, 32, 128, 136
    _, Kc, Vc = wl.make_attention_inputs(B, H, d, S, seed=1, config_id=501)
    Kd, Vd = _dev(Kc, gpu), _dev(Vc, gpu)
    Ko, Vo = Kc, Vc
    ws = sb.new_workspace(sb.attn_workspace_bytes(B, H, d, S), gpu)
    for step in range(8):
        qkv, _, _ = wl.make_attention_inputs(B, H, d, 1, seed=100 + step, config_id=501)
        out = sb.attn_decode(_dev(qkv, gpu), Kd, Vd, 128 + step, workspace=ws)
        want, Ko, Vo = orc.attn_decode(qkv, Ko, Vo, 128 + step)
        torch.cuda.synchronize()
        ok, rep = orc.check_close(out.cpu().numpy(), want, ulps=2, abs_tol=1e-3)
        assert ok, (step, rep)
    assert np.array_equal(Kd.cpu().numpy().view(np.uint16), Ko.view(np.uint16))
    assert np.array_equal(Vd.cpu().numpy().view(np.uint16), Vo.view(np.uint16))


def test_attention_special_cases(gpu):
    """Equal keys (uniform weights: the mean of the values), one dominating key (its value), an
    explicit scale, and scores large enough that a naive exponential would overflow."""
    import torch
    from paper_2207_00032_amd import binding as sb
    B, H, d, S, pos = 2, 3, 128, 64, 40
    qkv, Kc, Vc = wl.make_attention_inputs(B, H, d, S, seed=2, config_id=502)
    Kc[0] = Kc[0, :, :1]
    qkv[0, 1] = Kc[0, :, 0]
    Kc[1, 1, 7] = (qkv[1, 0, 1].astype(np.float32) * 30).astype(np.float16)          # score ~ 30 * |q|^2 / sqrt(d) >> others
    Kc[1, 2] = (Kc[1, 2].astype(np.float32) * 60).astype(np.float16)                 # scores in the hundreds
    for scale in (0.0, 0.25):
        want, _, _ = orc.attn_decode(qkv, Kc, Vc, pos, scale=None if scale == 0.0 else scale)
        out = sb.attn_decode(_dev(qkv, gpu), _dev(Kc, gpu), _dev(Vc, gpu), pos, scale=scale)
        torch.cuda.synchronize()
        o = out.cpu().numpy()
        assert np.isfinite(o.astype(np.float32)).all()
        ok, rep = orc.check_close(o, want, ulps=2, abs_tol=1e-3)
        assert ok, (scale, rep)
    mean = (Vc[0, :, :pos].astype(np.float64).sum(axis=1) + qkv[0, 2].astype(np.float64)) / (pos + 1)
    ok, rep = orc.check_close(o[0].reshape(H, d), mean.astype(np.float16), ulps=2, abs_tol=1e-3)
    assert ok, rep


# B, H, d, S, positions (one per sequence), bound handed to the call
RAGGED = [
    (4, 3, 128, 136, [135, 0, 17, 64], 135),
    (8, 32, 128, 2048, [2047, 5, 1000, 256, 255, 1, 1999, 640], 2047),      # long and short sequences side by side
    (5, 2, 64, 1200, [1100, 3, 700, 0, 512], 1150),                          # a bound above every position
    (3, 40, 128, 520, [100, 511, 300], 511),
    (64, 8, 64, 300, None, 299),                                             # drawn positions
    (1, 1, 64, 8, [0], 0),
]


@pytest.mark.parametrize("B,H,d,S,pos,bound", RAGGED)
def test_ragged_batch_matches_the_oracle_sequence_by_sequence(gpu, B, H, d, S, pos, bound):
    """sbi_attn_decode_ragged: sequences of one batch at different lengths.  The oracle is the same
    definition as for the common position, applied to each sequence with its own (a batch of one)."""
    import torch
    from paper_2207_00032_amd import binding as sb
    qkv, Kc, Vc = wl.make_attention_inputs(B, H, d, S, seed=B + H + S, config_id=510)
    if pos is None:
        pos = np.random.default_rng(B).integers(0, bound + 1, size=B).tolist()
        pos[0], pos[1] = bound, 0
    want = np.empty((B, H * d), dtype=np.float16)
    K2, V2 = Kc.copy(), Vc.copy()
    for b in range(B):
        want[b:b + 1], K2[b:b + 1], V2[b:b + 1] = orc.attn_decode(qkv[b:b + 1], Kc[b:b + 1], Vc[b:b + 1], pos[b])
    Kd, Vd = _dev(Kc, gpu), _dev(Vc, gpu)
    pd = torch.tensor(pos, dtype=torch.int32, device=gpu)
    ws = sb.new_workspace(sb.attn_workspace_bytes(B, H, d, S), gpu)
    first = None
    for rep in range(2):
        out = sb.attn_decode_ragged(_dev(qkv, gpu), Kd, Vd, pd, bound, workspace=ws)
        torch.cuda.synchronize()
        if first is None:
            first = out.clone()
        assert torch.equal(out.view(torch.int16), first.view(torch.int16))
    ok, rep = orc.check_close(first.cpu().numpy(), want, ulps=2, abs_tol=1e-3)
    assert ok, rep
    assert np.array_equal(Kd.cpu().numpy().view(np.uint16), K2.view(np.uint16))
    assert np.array_equal(Vd.cpu().numpy().view(np.uint16), V2.view(np.uint16))
    assert not ws[:256 * 1024].cpu().numpy().any()


def test_ragged_call_with_equal_positions_is_the_common_call_bit_for_bit(gpu):
    import torch
    from paper_2207_00032_amd import binding as sb
    B, H, d, S, pos = 8, 32, 128, 1100, 1029
    qkv, Kc, Vc = wl.make_attention_inputs(B, H, d, S, seed=3, config_id=511)
    a = sb.attn_decode(_dev(qkv, gpu), _dev(Kc, gpu), _dev(Vc, gpu), pos)
    pd = torch.full((B,), pos, dtype=torch.int32, device=gpu)
    b = sb.attn_decode_ragged(_dev(qkv, gpu), _dev(Kc, gpu), _dev(Vc, gpu), pd, pos)
    torch.cuda.synchronize()
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))


def test_ragged_positions_outside_the_bound_are_forced_into_it(gpu):
    """The host cannot see the device-side positions; the kernel forces an entry outside 0 .. bound to
    the nearer end, so the call stays inside the caches whatever the array holds."""
    import torch
    from paper_2207_00032_amd import binding as sb
    B, H, d, S, bound = 4, 2, 64, 96, 60
    qkv, Kc, Vc = wl.make_attention_inputs(B, H, d, S, seed=4, config_id=512)
    given, effective = [61, -1, 2 ** 31 - 1, 30], [60, 0, 60, 30]
    want = np.empty((B, H * d), dtype=np.float16)
    K2, V2 = Kc.copy(), Vc.copy()
    for b in range(B):
        want[b:b + 1], K2[b:b + 1], V2[b:b + 1] = orc.attn_decode(qkv[b:b + 1], Kc[b:b + 1], Vc[b:b + 1], effective[b])
    Kd, Vd = _dev(Kc, gpu), _dev(Vc, gpu)
    out = sb.attn_decode_ragged(_dev(qkv, gpu), Kd, Vd, torch.tensor(given, dtype=torch.int32, device=gpu), bound)
    torch.cuda.synchronize()
    ok, rep = orc.check_close(out.cpu().numpy(), want, ulps=2, abs_tol=1e-3)
    assert ok, rep
    assert np.array_equal(Kd.cpu().numpy().view(np.uint16), K2.view(np.uint16))
    assert np.array_equal(Vd.cpu().numpy().view(np.uint16), V2.view(np.uint16))
