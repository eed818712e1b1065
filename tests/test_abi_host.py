"""Host-only checks of the C-ABI library: it loads without a GPU, exports every symbol the
header declares, sizes and plans are consistent, and every argument error is reported by the
host-side validation before anything could reach a GPU (so fake device addresses are safe:
only calls that must fail are made here)."""
import ctypes
import os
import re

import pytest

from paper_2207_00032_amd import binding as sb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "sbi_gemm.h")

FAKE = 0x7F0000000000  # a 256-byte aligned non-null "device address"; never dereferenced


@pytest.fixture(scope="module")
def lib():
    return sb.load()


def test_library_exports_every_declared_symbol(lib):
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(sbi_[a-z_0-9]+)\s*\(", text))
    # the measurement helpers have a header of their own next to the sources
    calib = open(os.path.join(ROOT, "paper_2207_00032_amd", "csrc", "sbi_calib.h")).read()
    calib = set(re.findall(r"\b(sbi_calib_[a-z_0-9]+)\s*\(", re.sub(r"/\*.*?\*/", "", calib, flags=re.S)))
    assert calib == {"sbi_calib_read", "sbi_calib_copy"} and not (calib & declared)
    assert declared | calib == set(sb.EXPORTS), (declared | calib) ^ set(sb.EXPORTS)
    for name in declared | calib:
        assert getattr(lib, name) is not None
    assert lib.sbi_version() >= 100


def test_status_strings(lib):
    seen = set()
    for i, name in enumerate(sb.STATUS_NAMES):
        s = sb.status_string(i)
        assert s and s != "unknown status", name
        seen.add(s)
    assert len(seen) == len(sb.STATUS_NAMES)
    assert sb.status_string(99) == "unknown status"


def test_layout_bytes():
    assert sb.layout_bytes(32, 64) == 256 + 8 * 4096            # k-steps padded to a multiple of 8
    assert sb.layout_bytes(1, 1) == 256 + 8 * 4096
    assert sb.layout_bytes(257, 65) == 256 + 2 * 16 * 4096
    assert sb.layout_bytes(4096, 16384) == 256 + 2 * 4096 * 16384
    assert sb.layout_bytes(49152, 12288) == 256 + 2 * 49152 * 12288
    assert sb.layout_bytes(0, 64) == 0 and sb.layout_bytes(64, -1) == 0
    assert sb.layout_bytes(1 << 23, 64) == 0


@pytest.mark.parametrize("B", [1, 2, 4, 8, 16, 17, 32, 33, 48, 64])
@pytest.mark.parametrize("K,N", [(1, 1), (8, 1), (1024, 1024), (4096, 12288), (16384, 4096),
                                 (1536, 12288), (49152, 12288), (8192, 32768), (1000, 130), (1001, 130)])
def test_plan_invariants(B, K, N):
    KS, P = 8 * -(-(-(-K // 32)) // 8), -(-N // 64)
    for path in (sb.PATH_AUTO, sb.PATH_MFMA, sb.PATH_STREAM, sb.PATH_STREAMK):
        if (path == sb.PATH_STREAM and B > 8) or (path == sb.PATH_STREAMK and K % 8):
            with pytest.raises(sb.SbiError) as e:
                sb.plan(B, K, N, path)
            assert e.value.status == 10
            continue
        pl = sb.plan(B, K, N, path)
        assert pl["waves"] in (4, 8) and pl["depth"] in (2, 4, 8)
        assert pl["block"] == 64 * pl["waves"]
        if path == sb.PATH_AUTO:
            assert pl["path"] == sb.PATH_MFMA
            assert sb.workspace_bytes(B, K, N) == pl["workspace_bytes"]
        else:
            assert pl["path"] == path
        if pl["path"] == sb.PATH_STREAMK:
            upw = pl["ksteps_per_split"]
            nwaves = -(-KS * P // upw)
            assert upw % 8 == 0 and upw >= 8 and pl["split_k"] == 0 and pl["lds_bytes"] == 0
            assert pl["grid"] == -(-nwaves // pl["waves"]) and nwaves <= 2048
            assert pl["workspace_bytes"] == 256 * 1024 + nwaves * 2 * B * 64 * 4
            continue
        S, ksps, kc = pl["split_k"], pl["ksteps_per_split"], pl["ksteps_per_chunk"]
        assert 1 <= S <= KS and ksps * S >= KS and ksps * (S - 1) < KS      # covers K, no empty block
        pw = pl["panels"]
        assert pw in (1, 2) and (pw == 1 or B > 16)
        assert pl["grid"] == -(-P // pw) * S
        # k-steps per round: waves x depth, except the two-wave-group shape (8 waves, depth 4, 2 panels)
        rnd = 16 if (pw, pl["waves"], pl["depth"]) == (2, 8, 4) else pl["waves"] * pl["depth"]
        assert kc % rnd == 0 and kc >= rnd
        buffers = 1 if kc >= ksps else 2                         # X is double-buffered when chunked
        assert pl["lds_bytes"] <= (144 if pw == 2 else 72) * 1024 and pl["lds_bytes"] >= buffers * kc * (B | 1) * 64
        if S == 1:
            assert pl["workspace_bytes"] == 0
        else:
            assert pl["workspace_bytes"] >= 256 * 1024 + P * S * B * 64 * 4


def test_plan_tuning_overrides():
    pl = sb.plan(4, 4096, 4096, sb.PATH_MFMA, split_k=8, waves=4, depth=8)
    assert (pl["split_k"], pl["waves"], pl["depth"], pl["path"]) == (8, 4, 8, sb.PATH_MFMA)
    pl = sb.plan(4, 4096, 4096, sb.PATH_STREAM, split_k=1000)
    assert pl["split_k"] == 128                                  # clamped to the number of k-steps
    for bad in (dict(waves=3), dict(depth=5), dict(split_k=-1, path=sb.PATH_MFMA), dict(path=7), dict(blocks=-2)):
        with pytest.raises(sb.SbiError) as e:
            sb.plan(4, 4096, 4096, **bad)
        assert e.value.status == 10
    with pytest.raises(sb.SbiError) as e:                        # X chunks would not fit in LDS
        sb.plan(64, 4096, 4096, sb.PATH_MFMA, waves=8, depth=8)
    assert e.value.status == 10
    for B in (0, 65):
        with pytest.raises(sb.SbiError) as e:
            sb.plan(B, 64, 64)
        assert e.value.status == 4
    with pytest.raises(sb.SbiError) as e:
        sb.plan(1, 0, 64)
    assert e.value.status == 2


def _gemm(lib, W=FAKE, K=4096, N=4096, X=FAKE + (1 << 30), B=4, bias=None, res=None, epi=0,
          Y=FAKE + (2 << 30), ws=FAKE + (3 << 30), ws_bytes=1 << 30):
    return lib.sbi_gemm(W, K, N, X, B, bias, res, epi, Y, ws, ws_bytes, None)


def test_gemm_argument_validation(lib):
    assert _gemm(lib, W=None) == 1 and _gemm(lib, X=None) == 1 and _gemm(lib, Y=None) == 1
    assert _gemm(lib, K=0) == 2 and _gemm(lib, N=-5) == 2 and _gemm(lib, K=(1 << 22) + 1) == 2
    assert _gemm(lib, B=0) == 4 and _gemm(lib, B=65) == 4
    assert _gemm(lib, epi=17) == 7
    assert _gemm(lib, epi=sb.EPI_BIAS) == 7 and _gemm(lib, epi=sb.EPI_BIAS_GELU) == 7
    assert _gemm(lib, epi=sb.EPI_BIAS_RESIDUAL, bias=FAKE + (4 << 30)) == 7
    assert _gemm(lib, epi=sb.EPI_RESIDUAL) == 7
    assert _gemm(lib, W=FAKE + 128) == 3                          # laid-out buffer: 256-byte aligned
    assert _gemm(lib, X=FAKE + (1 << 30) + 8) == 3                # X: 16-byte aligned when K % 8 == 0
    assert _gemm(lib, Y=FAKE + (2 << 30) + 2) == 3                # Y: 4-byte aligned
    assert _gemm(lib, epi=sb.EPI_BIAS, bias=FAKE + (4 << 30) + 1) == 3
    assert _gemm(lib, Y=FAKE + (1 << 30) + 4096) == 9             # Y inside X
    need = sb.workspace_bytes(4, 4096, 4096)
    assert need > 256 * 1024                                      # this shape is split over K
    assert _gemm(lib, ws=None) == 6 and _gemm(lib, ws_bytes=need - 1) == 6
    assert _gemm(lib, ws=FAKE + (3 << 30) + 64, ws_bytes=need) == 3


def test_static_scratch_entry_point_validates_before_touching_the_device(lib):
    """sbi_gemm_static: the same argument checks as sbi_gemm, and a problem whose plan needs more than
    the library's scratch array is refused on the host (no GPU is present here, so any device call
    would come back as SBI_ERR_HIP instead)."""
    X, Y = FAKE + (1 << 30), FAKE + (2 << 30)
    call = lambda W=FAKE, K=4096, N=4096, x=X, B=4, bias=None, res=None, epi=sb.EPI_NONE, y=Y: \
        lib.sbi_gemm_static(W, K, N, x, B, bias, res, epi, y, None)
    assert call(W=None) == 1 and call(x=None) == 1 and call(y=None) == 1
    assert call(K=0) == 2 and call(B=65) == 4 and call(epi=sb.EPI_BIAS) == 7
    assert call(W=FAKE + 128) == 3 and call(y=X + 4096) == 9
    assert sb.workspace_bytes(64, 131072, 12288) > sb.STATIC_SCRATCH_BYTES
    assert call(K=131072, N=12288, B=64, y=FAKE + (2 << 40)) == 6
    text = open(HEADER).read()
    assert re.search(r"#define SBI_STATIC_SCRATCH_BYTES \((\d+)u << 20\)", text).group(1) == str(sb.STATIC_SCRATCH_BYTES >> 20)


def test_kernel_registers_argument_validation(lib):
    """sbi_kernel_registers refuses bad arguments and shapes without a kernel variant before it asks the
    runtime anything."""
    import ctypes
    a, m = ctypes.c_int32(0), ctypes.c_int32(0)
    pa, pm = ctypes.byref(a), ctypes.byref(m)
    assert lib.sbi_kernel_registers(8, 4, 2, 1, 0, None, pm) == 1
    assert lib.sbi_kernel_registers(8, 4, 2, 1, 0, pa, None) == 1
    assert lib.sbi_kernel_registers(0, 4, 2, 1, 0, pa, pm) == 4 and lib.sbi_kernel_registers(65, 4, 2, 1, 0, pa, pm) == 4
    assert lib.sbi_kernel_registers(8, 4, 2, 1, 4, pa, pm) == 10 and lib.sbi_kernel_registers(8, 4, 2, 1, -1, pa, pm) == 10
    # no such variants: 16 waves; a layer-norm kernel of two panels; 8 waves x depth 2 with the layer-norm; INT8 depth 8
    for B, w, d, pw, fl in ((8, 16, 4, 1, 0), (40, 8, 2, 2, 1), (8, 8, 2, 1, 1), (8, 4, 8, 1, 2), (8, 8, 4, 2, 0)):
        assert lib.sbi_kernel_registers(B, w, d, pw, fl, pa, pm) == 10, (B, w, d, pw, fl)


def test_int8_layernorm_argument_validation_and_plans(lib):
    """sbi_gemm_i8_ln: the layer-norm's and the INT8 call's checks both apply; its plans always run
    from codes in the workspace (a kernel of its own normalises and quantises the rows)."""
    sw = FAKE + (5 << 30)
    g, b = FAKE + (6 << 30), FAKE + (7 << 30)

    def call(**kw):
        ln = sb.LayerNorm(kw.get("gamma", g), kw.get("beta", b), kw.get("eps", 1e-5), kw.get("moments", None))
        return lib.sbi_gemm_i8_ln(kw.get("W", FAKE), kw.get("sw", sw), kw.get("K", 4096), 4096, FAKE + (1 << 30),
                                  kw.get("B", 4), None if kw.get("no_ln") else ctypes.byref(ln), None, None, 0,
                                  FAKE + (2 << 30), FAKE + (3 << 30), kw.get("wb", 1 << 30), None, None)
    assert call(no_ln=True) == 1 and call(gamma=None) == 1 and call(sw=None) == 1
    assert call(gamma=g + 8) == 3 and call(eps=-1.0) == 7
    assert call(K=4104) == 2 and call(B=0) == 4
    assert call(moments=FAKE + (8 << 30)) == 10                   # the fp64 statistics read the rows
    for B in (1, 8, 16, 40, 64):
        for K, N in ((4096, 12288), (16384, 4096), (1008, 130)):
            pl = sb.plan(B, K, N, int8=True, layernorm=True)
            plain = sb.plan(B, K, N, int8=True)
            assert pl["path"] == sb.PATH_MFMA
            assert pl["workspace_bytes"] >= 256 * 1024 + B * K      # counters, codes, row scales
            if B > 8:
                assert pl == plain                                  # above 8 rows the INT8 call runs from codes anyway
    need = sb.plan(4, 4096, 4096, int8=True, layernorm=True)["workspace_bytes"]
    assert call(wb=need - 1) == 6
    # an INT8 layer may carry layer-norms now
    L = sb.Layer()
    L.Wqkv = L.Wout = L.Wffn1 = L.Wffn2 = FAKE
    L.h, L.n_qkv, L.k_out, L.n_ffn1, L.k_ffn2 = 256, 768, 256, 1024, 1024
    L.sqkv = L.sout = L.sffn1 = L.sffn2 = sw
    L.ln1_gamma, L.ln1_beta, L.ln2_gamma, L.ln2_beta, L.ln_eps = g, b, g, b, 1e-5
    assert lib.sbi_layer_workspace_bytes(ctypes.byref(L), 4) >= 256 * 1024 + 4 * (256 + 256 + 256 + 1024)
    L.ln1_beta = None
    assert lib.sbi_layer_workspace_bytes(ctypes.byref(L), 4) == 0   # gamma without beta


def test_tuner_argument_validation(lib):
    """sbi_layer_tune / sbi_gemm_tune refuse bad arguments on the host (nothing is launched or timed)."""
    L = sb.Layer()
    L.Wqkv = L.Wout = L.Wffn1 = L.Wffn2 = FAKE
    L.h, L.n_qkv, L.k_out, L.n_ffn1, L.k_ffn2 = 256, 768, 256, 1024, 1024
    X, Y = FAKE + (1 << 30), FAKE + (2 << 30)
    tune = lambda arr, n, B=2: lib.sbi_layer_tune(arr, n, B, X, X, X, X, None, Y, Y + (1 << 20), Y + (2 << 20), Y + (3 << 20),
                                                  FAKE + (3 << 30), 1 << 26, None, None)
    one = (sb.Layer * 1)(L)
    assert tune(None, 1) == 1 and tune(one, 0) == 1
    assert tune(one, 1, B=0) == 4 and tune(one, 1, B=65) == 4
    L2 = sb.Layer()
    ctypes.memmove(ctypes.byref(L2), ctypes.byref(L), ctypes.sizeof(L))
    L2.n_ffn1 = L2.k_ffn2 = 2048
    assert tune((sb.Layer * 2)(L, L2), 2) == 2                      # two shapes in one call
    bad = sb.Layer()
    ctypes.memmove(ctypes.byref(bad), ctypes.byref(L), ctypes.sizeof(L))
    bad.Wout = None
    assert tune((sb.Layer * 1)(bad), 1) == 1
    ptrs = (ctypes.c_void_p * 2)(FAKE, FAKE + 128)
    gt = lambda p, n, K=256, B=2: lib.sbi_gemm_tune(p, n, K, 256, X, B, None, None, sb.EPI_NONE, Y, FAKE + (3 << 30),
                                                    1 << 26, None, None)
    assert gt(None, 1) == 1 and gt(ptrs, 0) == 1
    assert gt(ptrs, 2) == 3                                         # second weight set not 256-byte aligned
    assert gt((ctypes.c_void_p * 1)(None), 1) == 1
    assert gt(ptrs, 1, K=0) == 2 and gt(ptrs, 1, B=99) == 4


def test_layout_argument_validation(lib):
    nb = sb.layout_bytes(64, 64)
    assert lib.sbi_gemm_layout_weights(None, 64, 64, FAKE, nb, None) == 1
    assert lib.sbi_gemm_layout_weights(FAKE, 64, 64, None, nb, None) == 1
    assert lib.sbi_gemm_layout_weights(FAKE, 0, 64, FAKE + 4096, nb, None) == 2
    assert lib.sbi_gemm_layout_weights(FAKE + 1, 64, 64, FAKE + 4096, nb, None) == 3
    assert lib.sbi_gemm_layout_weights(FAKE, 64, 64, FAKE + 4096 + 16, nb, None) == 3
    assert lib.sbi_gemm_layout_weights(FAKE, 64, 64, FAKE + 4096, nb - 1, None) == 5
    assert lib.sbi_gemm_unlayout_weights(None, 64, 64, FAKE, None) == 1
    assert lib.sbi_gemm_unlayout_weights(FAKE, 64, 0, FAKE + 4096, None) == 2
    assert lib.sbi_gemm_layout_check(None, 64, 64, None) == 1
    assert lib.sbi_gemm_layout_check(FAKE + 8, 64, 64, None) == 3


def test_layer_argument_validation(lib):
    L = sb.Layer()
    L.Wqkv = L.Wout = L.Wffn1 = L.Wffn2 = FAKE
    L.h, L.n_qkv, L.k_out, L.n_ffn1, L.k_ffn2 = 1024, 3072, 1024, 4096, 4096
    ws = sb.layer_workspace_bytes(L, 1)
    assert ws >= max(sb.workspace_bytes(1, 1024, 3072), sb.workspace_bytes(1, 1024, 1024),
                     sb.workspace_bytes(1, 1024, 4096), sb.workspace_bytes(1, 4096, 1024)) > 0
    args = [FAKE + (i << 28) for i in range(1, 10)]
    call = lambda layer, B, a, w=FAKE, wb=1 << 30: lib.sbi_layer_gemms(layer, B, *a, w, wb, None)
    assert call(None, 1, args) == 1
    assert call(ctypes.byref(L), 0, args) == 4
    a = list(args); a[0] = None
    assert call(ctypes.byref(L), 1, a) == 1
    # a call needs what its own launches need (the four-GeMM launch here), never more than `ws`
    plans, _ = sb.layer_plan(L, 1, chained=False)
    assert any(p["split_k"] > 1 for p in plans)
    need = 256 * 1024 + sum(p["workspace_bytes"] for p in plans)
    assert 0 < need <= ws
    assert call(ctypes.byref(L), 1, args, wb=need - 1) == 6
    L2 = sb.Layer.from_buffer_copy(L)
    L2.k_ffn2 = 2048                                              # chaining needs n_ffn1 == k_ffn2
    a = list(args); a[3] = None
    assert call(ctypes.byref(L2), 1, a) == 2
    L3 = sb.Layer.from_buffer_copy(L)
    L3.Wout = None
    assert call(ctypes.byref(L3), 1, args) == 1
    L4 = sb.Layer.from_buffer_copy(L)
    L4.h = 0
    assert call(ctypes.byref(L4), 1, args) == 2


def _gemm_ln(lib, gamma=FAKE + (5 << 30), beta=FAKE + (6 << 30), eps=1e-5, K=4096, N=4096, B=4, ln=True,
             tune=None, ws_bytes=1 << 30, moments=None):
    lnp = ctypes.byref(sb.LayerNorm(gamma, beta, eps, moments)) if ln else None
    return lib.sbi_gemm_ln(FAKE, K, N, FAKE + (1 << 30), B, lnp, None, None, 0, FAKE + (2 << 30),
                           FAKE + (3 << 30), ws_bytes, None, tune)


def test_layernorm_argument_validation(lib):
    assert _gemm_ln(lib, ln=False) == 1
    assert _gemm_ln(lib, gamma=None) == 1 and _gemm_ln(lib, beta=None) == 1
    assert _gemm_ln(lib, gamma=FAKE + 8) == 3 and _gemm_ln(lib, beta=FAKE + 2) == 3
    assert _gemm_ln(lib, K=4100) == 2                              # rows must split into 128-bit pieces
    assert _gemm_ln(lib, eps=-1.0) == 7 and _gemm_ln(lib, eps=float("nan")) == 7
    assert _gemm_ln(lib, eps=float("inf")) == 7
    for bad in (sb.Tuning(sb.PATH_STREAM, 0, 0, 0, 0, 0, 0), sb.Tuning(sb.PATH_STREAMK, 0, 0, 0, 0, 0, 0),
                sb.Tuning(sb.PATH_MFMA, 0, 0, 0, 0, 2, 0), sb.Tuning(sb.PATH_MFMA, 0, 4, 8, 0, 0, 0),
                sb.Tuning(sb.PATH_MFMA, 0, 8, 8, 0, 0, 0)):
        assert _gemm_ln(lib, tune=ctypes.byref(bad)) == 10
    need = sb.ln_workspace_bytes(4, 4096, 4096)
    assert need == sb.plan(4, 4096, 4096, layernorm=True)["workspace_bytes"] > 0
    assert _gemm_ln(lib, ws_bytes=need - 1) == 6
    # the plain entry point has no layer-norm parameters and refuses the request
    t = sb.Tuning(0, 0, 0, 0, 0, 0, 1)
    assert lib.sbi_gemm_ex(FAKE, 4096, 4096, FAKE + (1 << 30), 4, None, None, 0, FAKE + (2 << 30),
                           FAKE + (3 << 30), 1 << 30, None, ctypes.byref(t)) == 10


@pytest.mark.parametrize("B", [1, 4, 8, 16, 33, 64])
@pytest.mark.parametrize("K,N", [(8, 1), (1024, 3072), (4096, 12288), (4096, 16384), (12288, 4608), (1000, 130)])
def test_layernorm_plan_invariants(B, K, N):
    KS, P = 8 * -(-(-(-K // 32)) // 8), -(-N // 64)
    pl = sb.plan(B, K, N, layernorm=True)
    if B > 8:
        # above 8 rows (4 on launches of gigabytes) the rows are normalised once by a kernel of their own, into the workspace,
        # and the launch is the plain one
        plain = sb.plan(B, K, N, sb.PATH_MFMA)
        same = ("path", "waves", "depth", "panels", "split_k", "ksteps_per_split", "ksteps_per_chunk", "grid", "lds_bytes")
        assert all(pl[k] == plain[k] for k in same)
        rows = -(-B * K * 2 // 256) * 256
        assert pl["workspace_bytes"] == max(plain["workspace_bytes"], 256 * 1024) + rows
    else:
        assert pl["path"] == sb.PATH_MFMA and pl["panels"] == 1
        assert (pl["waves"], pl["depth"]) in ((4, 2), (4, 4), (8, 4))
        S, ksps, kc = pl["split_k"], pl["ksteps_per_split"], pl["ksteps_per_chunk"]
        assert 1 <= S <= KS and ksps * S >= KS and ksps * (S - 1) < KS and pl["grid"] == P * S
        buffers = 1 if kc >= ksps else 2
        # statistics ahead of the X buffers; each buffer also holds its k-steps of gamma and beta
        assert 512 + buffers * kc * ((B | 1) + 2) * 64 <= pl["lds_bytes"] <= 144 * 1024
    with pytest.raises(sb.SbiError) as e:
        sb.plan(B, K + 4, N, layernorm=True)
    assert e.value.status == 10


def test_layer_layernorm_validation(lib):
    L = sb.Layer()
    L.Wqkv = L.Wout = L.Wffn1 = L.Wffn2 = FAKE
    L.h, L.n_qkv, L.k_out, L.n_ffn1, L.k_ffn2 = 1024, 3072, 1024, 4096, 4096
    L.ln_eps = 1e-5
    args = [FAKE + (i << 28) for i in range(1, 10)]
    call = lambda layer: lib.sbi_layer_gemms(ctypes.byref(layer), 2, *args, FAKE, 1 << 30, None)
    L.ln1_gamma = FAKE + (11 << 28)
    assert call(L) == 1                                            # gamma without beta
    L.ln1_beta = FAKE + (12 << 28) + 4
    assert call(L) == 3
    L.ln1_beta = FAKE + (12 << 28)
    L.ln_eps = -1.0
    assert call(L) == 7
    L.ln_eps = 1e-5
    L.ln2_beta = FAKE + (13 << 28)
    assert call(L) == 1
    L.ln2_beta = None
    plans, grid = sb.layer_plan(L, 2, chained=True)
    assert all(p["panels"] == 1 and p["lds_bytes"] >= 512 for p in plans)
    L.h = 1028; L.k_out = 1028                                     # h % 8 != 0 cannot be layer-normalised
    assert call(L) == 2


def test_binding_fails_loudly_without_library(monkeypatch, tmp_path):
    monkeypatch.setattr(sb, "_lib", None)
    monkeypatch.setattr(sb, "LIB_PATH", str(tmp_path / "libsbi_gemm.so"))
    with pytest.raises(ImportError):
        sb.load()


def test_int8_argument_validation_and_plans(lib):
    sw = FAKE + (7 << 30)
    call = lambda **kw: lib.sbi_gemm_i8(kw.get("W", FAKE), kw.get("sw", sw), kw.get("K", 4096), kw.get("N", 4096),
                                        kw.get("X", FAKE + (1 << 30)), kw.get("B", 4), None, None, 0,
                                        FAKE + (2 << 30), FAKE + (3 << 30), kw.get("wb", 1 << 30), None,
                                        kw.get("tune"))
    assert call(sw=None) == 1 and call(W=None) == 1
    assert call(K=4104) == 2                                      # rows must split into 32-byte pieces
    assert call(sw=sw + 2) == 3
    assert call(B=65) == 4
    for bad in (sb.Tuning(sb.PATH_STREAM, 0, 0, 0, 0, 0, 0, 0), sb.Tuning(sb.PATH_MFMA, 0, 0, 0, 0, 2, 0, 0),
                sb.Tuning(sb.PATH_MFMA, 0, 8, 8, 0, 0, 0, 0), sb.Tuning(sb.PATH_MFMA, 0, 0, 0, 0, 0, 1, 0)):
        assert call(tune=ctypes.byref(bad)) == 10
    need = sb.i8_workspace_bytes(4, 4096, 4096)
    assert need == sb.plan(4, 4096, 4096, int8=True)["workspace_bytes"] > 0
    assert call(wb=need - 1) == 6
    t = sb.Tuning(0, 0, 0, 0, 0, 0, 0, 1)
    assert lib.sbi_gemm_ex(FAKE, 4096, 4096, FAKE + (1 << 30), 4, None, None, 0, FAKE + (2 << 30),
                           FAKE + (3 << 30), 1 << 30, None, ctypes.byref(t)) == 10
    # weight preparation
    assert sb.i8_layout_bytes(4096, 4096) == 256 + 64 * 64 * 4096 and sb.i8_layout_bytes(0, 4) == 0
    assert sb.i8_layout_bytes(100, 65) == 256 + 8 * 2 * 4096
    assert lib.sbi_gemm_i8_layout_weights(None, 64, 64, FAKE, 1 << 20, None) == 1
    assert lib.sbi_gemm_i8_layout_weights(FAKE, 64, 64, FAKE + 4096 + 8, 1 << 20, None) == 3
    assert lib.sbi_gemm_i8_layout_weights(FAKE, 64, 64, FAKE + 4096, sb.i8_layout_bytes(64, 64) - 1, None) == 5
    assert lib.sbi_gemm_i8_quantize_weights(FAKE, 64, 64, None, FAKE, None) == 1
    assert lib.sbi_gemm_i8_quantize_weights(FAKE + 1, 64, 64, FAKE, FAKE, None) == 3
    assert lib.sbi_gemm_i8_layout_check(None, 64, 64, None) == 1
    for B in (1, 8, 16, 33, 64):
        for K, N in ((16, 1), (4096, 12288), (16384, 4096), (1008, 130)):
            KS, P = 8 * -(-(-(-K // 64)) // 8), -(-N // 64)
            pl = sb.plan(B, K, N, int8=True)
            pw = pl["panels"]
            assert pl["path"] == sb.PATH_MFMA and pw in (1, 2) and (pw == 1 or B > 16)
            assert (pl["waves"], pl["depth"]) in (((4, 2), (4, 4), (8, 4)) if pw == 1 else ((8, 2), (8, 4)))
            S, ksps, kc = pl["split_k"], pl["ksteps_per_split"], pl["ksteps_per_chunk"]
            assert 1 <= S <= KS and ksps * S >= KS and ksps * (S - 1) < KS and pl["grid"] == -(-P // pw) * S
            buffers = 1 if kc >= ksps else 2
            assert 512 + max(buffers * kc * (B | 1) * 64, pl["waves"] * 16 * 68 * 4) <= pl["lds_bytes"] <= 144 * 1024


def test_moments_argument_validation(lib):
    mom = FAKE + (8 << 30)
    assert _gemm_ln(lib, moments=mom, ws_bytes=0) == 6             # (no launch without a workspace)
    assert _gemm_ln(lib, moments=mom + 4, ws_bytes=0) == 3         # float2 entries: 8-byte aligned
    assert _gemm_ln(lib, moments=mom, K=4128, ws_bytes=0) == 2     # moments come in 64-feature panels
    call = lambda out=mom, tune=None, ws_bytes=0: lib.sbi_gemm_moments(
        FAKE, 4096, 4096, FAKE + (1 << 30), 4, None, None, None, 0, FAKE + (2 << 30), out, FAKE + (3 << 30),
        ws_bytes, None, tune)
    assert call(out=None) == 1 and call(out=mom + 2) == 3 and call() == 6
    for bad in (sb.Tuning(sb.PATH_STREAM, 0, 0, 0, 0, 0, 0, 0), sb.Tuning(sb.PATH_STREAMK, 0, 0, 0, 0, 0, 0, 0),
                sb.Tuning(0, 0, 0, 0, 0, 0, 0, 1)):
        assert call(tune=ctypes.byref(bad), ws_bytes=1 << 30) == 10


def test_attention_argument_validation(lib):
    q, k, v, o, w = (FAKE + (i << 30) for i in range(1, 6))
    call = lambda **kw: lib.sbi_attn_decode(kw.get("q", q), kw.get("k", k), kw.get("v", v), kw.get("B", 2), kw.get("H", 4),
                                            kw.get("d", 128), kw.get("S", 4096), kw.get("pos", 4000),
                                            ctypes.c_float(kw.get("scale", 0.0)), kw.get("o", o), kw.get("w", w),
                                            kw.get("wb", 0), None)
    assert call(q=None) == 1 and call(k=None) == 1 and call(v=None) == 1 and call(o=None) == 1
    assert call(B=0) == 4 and call(B=65) == 4
    assert call(H=0) == 2 and call(d=96) == 2 and call(S=0) == 2 and call(pos=-1) == 2 and call(pos=4096) == 2
    assert call(scale=-1.0) == 7 and call(scale=float("nan")) == 7
    assert call(q=q + 8) == 3 and call(k=k + 2) == 3 and call(o=o + 1) == 3
    need = sb.attn_workspace_bytes(2, 4, 128, 4096)
    assert need == 256 * 1024 + 2 * 4 * 16 * 130 * 4            # 16 position ranges of 256 per (sequence, head)
    full = dict(pos=4095)                                        # the requirement follows the filled length
    assert call(wb=need - 1, **full) == 6 and call(w=None, wb=need, **full) == 6 and call(w=w + 64, wb=need, **full) == 3
    assert sb.attn_workspace_bytes(8, 32, 128, 136) == 0         # short caches: one block per (sequence, head)
    assert sb.attn_workspace_bytes(2, 4, 100, 64) == 0 and sb.attn_workspace_bytes(0, 4, 128, 64) == 0


def test_ragged_attention_argument_validation(lib):
    q, k, v, o, w, pp = (FAKE + (i << 30) for i in range(1, 7))
    call = lambda **kw: lib.sbi_attn_decode_ragged(kw.get("q", q), kw.get("k", k), kw.get("v", v), kw.get("B", 2),
                                                   kw.get("H", 4), kw.get("d", 128), kw.get("S", 4096), kw.get("p", pp),
                                                   kw.get("bound", 4095), ctypes.c_float(kw.get("scale", 0.0)),
                                                   kw.get("o", o), kw.get("w", w), kw.get("wb", 0), None)
    assert call() == 6                                           # every call here stops at a check: no launch
    assert call(p=None) == 1 and call(p=pp + 2) == 3 and call(q=None) == 1 and call(o=None) == 1
    assert call(bound=-1) == 2 and call(bound=4096) == 2 and call(B=65) == 4 and call(d=96) == 2
    assert call(scale=-1.0) == 7 and call(k=k + 2) == 3
    need = sb.attn_workspace_bytes(2, 4, 128, 4096)
    assert call(wb=need - 1) == 6 and call(w=None, wb=need) == 6 and call(w=w + 64, wb=need) == 3
