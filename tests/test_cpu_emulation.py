"""The library's host code and MFMA kernels compiled for the CPU under AddressSanitizer
(tests/cpu_emulation/): every global and LDS access of every thread of every block is checked
against buffers of exactly the documented size, and the results against an fp64 reference
written out in the drivers.  No GPU, no oracle involved: this guards addressing (the kind of
mistake that is a memory fault on the GPU), not numerics.

The build takes about two minutes, so the test only runs on request:
    SBI_RUN_EMULATION=1 python -m pytest tests/test_cpu_emulation.py -q
"""
import os
import subprocess

import pytest

pytestmark = pytest.mark.skipif(os.environ.get("SBI_RUN_EMULATION") != "1",
                                reason="set SBI_RUN_EMULATION=1 (two-minute sanitizer build)")


@pytest.fixture(scope="module")
def drivers(tmp_path_factory):
    import importlib.util
    here = os.path.dirname(os.path.abspath(__file__))
    spec = importlib.util.spec_from_file_location("emu_build", os.path.join(here, "cpu_emulation", "build.py"))
    build = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(build)
    out = tmp_path_factory.mktemp("emu")
    return build.build(str(out))


def run(cmd):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0")
    env.pop("EMU_BLOCKS", None)
    r = subprocess.run(cmd, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600)
    assert r.returncode == 0 and "AddressSanitizer" not in r.stdout, r.stdout[-3000:]


# B K N waves depth split panels mode (0 plain, 1 layer-norm, 2 int8, 3 moments out, 4 layer-norm from moments,
# 5 layer-norm in front of int8)
# (waves 0 = automatic plan)
GEMM_CASES = [
    (1, 64, 64, 0, 0, 0, 0, 0), (3, 264, 200, 0, 0, 0, 0, 0), (5, 1001, 130, 4, 4, 2, 1, 0),
    (8, 2048, 128, 8, 4, 1, 1, 0), (17, 1024, 136, 4, 2, 3, 1, 0), (33, 520, 192, 4, 4, 1, 2, 0),
    (64, 512, 128, 8, 2, 2, 2, 0), (1, 12288, 128, 4, 4, 1, 1, 0),
    (64, 2048, 192, 8, 2, 1, 2, 0), (48, 1100, 128, 8, 2, 1, 2, 0), (40, 1544, 136, 8, 2, 2, 2, 0), (33, 3072, 128, 8, 2, 1, 2, 0),
    # two wave groups, one panel each (waves 8, depth 4, panels 2)
    (64, 2048, 192, 8, 4, 1, 2, 0), (48, 1100, 128, 8, 4, 1, 2, 0), (40, 1544, 136, 8, 4, 2, 2, 0), (33, 3072, 128, 8, 4, 1, 2, 0), (17, 520, 72, 8, 4, 3, 2, 0),
    (64, 2048, 128, 8, 4, 2, 2, 2), (40, 4096, 136, 8, 4, 1, 2, 2), (24, 1040, 72, 8, 4, 1, 2, 2),
    # several rounds with the X staging passes spread over the steps of a round (batches above 16)
    (40, 4096, 72, 4, 2, 1, 1, 0), (40, 4096, 72, 4, 4, 1, 1, 1), (40, 4096, 72, 4, 4, 1, 1, 2),
    (40, 4096, 136, 8, 2, 1, 2, 2), (64, 2048, 128, 8, 2, 2, 2, 2), (24, 1040, 72, 8, 2, 1, 2, 2),
    (24, 4096, 72, 4, 4, 1, 1, 0), (24, 4096, 72, 8, 4, 1, 1, 1), (24, 4100, 72, 4, 4, 1, 1, 0), (24, 4096, 72, 8, 4, 1, 1, 2), (64, 8192, 64, 4, 4, 1, 1, 2),
    (1, 64, 64, 0, 0, 0, 0, 1), (3, 264, 200, 0, 0, 0, 0, 1), (8, 2048, 128, 8, 4, 1, 1, 1),
    (17, 1024, 136, 4, 2, 3, 1, 1), (40, 1024, 72, 4, 4, 2, 1, 1), (64, 512, 128, 4, 2, 2, 1, 1),
    (2, 6144, 64, 4, 4, 1, 1, 1),
    # above 16 rows the automatic plan normalises the rows with a kernel of its own first
    (33, 1024, 200, 0, 0, 0, 0, 1), (64, 520, 72, 0, 0, 0, 0, 1), (40, 1024, 72, 0, 0, 0, 0, 4),
    (1, 64, 64, 0, 0, 0, 0, 2), (3, 272, 200, 0, 0, 0, 0, 2), (8, 2048, 128, 8, 4, 1, 1, 2),
    (17, 1024, 136, 4, 2, 3, 1, 2), (40, 1024, 72, 4, 4, 2, 1, 2), (64, 512, 128, 4, 2, 2, 1, 2),
    (5, 4096, 64, 4, 4, 1, 1, 2), (2, 8192, 64, 0, 0, 0, 0, 2), (17, 1024, 136, 4, 2, 3, 1, 2), (33, 4096, 64, 0, 0, 0, 0, 2),
    (3, 264, 200, 0, 0, 0, 0, 3), (17, 1024, 136, 4, 2, 3, 1, 3), (64, 512, 128, 4, 2, 1, 1, 3), (5, 512, 72, 4, 4, 1, 1, 3),
    (3, 320, 200, 0, 0, 0, 0, 4), (40, 1024, 72, 4, 4, 2, 1, 4), (2, 6144, 64, 4, 4, 1, 1, 4),
    # 8 waves, depth 2, one panel
    (8, 2048, 128, 8, 2, 1, 1, 0), (1, 4096, 64, 8, 2, 2, 1, 0),
    (1, 64, 64, 0, 0, 0, 0, 5), (3, 272, 200, 0, 0, 0, 0, 5), (8, 2048, 128, 8, 4, 1, 1, 5), (17, 1024, 136, 4, 2, 3, 1, 5),
    (40, 1024, 72, 0, 0, 0, 0, 5), (64, 2048, 128, 8, 4, 2, 2, 5),
]


@pytest.mark.parametrize("case", GEMM_CASES)
def test_single_gemm_under_asan(drivers, case):
    run([drivers[0], *[str(v) for v in case]])


@pytest.mark.parametrize("B,h,ln", [(2, 256, 0), (5, 512, 1), (33, 256, 1), (9, 1024, 1)])
def test_layer_launch_under_asan(drivers, B, h, ln):
    run([drivers[1], str(B), str(h), str(ln), "1"])


# B heads head_dim max_seq pos
@pytest.mark.parametrize("case", [(1, 1, 64, 4, 0), (2, 3, 128, 40, 17), (1, 2, 64, 300, 299), (3, 2, 128, 130, 64),
                                  (1, 1, 128, 1100, 1030), (2, 1, 64, 600, 520), (1, 1, 128, 2600, 2570), (1, 2, 64, 1600, 1590)])
def test_attention_decode_under_asan(drivers, case):
    run([drivers[2], *[str(v) for v in case]])


# the same with one position per sequence (sbi_attn_decode_ragged); `pos` is the bound
@pytest.mark.parametrize("case", [(5, 2, 64, 40, 17), (6, 1, 128, 1100, 1030), (7, 2, 64, 1600, 1590), (2, 1, 128, 300, 299),
                                  (1, 1, 64, 4, 0)])
def test_ragged_attention_decode_under_asan(drivers, case):
    run([drivers[2], *[str(v) for v in case], "1"])
