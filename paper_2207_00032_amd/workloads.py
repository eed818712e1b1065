"""Seeded synthetic inputs for the small-batch GeMM workloads (numpy only).

This module holds NO arithmetic of the method: it only names the GeMM shapes of the
benchmark configurations and draws their fp16 inputs.  Both the CPU oracle's tests and
the GPU path's tests / benchmark feed on these same host arrays.

The shapes stand in for the dense GPT-style models the paper evaluates (Table I:
hidden sizes 4096, 8192 and 12288, the last with tensor-parallel degree 8); value
distributions follow the GPT initialisation convention (weights and biases
N(0, sigma=0.02), activations and residuals N(0, 1)), drawn in fp64 and rounded to fp16.
"""
from dataclasses import dataclass
from typing import Dict, List, Optional, Tuple

import numpy as np

# epilogue names used by the workload tables (strings, mapped by each consumer)
NONE, BIAS, BIAS_GELU, BIAS_RESIDUAL, GELU, RESIDUAL = (
    "none", "bias", "bias_gelu", "bias_residual", "gelu", "residual")


@dataclass(frozen=True)
class GemmSpec:
    name: str
    K: int
    N: int
    epilogue: str

    @property
    def weight_bytes(self) -> int:
        return 2 * self.K * self.N

    def algorithmic_bytes(self, B: int, int8: bool = False) -> int:
        """HBM bytes one GeMM must move: W once, X, Y, plus bias / residual if used.  INT8: one byte
        per weight plus a binary32 scale per column; the activations stay fp16 at the boundary."""
        n = (self.K * self.N + 4 * self.N if int8 else 2 * self.K * self.N) + 2 * B * self.K + 2 * B * self.N
        if self.epilogue in (BIAS, BIAS_GELU, BIAS_RESIDUAL):
            n += 2 * self.N
        if self.epilogue in (BIAS_RESIDUAL, RESIDUAL):
            n += 2 * B * self.N
        return n

    def flops(self, B: int) -> int:
        return 2 * B * self.K * self.N


@dataclass(frozen=True)
class Config:
    config_id: int
    name: str
    gemms: Tuple[GemmSpec, ...]
    batches: Tuple[int, ...]
    seeds: Tuple[int, ...]
    outlier_channels: float = 0.0   # fraction of input channels of X scaled by outlier_scale
    outlier_scale: float = 1.0


def _layer(h: int, n_qkv: int, k_out: int, n_ffn1: int, k_ffn2: int,
           epis=(NONE, NONE, BIAS_GELU, BIAS_RESIDUAL)) -> Tuple[GemmSpec, ...]:
    return (GemmSpec("qkv", h, n_qkv, epis[0]),
            GemmSpec("attn_out", k_out, h, epis[1]),
            GemmSpec("ffn1", h, n_ffn1, epis[2]),
            GemmSpec("ffn2", k_ffn2, h, epis[3]))


CONFIGS: Dict[int, Config] = {
    # one GPT-style layer at h=1024, batch 1
    1: Config(1, "h1024_layer", _layer(1024, 3072, 1024, 4096, 4096), (1,), (0,)),
    # the same layer at h=4096 (GPT-J-6B-like), batch sweep, four seeds
    2: Config(2, "h4096_layer", _layer(4096, 12288, 4096, 16384, 16384), (1, 2, 4, 8), (0, 1, 2, 3)),
    # one GPU's 1/8 tensor-parallel share of an h=12288 layer; the row-parallel GeMMs
    # (attn_out, ffn2) get no epilogue: bias/residual follow the all-reduce that is left out
    3: Config(3, "h12288_tp8_slice", _layer(12288, 4608, 1536, 6144, 6144,
                                            (NONE, NONE, BIAS_GELU, NONE)), (1, 4, 16), (0,)),
    # the full h=12288 layer on one GPU (3.6 GB of weights)
    4: Config(4, "h12288_layer", _layer(12288, 36864, 12288, 49152, 49152,
                                        (NONE, NONE, GELU, NONE)), (1, 8), (0,)),
    # batch crossover sweep on an h=8192 FFN1 with outlier input channels
    5: Config(5, "h8192_ffn1_crossover", (GemmSpec("ffn1", 8192, 32768, BIAS_GELU),),
              (1, 2, 4, 8, 16, 32, 48, 64), (0,), outlier_channels=0.01, outlier_scale=50.0),
}

_CHUNK = 1 << 24  # elements drawn per call; sequential calls continue the same stream


def _normal_fp16(rng: np.random.Generator, shape, sigma: float) -> np.ndarray:
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.float16)
    for s in range(0, n, _CHUNK):
        e = min(n, s + _CHUNK)
        out[s:e] = (rng.standard_normal(e - s) * sigma).astype(np.float16)
    return out.reshape(shape)


def make_gemm_inputs(K: int, N: int, B: int, seed: int = 0, config_id: int = 0, gemm_id: int = 0,
                     outlier_channels: float = 0.0, outlier_scale: float = 1.0,
                     want_bias: bool = True, want_residual: bool = True, outlier_rows: float = 0.0):
    """Draw (W[K,N], bias[N], X[B,K], R[B,N]) as fp16, always in that order.

    Weights/bias sigma = 0.02, activations/residual sigma = 1.  When outlier_channels > 0,
    ceil(outlier_channels*K) input channels (columns of X) picked by the same generator are
    multiplied by outlier_scale before the fp16 rounding.  outlier_rows > 0 is the other reading
    of "1 % of rows": ceil(outlier_rows*B) batch rows of X, picked after the channels, are scaled.
    """
    rng = np.random.default_rng(np.random.SeedSequence([seed, config_id, gemm_id]))
    W = _normal_fp16(rng, (K, N), 0.02)
    bias = _normal_fp16(rng, (N,), 0.02)
    Xf = rng.standard_normal((B, K))
    if outlier_channels > 0.0:
        n_out = int(np.ceil(outlier_channels * K))
        ch = rng.choice(K, size=n_out, replace=False)
        Xf[:, ch] *= outlier_scale
    if outlier_rows > 0.0:
        rows = rng.choice(B, size=int(np.ceil(outlier_rows * B)), replace=False)
        Xf[rows, :] *= outlier_scale
    X = Xf.astype(np.float16)
    R = _normal_fp16(rng, (B, N), 1.0)
    assert np.isfinite(W.astype(np.float32)).all() and np.isfinite(X.astype(np.float32)).all()
    return W, (bias if want_bias else None), X, (R if want_residual else None)


def make_layernorm_inputs(K: int, B: int, seed: int = 0, config_id: int = 0, gemm_id: int = 0,
                          row_shift: float = 0.5, row_scale: float = 2.0):
    """Draw (gamma[K], beta[K], X[B,K]) as fp16 for a layer-norm in front of a GeMM.

    gamma ~ 1 + 0.1 N(0,1), beta ~ 0.1 N(0,1) (trained layer-norm parameters stay close to their
    initial 1 and 0).  X is the residual stream entering the norm: row b is
    N(m_b, s_b^2) with m_b ~ row_shift * N(0,1) and s_b log-uniform in [1/row_scale, row_scale],
    so rows differ in mean and spread.  Own generator stream (a fourth seed word), so the
    draws of make_gemm_inputs for the same (seed, config, gemm) are unchanged.
    """
    rng = np.random.default_rng(np.random.SeedSequence([seed, config_id, gemm_id, 1]))
    gamma = (1.0 + 0.1 * rng.standard_normal(K)).astype(np.float16)
    beta = (0.1 * rng.standard_normal(K)).astype(np.float16)
    m = row_shift * rng.standard_normal((B, 1))
    sc = np.exp(rng.uniform(-np.log(row_scale), np.log(row_scale), size=(B, 1)))
    X = (m + sc * rng.standard_normal((B, K))).astype(np.float16)
    return gamma, beta, X


def make_attention_inputs(B: int, heads: int, head_dim: int, max_seq: int, seed: int = 0, config_id: int = 0,
                          key_scale: float = 1.0):
    """Draw (qkv[B,3,H,d], K_cache[B,H,S,d], V_cache[B,H,S,d]) as fp16 for single-token attention:
    N(0,1) queries, keys and values (the scale layer-normed activations give the QKV projection's
    outputs); key_scale > 1 widens the score distribution, i.e. makes the softmax more peaked.
    The whole cache is drawn; a test decides how many positions count as filled."""
    rng = np.random.default_rng(np.random.SeedSequence([seed, config_id, 7]))
    qkv = rng.standard_normal((B, 3, heads, head_dim))
    qkv[:, 1] *= key_scale
    K = _normal_fp16(rng, (B, heads, max_seq, head_dim), key_scale)
    V = _normal_fp16(rng, (B, heads, max_seq, head_dim), 1.0)
    return qkv.astype(np.float16), K, V


def make_config_gemm(config_id: int, gemm_index: int, seed: int = 0, B: Optional[int] = None):
    """Inputs for one GeMM of a named configuration.

    X and R are drawn for the configuration's largest batch and their first B rows
    returned, so a batch sweep shares data.
    """
    cfg = CONFIGS[config_id]
    spec = cfg.gemms[gemm_index]
    Bmax = max(cfg.batches)
    B = Bmax if B is None else B
    if not 1 <= B <= Bmax:
        raise ValueError(f"B={B} outside 1..{Bmax} for config {config_id}")
    W, bias, X, R = make_gemm_inputs(spec.K, spec.N, Bmax, seed, config_id, gemm_index,
                                     cfg.outlier_channels, cfg.outlier_scale)
    return spec, W, bias, np.ascontiguousarray(X[:B]), np.ascontiguousarray(R[:B])


def ragged_shapes() -> List[Tuple[int, int, int]]:
    """(B, K, N) cases that span several tiles and end in ragged tails, small enough for
    the oracle to finish in well under a second each."""
    return [
        (1, 8, 1), (1, 1, 1), (1, 32, 16), (2, 40, 24), (3, 103, 71), (4, 77, 65), (3, 104, 72), (5, 264, 200),
        (7, 1000, 130), (8, 520, 1032), (13, 776, 328), (16, 2056, 520),
        (17, 296, 136), (31, 1032, 264), (33, 520, 72), (48, 264, 328), (64, 1096, 200),
    ]
