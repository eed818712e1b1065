"""One token-generation step of a pre-layer-norm transformer layer as the sequence of library
calls the paper's Deep-Fusion draws for small batches (Sec. III-D, Fig. 1(c): four fused regions):

  1. input layer-norm + QKV GeMM + bias                         sbi_gemm_ln
  2. transposition + attention over the KV cache                sbi_attn_decode
  3. attention-output GeMM + bias + residual                    sbi_gemm_moments (leaves the row moments)
     post-attention layer-norm + FFN1 GeMM + bias + GeLU        sbi_gemm_ln (statistics from the moments)
  4. FFN2 GeMM + bias + residual                                sbi_gemm_moments (leaves the row moments
                                                                of the layer's output for the next layer's step 1)

Sequencing only: every value is produced by the kernels behind those calls.  All buffers are
allocated once (`DecoderLayer.__init__`, `new_state`), so a step allocates nothing and can be
captured into a HIP graph.
"""
from dataclasses import dataclass

from . import binding as sb


@dataclass
class DecoderState:
    """Per-batch buffers of a layer: the KV cache and the step's intermediates."""
    k_cache: object
    v_cache: object
    qkv: object
    ctx: object
    x2: object
    moments: object
    f: object
    y: object
    workspace: object
    y_moments: object = None      # per-panel row moments of y: the next layer's input layer-norm can start from them


class DecoderLayer:
    """Laid-out fp16 weights of one layer (W[K,N] row-major in, as everywhere in this library)."""

    def __init__(self, h, heads, Wqkv, bqkv, Wout, bout, Wffn1, bffn1, Wffn2, bffn2,
                 ln1_gamma, ln1_beta, ln2_gamma, ln2_beta, eps=1e-5):
        assert h % heads == 0 and h // heads in (64, 128) and h % 64 == 0
        self.h, self.heads, self.d, self.eps = h, heads, h // heads, eps
        self.f = Wffn1.shape[1]
        assert tuple(Wqkv.shape) == (h, 3 * h) and tuple(Wout.shape) == (h, h)
        assert tuple(Wffn1.shape) == (h, self.f) and tuple(Wffn2.shape) == (self.f, h)
        self.Wqkv, self.Wout = sb.layout_weights(Wqkv), sb.layout_weights(Wout)
        self.Wffn1, self.Wffn2 = sb.layout_weights(Wffn1), sb.layout_weights(Wffn2)
        self.bqkv, self.bout, self.bffn1, self.bffn2 = bqkv, bout, bffn1, bffn2
        self.ln1, self.ln2 = (ln1_gamma, ln1_beta, eps), (ln2_gamma, ln2_beta, eps)

    def workspace_bytes(self, B, max_seq):
        h, f = self.h, self.f
        return max(sb.ln_workspace_bytes(B, h, 3 * h), sb.workspace_bytes(B, h, h), sb.ln_workspace_bytes(B, h, f),
                   sb.workspace_bytes(B, f, h), sb.attn_workspace_bytes(B, self.heads, self.d, max_seq), 256)

    def new_state(self, B, max_seq, device, k_cache=None, v_cache=None):
        import torch
        h, f = self.h, self.f
        half = dict(dtype=torch.float16, device=device)
        if k_cache is None:
            k_cache = torch.zeros((B, self.heads, max_seq, self.d), **half)
            v_cache = torch.zeros((B, self.heads, max_seq, self.d), **half)
        return DecoderState(k_cache, v_cache, torch.empty((B, 3, self.heads, self.d), **half),
                            torch.empty((B, h), **half), torch.empty((B, h), **half),
                            torch.empty((B, h // 64, 2), dtype=torch.float32, device=device),
                            torch.empty((B, f), **half), torch.empty((B, h), **half),
                            sb.new_workspace(self.workspace_bytes(B, max_seq), device),
                            torch.empty((B, h // 64, 2), dtype=torch.float32, device=device))

    def step(self, x, pos, st, pos_bound=None, x_moments=None):
        """x fp16 [B,h]: the layer's input for the token at position pos.  Returns st.y [B,h].
        pos: one position for the whole batch (int), or an int32 device tensor [B] with one position
        per sequence together with pos_bound >= every entry (a batch of sequences of different lengths).
        x_moments: the previous layer's st.y_moments when x is that layer's st.y - the input layer-norm
        then takes its statistics from them instead of reading the rows again."""
        h, f = self.h, self.f
        B = x.shape[0]
        ws = st.workspace
        sb.gemm(self.Wqkv, h, 3 * h, x, self.bqkv, None, "bias", out=st.qkv.view(B, 3 * h), workspace=ws,
                layernorm=self.ln1, moments_in=x_moments)
        if pos_bound is None:
            sb.attn_decode(st.qkv, st.k_cache, st.v_cache, pos, out=st.ctx, workspace=ws)
        else:
            sb.attn_decode_ragged(st.qkv, st.k_cache, st.v_cache, pos, pos_bound, out=st.ctx, workspace=ws)
        sb.gemm(self.Wout, h, h, st.ctx, self.bout, x, "bias_residual", out=st.x2, workspace=ws,
                moments_out=st.moments)
        sb.gemm(self.Wffn1, h, f, st.x2, self.bffn1, None, "bias_gelu", out=st.f, workspace=ws,
                layernorm=self.ln2, moments_in=st.moments)
        sb.gemm(self.Wffn2, f, h, st.f, self.bffn2, st.x2, "bias_residual", out=st.y, workspace=ws,
                moments_out=st.y_moments)
        return st.y
