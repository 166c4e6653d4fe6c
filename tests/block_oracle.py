"""One block of Eq. 2 / Eq. 3 on chosen rows, assembled from the oracle's routines (CPU only).

Two modes:
  * exact (default): float64 throughout -- the oracle proper;
  * stored_bf16=True: the same routines with one round-to-bf16 wherever a bf16 pipeline stores a
    tensor (LayerNorm output, Q (after the softmax scale), K, V, the attention output, the
    out-projection feature, the FFN hidden activation, the feature sum S).  No value of this mode
    ever comes from the GPU: it is what an ideal bf16-operand pipeline computes -- every
    contraction exact, one rounding per stored tensor -- and serves to tell the error that bf16
    storage forces on any implementation from an error of this one.
"""
import math

import numpy as np

from oracle import hero_oracle as O
from workloads import round_to_bf16


def r16(a):
    """Round to the nearest bf16-representable value (ties to even), back in float64."""
    return round_to_bf16(np.asarray(a, np.float32)).astype(np.float64)


class BlockOracle:
    def __init__(self, cfg, w, stored_bf16=False):
        self.cfg = cfg
        self.w = {k: v.astype(np.float64) for k, v in w.items()}
        d = cfg.hidden
        self.wq, self.bq = self.w["w_qkv"][:d], self.w["b_qkv"][:d]
        self.wkv, self.bkv = self.w["w_qkv"][d:], self.w["b_qkv"][d:]
        self.ext = O.BlockExt(cfg) if cfg.block_flags else None      # the modulated block's parts, if any
        self.R = r16 if stored_bf16 else (lambda a: a)
        # the pipeline stores Q multiplied by log2(e) / sqrt(head_dim): rounding happens at that scale
        self.q_scale = math.log2(math.e) / math.sqrt(cfg.head_dim)

    def _ln(self, x_rows, rows, which):
        w, c = self.w, self.cfg
        if self.ext is None:
            return self.R(O.layer_norm(x_rows, w[f"ln{which}_g"], w[f"ln{which}_b"], c.ln_eps))
        return self.R(self.ext.ln(x_rows, rows, w, which, c.ln_eps))

    def _gate(self, g, rows, which):
        return g if self.ext is None else self.ext.gate(g, rows, self.w, which)

    def kv(self, x_rows, rows):
        """K, V of the input rows x_rows, which sit at joint-sequence rows `rows`."""
        d, R = self.cfg.hidden, self.R
        kv = R(O.linear(self._ln(x_rows, rows, 1), self.wkv, self.bkv))
        if self.ext is None:
            return kv[:, :d], kv[:, d:]
        # (q is not needed here: normalise / rotate k alone by passing it as both arguments)
        _, k = self.ext.qk(kv[:, :d], kv[:, :d], rows, {**self.w, "qn_g": self.w.get("kn_g"), "qn_b": self.w.get("kn_b")})
        return (R(k) if self.ext.flags & (O.BLOCK_QKNORM | O.BLOCK_ROPE) else k), kv[:, d:]

    def rows(self, x_rows, rows, k_all, v_all):
        """(g_attn, g_ffn, S) of the given input rows against the given keys / values (Eq. 2 / Eq. 3);
        S = g_attn + g_ffn as the feature cache holds it."""
        c, w, R, s = self.cfg, self.w, self.R, self.q_scale
        q = O.linear(self._ln(x_rows, rows, 1), self.wq, self.bq)
        if self.ext is not None and self.ext.flags & (O.BLOCK_QKNORM | O.BLOCK_ROPE):
            q = R(q)                                            # stored once before the q/k pass
            q, _ = self.ext.qk(q, q, rows, {**w, "kn_g": w.get("qn_g"), "kn_b": w.get("qn_b")})
        q = R(q * s) / s
        o = R(O.attention(q, k_all, v_all, c.n_heads))
        g_attn = R(self._gate(O.linear(o, w["w_o"], w["b_o"]), rows, 1))
        h = R(O.gelu_tanh(O.linear(self._ln(x_rows + g_attn, rows, 2), w["w_ff1"], w["b_ff1"])))
        g_ffn = self._gate(O.linear(h, w["w_ff2"], w["b_ff2"]), rows, 2)
        return g_attn, g_ffn, R(g_attn + g_ffn)
