"""Rounding-noise model of a bf16 configuration (test helper, NOT part of the oracle).

The oracle computes the exact method in one working precision.  A bf16 configuration of the
library stores some tensors in bf16: the input of every weight multiplication, the rotated
queries and keys, the values (the K/V cache) and the attention probabilities that multiply the
values.  This module re-runs the oracle's decoder with those tensors rounded to bf16 at the
point where they are stored, each tensor class switchable on its own, so that a test (or a
study on the CPU) can say how far the storage formats ALONE move the logits of a deep model, and
which tensor class contributes what.  It mirrors where the library rounds, so it is evidence
about the formats, never a reference: parity is always measured against oracle/ itself.

Tensor classes:
  xin_qkv   x * gain before the q/k/v projections      (GEMM input)
  xin_gu    x * gain before the gate/up projections    (GEMM input)
  xin_head  x * gain before the LM head                (GEMM input)
  attn      attention output before the O projection   (GEMM input)
  act       silu(gate) * up before the down projection (GEMM input)
  k, v      rotated keys and values                    (the K/V cache)
  q         rotated queries
  p         un-normalised attention probabilities exp(s - max) (their normaliser is summed unrounded)
"""
import numpy as np

from oracle import falcon_oracle as fo

GEMM_INPUTS = ("xin_qkv", "xin_gu", "xin_head", "attn", "act")
KV_CACHE = ("k", "v")
OTHER = ("q", "p")
ALL_CLASSES = GEMM_INPUTS + KV_CACHE + OTHER


def round_bf16(x):
    """Round to the nearest bf16 value, ties to even, through fp32 (the value is first an fp32
    number, as on a device that computes in fp32); returned in x's own dtype."""
    a = np.ascontiguousarray(x, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    u = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16) << 16
    return u.astype(np.uint32).view(np.float32).astype(np.asarray(x).dtype)


class StorageNoiseModel(fo.Oracle):
    """fo.Oracle with the tensor classes in `rounded` stored as bf16.  prefill / verify_tree /
    rollback and the acceptance rule are the oracle's own; only the decoder pass is replaced."""

    def __init__(self, shape, weights, max_seq, dtype=np.float64, rounded=ALL_CLASSES):
        unknown = set(rounded) - set(ALL_CLASSES)
        if unknown:
            raise ValueError(f"unknown tensor classes {sorted(unknown)}")
        super().__init__(shape, weights, max_seq, dtype=dtype)
        self.rounded = frozenset(rounded)

    def _st(self, cls, t):
        return round_bf16(t) if cls in self.rounded else t

    def _gemm_in(self, cls, x, gain):
        """RMSNorm as the input of a weight multiplication, the way the library stores it: the
        stored tensor is x * gain and the per-row factor 1/sqrt(mean(x^2) + eps) multiplies the
        product -- the same thing in exact arithmetic.  Returns (stored input, factor)."""
        rinv = 1.0 / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + self.s.rms_eps)
        return self._st(cls, x * gain), rinv

    def _forward_rows(self, tokens, pos, visible):
        s, dt, L = self.s, self.dtype, self.L
        n = len(tokens)
        x = fo._up(self.w["embed"], dt)[np.asarray(tokens)]
        newK = np.zeros((s.n_layers, n, s.n_kv_heads, s.head_dim), dtype=dt)
        newV = np.zeros_like(newK)
        grp = s.n_q_heads // s.n_kv_heads
        lin, st = fo.linear, self._st
        for l in range(s.n_layers):
            W = lambda k: self.w[f"l{l}.{k}"]
            xin, rinv = self._gemm_in("xin_qkv", x, W("g_attn").astype(dt))
            q = st("q", fo.rope((lin(xin, W("wq"), dt) * rinv).reshape(n, s.n_q_heads, s.head_dim), pos, s.rope_base))
            k = st("k", fo.rope((lin(xin, W("wk"), dt) * rinv).reshape(n, s.n_kv_heads, s.head_dim), pos, s.rope_base))
            v = st("v", (lin(xin, W("wv"), dt) * rinv).reshape(n, s.n_kv_heads, s.head_dim))
            newK[l], newV[l] = k, v
            att = np.zeros((n, s.n_q_heads, s.head_dim), dtype=dt)
            scale = 1.0 / np.sqrt(s.head_dim)
            for qh in range(s.n_q_heads):
                kh = qh // grp
                if visible is None:   # a prompt: causal, written with a triangular mask
                    keys = np.concatenate([self.K[l, :L, kh], k[:, kh]], axis=0)
                    vals = np.concatenate([self.V[l, :L, kh], v[:, kh]], axis=0)
                    seen = np.concatenate([np.ones((n, L), dtype=bool), np.tril(np.ones((n, n), dtype=bool))], axis=1)
                    sc = np.where(seen, q[:, qh] @ keys.T * scale, -np.inf)
                    e = np.exp(sc - np.max(sc, axis=-1, keepdims=True))
                    att[:, qh] = (st("p", e) @ vals) / np.sum(e, axis=-1, keepdims=True)
                else:
                    for i in range(n):
                        keys = np.concatenate([self.K[l, :L, kh], k[visible[i], kh]], axis=0)
                        vals = np.concatenate([self.V[l, :L, kh], v[visible[i], kh]], axis=0)
                        sc = keys @ q[i, qh] * scale
                        e = np.exp(sc - np.max(sc))
                        att[i, qh] = (st("p", e) @ vals) / np.sum(e)
            x = x + lin(st("attn", att.reshape(n, -1)), W("wo"), dt)
            xin, rinv = self._gemm_in("xin_gu", x, W("g_mlp").astype(dt))
            a = fo.silu(lin(xin, W("wg"), dt) * rinv) * (lin(xin, W("wu"), dt) * rinv)
            x = x + lin(st("act", a), W("wd"), dt)
        self.last_hidden = fo.rmsnorm(x, self.w["g_final"].astype(dt), s.rms_eps)
        xin, rinv = self._gemm_in("xin_head", x, self.w["g_final"].astype(dt))
        return lin(xin, self.w["lm_head"], dt) * rinv, newK, newV
