"""CPU oracle for the tree-verification step of Falcon's speculative decoding loop.

TEST INFRASTRUCTURE ONLY.  This file is a plain, slow, from-the-definition numpy
implementation (fp64 by default) used by the tests, the smoke check and the
benchmark's CPU-baseline leg.  It shares no code with the HIP library and the
library never calls it.

What it computes.  The paper's verification phase (section "Custom-Designed
Decoding Tree") hands the drafted token tree, every node of which stands for the
candidate sequence spelled by its root path, to the target LLM, which checks all
candidates in one tree-based parallel decoding pass in the SpecInfer manner; only
tokens the LLM itself validates are kept, so the output equals plain decoding
(Abstract and Introduction: the speed-up is lossless).  With the paper's greedy
setting (Experiments, "Models and Tasks": temperature 0, batch size 1) this means:

  * every node's logits are the target model's next-token logits after
    prefix ++ tokens on the node's root path;
  * a child is accepted iff its parent is accepted and its token is the argmax of
    the parent's logits; the longest accepted path wins;
  * the accepted tokens and the K/V the target computed for them are recorded for
    the next round.

The target model is the Llama-style decoder of the evaluated model families
(Vicuna / LLaMA2-Chat): RMSNorm, rotary positions in the rotate-half pairing,
causal softmax attention with optional grouped KV heads, SwiGLU FFN, no biases,
untied LM head.

Pins (tests/test_oracle_pins.py): `causal_forward` against an independent library
implementation of the same architecture; `verify_tree` node logits against
`causal_forward` over each root path by brute force; chain trees against plain
greedy decoding; closed forms for the ancestor mask; cache contents after
compaction against a fresh prefill of the extended sequence.

Readings where the paper is silent are listed with each function.

Precision.  The paper states none; the default is fp64 throughout.  `Oracle(storage="bf16")`
is the same computation with the STORAGE FORMATS of the bf16 configuration written in: every
tensor that such a configuration keeps in bf16 (the input of each weight multiplication, the
rotated queries and keys, the values, i.e. the K/V cache, and the attention probabilities that
multiply the values) is rounded to bf16 (round to nearest even) at the point where it is
stored; all arithmetic stays in the working precision.  It exists for deep models, where the
rounding noise of those formats alone (about 2^-9 relative per stored tensor, adding in
quadrature over ~9 tensors per layer) exceeds the tolerance that is demanded of shallow ones;
pinned in tests/test_oracle_pins.py (rounding against a library conversion; storage=None
unchanged; exactly representable data unaffected).
"""
import numpy as np


# ----------------------------------------------------------------------------- helpers

def round_bf16(x):
    """Round to the nearest bf16 value, ties to even, through fp32 (the value is first an fp32
    number, as on a device that computes in fp32); returned in x's own dtype."""
    a = np.ascontiguousarray(x, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    u = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16) << 16
    return u.astype(np.uint32).view(np.float32).astype(np.asarray(x).dtype)


def _up(w, dtype):
    """Weights arrive as float32 or as bf16 bit patterns (uint16); both are widened
    exactly to the working precision."""
    if w.dtype == np.uint16:
        w = (w.astype(np.uint32) << np.uint32(16)).view(np.float32)
    return w.astype(dtype, copy=False)


def linear(x, w, dtype):
    """y = x W^T for a weight stored [out_features, in_features]."""
    return x @ _up(w, dtype).T


def rmsnorm(x, gain, eps):
    """Root-mean-square layer norm over the last axis: x / sqrt(mean(x^2) + eps) * gain.
    (Reading: eps inside the square root, as in the Llama family.)"""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * gain


def rope(x, pos, base):
    """Rotary position embedding, rotate-half pairing.  x: [n, heads, d]; pos: [n].
    Dimension i (0 <= i < d/2) is paired with i + d/2 and the pair is rotated by the
    angle pos * base^(-2i/d)."""
    n, _, d = x.shape
    half = d // 2
    inv_freq = base ** (-2.0 * np.arange(half, dtype=np.float64) / d)
    ang = np.asarray(pos, dtype=np.float64)[:, None] * inv_freq[None, :]
    c = np.cos(ang).astype(x.dtype)[:, None, :]
    s = np.sin(ang).astype(x.dtype)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def silu(x):
    return x / (1.0 + np.exp(-x))


def softmax_lastaxis(s):
    m = np.max(s, axis=-1, keepdims=True)
    e = np.exp(s - m)
    return e / np.sum(e, axis=-1, keepdims=True)


def first_argmax(row):
    """Greedy choice; the lowest token id wins ties (reading: the paper is silent)."""
    if not np.all(np.isfinite(row)):
        raise FloatingPointError("non-finite logits")
    return int(np.argmax(row))


def ancestor_mask(parent):
    """mask[i] = set of tree indices on the parent chain of i, i included, as four
    64-bit words, bit j of the set stored in word j // 64 at bit j % 64."""
    n = len(parent)
    out = np.zeros((n, 4), dtype=np.uint64)
    for i in range(n):
        j = i
        while j >= 0:
            out[i, j // 64] |= np.uint64(1) << np.uint64(j % 64)
            j = int(parent[j])
    return out


def root_path(parent, i):
    p = []
    while i >= 0:
        p.append(int(i))
        i = int(parent[i])
    return p[::-1]


# ----------------------------------------------------------------------------- the model from scratch

def _kv_head_of(qh, shape):
    """Grouped-query attention: query head qh reads KV head floor(qh * Hkv / Hq)."""
    return qh * shape.n_kv_heads // shape.n_q_heads


def causal_forward(shape, weights, tokens, dtype=np.float64, return_hidden=False):
    """Logits [n, V] of the decoder over a whole token sequence with a lower-
    triangular mask, computed from scratch with no cache.  With return_hidden also the
    LM head's input [n, hidden] (the last layer's output after the final norm)."""
    s = shape
    n = len(tokens)
    x = _up(weights["embed"], dtype)[np.asarray(tokens)]
    pos = np.arange(n)
    for l in range(s.n_layers):
        W = lambda k: weights[f"l{l}.{k}"]
        xn = rmsnorm(x, W("g_attn").astype(dtype), s.rms_eps)
        q = linear(xn, W("wq"), dtype).reshape(n, s.n_q_heads, s.head_dim)
        k = linear(xn, W("wk"), dtype).reshape(n, s.n_kv_heads, s.head_dim)
        v = linear(xn, W("wv"), dtype).reshape(n, s.n_kv_heads, s.head_dim)
        q, k = rope(q, pos, s.rope_base), rope(k, pos, s.rope_base)
        att = np.zeros((n, s.n_q_heads, s.head_dim), dtype=dtype)
        for qh in range(s.n_q_heads):
            kh = _kv_head_of(qh, s)
            sc = q[:, qh, :] @ k[:, kh, :].T / np.sqrt(s.head_dim)
            sc = np.where(np.tril(np.ones((n, n), dtype=bool)), sc, -np.inf)
            att[:, qh, :] = softmax_lastaxis(sc) @ v[:, kh, :]
        x = x + linear(att.reshape(n, -1), W("wo"), dtype)
        xn = rmsnorm(x, W("g_mlp").astype(dtype), s.rms_eps)
        a = silu(linear(xn, W("wg"), dtype)) * linear(xn, W("wu"), dtype)
        x = x + linear(a, W("wd"), dtype)
    xn = rmsnorm(x, weights["g_final"].astype(dtype), s.rms_eps)
    logits = linear(xn, weights["lm_head"], dtype)
    return (logits, xn) if return_hidden else logits


def greedy_decode(shape, weights, tokens, n_new, dtype=np.float64):
    """Plain autoregressive greedy decoding by repeated full forwards."""
    seq = [int(t) for t in tokens]
    out = []
    for _ in range(n_new):
        nxt = first_argmax(causal_forward(shape, weights, seq, dtype)[-1])
        out.append(nxt)
        seq.append(nxt)
    return out


# ----------------------------------------------------------------------------- cached decoding + tree verification

class TreeVerifyError(ValueError):
    pass


class Oracle:
    """prefill / verify_tree with a per-layer K/V cache (K stored after rotation)."""

    def __init__(self, shape, weights, max_seq, dtype=np.float64, storage=None):
        if storage not in (None, "bf16"):
            raise ValueError("storage must be None or 'bf16'")
        self.s, self.w, self.dtype = shape, weights, dtype
        self.st = round_bf16 if storage == "bf16" else (lambda t: t)
        self.storage = storage
        s = shape
        self.K = np.zeros((s.n_layers, max_seq, s.n_kv_heads, s.head_dim), dtype=dtype)
        self.V = np.zeros_like(self.K)
        self.L = 0          # committed prefix length
        self.pending = None  # token produced last, not yet in the cache (the next root)

    # -- one decoder pass over `n` new rows; row i attends cache slots [0, L) plus the
    #    new rows listed in visible[i] (indices into the new rows, in any order)
    def _forward_rows(self, tokens, pos, visible):
        s, dt, L = self.s, self.dtype, self.L
        n = len(tokens)
        x = _up(self.w["embed"], dt)[np.asarray(tokens)]
        newK = np.zeros((s.n_layers, n, s.n_kv_heads, s.head_dim), dtype=dt)
        newV = np.zeros_like(newK)
        grp = s.n_q_heads // s.n_kv_heads
        st = self.st
        for l in range(s.n_layers):
            W = lambda k: self.w[f"l{l}.{k}"]
            xn, post = self._norm_in(x, W("g_attn").astype(dt))
            q = st(rope((linear(xn, W("wq"), dt) * post).reshape(n, s.n_q_heads, s.head_dim), pos, s.rope_base))
            k = st(rope((linear(xn, W("wk"), dt) * post).reshape(n, s.n_kv_heads, s.head_dim), pos, s.rope_base))
            v = st((linear(xn, W("wv"), dt) * post).reshape(n, s.n_kv_heads, s.head_dim))
            newK[l], newV[l] = k, v
            att = np.zeros((n, s.n_q_heads, s.head_dim), dtype=dt)
            for i in range(n):
                vis = visible[i]
                keys = np.concatenate([self.K[l, :L], k[vis]], axis=0)   # [m, Hkv, d]
                vals = np.concatenate([self.V[l, :L], v[vis]], axis=0)
                # query head qh uses KV head qh // grp  (== floor(qh*Hkv/Hq))
                kq = np.repeat(keys, grp, axis=1)                         # [m, Hq, d]
                vq = np.repeat(vals, grp, axis=1)
                sc = np.einsum("hd,mhd->hm", q[i], kq) / np.sqrt(s.head_dim)
                if self.storage is None:
                    p = softmax_lastaxis(sc)
                    att[i] = np.einsum("hm,mhd->hd", p, vq)
                else:
                    # stored probabilities are the un-normalised exp(s - max); the sum that
                    # normalises them is taken before they are rounded
                    e = np.exp(sc - np.max(sc, axis=-1, keepdims=True))
                    att[i] = np.einsum("hm,mhd->hd", st(e), vq) / np.sum(e, axis=-1, keepdims=True)
            x = x + linear(st(att.reshape(n, -1)), W("wo"), dt)
            xn, post = self._norm_in(x, W("g_mlp").astype(dt))
            a = silu(linear(xn, W("wg"), dt) * post) * (linear(xn, W("wu"), dt) * post)
            x = x + linear(st(a), W("wd"), dt)
        xn, post = self._norm_in(x, self.w["g_final"].astype(dt))
        # features: what the LM head consumes (the last layer's output after the final norm)
        self.last_hidden = rmsnorm(x, self.w["g_final"].astype(dt), s.rms_eps)
        return linear(xn, self.w["lm_head"], dt) * post, newK, newV

    def _norm_in(self, x, gain):
        """RMSNorm as the input of a weight multiplication: returns (input, factor) with
        norm(x) W^T == (input W^T) * factor.  Default: (rmsnorm(x), 1).  With bf16 storage the
        stored tensor is x * gain (rounded), and the per-row factor 1/sqrt(mean(x^2) + eps)
        multiplies the product, which is the same thing in exact arithmetic."""
        if self.storage is None:
            return rmsnorm(x, gain, self.s.rms_eps), 1.0
        rinv = 1.0 / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + self.s.rms_eps)
        return self.st(x * gain), rinv

    def prefill(self, tokens):
        """Run the prompt, fill cache slots 0..n-1, return the greedy next token (the
        root of the first tree)."""
        n = len(tokens)
        if n < 1 or n > self.K.shape[1]:
            raise TreeVerifyError("bad prompt length")
        self.L = 0
        visible = [list(range(i + 1)) for i in range(n)]
        logits, newK, newV = self._forward_rows(tokens, np.arange(n), visible)
        self.K[:, :n], self.V[:, :n] = newK, newV
        self.L = n
        self.pending = first_argmax(logits[-1])
        self.last_logits = logits
        return self.pending

    @staticmethod
    def check_tree(tokens, parent, depth, vocab, pending, L, max_seq, max_tree=256):
        """Input rules (Appendix "Tree Structure": one token per non-root node; the
        root is the token the LLM generated).  Reading: nodes come in an order with
        parent[i] < i and depth is redundant but checked."""
        n = len(tokens)
        if n < 1 or len(parent) != n or len(depth) != n:
            raise TreeVerifyError("bad sizes")
        if n > max_tree:
            raise TreeVerifyError("tree too big")
        if L + n > max_seq:
            raise TreeVerifyError("cache full")
        if parent[0] != -1 or depth[0] != 0:
            raise TreeVerifyError("node 0 must be the root")
        for i in range(1, n):
            if not (0 <= parent[i] < i):
                raise TreeVerifyError("parent order")
            if depth[i] != depth[parent[i]] + 1:
                raise TreeVerifyError("depth mismatch")
        if np.any(np.asarray(tokens) < 0) or np.any(np.asarray(tokens) >= vocab):
            raise TreeVerifyError("token range")
        if int(tokens[0]) != int(pending):
            raise TreeVerifyError("root mismatch")

    def verify_tree(self, tokens, parent, depth):
        """One verification step.  Returns a dict with
        logits [T,V], argmax [T], mask [T,4] u64, accepted_len a, accepted_tokens [a],
        next_token, path [a+1] (tree indices root..best), src_slot / dst_slot [a+1],
        features [a+1, hidden]: the LM head's input of every path node, recorded with the
        accepted tokens for the next drafting round (section "Custom-Designed Decoding Tree";
        reading: after the final norm, i.e. exactly what the shared LM head consumes)."""
        s, L = self.s, self.L
        if self.pending is None:
            raise TreeVerifyError("no prefill")
        self.check_tree(tokens, parent, depth, s.vocab, self.pending, L, self.K.shape[1])
        T = len(tokens)
        # each node sees the committed prefix and the nodes on its own root path,
        # found by walking parent pointers; its position is prefix length + depth
        visible = [root_path(parent, i) for i in range(T)]
        pos = L + np.asarray(depth)
        logits, newK, newV = self._forward_rows(tokens, pos, visible)
        am = np.array([first_argmax(logits[i]) for i in range(T)], dtype=np.int32)
        # greedy acceptance: the root always; a child iff parent accepted and token
        # equals the parent's argmax
        acc = np.zeros(T, dtype=bool)
        acc[0] = True
        for i in range(1, T):
            acc[i] = acc[parent[i]] and int(tokens[i]) == int(am[parent[i]])
        best = 0
        for i in range(T):  # deepest accepted node, lowest index among equals
            if acc[i] and depth[i] > depth[best]:
                best = i
        path = root_path(parent, best)
        a = int(depth[best])
        accepted_tokens = np.array([tokens[j] for j in path[1:]], dtype=np.int32)
        next_token = int(am[best])
        # compaction: the K/V of path node j goes to cache slot L + j
        src = np.array(path, dtype=np.int32)
        dst = L + np.arange(a + 1, dtype=np.int32)
        for j in range(a + 1):
            self.K[:, dst[j]] = newK[:, src[j]]
            self.V[:, dst[j]] = newV[:, src[j]]
        self.L = L + a + 1
        self.pending = next_token
        return dict(logits=logits, argmax=am, mask=ancestor_mask(parent), accepted_len=a,
                    accepted_tokens=accepted_tokens, next_token=next_token,
                    path=src, src_slot=src, dst_slot=dst, tree_k=newK, tree_v=newV,
                    features=self.last_hidden[src].copy())

    def rollback(self, new_len, pending):
        self.L, self.pending = int(new_len), int(pending)


def top2_margin(row):
    """Gap between the largest and second-largest logit of a row."""
    part = np.partition(row, -2)
    return float(part[-1] - part[-2])
