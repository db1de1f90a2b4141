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

Precision.  The paper states none; the default working precision is fp64 (`dtype`), and
nothing in this file rounds to a narrower format.  Full-size test cases pass dtype=np.float32
to bound the run time; that moves the logits by about 1e-6 of a row's maximum.

Pins added with the acceptance rule as a function of its own (`greedy_accept`): the parent-
pointer walk on hand-made trees, chains, ties and empty acceptance, and invariance under
relabelling; `top2_margin` against a sorted array.
"""
import numpy as np


# ----------------------------------------------------------------------------- helpers

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


def greedy_accept(tokens, parent, depth, argmax, L):
    """The acceptance and compaction rule of one verification step, as a function of the tree
    and of the target's greedy choice at every node (section "Custom-Designed Decoding Tree":
    candidates are checked by the LLM in the SpecInfer manner and only what it validates is
    kept; Experiments, "Models and Tasks": temperature 0).

    The root is accepted; a child is accepted iff its parent is accepted and its token is the
    target's argmax at the parent.  The deepest accepted node wins (reading: the lowest index
    among equally deep ones).  Returns a dict:
      accepted_len a   number of accepted draft nodes (= depth of the best node)
      path [a+1]       tree indices root .. best, found by walking parent pointers
      accepted_tokens  tokens of path[1:]
      next_token       the target's choice after the best node (the bonus token)
      src_slot / dst_slot [a+1]   compaction: the K/V of path node j goes to cache slot L + j
    """
    T = len(tokens)
    acc = np.zeros(T, dtype=bool)
    acc[0] = True
    for i in range(1, T):
        acc[i] = acc[parent[i]] and int(tokens[i]) == int(argmax[parent[i]])
    best = 0
    for i in range(T):  # deepest accepted node, lowest index among equals
        if acc[i] and depth[i] > depth[best]:
            best = i
    path = root_path(parent, best)
    a = int(depth[best])
    return dict(accepted_len=a, path=np.array(path, dtype=np.int32),
                accepted_tokens=np.array([tokens[j] for j in path[1:]], dtype=np.int32),
                next_token=int(argmax[best]),
                src_slot=np.array(path, dtype=np.int32),
                dst_slot=(L + np.arange(a + 1)).astype(np.int32))


def sampled_accept(logits, tokens, parent, depth, L, temperature, u_accept, u_sample, draft_probs=None):
    """Non-greedy verification of a token tree (Appendix "Tree Structure": in a non-greedy setting the
    children of a node are sampled instead of being the top-m tokens; section "Custom-Designed
    Decoding Tree": verification is consistent with SpecInfer, i.e. its multi-step speculative
    sampling over the tree).  A pure function of the target's logits and of uniform random numbers
    that are passed in, so that it can be applied to any logits.

    Starting at the root with the target distribution p = softmax(logits[node] / temperature):
    the children of the current node are tried in index order; child c with token x is accepted
    with probability min(1, p[x] / q[x]) (the test is  u_accept[c] * q[x] <= p[x]); on rejection
    p becomes the normalised positive part of p - q and the next child is tried against it.  An
    accepted child becomes the current node.  When no child is accepted (or the node is a leaf) the
    next token is drawn from what is left of p by inverting its cumulative sum over increasing
    token ids at u_sample[node].  q is the distribution the drafter drew that node's children from:
    row `node` of draft_probs [T, V]; with draft_probs=None every child is its own point-mass
    proposal (q[x] = 1, the case of deterministic top-m children), for which the rule reads: accept
    with probability p[x], else strike x from p and renormalise.  Either way every emitted token
    is distributed exactly as the target's own sampling would have it.

    Returns the fields of greedy_accept() plus `min_margin`: the smallest relative distance of any
    test from its threshold, and of the final draw from a boundary of the cumulative sum (a caller
    comparing two implementations rejects instances where that is within their rounding error)."""
    T = len(tokens)
    children = [[] for _ in range(T)]
    for i in range(1, T):
        children[int(parent[i])].append(i)
    cur, path, min_margin = 0, [0], np.inf
    while True:
        z = np.asarray(logits[cur], dtype=np.float64) / float(temperature)
        if not np.all(np.isfinite(z)):
            raise FloatingPointError("non-finite logits")
        w = np.exp(z - np.max(z))          # unnormalised target distribution after `cur`
        S = float(np.sum(w))
        taken = None
        for c in children[cur]:
            x = int(tokens[c])
            qx = 1.0 if draft_probs is None else float(draft_probs[cur][x])
            lhs, rhs = float(u_accept[c]) * qx * S, float(w[x])
            min_margin = min(min_margin, abs(lhs - rhs) / max(lhs, rhs, 1e-300))
            if lhs <= rhs:
                taken = c
                break
            if draft_probs is None:
                w[x] = 0.0
            else:
                w = np.maximum(w - S * np.asarray(draft_probs[cur], dtype=np.float64), 0.0)
            S2 = float(np.sum(w))
            if S2 <= 0.0:     # nothing is left besides what was rejected (probability zero): keep the last p
                w = np.exp(z - np.max(z))
                S2 = float(np.sum(w))
            S = S2
        if taken is None:
            cdf = np.cumsum(w)
            target = float(u_sample[cur]) * S
            nxt = int(np.searchsorted(cdf, target, side="right"))
            nxt = min(nxt, len(w) - 1)
            while w[nxt] == 0.0 and nxt > 0:   # a struck token has zero width: it cannot be drawn
                nxt -= 1
            lo = cdf[nxt - 1] if nxt > 0 else 0.0
            min_margin = min(min_margin, min(abs(target - lo), abs(cdf[nxt] - target)) / S)
            break
        cur = taken
        path.append(cur)
    a = len(path) - 1
    return dict(accepted_len=a, path=np.array(path, dtype=np.int32),
                accepted_tokens=np.array([tokens[j] for j in path[1:]], dtype=np.int32),
                next_token=nxt, src_slot=np.array(path, dtype=np.int32),
                dst_slot=(L + np.arange(a + 1)).astype(np.int32), min_margin=float(min_margin))


class Oracle:
    """prefill / verify_tree with a per-layer K/V cache (K stored after rotation)."""

    def __init__(self, shape, weights, max_seq, dtype=np.float64):
        self.s, self.w, self.dtype = shape, weights, dtype
        s = shape
        self.K = np.zeros((s.n_layers, max_seq, s.n_kv_heads, s.head_dim), dtype=dtype)
        self.V = np.zeros_like(self.K)
        self.L = 0          # committed prefix length
        self.pending = None  # token produced last, not yet in the cache (the next root)

    # -- one decoder pass over `n` new rows; row i attends cache slots [0, L) plus the
    #    new rows listed in visible[i] (indices into the new rows, in any order).
    #    visible=None means the causal case visible[i] = [0..i] (a prompt), which is written
    #    with a lower-triangular mask instead of a Python loop over rows: same sums.
    def _forward_rows(self, tokens, pos, visible):
        s, dt, L = self.s, self.dtype, self.L
        n = len(tokens)
        x = _up(self.w["embed"], dt)[np.asarray(tokens)]
        newK = np.zeros((s.n_layers, n, s.n_kv_heads, s.head_dim), dtype=dt)
        newV = np.zeros_like(newK)
        scale = 1.0 / np.sqrt(s.head_dim)
        for l in range(s.n_layers):
            W = lambda k: self.w[f"l{l}.{k}"]
            xn = rmsnorm(x, W("g_attn").astype(dt), s.rms_eps)
            q = rope(linear(xn, W("wq"), dt).reshape(n, s.n_q_heads, s.head_dim), pos, s.rope_base)
            k = rope(linear(xn, W("wk"), dt).reshape(n, s.n_kv_heads, s.head_dim), pos, s.rope_base)
            v = linear(xn, W("wv"), dt).reshape(n, s.n_kv_heads, s.head_dim)
            newK[l], newV[l] = k, v
            att = np.zeros((n, s.n_q_heads, s.head_dim), dtype=dt)
            for qh in range(s.n_q_heads):
                kh = _kv_head_of(qh, s)
                if visible is None:
                    keys = np.concatenate([self.K[l, :L, kh], k[:, kh]], axis=0)      # [L + n, d]
                    vals = np.concatenate([self.V[l, :L, kh], v[:, kh]], axis=0)
                    sc = q[:, qh] @ keys.T * scale                                    # [n, L + n]
                    seen = np.concatenate([np.ones((n, L), dtype=bool), np.tril(np.ones((n, n), dtype=bool))], axis=1)
                    att[:, qh] = softmax_lastaxis(np.where(seen, sc, -np.inf)) @ vals
                else:
                    for i in range(n):
                        keys = np.concatenate([self.K[l, :L, kh], k[visible[i], kh]], axis=0)
                        vals = np.concatenate([self.V[l, :L, kh], v[visible[i], kh]], axis=0)
                        att[i, qh] = softmax_lastaxis(keys @ q[i, qh] * scale) @ vals
            x = x + linear(att.reshape(n, -1), W("wo"), dt)
            xn = rmsnorm(x, W("g_mlp").astype(dt), s.rms_eps)
            x = x + linear(silu(linear(xn, W("wg"), dt)) * linear(xn, W("wu"), dt), W("wd"), dt)
        # features: what the LM head consumes (the last layer's output after the final norm)
        self.last_hidden = rmsnorm(x, self.w["g_final"].astype(dt), s.rms_eps)
        return linear(self.last_hidden, self.w["lm_head"], dt), newK, newV

    def prefill(self, tokens):
        """Run the prompt, fill cache slots 0..n-1, return the greedy next token (the
        root of the first tree)."""
        n = len(tokens)
        if n < 1 or n > self.K.shape[1]:
            raise TreeVerifyError("bad prompt length")
        self.L = 0
        logits, newK, newV = self._forward_rows(tokens, np.arange(n), None)
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

    def tree_logits(self, tokens, parent, depth):
        """Logits [T, V] of every node and the K/V the target computes for it ([NL, T, Hkv, d]
        each), without touching the state: each node sees the committed prefix and the nodes on
        its own root path, found by walking parent pointers; its position is prefix length +
        depth."""
        visible = [root_path(parent, i) for i in range(len(tokens))]
        return self._forward_rows(tokens, self.L + np.asarray(depth), visible)

    def verify_tree(self, tokens, parent, depth):
        """One verification step.  Returns a dict with
        logits [T,V], argmax [T], mask [T,4] u64, the fields of greedy_accept(), tree_k / tree_v
        (the K/V of every node), and features [a+1, hidden]: the LM head's input of every path
        node, recorded with the accepted tokens for the next drafting round (section
        "Custom-Designed Decoding Tree"; reading: after the final norm, i.e. exactly what the
        shared LM head consumes)."""
        s, L = self.s, self.L
        if self.pending is None:
            raise TreeVerifyError("no prefill")
        self.check_tree(tokens, parent, depth, s.vocab, self.pending, L, self.K.shape[1])
        T = len(tokens)
        logits, newK, newV = self.tree_logits(tokens, parent, depth)
        am = np.array([first_argmax(logits[i]) for i in range(T)], dtype=np.int32)
        out = greedy_accept(tokens, parent, depth, am, L)
        self.commit(out, newK, newV)
        out.update(logits=logits, argmax=am, mask=ancestor_mask(parent), tree_k=newK, tree_v=newV,
                   features=self.last_hidden[out["path"]].copy())
        return out

    def verify_tree_sampled(self, tokens, parent, depth, temperature, u_accept, u_sample, draft_probs=None):
        """One non-greedy verification step: the tree's logits as in verify_tree, acceptance by
        sampled_accept(), then the same compaction and state update."""
        s, L = self.s, self.L
        if self.pending is None:
            raise TreeVerifyError("no prefill")
        self.check_tree(tokens, parent, depth, s.vocab, self.pending, L, self.K.shape[1])
        logits, newK, newV = self.tree_logits(tokens, parent, depth)
        out = sampled_accept(logits, tokens, parent, depth, L, temperature, u_accept, u_sample, draft_probs)
        self.commit(out, newK, newV)
        out.update(logits=logits, mask=ancestor_mask(parent), tree_k=newK, tree_v=newV,
                   features=self.last_hidden[out["path"]].copy())
        return out

    def commit(self, decision, newK, newV):
        """Compaction and state update: the K/V of path node j goes to cache slot L + j, the
        committed length grows by accepted_len + 1 and the bonus token becomes the next root."""
        for src, dst in zip(decision["src_slot"], decision["dst_slot"]):
            self.K[:, dst] = newK[:, src]
            self.V[:, dst] = newV[:, src]
        self.L = self.L + decision["accepted_len"] + 1
        self.pending = decision["next_token"]

    def rollback(self, new_len, pending):
        self.L, self.pending = int(new_len), int(pending)


def top2_margin(row):
    """Gap between the largest and second-largest logit of a row (0 if the maximum is attained twice)."""
    part = np.partition(row, -2)
    return float(part[-1] - part[-2])
