"""Non-greedy verification (fv_verify_tree_sampled) against the oracle's multi-step speculative
sampling rule, through the C ABI.  The acceptance decisions are thresholds on floating-point
sums, so both sides take them in the same precision from the same numbers: the oracle's rule
(fp64) is applied to the logits the DEVICE produced (whose parity with the oracle's logits is
tested elsewhere), with the same uniforms; instances in which some decision lies within 1e-7
(relative) of its threshold are re-drawn.  Then everything is demanded bit-exact."""
import numpy as np
import pytest

import fv_inputs as fi
from oracle import falcon_oracle as fo
from tests import helpers as H

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fvmod():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2412_12639_amd as m
    m.load_library()
    return m


def _softmax(z):
    e = np.exp(z - np.max(z))
    return e / e.sum()


def _draft_tree(o, s, rng, root, n, branching, temperature, mode, seed):
    """A tree whose children are drawn level by level from a stand-in drafter: q_i = the target's
    own distribution at node i (from the oracle) flattened by noise.  mode "pointmass": the top-m
    tokens of q_i (distinct); mode "draft": m i.i.d. draws from q_i.  Returns tokens and q [n, V] float32."""
    parent, depth, _ = fi.gen_tree(seed, n, branching)
    tokens = np.zeros(n, dtype=np.int32)
    tokens[0] = root
    q = np.zeros((n, s.vocab), dtype=np.float32)
    for lvl in range(int(depth.max()) + 1):
        known = [i for i in range(n) if depth[i] <= lvl]
        new_of = {old: k for k, old in enumerate(known)}
        sub_parent = np.array([-1 if parent[i] < 0 else new_of[int(parent[i])] for i in known], dtype=np.int32)
        lg = o.tree_logits(tokens[known], sub_parent, depth[known])[0]
        for i in known:
            if depth[i] != lvl:
                continue
            kids = [c for c in range(n) if parent[c] == i]
            qi = _softmax(lg[new_of[i]] / temperature + rng.standard_normal(s.vocab) * 0.7)
            q[i] = qi.astype(np.float32)
            if not kids:
                continue
            if mode == "pointmass":
                picks = np.argsort(-qi)[:len(kids)]
            else:
                picks = rng.choice(s.vocab, size=len(kids), p=qi / qi.sum())
            for c, t in zip(kids, picks):
                tokens[c] = int(t)
    return tokens, parent, depth, q


@pytest.mark.parametrize("name", ["tiny", "small-gqa-f32", "small-gqa", "7b-L2"])
@pytest.mark.parametrize("mode", ["pointmass", "draft"])
def test_sampled_verification_takes_the_oracle_rule_decisions(fvmod, name, mode):
    """7b-L2: the benchmark's width and vocabulary (32000 tokens: the sums the decisions rest on are
    over the full vocabulary), two layers, 64 nodes, fewer trials."""
    import torch
    big = name == "7b-L2"
    s = fi.SHAPES["7b"].with_layers(2) if big else fi.SHAPES[name]
    w = fi.gen_weights(s, seed=0, gain_jitter=0.1)
    tol = H.tol_for(s)
    L, n = (200, 64) if big else (50, 24)
    temperature = np.float32(0.9 if mode == "draft" else 0.05)   # deterministic children are accepted with probability p[x]: a sharp p
    prefix = fi.gen_prefix(17, L, s.vocab)
    wo = {k: (fi.f32_from_bf16_bits(v) if v.dtype == np.uint16 else v) for k, v in w.items()}   # widened once, exactly
    o = fo.Oracle(s, wo, max_seq=L + n + 16, dtype=np.float32 if big else np.float64)
    root = o.prefill(prefix)
    g = fvmod.FalconVerifier(s, max_seq=L + n + 16, max_tree=64)
    g.init_weights(w)
    groot = g.prefill(prefix)
    if groot != root:
        g.rollback(L, root)
    rng = np.random.default_rng(123)
    n_checked = n_accepting = n_rejecting = 0
    for trial in range(3 if big else 10):
        tokens, parent, depth, q = _draft_tree(o, s, rng, root, n, [8, 4, 2, 2, 1, 1] if big else [3, 3, 2, 2, 1], temperature, mode, seed=trial)
        ua, us = rng.random(n), rng.random(n)
        qdev = torch.from_numpy(q).cuda() if mode == "draft" else None
        a, acc, nxt = g.verify_tree_sampled(tokens, parent, depth, temperature, ua, us, qdev)
        dev_logits = g.logits(n)
        d = fo.sampled_accept(dev_logits.astype(np.float64), tokens, parent, depth, L, temperature, ua, us,
                              q if mode == "draft" else None)
        if d["min_margin"] < 1e-7:       # a decision too close to its threshold to demand anything of it
            g.rollback(L, root)
            continue
        n_checked += 1
        assert a == d["accepted_len"], f"trial {trial}: accepted_len {a} vs {d['accepted_len']}"
        assert list(acc) == list(d["accepted_tokens"]) and nxt == d["next_token"]
        src, dst = g.kv_moves()
        assert list(src) == list(d["src_slot"]) and list(dst) == list(d["dst_slot"])
        assert g.state() == (L + a + 1, nxt)
        assert np.array_equal(g.tree_mask(n), fo.ancestor_mask(parent))
        # the forward pass is the greedy step's: logits, compacted K/V and features against the oracle
        lg, tk, tv = o.tree_logits(tokens, parent, depth)
        assert H.row_rel_err(dev_logits.astype(np.float64), lg).max() <= tol
        H.check_path_cache(g, s, L, d["path"], tk, tv, tol)
        feat = g.features(a + 1).astype(np.float64)
        assert H.row_rel_err(feat, o.last_hidden[d["path"]]).max() <= tol
        n_accepting += a >= 1
        n_rejecting += a < int(depth.max())
        g.rollback(L, root)
    if big:
        assert n_checked >= 2
    else:
        assert n_checked >= 6 and n_accepting >= 2 and n_rejecting >= 2, (n_checked, n_accepting, n_rejecting)
    g.close()


def test_sampled_verification_limits_and_errors(fvmod):
    s = fi.SHAPES["tiny"]
    w = fi.gen_weights(s, seed=0)
    L = 30
    prefix = fi.gen_prefix(3, L, s.vocab)
    g = fvmod.FalconVerifier(s, max_seq=80, max_tree=16)
    g.init_weights(w)
    root = g.prefill(prefix)
    parent, depth, _ = fi.gen_tree(2, 12, [3, 2, 2])
    rng = np.random.default_rng(0)
    # greedy tokens planted along one path; a very low temperature with point-mass proposals is greedy verification
    p1, d1 = fi.chain_tree(1)
    greedy, tk = [], root
    for _ in range(3):
        _, _, tk = g.verify_tree([tk], p1, d1)
        greedy.append(tk)
    g.rollback(L, root)
    from fv_inputs.trees import fill_tokens
    _, _, planted = fi.gen_tree(2, 12, [3, 2, 2], 2)
    tokens = fill_tokens(2, parent, s.vocab, root, planted, greedy[:2])
    want = g.verify_tree(tokens, parent, depth)
    g.rollback(L, root)
    got = g.verify_tree_sampled(tokens, parent, depth, 1e-4, rng.random(12), rng.random(12))
    assert got[0] == want[0] == 2 and list(got[1]) == list(want[1]) and got[2] == want[2]
    g.rollback(L, root)
    # a single node: the draw is the inverse cumulative sum of softmax(logits / T) at u_sample[0]
    for u in (0.0, 0.31, 0.77, 1.0):
        a, acc, nxt = g.verify_tree_sampled([root], p1, d1, 1.3, [0.5], [u])
        p = np.exp(g.logits(1)[0].astype(np.float64) / np.float64(np.float32(1.3)))
        cdf = np.cumsum(p / p.sum())
        lo = cdf[nxt - 1] if nxt > 0 else 0.0
        assert a == 0 and lo - 1e-9 <= u <= cdf[nxt] + 1e-9
        g.rollback(L, root)
    # refused inputs change nothing
    for kw in (dict(temperature=0.0), dict(temperature=float("nan")), dict(ua=[1.5] + [0.5] * 11), dict(us=[float("nan")] + [0.5] * 11)):
        with pytest.raises(fvmod.FvError) as ei:
            g.verify_tree_sampled(tokens, parent, depth, kw.get("temperature", 1.0), kw.get("ua", [0.5] * 12), kw.get("us", [0.5] * 12))
        assert ei.value.status == -1 and g.state() == (L, root)
    g.close()
