"""Pins of the drafting-phase oracle (oracle/drafter_oracle.py) against things other than itself:
a library LSTM, the verification oracle's decoder (itself pinned against an independent
implementation), hand-derived masks, a stable sort, and brute-force recomputation per path."""
import copy
import os

import numpy as np
import pytest

from fv_inputs.shapes import ModelShape, shape_by_name
from fv_inputs.trees import chain_tree, gen_tree, sibling_ranks, tree_depths
from fv_inputs.weights import gen_drafter_weights, gen_features, gen_weights
from oracle import drafter_oracle as do
from oracle import falcon_oracle as fo

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
TINY = ModelShape("tiny-d", 1, 64, 2, 1, 32, 96, 50, "f32")   # grouped KV heads, small enough for brute force


def _setup(shape=TINY, k=2, seed=3, max_seq=64):
    lw = gen_weights(shape, seed=seed, gain_jitter=0.1)
    dw = gen_drafter_weights(shape, seed=seed + 1, gain_jitter=0.1)
    return do.DrafterOracle(shape, lw, dw, k, max_seq), lw, dw


# ----------------------------------------------------------------------------- LSTM (reading D1)

def test_lstm_stack_equals_library_lstm_on_a_chain():
    torch = pytest.importorskip("torch")
    s = TINY
    dw = gen_drafter_weights(s, seed=5, bias_std=0.3)
    h = s.hidden
    ref = torch.nn.LSTM(input_size=2 * h, hidden_size=h, num_layers=2, batch_first=True).double()
    with torch.no_grad():
        for l in range(2):
            getattr(ref, f"weight_ih_l{l}").copy_(torch.from_numpy(dw[f"lstm{l}.w_ih"].astype(np.float64)))
            getattr(ref, f"weight_hh_l{l}").copy_(torch.from_numpy(dw[f"lstm{l}.w_hh"].astype(np.float64)))
            getattr(ref, f"bias_ih_l{l}").copy_(torch.from_numpy(dw[f"lstm{l}.b"].astype(np.float64)))
            getattr(ref, f"bias_hh_l{l}").zero_()
    rng = np.random.default_rng(0)
    z = rng.standard_normal((7, 2 * h))
    h0 = rng.standard_normal((2, h)) * 0.5
    c0 = rng.standard_normal((2, h)) * 0.5
    with torch.no_grad():
        out, (hn, cn) = ref(torch.from_numpy(z)[None], (torch.from_numpy(h0)[:, None], torch.from_numpy(c0)[:, None]))
    st = [(h0[0], c0[0]), (h0[1], c0[1])]
    mine = []
    for t in range(7):
        a = do.lstm_cell(z[t], st[0][0], st[0][1], dw["lstm0.w_ih"], dw["lstm0.w_hh"], dw["lstm0.b"], np.float64)
        b = do.lstm_cell(a[0], st[1][0], st[1][1], dw["lstm1.w_ih"], dw["lstm1.w_hh"], dw["lstm1.b"], np.float64)
        st = [a, b]
        mine.append(b[0])
    np.testing.assert_allclose(np.array(mine), out[0].numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(st[0][1], cn[0, 0].numpy(), atol=1e-12)
    np.testing.assert_allclose(st[1][1], cn[1, 0].numpy(), atol=1e-12)


def test_lstm_cell_closed_forms():
    h = 4
    z = np.zeros((4 * h, 3))
    # zero weights: gates are the biases alone
    b = np.concatenate([np.full(h, 50.0), np.full(h, -50.0), np.full(h, 0.5), np.full(h, 50.0)])   # i=1, f=0, g=tanh(.5), o=1
    hh, cc = do.lstm_cell(np.ones(3), np.ones(h), np.full(h, 7.0), z, np.zeros((4 * h, h)), b, np.float64)
    np.testing.assert_allclose(cc, np.tanh(0.5), atol=1e-12)          # the old cell is forgotten
    np.testing.assert_allclose(hh, np.tanh(np.tanh(0.5)), atol=1e-12)
    b = np.concatenate([np.full(h, -50.0), np.full(h, 50.0), np.zeros(h), np.full(h, -50.0)])      # i=0, f=1, o=0
    hh, cc = do.lstm_cell(np.ones(3), np.ones(h), np.full(h, 7.0), z, np.zeros((4 * h, h)), b, np.float64)
    np.testing.assert_allclose(cc, 7.0, atol=1e-12)                    # the old cell is kept
    np.testing.assert_allclose(hh, 0.0, atol=1e-12)


# ----------------------------------------------------------------------------- relaxed causal mask

def test_relaxed_mask_equals_the_rule_written_out_by_hand():
    """tests/golden/relaxed_mask_k2.txt: a phase of 2 chain rows and three blocks of two rows,
    visibility derived by hand from the rule of section 'Custom-Designed Decoding Tree'."""
    rows = [l.split() for l in open(os.path.join(GOLDEN, "relaxed_mask_k2.txt")) if l.strip() and not l.startswith("#")]
    pred = [int(r[0]) for r in rows]
    block = [int(r[1]) for r in rows]
    want = [sorted(int(c) for c in r[2].split(",")) for r in rows]
    assert do.relaxed_visible(pred, block) == want


def test_relaxed_mask_with_singleton_blocks_is_the_ancestor_mask():
    parent, depth, _ = gen_tree(4, 40, [4, 3, 2, 2, 1, 1], 0)
    vis = do.relaxed_visible(parent, np.arange(40))
    m = fo.ancestor_mask(parent)
    for i in range(40):
        bits = [j for j in range(40) if (int(m[i, j // 64]) >> (j % 64)) & 1]
        assert vis[i] == bits


def test_relaxed_mask_properties():
    rng = np.random.default_rng(1)
    for _ in range(20):
        n_blocks, k = int(rng.integers(1, 6)), int(rng.integers(1, 5))
        pred, block = [], []
        last_of = []
        for b in range(n_blocks):
            up = -1 if b == 0 else last_of[int(rng.integers(0, b))]
            for j in range(k):
                pred.append(up if j == 0 else len(pred) - 1)
                block.append(b)
            last_of.append(len(pred) - 1)
        vis = do.relaxed_visible(pred, block)
        for r in range(len(pred)):
            assert r in vis[r]
            mates = [j for j in range(len(pred)) if block[j] == block[r]]
            assert set(mates) <= set(vis[r])                       # the whole k x k block
            assert all(set(vis[r]) == set(vis[j]) for j in mates)  # rows of a block see the same set
            assert all(block[j] <= block[r] for j in vis[r])       # nothing later than the own block


# ----------------------------------------------------------------------------- decoder block (reading D2)

def test_block_equals_the_verification_oracles_decoder_layer():
    d, lw, dw = _setup()
    s = TINY
    rng = np.random.default_rng(2)
    n = 6
    x = rng.standard_normal((n, s.hidden))
    parent, depth = np.array([-1, 0, 0, 1, 1, 2]), np.array([0, 1, 1, 2, 2, 2])
    # the same layer inside the verification oracle: the rows come in through its embedding table
    w = {"embed": x.astype(np.float32), "g_final": np.ones(s.hidden, np.float32), "lm_head": lw["lm_head"]}
    for name in ("wq", "wk", "wv", "wo", "wg", "wu", "wd", "g_attn", "g_mlp"):
        w[f"l0.{name}"] = dw[f"d.{name}"]
    ref = fo.Oracle(s, w, 32, dtype=np.float64)
    vis = [fo.root_path(parent, i) for i in range(n)]
    ref._forward_rows(np.arange(n), 3 + depth, vis)
    d.L0 = 0
    out = d._block(x.astype(np.float32).astype(np.float64), 3 + depth, vis, [], [])
    np.testing.assert_allclose(fo.rmsnorm(out, np.ones(s.hidden), s.rms_eps), ref.last_hidden, atol=1e-10)


def test_block_scale_on_a_single_row_written_out():
    """One row with no context: attention returns that row's v, so the block is
    x + Wo.rep(v) + MLP(...) -- written out here with plain matrix products."""
    d, lw, dw = _setup()
    s = TINY
    x = np.random.default_rng(3).standard_normal((1, s.hidden))
    d.L0 = 0
    out = d._block(x, np.array([5]), [[0]], [], [])
    f64 = lambda a: a.astype(np.float64)
    nrm = lambda v, g: v / np.sqrt(np.mean(v * v) + s.rms_eps) * f64(g)
    v = f64(dw["d.wv"]) @ nrm(x[0], dw["d.g_attn"])
    rep = np.repeat(v.reshape(s.n_kv_heads, s.head_dim), s.n_q_heads // s.n_kv_heads, axis=0).reshape(-1)
    y = x[0] + f64(dw["d.wo"]) @ rep
    yn = nrm(y, dw["d.g_mlp"])
    g, u = f64(dw["d.wg"]) @ yn, f64(dw["d.wu"]) @ yn
    want = y + f64(dw["d.wd"]) @ (g / (1 + np.exp(-g)) * u)
    np.testing.assert_allclose(out[0], want, atol=1e-12)


# ----------------------------------------------------------------------------- top-m (reading D6)

def test_top_m_against_a_stable_sort_and_ties():
    rng = np.random.default_rng(4)
    row = rng.standard_normal(500)
    row[[7, 100, 300]] = row.max() + 1.0          # a three-way tie at the top
    row[[9, 8]] = row.min() - 1.0
    want = np.argsort(-row, kind="stable")[:20]
    np.testing.assert_array_equal(do.top_m(row, 20), want)
    assert list(do.top_m(row, 3)) == [7, 100, 300]
    assert do.top_m(row, 1)[0] == fo.first_argmax(row)
    with pytest.raises(FloatingPointError):
        do.top_m(np.array([0.0, np.nan, 1.0]), 2)
    with pytest.raises(FloatingPointError):
        do.top_m(np.array([0.0, np.inf, 1.0]), 2)


# ----------------------------------------------------------------------------- structure (readings D4, D5)

def test_sar_structure_on_a_hand_made_tree():
    #        0
    #      /   \
    #     1     2          depth 1
    #    / \    |
    #   3   4   5          depth 2
    #   |       |
    #   6       7          depth 3
    #   |
    #   8                  depth 4
    parent = [-1, 0, 0, 1, 1, 2, 3, 5, 6]
    depth = tree_depths(parent)
    blocks, gen = do.sar_structure(parent, depth, 2)
    assert blocks == [(0, 2), (3, 2), (5, 1)]          # node 4 is a leaf: no block; node 5 reaches one level
    assert gen[1] == (0, 0) and gen[2] == (0, 0)        # depth 1: row 0 of the root block
    assert gen[3] == gen[4] == gen[5] == (0, 1)         # depth 2: row 1 of the root block
    assert gen[6] == (1, 0) and gen[8] == (1, 1) and gen[7] == (2, 0)
    blocks, gen = do.sar_structure(parent, depth, 3)
    assert blocks == [(0, 3), (6, 1)]
    assert gen[6] == (0, 2) and gen[7] == (0, 2) and gen[8] == (1, 0)
    blocks, gen = do.sar_structure(parent, depth, 1)     # k = 1: every inner node has a block of one row
    assert [a for a, _ in blocks] == [0, 1, 2, 3, 5, 6] and all(r == 1 for _, r in blocks)


def test_number_of_passes_and_proposed_tokens():
    """Section 'Custom-Designed Decoding Tree': every pass yields k levels of the tree, so a tree
    of height H takes ceil(H / k) passes (k = 2, height 8: four passes, Appendix 'Tree Structure')."""
    parent, depth, _ = gen_tree(6, 64, [8, 4, 2, 2, 1, 1, 1, 1], 8)
    assert max(depth) == 8
    for k, want in ((2, 4), (3, 3), (4, 2)):
        blocks, gen = do.sar_structure(parent, depth, k)
        passes = 1 + max(depth[a] for a, _ in blocks) // k
        assert passes == want
        assert all(g is not None for g in gen[1:])


# ----------------------------------------------------------------------------- drafting

def _commit_some(d, s, n, seed):
    feats = gen_features(seed, n, s.hidden)
    toks = np.random.default_rng(seed).integers(0, s.vocab, n)
    d.commit(feats, toks)
    return feats, toks


def test_commit_in_pieces_equals_commit_at_once():
    a, _, _ = _setup()
    b, _, _ = _setup()
    feats = gen_features(1, 9, TINY.hidden)
    toks = np.random.default_rng(1).integers(0, TINY.vocab, 9)
    fa, la = a.commit(feats, toks)
    out = [b.commit(feats[:4], toks[:4]), b.commit(feats[4:5], toks[4:5]), b.commit(feats[5:], toks[5:])]
    np.testing.assert_allclose(np.concatenate([o[1] for o in out]), la, atol=1e-10)
    np.testing.assert_allclose(b.K[:9], a.K[:9], atol=1e-12)
    np.testing.assert_allclose(b.tail[0][0], a.tail[0][0], atol=1e-10)
    np.testing.assert_allclose(b.tail[1][1], a.tail[1][1], atol=1e-10)


def test_k1_chain_drafting_is_plain_autoregressive_drafting():
    """k = 1 and a chain: each pass has one row that sees all its predecessors -- the same as
    committing the drafter's own predicted feature and chosen token one pair at a time."""
    d, _, _ = _setup(k=1)
    ref, _, _ = _setup(k=1)
    _commit_some(d, TINY, 5, 7)
    _, toks = _commit_some(ref, TINY, 5, 7)
    parent, depth = chain_tree(5)
    got = d.draft(parent, depth, np.zeros(5, np.int64), int(toks[-1]))
    f, lg = ref.tail[-1]
    want = [int(toks[-1])]
    for _ in range(4):
        t = int(do.top_m(lg, 1)[0])
        want.append(t)
        fh, lgs = ref.commit(f[None], [t])
        f, lg = fh[0], lgs[0]
    assert list(got) == want


@pytest.mark.parametrize("k", [2, 3])
def test_draft_tokens_equal_per_path_recomputation(k):
    """Every block's rows recomputed in isolation: a fresh phase that holds only the committed chain
    and the blocks on that block's own path.  Rows off the path must not matter."""
    d, _, _ = _setup(k=k)
    _, toks = _commit_some(d, TINY, 6, 11)
    base = copy.deepcopy(d)
    parent, depth, _ = gen_tree(8, 30, [3, 2, 2, 2, 1, 1], 6)
    rank = sibling_ranks(parent)
    tokens = d.draft(parent, depth, rank, int(toks[-1]))
    blocks, gen = do.sar_structure(parent, depth, k)
    for bi, (a, rows) in enumerate(blocks):
        if bi == 0:
            continue
        # blocks on the path from the root block to this one
        chain = []
        j = a
        while depth[j] > 0:
            if depth[j] % k == 0:
                chain.append(j)
            j = parent[j]
        chain = chain[::-1]
        one = copy.deepcopy(base)
        up_rows, last = None, one.n_chain - 1
        for p, anc in enumerate(chain, start=1):
            path = []
            j = anc
            while depth[j] > (p - 1) * k:
                path.append(j)
                j = parent[j]
            path = path[::-1]
            nrows = dict(blocks)[anc]
            feat = [(one.tail[jj][0] if up_rows is None else one.phase["f"][up_rows[jj]]) for jj in range(nrows)]
            r0 = len(one.phase["pred"])
            pred = [last] + [r0 + jj - 1 for jj in range(1, nrows)]
            one._pass(np.array(feat), [tokens[q] for q in path[:nrows]], pred, [99 + p] * nrows,
                      [one.L - 1 + (p - 1) * k + jj + 1 for jj in range(nrows)])
            up_rows = list(range(r0, r0 + nrows))
            last = up_rows[-1] if nrows == k else None
        for i in range(1, len(parent)):
            if gen[i][0] == bi:
                lg = one.phase["logits"][up_rows[gen[i][1]]]
                assert tokens[i] == do.top_m(lg, int(rank[i]) + 1)[int(rank[i])]
                np.testing.assert_allclose(lg, d.phase["logits"][d.rows_of[bi][gen[i][1]]], atol=1e-9)


def test_nodes_of_one_depth_under_one_block_share_their_candidates():
    d, _, _ = _setup(k=2)
    _, toks = _commit_some(d, TINY, 4, 13)
    parent, depth, _ = gen_tree(9, 40, [4, 3, 2, 2], 0)
    rank = sibling_ranks(parent)
    tokens = d.draft(parent, depth, rank, int(toks[-1]))
    _, gen = do.sar_structure(parent, depth, 2)
    seen = {}
    for i in range(1, len(parent)):
        key = (gen[i], int(rank[i]))
        assert seen.setdefault(key, int(tokens[i])) == int(tokens[i])
    # siblings are distinct tokens
    for p in set(parent[1:]):
        kids = [int(tokens[i]) for i in range(1, len(parent)) if parent[i] == p]
        assert len(set(kids)) == len(kids)


def test_first_levels_come_from_the_last_k_committed_rows():
    d, lw, _ = _setup(k=2)
    _commit_some(d, TINY, 5, 17)
    f, toks = gen_features(18, 1, TINY.hidden), [3]
    d.commit(f, toks)                                   # one more pair: the root block spans two commits
    parent = np.array([-1, 0, 0, 1, 2])
    depth = tree_depths(parent)
    tokens = d.draft(parent, depth, sibling_ranks(parent), 3)
    l0, l1 = d.tail[0][1], d.tail[1][1]
    assert list(tokens[1:3]) == list(do.top_m(l0, 2))
    assert tokens[3] == tokens[4] == do.top_m(l1, 1)[0]
