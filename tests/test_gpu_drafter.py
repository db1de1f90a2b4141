"""Drafting phase on the GPU against oracle/drafter_oracle.py, through the C ABI.

Every phase row's predicted feature and logits are compared element by element; the integer work
(top lists, the tokens of the tree) is checked bit-exactly: a top list must be the oracle's top_m
applied to the device's own logits (the decision taken in the device's precision), and the tree's
tokens must be those lists expanded by the oracle's structure function.  The oracle runs its later
passes on the device's tokens, so that a near-tie cannot make the two sides drift apart."""
import numpy as np
import pytest

from fv_inputs.shapes import shape_by_name
from fv_inputs.trees import gen_tree, sibling_ranks
from fv_inputs.weights import gen_drafter_weights, gen_features, gen_weights, sub_model
from oracle import drafter_oracle as do

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


def _make(shape_name, k, max_seq=160, seed=21, layers=None):
    import torch
    from paper_2412_12639_amd.binding import FalconDrafter, FalconVerifier
    s = shape_by_name(shape_name)
    if layers is not None:
        s = s.with_layers(layers)
    lw = gen_weights(s, seed=seed, gain_jitter=0.1)
    dw = gen_drafter_weights(s, seed=seed + 1, gain_jitter=0.1)
    tgt = FalconVerifier(s, max_seq, 64)
    tgt.init_weights(lw)
    dr = FalconDrafter(tgt, k)
    dr.init_weights(dw)
    return s, lw, dw, tgt, dr


def _oracle_weights(w):
    """bf16 bit patterns widened to fp32 once (exact), so that the oracle does not widen per product."""
    return {n: ((a.astype(np.uint32) << 16).view(np.float32) if a.dtype == np.uint16 else a) for n, a in w.items()}


def _rel(a, b):
    return float(np.max(np.abs(a - b)) / max(1e-30, np.max(np.abs(b))))


def _tol_of_pass(tol, p):
    """Rows of pass p (the commit's rows are pass 0) are computed from the outputs of pass p - 1: its predicted
    features and its LSTM states, two channels that carry the same rounding errors, so the errors of successive
    passes add up rather than average out (measured at the 7B width: 0.5e-2 of the largest logit per pass).
    The 2e-2 bar is kept for the commit's rows and the first tree pass and widened by 1e-2 per further pass
    (bf16 builds only; fp32 builds keep their flat tolerance)."""
    return tol if tol < 1e-3 else tol * max(1.0, (p + 1) / 2)


def _check_phase(s, dr, orc, n_chain, tokens_dev, parent, depth, rank, tol):
    """Rows of the open phase: features, logits, top lists, tree tokens."""
    _, n_rows, chain = dr.state()
    assert chain == n_chain and n_rows == len(orc.phase["f"])
    f_dev, l_dev = dr.rows("features", 0, n_rows), dr.rows("logits", 0, n_rows)
    f_ref, l_ref = np.array(orc.phase["f"]), np.array(orc.phase["logits"])
    pass_of = np.zeros(n_rows, dtype=int)
    if parent is not None:
        for bi, (a, _) in enumerate(orc.blocks):
            if bi > 0:
                pass_of[orc.rows_of[bi]] = depth[a] // orc.k
    for p in range(int(pass_of.max()) + 1):
        rows = np.nonzero(pass_of == p)[0]
        ef, el = _rel(f_dev[rows], f_ref[rows]), _rel(l_dev[rows], l_ref[rows])
        say(f"    pass {p}: {len(rows)} rows, features rel err {ef:.2e}, logits rel err {el:.2e} (tol {_tol_of_pass(tol, p):.2g})")
        assert ef <= _tol_of_pass(tol, p) and el <= _tol_of_pass(tol, p)
    tops = dr.top(0, n_rows)
    for r in range(n_rows):
        np.testing.assert_array_equal(tops[r], do.top_m(l_dev[r], tops.shape[1]), err_msg=f"top list of row {r}")
    if parent is None:
        return
    # the tree's tokens: the lists expanded by the oracle's structure function (history rows: the last k committed rows)
    blocks, gen = do.sar_structure(parent, depth, orc.k)
    hist = dr.top(256, orc.k)   # history slots (valid for the k-1 first ones)
    for i in range(1, len(parent)):
        bi, j = gen[i]
        if bi == 0:
            c = n_chain - 1 + j
            lst = hist[c] if c < orc.k - 1 else tops[c - (orc.k - 1)]
        else:
            lst = tops[orc.rows_of[bi][j]]
        assert tokens_dev[i] == lst[rank[i]], f"node {i}"


CASES = [("tiny", 2, 1e-4), ("tiny", 3, 1e-4), ("tiny", 1, 1e-4), ("tiny-bf16", 2, 2e-2), ("small-gqa", 2, 2e-2),
         ("small-gqa-f32", 4, 1e-4)]


@pytest.mark.parametrize("shape_name,k,tol", CASES)
def test_drafting_phases_elementwise(shape_name, k, tol):
    import torch
    s, lw, dw, tgt, dr = _make(shape_name, k)
    orc = do.DrafterOracle(s, lw, dw, k, 160)
    rng = np.random.default_rng(5)
    trees = [gen_tree(31, 40, [4, 3, 2, 2, 1, 1], 6), gen_tree(32, 25, [5, 2, 2, 1, 1, 1, 1, 1], 8), gen_tree(33, 12, [3, 2, 1], 3)]
    hist_ref = []                                           # top lists of all committed rows so far (oracle side, from device logits)
    for phase, (n_new, tree) in enumerate(zip([7, 1, 3], trees)):
        say(f"  {shape_name} k={k} phase {phase}: commit {n_new} pairs")
        feats = gen_features(100 + phase, n_new, s.hidden)
        toks = rng.integers(0, s.vocab, n_new)
        dr.commit(toks, torch.from_numpy(feats).cuda())
        orc.commit(feats, toks)
        _check_phase(s, dr, orc, n_new, None, None, None, None, tol)
        kd, vd = dr.read_kv(orc.L - n_new, n_new)
        assert _rel(kd, orc.K[orc.L - n_new:orc.L]) <= tol and _rel(vd, orc.V[orc.L - n_new:orc.L]) <= tol
        parent, depth, _ = tree
        rank = sibling_ranks(parent)
        tokens_dev = dr.draft_tree(parent, depth, rank, int(toks[-1]))
        tokens_ref = orc.draft(parent, depth, rank, int(toks[-1]), force_tokens=tokens_dev)
        _check_phase(s, dr, orc, n_new, tokens_dev, parent, depth, rank, tol)
        # where the oracle's own pick is clear of its neighbours by more than the tolerance, it is the device's pick
        agree = int(np.sum(tokens_dev == tokens_ref))
        say(f"    tree of {len(parent)} nodes: {agree} tokens equal the oracle's own picks")
        assert tokens_dev[0] == toks[-1]
        assert agree >= len(parent) - 2
    dr.close()
    tgt.close()


def test_wide_pass_and_degenerate_trees():
    """A pass of more than 64 rows (the shared-activation GEMM kernel and its separate reduction launch),
    a tree no deeper than k (no pass at all: the commit's rows give every token) and the one-node tree."""
    import torch
    s, lw, dw, tgt, dr = _make("tiny", 2, max_seq=400)
    orc = do.DrafterOracle(s, lw, dw, 2, 400)
    rng = np.random.default_rng(6)
    shapes = [gen_tree(41, 205, [4, 10, 2, 1], 0), gen_tree(42, 9, [4, 1], 2), (np.array([-1]), np.array([0]), None)]
    for phase, (n_new, tree) in enumerate(zip([4, 2, 1], shapes)):
        feats = gen_features(200 + phase, n_new, s.hidden)
        toks = rng.integers(0, s.vocab, n_new)
        dr.commit(toks, torch.from_numpy(feats).cuda())
        orc.commit(feats, toks)
        parent, depth, _ = tree
        rank = sibling_ranks(parent)
        got = dr.draft_tree(parent, depth, rank, int(toks[-1]))
        want = orc.draft(parent, depth, rank, int(toks[-1]), force_tokens=got)
        say(f"  tree of {len(parent)} nodes: phase rows {dr.state()[1]}")
        _check_phase(s, dr, orc, n_new, got, parent, depth, rank, 1e-4)
        np.testing.assert_array_equal(got, want)
        if phase == 0:
            assert dr.state()[1] - n_new > 64
    dr.close()
    tgt.close()


def test_benchmark_width_drafter_rows():
    """The 7B width (hidden 4096, 32 heads, FFN 11008, vocabulary 32000) with k = 2 and a 64-node tree of
    depth 8: what the benchmark times.  The oracle runs in fp32 on weights widened once."""
    import torch
    s, lw, dw, tgt, dr = _make("7b", 2, max_seq=256, layers=1)
    orc = do.DrafterOracle(s, _oracle_weights(lw), _oracle_weights(dw), 2, 256, dtype=np.float32)
    rng = np.random.default_rng(9)
    trees = [gen_tree(51, 64, [8, 4, 2, 2, 1, 1, 1, 1], 8), gen_tree(52, 64, [6, 3, 2, 2, 2, 1, 1, 1], 8)]
    for phase, (n_new, tree) in enumerate(zip([5, 2], trees)):
        feats = gen_features(300 + phase, n_new, s.hidden)
        toks = rng.integers(0, s.vocab, n_new)
        dr.commit(toks, torch.from_numpy(feats).cuda())
        say(f"  7b phase {phase}: commit {n_new} pairs {dr.last_ms():.3f} ms")
        orc.commit(feats, toks)
        parent, depth, _ = tree
        rank = sibling_ranks(parent)
        got = dr.draft_tree(parent, depth, rank, int(toks[-1]))
        say(f"    tree: {dr.state()[1] - n_new} rows in {int(max(depth) + 1) // 2 - 1} passes, {dr.last_ms():.3f} ms")
        want = orc.draft(parent, depth, rank, int(toks[-1]), force_tokens=got)
        _check_phase(s, dr, orc, n_new, got, parent, depth, rank, 2e-2)
        say(f"    {int(np.sum(got == want))} of {len(parent)} tokens equal the oracle's own picks")
        assert int(np.sum(got == want)) >= len(parent) - 3
    dr.close()
    tgt.close()


@pytest.mark.parametrize("head", ["ties", "zero"])
def test_top_lists_with_equal_logits(head):
    """Equal logits are ordered by token id: three LM-head rows made identical (and large, so that they
    often make the list), and an all-zero head (every logit equal: the list is 0, 1, 2, ...)."""
    import torch
    from paper_2412_12639_amd.binding import FalconDrafter, FalconVerifier
    s = shape_by_name("tiny")
    lw = gen_weights(s, seed=2)
    lw["lm_head"] = lw["lm_head"].copy()
    if head == "ties":
        lw["lm_head"][[100, 300]] = lw["lm_head"][7]
        lw["lm_head"][[7, 100, 300]] *= 6.0
    else:
        lw["lm_head"][:] = 0.0
    dw = gen_drafter_weights(s, seed=3)
    tgt = FalconVerifier(s, 64, 64)
    tgt.init_weights(lw)
    dr = FalconDrafter(tgt, 2)
    dr.init_weights(dw)
    feats = gen_features(4, 9, s.hidden)
    toks = np.random.default_rng(4).integers(0, s.vocab, 9)
    dr.commit(toks, torch.from_numpy(feats).cuda())
    logits, tops = dr.rows("logits", 0, 9), dr.top(0, 9)
    for r in range(9):
        np.testing.assert_array_equal(tops[r], do.top_m(logits[r], 32))
        if head == "zero":
            assert list(tops[r]) == list(range(32))
        else:
            assert logits[r][7] == logits[r][100] == logits[r][300]
            lst = tops[r].tolist()
            if 7 in lst and lst.index(7) + 2 < len(lst):     # the three equal logits are neighbours, in id order
                assert lst[lst.index(7):lst.index(7) + 3] == [7, 100, 300]
    parent, depth, _ = gen_tree(3, 20, [6, 3, 1], 0)
    got = dr.draft_tree(parent, depth, sibling_ranks(parent), int(toks[-1]))
    if head == "zero":
        np.testing.assert_array_equal(got[1:], sibling_ranks(parent)[1:])   # rank r takes token r everywhere
    dr.close()
    tgt.close()


def test_long_commit_in_pieces_and_errors():
    import torch
    from paper_2412_12639_amd.binding import FvError
    s, lw, dw, tgt, dr = _make("tiny", 2, max_seq=256)
    orc = do.DrafterOracle(s, lw, dw, 2, 256)
    n = 150                                                  # three pieces: 64 + 64 + 22
    feats = gen_features(7, n, s.hidden)
    toks = np.random.default_rng(8).integers(0, s.vocab, n)
    dr.commit(toks, torch.from_numpy(feats).cuda())
    _, l_ref = orc.commit(feats, toks)
    committed, n_rows, chain = dr.state()
    assert committed == n and chain == 22
    assert _rel(dr.rows("logits", 0, 22), l_ref[-22:]) <= 1e-4
    kd, vd = dr.read_kv(0, n)
    assert _rel(kd, orc.K[:n]) <= 1e-4 and _rel(vd, orc.V[:n]) <= 1e-4
    parent, depth, _ = gen_tree(3, 20, [3, 2, 2, 1], 4)
    rank = sibling_ranks(parent)
    with pytest.raises(FvError) as e:                        # rank beyond the list
        dr.draft_tree(parent, depth, np.full(20, 40), int(toks[-1]))
    assert e.value.status == -1
    with pytest.raises(FvError) as e:                        # a tree that is no tree
        dr.draft_tree(np.array([-1, 1, 0]), np.array([0, 1, 1]), np.zeros(3), int(toks[-1]))
    assert e.value.status == -2
    got = dr.draft_tree(parent, depth, rank, int(toks[-1]))
    want = orc.draft(parent, depth, rank, int(toks[-1]), force_tokens=got)
    assert int(np.sum(got == want)) >= 19
    with pytest.raises(FvError) as e:                        # one tree per phase
        dr.draft_tree(parent, depth, rank, int(toks[-1]))
    assert e.value.status == -8
    dr.reset()
    with pytest.raises(FvError) as e:                        # no committed pairs
        dr.draft_tree(parent, depth, rank, 1)
    assert e.value.status == -8
    dr.commit(toks[:1], torch.from_numpy(feats[:1]).cuda())
    with pytest.raises(FvError) as e:                        # fewer than k committed pairs
        dr.draft_tree(parent, depth, rank, int(toks[0]))
    assert e.value.status == -8
    dr.close()
    tgt.close()


def test_drafted_tree_goes_through_verification():
    """The drafted tokens are a valid tree for the verification step, fed by the features it exports."""
    import torch
    from paper_2412_12639_amd.binding import features_device_ptr
    s, lw, dw, tgt, dr = _make("small-gqa", 2, max_seq=200)
    prompt = np.random.default_rng(3).integers(0, s.vocab, 12)
    root = tgt.prefill(prompt)
    # stand-in features for the prompt pairs (the prefill does not export them); afterwards the real ones
    feats = gen_features(9, len(prompt), s.hidden)
    dr.commit(np.concatenate([prompt[1:], [root]]), torch.from_numpy(feats).cuda())
    parent, depth, _ = gen_tree(5, 30, [4, 2, 2, 1, 1, 1], 6)
    rank = sibling_ranks(parent)
    for step in range(3):
        tokens = dr.draft_tree(parent, depth, rank, root)
        a, acc, nxt = tgt.verify_tree(tokens, parent, depth)
        say(f"  step {step}: accepted {a}")
        new = list(acc[:a]) + [nxt]
        dr.commit(new, features_device_ptr(tgt))
        root = nxt
        assert dr.state()[0] == tgt.state()[0]
    dr.close()
    tgt.close()
