"""HIP path vs CPU oracle, through the C ABI, on a real MI355X."""
import sys

import numpy as np
import pytest

import fv_inputs as fi
from fv_inputs.shapes import ModelShape
from oracle import falcon_oracle as fo
from tests import helpers as H

pytestmark = pytest.mark.gpu


def say(*a):
    """Progress line on stdout (run pytest with -s or -v to see it; nothing is written to disk)."""
    print("[case]", *a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def fvmod():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2412_12639_amd as m
    m.load_library()   # fails loudly if the HIP library is not built
    return m


def make_gpu(fvmod, shape, weights, max_seq, max_tree, invariant=False):
    g = fvmod.FalconVerifier(shape, max_seq=max_seq, max_tree=max_tree)
    g.init_weights(weights)
    if invariant:
        g.set_step_invariant(True)   # the step-invariant form of the attention, held to the same oracle
    return g


SHAPES = {
    "tiny": fi.SHAPES["tiny"],
    "tiny-bf16": fi.SHAPES["tiny-bf16"],
    "small-gqa-f32": fi.SHAPES["small-gqa-f32"],
    "small-gqa": fi.SHAPES["small-gqa"],
}
_W = {}


def weights_of(name):
    if name not in _W:
        _W[name] = fi.gen_weights(SHAPES[name], seed=0, gain_jitter=0.1)
    return _W[name]


@pytest.mark.parametrize("name", ["tiny", "small-gqa-f32", "tiny-bf16", "small-gqa"])
def test_prefill_logits_and_layer_intermediates(fvmod, name):
    """One chunk of prompt: logits of every row, and for the 1-layer shapes the rotated queries,
    attention output, FFN activation and residual stream, against oracle building blocks."""
    s, w = SHAPES[name], weights_of(name)
    tol = H.tol_for(s)
    say("prefill", name)
    prefix = fi.gen_prefix(3, 40, s.vocab)
    o = fo.Oracle(s, w, max_seq=64)
    o.prefill(prefix)
    g = make_gpu(fvmod, s, w, max_seq=64, max_tree=64)
    nxt = g.prefill(prefix)
    logits = g.logits(40)
    err = H.row_rel_err(logits.astype(np.float64), o.last_logits)
    say("prefill logits err", err.max())
    if s.n_layers == 1:
        dt = np.float64
        x0 = fo._up(w["embed"], dt)[prefix]
        xn = fo.rmsnorm(x0, w["l0.g_attn"].astype(dt), s.rms_eps)
        q = fo.rope(fo.linear(xn, w["l0.wq"], dt).reshape(40, s.n_q_heads, s.head_dim), np.arange(40), s.rope_base)
        gq = g.activation("q", 40)
        eq = np.max(np.abs(gq - q.reshape(40, -1))) / np.max(np.abs(q))
        say("q err", eq)
        assert eq <= tol
        k = fo.rope(fo.linear(xn, w["l0.wk"], dt).reshape(40, s.n_kv_heads, s.head_dim), np.arange(40), s.rope_base)
        gk, gv = g.read_kv(0, 0, 40)
        ek = np.max(np.abs(gk - k)) / np.max(np.abs(k))
        ev = np.max(np.abs(gv - o.V[0, :40])) / np.max(np.abs(o.V[0, :40]))
        say("k err", ek, "v err", ev)
        assert ek <= tol and ev <= tol
    assert err.max() <= tol
    assert np.isfinite(logits).all()
    if fo.top2_margin(o.last_logits[-1]) > tol * np.max(np.abs(o.last_logits[-1])):
        assert nxt == o.pending
    e = H.check_cache(g, o, s, 40, tol)
    say("cache err", e)
    g.close()


@pytest.mark.parametrize("name,n,br,plant,L", [
    ("tiny", 16, [4, 2, 1, 1], 4, 64),             # the small configuration of the benchmark list
    ("small-gqa-f32", 64, [8, 4, 2, 2, 1, 1], 3, 70),
    ("tiny-bf16", 16, [4, 2, 1, 1], 4, 64),
    ("small-gqa", 64, [8, 4, 2, 2, 1, 1], 3, 70),
])
@pytest.mark.parametrize("invariant", [False, True])
def test_verify_planted_tree(fvmod, name, n, br, plant, L, invariant):
    s, w = SHAPES[name], weights_of(name)
    tol = H.tol_for(s)
    say("verify", name, n, br, plant, L, "step-invariant rows" if invariant else "")
    case = H.planted_case(s, w, L, n, br, plant, seed=0)
    g = make_gpu(fvmod, s, w, max_seq=L + n + 8, max_tree=max(n, 64), invariant=invariant)
    root = g.prefill(case["prefix"])
    assert root == case["root"]
    got = g.verify_tree(case["tokens"], case["parent"], case["depth"])
    e = H.check_step(g, case, got, tol)
    say("logits err", e, "accepted", got[0])
    assert got[0] == plant
    assert g.state() == (L + plant + 1, case["res"]["next_token"])
    ec = H.check_cache(g, case["oracle"], s, L + plant + 1, tol)
    say("cache err after compaction", ec)
    g.close()


@pytest.mark.parametrize("name", ["small-gqa-f32", "small-gqa"])
def test_long_prefix_large_tree(fvmod, name):
    """A prefix long enough that every attention wavefront walks several key blocks, under a 200-node tree."""
    L, n = 1700, 200
    s, w = SHAPES[name], weights_of(name)
    tol = H.tol_for(s)
    say("long prefix", name, L, n)
    case = H.planted_case(s, w, L, n, fi.random_branching(n, n), 3, seed=L + n)
    g = make_gpu(fvmod, s, w, max_seq=L + n + 8, max_tree=256)
    assert g.prefill(case["prefix"]) == case["root"]
    got = g.verify_tree(case["tokens"], case["parent"], case["depth"])
    e = H.check_step(g, case, got, tol)
    say("logits err", e, "accepted", got[0])
    assert got[0] == 3
    H.check_cache(g, case["oracle"], s, L + 3 + 1, tol)
    g.close()


@pytest.mark.parametrize("name", ["small-gqa-f32", "small-gqa"])
@pytest.mark.parametrize("n", [1, 2, 16, 33, 64, 100, 128, 200, 256])
def test_tree_sizes_and_ragged_rows(fvmod, name, n):
    """All token-block instantiations (32/64/128/256 padded rows) with ragged fills."""
    s, w = SHAPES[name], weights_of(name)
    tol = H.tol_for(s)
    say("sizes", name, n)
    br = fi.random_branching(n, n) if n > 1 else [1]
    plant = min(3, n - 1) if n < 4 else 3
    if n == 2:
        br, plant = [1], 1
    case = H.planted_case(s, w, 45, n, br, plant, seed=n)
    g = make_gpu(fvmod, s, w, max_seq=45 + n + 8, max_tree=256)
    assert g.prefill(case["prefix"]) == case["root"]
    got = g.verify_tree(case["tokens"], case["parent"], case["depth"])
    e = H.check_step(g, case, got, tol)
    say("logits err", e, "accepted", got[0])
    g.close()


@pytest.mark.parametrize("name", ["small-gqa-f32", "small-gqa"])
def test_multi_chunk_prefill_and_multi_step_decode(fvmod, name):
    """Prompt longer than max_tree (several chain chunks, ragged last one), then several
    verification steps in a row, each from the state the previous one left."""
    s, w = SHAPES[name], weights_of(name)
    tol = H.tol_for(s)
    say("multi", name)
    L0 = 2 * 32 + 7
    prefix = fi.gen_prefix(13, L0, s.vocab)   # a prompt after which five steps in a row have clear argmax gaps
    o = fo.Oracle(s, w, max_seq=L0 + 200)
    root = o.prefill(prefix)
    g = make_gpu(fvmod, s, w, max_seq=L0 + 200, max_tree=32)
    groot = g.prefill(prefix)
    err = H.row_rel_err(g.logits(7).astype(np.float64), o.last_logits[-7:])
    say("last chunk logits err", err.max())
    assert err.max() <= tol
    e = H.check_cache(g, o, s, L0, tol)
    say("prefill cache err", e)
    assert groot == root or fo.top2_margin(o.last_logits[-1]) <= tol * np.max(np.abs(o.last_logits[-1]))
    if groot != root:
        pytest.skip("prefill argmax inside tolerance band")
    from fv_inputs.trees import fill_tokens
    emitted_g, emitted_o = [], []
    for step in range(5):
        L = o.L
        # plant the oracle's greedy continuation of length step % 4
        plant = step % 4
        greedy, tk = [], o.pending
        for _ in range(plant):
            p1, d1 = fi.chain_tree(1)
            tk = o.verify_tree(np.array([tk], dtype=np.int32), p1, d1)["next_token"]
            greedy.append(tk)
        pending = g.state()[1]
        for attempt in range(30):   # a tree whose decisive argmax gaps clear the tolerance
            o.rollback(L, pending)
            sd = 100 + step + 50 * attempt
            parent, depth, planted = fi.gen_tree(sd, 24, [3, 3, 2, 2, 1], plant)
            tokens = fill_tokens(sd, parent, s.vocab, pending, planted, greedy)
            res = o.verify_tree(tokens, parent, depth)
            if H.decision_margins_ok(res, tokens, parent, tol):
                break
        else:
            # the greedy path itself has a near-tie here: nothing decisive can be demanded past this point
            o.rollback(L, pending)
            say("step", step, "near-tie on the greedy path: stop here")
            break
        a, acc, nxt = g.verify_tree(tokens, parent, depth)
        case = dict(res=res, parent=parent, tokens=tokens, depth=depth, hidden=o.last_hidden.copy())
        e = H.check_step(g, case, (a, acc, nxt), tol)
        say("step", step, "err", e, "accepted", a)
        emitted_g += list(acc) + [nxt]
        emitted_o += list(res["accepted_tokens"]) + [res["next_token"]]
        assert g.state() == (o.L, o.pending)
    assert emitted_g == emitted_o and step >= 4 and len(emitted_g) >= 5
    e = H.check_cache(g, o, s, o.L, tol)
    say("final cache err", e)
    g.close()


def test_chain_equals_single_token_decoding_on_device(fvmod):
    """Losslessness on the device alone: verifying a chain of the device's own greedy tokens
    accepts all of it, and single-node steps reproduce the same tokens."""
    s, w = SHAPES["small-gqa"], weights_of("small-gqa")
    say("chain-vs-AR")
    prefix = fi.gen_prefix(21, 50, s.vocab)
    g = make_gpu(fvmod, s, w, max_seq=128, max_tree=32)
    root = g.prefill(prefix)
    ar, tk = [], root
    p1, d1 = fi.chain_tree(1)
    for _ in range(6):
        a, acc, tk = g.verify_tree([tk], p1, d1)
        assert a == 0
        ar.append(tk)
    g.rollback(50, root)
    p, d = fi.chain_tree(6)
    a, acc, nxt = g.verify_tree([root] + ar[:5], p, d)
    assert a == 5 and list(acc) == ar[:5] and nxt == ar[5]
    assert g.state() == (56, ar[5])
    g.close()


def test_two_runs_are_bitwise_identical(fvmod):
    s, w = SHAPES["small-gqa"], weights_of("small-gqa")
    say("determinism")
    case = H.planted_case(s, w, 60, 64, [8, 4, 2, 2, 1, 1], 3, seed=5)
    g = make_gpu(fvmod, s, w, max_seq=160, max_tree=64)
    g.prefill(case["prefix"])
    g.verify_tree(case["tokens"], case["parent"], case["depth"])
    l1 = g.logits(64).copy()
    g.rollback(60, case["root"])
    g.verify_tree(case["tokens"], case["parent"], case["depth"])
    l2 = g.logits(64)
    assert np.array_equal(l1.view(np.uint32), l2.view(np.uint32))
    g.close()


def test_rejected_calls_change_nothing(fvmod):
    s, w = SHAPES["tiny"], weights_of("tiny")
    say("errors")
    g = fvmod.FalconVerifier(s, max_seq=70, max_tree=16)
    with pytest.raises(fvmod.FvError) as ei:
        g.prefill([1, 2, 3])
    assert ei.value.status == -8   # weights missing
    g.init_weights(w)
    with pytest.raises(fvmod.FvError) as ei:
        g.verify_tree([1], [-1], [0])
    assert ei.value.status == -8   # no prefill yet
    root = g.prefill(fi.gen_prefix(0, 64, s.vocab))
    bad = [
        ([root, 1, 2], [-1, 0, 2], [0, 1, 2], -2),
        ([root, 1, 2], [0, 0, 1], [0, 1, 2], -2),
        ([root, 1, 2], [-1, 0, 1], [0, 1, 1], -3),
        ([root, 1, s.vocab], [-1, 0, 1], [0, 1, 2], -4),
        ([(root + 1) % s.vocab, 1, 2], [-1, 0, 1], [0, 1, 2], -7),
        ([root] + [1] * 16, list(range(-1, 16)), list(range(17)), -5),
        ([root] + [1] * 6, list(range(-1, 6)), list(range(7)), -6),
    ]
    for tok, par, dep, code in bad:
        with pytest.raises(fvmod.FvError) as ei:
            g.verify_tree(tok, par, dep)
        assert ei.value.status == code, (tok, par, dep)
        assert g.state() == (64, root)
    a, acc, nxt = g.verify_tree([root, 1, 2], [-1, 0, 1], [0, 1, 2])
    assert 0 <= a <= 2
    g.close()


def test_non_finite_logits_are_an_error_not_a_choice(fvmod):
    """A NaN among the logits leaves no greedy choice: the oracle raises, the library returns
    FV_E_NONFINITE and leaves the committed length and pending root as they were."""
    from fv_inputs.trees import fill_tokens
    s = SHAPES["tiny-bf16"]
    say("non-finite")
    prefix = fi.gen_prefix(0, 20, s.vocab)
    # (a) prompt: a row of NaNs in the LM head makes token 7's logit NaN in every row
    w = dict(weights_of("tiny-bf16"))
    bad = w["lm_head"].copy()
    bad[7, :] = 0x7FC0
    w["lm_head"] = bad
    with pytest.raises(FloatingPointError):
        fo.Oracle(s, w, max_seq=64).prefill(prefix)
    g = make_gpu(fvmod, s, w, max_seq=64, max_tree=16)
    with pytest.raises(fvmod.FvError) as ei:
        g.prefill(prefix)
    assert ei.value.status == -10
    g.close()
    # (b) verification: the embedding of a token that only one tree node carries is NaN, so that
    # node's logits are NaN and the step has no decision
    w = dict(weights_of("tiny-bf16"))
    poison = next(t for t in range(s.vocab) if t not in set(int(x) for x in prefix))
    emb = w["embed"].copy()
    emb[poison, :] = 0x7FC0
    w["embed"] = emb
    o = fo.Oracle(s, w, max_seq=64)
    root = o.prefill(prefix)
    assert root != poison
    parent, depth, _ = fi.gen_tree(1, 9, [3, 2, 1])
    tok = fill_tokens(1, parent, s.vocab, root)
    tok[5] = poison
    with pytest.raises(FloatingPointError):
        o.verify_tree(tok, parent, depth)
    g = make_gpu(fvmod, s, w, max_seq=64, max_tree=16)
    assert g.prefill(prefix) == root
    with pytest.raises(fvmod.FvError) as ei:
        g.verify_tree(tok, parent, depth)
    assert ei.value.status == -10 and g.state() == (20, root)
    g.close()


@pytest.mark.parametrize("kind", ["direct", "paired", "shared"])
@pytest.mark.parametrize("name", ["tiny", "small-gqa", "small-gqa-f32"])
def test_alternative_gemm_kernels_match_the_oracle(fvmod, name, kind, monkeypatch):
    """Up to 64 tokens the GEMMs default to the paired form of the direct-operand kernel wherever the
    K range is long enough for it (all matrices of small-gqa-f32, O and down of small-gqa, down of
    tiny) and to the one-strip form elsewhere; FV_GEMM forces the one-strip form ("direct") or the
    LDS-shared-activation kernel ("shared").  Same bar against the oracle for each."""
    s, w = SHAPES[name], weights_of(name)
    tol = H.tol_for(s)
    say("gemm-kind", kind, name)
    monkeypatch.setenv("FV_GEMM", kind)
    for n_nodes in (48, 17):
        case = H.planted_case(s, w, 70, n_nodes, [6, 3, 2, 2, 1, 1], 3, seed=4)
        g = make_gpu(fvmod, s, w, max_seq=160, max_tree=64)
        assert g.prefill(case["prefix"]) == case["root"]
        got = g.verify_tree(case["tokens"], case["parent"], case["depth"])
        e = H.check_step(g, case, got, tol)
        say("FV_GEMM=" + kind, n_nodes, "nodes: err", e)
        H.check_cache(g, case["oracle"], s, 70 + got[0] + 1, tol)
        g.close()


@pytest.mark.parametrize("name", ["small-gqa-f32", "small-gqa"])
@pytest.mark.parametrize("mode", ["0", "1", "2"])
def test_partial_tile_reduction_modes_above_64_rows(fvmod, name, mode, monkeypatch):
    """Steps of 128 / 256 rows: the partial tiles of a row group are reduced by the last workgroup to
    arrive inside the GEMM launch (FV_GEMM_FIX=0), by a second launch with one wavefront per tile for
    QKV, O and down (1, the default), or by that launch for every GEMM (2).  Same bar for each.  All
    three sum in ascending workgroup order, but the epilogue is compiled into two kernels whose
    multiply-adds may be contracted differently, so across modes the fp32 logits are only required to
    agree to rounding (1e-5 of the row maximum), not bit for bit."""
    s, w = SHAPES[name], weights_of(name)
    tol = H.tol_for(s)
    monkeypatch.setenv("FV_GEMM_FIX", mode)
    for n_nodes in (100, 256):
        say("reduction mode", mode, name, n_nodes)
        case = H.planted_case(s, w, 45, n_nodes, fi.random_branching(n_nodes, n_nodes), 3, seed=n_nodes)
        g = make_gpu(fvmod, s, w, max_seq=45 + n_nodes + 8, max_tree=256)
        assert g.prefill(case["prefix"]) == case["root"]
        got = g.verify_tree(case["tokens"], case["parent"], case["depth"])
        e = H.check_step(g, case, got, tol)
        say("FV_GEMM_FIX=" + mode, n_nodes, "nodes: err", e)
        logits = g.logits(n_nodes).copy()
        key = (name, n_nodes)
        if key in _REDUCTION_LOGITS:
            if s.dtype == "f32":
                d = H.row_rel_err(logits.astype(np.float64), _REDUCTION_LOGITS[key].astype(np.float64))
                say("distance to the first mode's logits", d.max())
                assert d.max() <= 1e-5
        else:
            _REDUCTION_LOGITS[key] = logits
        g.close()


_REDUCTION_LOGITS = {}


def _oracle_weights(w):
    """The same weights widened to fp32 once (exact), so that the oracle does not widen a matrix again
    at every use: matters at benchmark widths."""
    return {k: (fi.f32_from_bf16_bits(v) if v.dtype == np.uint16 else v) for k, v in w.items()}


def _wide_case(s, w, L, n_nodes, branching, plant, seed, tol, max_last_tokens=400):
    """One instance at a benchmark width whose deciding rows have clear margins, found cheaply: the
    oracle's pass over the first L-1 prompt tokens (the slow part; fp32 working precision bounds it)
    runs once, then candidates for the LAST prompt token are tried with single-row steps until the
    rows that decide the root and the planted greedy tokens all have a top-2 gap above
    2*tol*max|row| (so that a device within tol of the oracle must take the same decisions).
    max_last_tokens=1 takes the first candidate whatever its margins."""
    from fv_inputs.trees import fill_tokens
    prefix = fi.gen_prefix(seed, L, s.vocab)
    o = fo.Oracle(s, _oracle_weights(w), max_seq=L + n_nodes + 8, dtype=np.float32)
    o.prefill(prefix[:L - 1])
    say("oracle prompt pass done")
    p1, d1 = fi.chain_tree(1)
    rng = np.random.Generator(np.random.Philox(key=[seed, 7100]))
    for attempt in range(max_last_tokens):
        cand = int(prefix[L - 1]) if attempt == 0 else int(rng.integers(0, s.vocab))
        o.rollback(L - 1, cand)
        chain, tk, clear, rows = [], cand, True, []
        for j in range(plant + 2):   # rows of: the last prompt token, the root, the planted nodes
            r = o.verify_tree(np.array([tk], dtype=np.int32), p1, d1)
            row = r["logits"][0]
            rows.append(row.copy())
            clear = clear and fo.top2_margin(row) > 2 * tol * np.max(np.abs(row))
            if not clear and max_last_tokens > 1:
                break
            tk = r["next_token"]
            chain.append(tk)
        if clear or max_last_tokens == 1:
            break
    else:
        raise RuntimeError("no last prompt token with clear margins found")
    prefix = np.concatenate([prefix[:L - 1], np.array([cand], dtype=np.int32)])
    root, greedy = chain[0], chain[1:plant + 1]
    say("last prompt token candidates tried:", attempt + 1)
    for t in range(12):
        o.rollback(L, root)
        sd = seed + 1000 * t
        parent, depth, planted = fi.gen_tree(sd, n_nodes, branching, plant)
        tokens = fill_tokens(sd, parent, s.vocab, root, planted, greedy)
        res = o.verify_tree(tokens, parent, depth)
        clear = H.decision_margins_ok(res, tokens, parent, tol)
        if clear or max_last_tokens == 1:
            break
    say("oracle verify done; tree draws:", t + 1, "deciding margins clear:", clear)
    return dict(prefix=prefix, root=root, parent=parent, depth=depth, tokens=tokens, oracle=o, res=res,
                prefill_last=rows[0], hidden=o.last_hidden.copy(), clear=clear, plant=plant)


def _run_wide(fvmod, s, w, case, L, T, tol, max_tree=256, invariant=False):
    """Device step on a _wide_case instance, in the launch configuration bench.py times (max_tree 256)."""
    g = make_gpu(fvmod, s, w, max_seq=L + max_tree + 8, max_tree=max_tree, invariant=invariant)
    groot = g.prefill(case["prefix"])
    pl = case["prefill_last"]
    if fo.top2_margin(pl) > tol * np.max(np.abs(pl)):
        assert groot == case["root"]
    ec = H.check_cache(g, case["oracle"], s, 0 + L, tol) if s.n_layers <= 4 else None
    if groot != case["root"]:
        g.rollback(L, case["root"])
    got = g.verify_tree(case["tokens"], case["parent"], case["depth"])
    return g, got, ec


@pytest.mark.parametrize("name,L,T,br,plant", [
    ("7b", 512, 64, [8, 4, 2, 2, 1, 1], 3),        # the benchmark's headline shape
    ("7b", 2048, 128, "random", 2),                # tree-size sweep: the LDS-shared GEMM + separate reduction launch
    ("7b", 2048, 256, "random", 2),
    ("13b", 1024, 64, [8, 4, 2, 2, 1, 1], 2),      # hidden 5120, 40 heads, FFN 13824
    ("70b", 2048, 32, [4, 2, 2, 1, 1], 2),         # hidden 8192, 64 query / 8 KV heads, FFN 28672
])
def test_benchmark_widths_two_layers_elementwise(fvmod, name, L, T, br, plant):
    """Every shape of the benchmark list truncated to two layers, so that the oracle finishes in
    seconds to a minute: every logit of every node within 2e-2, prompt cache, compacted cache, and
    the integer outputs bit-exact against the oracle (the tree is re-drawn until the deciding
    margins are clear of the tolerance)."""
    s = fi.SHAPES[name].with_layers(2)
    tol = H.tol_for(s)
    say("width", name, "x 2 layers, prefix", L, "nodes", T)
    w = fi.gen_weights(s, seed=0)
    branching = fi.random_branching(T, T) if br == "random" else br
    case = _wide_case(s, w, L, T, branching, plant, seed=T, tol=tol)
    assert case["clear"], "no tree with clear deciding margins in 12 draws"
    # steps of up to 64 nodes also in the step-invariant form of the attention (same oracle, same bars)
    for invariant in ([False, True] if T <= 64 else [False]):
        g, got, ec = _run_wide(fvmod, s, w, case, L, T, tol, invariant=invariant)
        e = H.check_step(g, case, got, tol, L=L)
        say("step-invariant rows:" if invariant else "default:", "logits err", e, "(bar 2e-2); prompt cache err", ec, "; accepted", got[0])
        assert got[0] == plant
        H.check_cache(g, case["oracle"], s, L + plant + 1, tol)
        g.close()


_DEEP = {}


@pytest.mark.timeout(1500)
def test_benchmark_configuration_all_layers(fvmod):
    """The benchmark's own configuration, all 32 layers (minutes of CPU for the oracle and the noise model).

    Integer outputs: bit-exact, unconditionally, against the oracle's acceptance rule applied to the
    device's argmax; and equal to the oracle's own decisions where the oracle's deciding margins are
    clear of the error measured on this instance.  Compacted K/V of the path taken: against the
    oracle's per-node K/V.  Logits: the 2e-2 bar of the shallow shapes is NOT met at this depth (see
    test_all_layers_logits_against_the_2e-2_bar, which reports it); what is asserted here is that the
    device is no further from the exact logits than 1.1x what the bf16 formats that the configuration
    fixes (GEMM inputs and K/V cache) put between the noise model and the exact logits, and the
    depth-scaled bound 2e-2*sqrt(NL/4)."""
    from tests import bf16_noise_model as nm
    s = fi.SHAPES["7b"]
    L, T = 512, 64
    w = fi.gen_weights(s, seed=0)
    say("7b, 32 layers: oracle prompt pass + verify on the host ...")
    tol = H.tol_for(s)
    case = _wide_case(s, w, L, T, [8, 4, 2, 2, 1, 1], 3, seed=0, tol=tol, max_last_tokens=1)
    g, got, _ = _run_wide(fvmod, s, w, case, L, T, tol)
    res = case["res"]
    assert np.array_equal(g.tree_mask(T), res["mask"])
    logits = g.logits(T)
    ref = res["logits"].astype(np.float64)
    err = H.row_rel_err(logits.astype(np.float64), ref)
    _DEEP["err"] = err
    bound = tol * float(np.sqrt(s.n_layers / 4.0))
    say("all-layers logits err: max", err.max(), "median", float(np.median(err)), "-- the 2e-2 bar is",
        "met" if err.max() <= tol else "NOT met", "; depth-scaled bound", bound)
    d = H.check_decisions(g, case["tokens"], case["parent"], case["depth"], L, got)
    ek = H.check_path_cache(g, s, L, d["path"], res["tree_k"], res["tree_v"], bound)
    say("decisions = acceptance rule of the device argmax; accepted", d["accepted_len"], "; compacted K/V err", ek)
    feat = g.features(d["accepted_len"] + 1).astype(np.float64)
    assert H.row_rel_err(feat, case["hidden"][d["path"]].astype(np.float64)).max() <= bound
    am = g.argmax(T)
    clear = [i for i in range(T) if fo.top2_margin(res["logits"][i]) > 2 * err[i] * np.max(np.abs(res["logits"][i]))]
    for i in clear:   # a row's argmax cannot move if its top-2 gap exceeds twice that row's own error
        assert am[i] == res["argmax"][i], f"argmax of node {i}"
    say("argmax equals the oracle's on the", len(clear), "of", T, "rows whose gap exceeds twice their measured error")
    if H.decision_margins_ok(res, case["tokens"], case["parent"], float(err.max()) * 1.01):
        assert d["accepted_len"] == res["accepted_len"] and list(d["path"]) == list(res["path"]) and d["next_token"] == res["next_token"]
        say("decisions also equal the oracle's own")
    else:
        say("a deciding row of the ORACLE is a near-tie at this depth: oracle decisions not demanded")
    g.close()
    assert err.max() <= bound
    # the formats the configuration fixes, alone, in the noise model
    fl = nm.StorageNoiseModel(s, _oracle_weights(w), max_seq=L + T + 8, dtype=np.float32, rounded=nm.GEMM_INPUTS + nm.KV_CACHE)
    fl.prefill(case["prefix"])
    fl.rollback(L, case["root"])
    floor = H.row_rel_err(fl.tree_logits(case["tokens"], case["parent"], case["depth"])[0].astype(np.float64), ref)
    say("noise model, bf16 GEMM inputs + K/V cache only: max", floor.max(), "median", float(np.median(floor)))
    _DEEP["floor"] = floor
    assert np.median(err) <= 1.1 * np.median(floor) and err.max() <= 1.25 * floor.max()


def test_all_layers_logits_against_the_2e_2_bar():
    """The stated bar, 2e-2 of the row maximum, on the 32-layer benchmark configuration.  Recorded as
    an expected failure while the measured error exceeds it: with bf16 GEMM inputs and a bf16 K/V
    cache, which the configuration fixes, the rounding noise of those formats alone is above the bar
    at this depth (the previous test measures both figures)."""
    if "err" not in _DEEP:
        pytest.skip("needs the all-layers test of this module to have run")
    e = float(_DEEP["err"].max())
    if e > 2e-2:
        pytest.xfail(f"2e-2 bar NOT met at 32 layers: measured {e:.3e}"
                     + (f"; bf16 GEMM inputs + K/V cache alone give {float(_DEEP['floor'].max()):.3e}" if "floor" in _DEEP else ""))


@pytest.mark.parametrize("name", ["small-gqa-f32", "small-gqa"])
def test_multi_step_decoding_with_a_synthetic_drafter_is_lossless(fvmod, name):
    """Decoding loop: trees from a synthetic drafter that gets a geometric number of tokens right per
    step; the concatenation of accepted tokens and bonus tokens must be exactly the target's greedy
    sequence (the oracle's, and the device's own one-token-at-a-time decoding), and every step must
    accept exactly the number of tokens the drafter got right."""
    s, w = SHAPES[name], weights_of(name)
    tol = H.tol_for(s)
    say("decode-loop", name)
    N, L0 = 40, 37
    prefix = fi.gen_prefix(41, L0, s.vocab)   # a prompt whose first greedy tokens have clear margins in bf16 too
    o_seq = fo.greedy_decode(s, w, list(prefix), N + 1)          # root, then N more tokens
    g = make_gpu(fvmod, s, w, max_seq=L0 + N + 64, max_tree=32)
    root = g.prefill(prefix)
    # where the oracle's own top-2 gap is inside the tolerance nothing can be demanded beyond that point
    o_chk = fo.Oracle(s, w, max_seq=L0 + N + 8)
    o_chk.prefill(list(prefix) + [int(t) for t in o_seq[:N]])
    lg = o_chk.last_logits[L0 - 1:]                               # row j decides o_seq[j]
    clear = [fo.top2_margin(lg[j]) > 2 * tol * np.max(np.abs(lg[j])) for j in range(N + 1)]
    n_sure = clear.index(False) if False in clear else N + 1   # o_seq[:n_sure] are beyond doubt
    say("greedy tokens with a clear margin before the first near-tie:", n_sure, "of", N + 1)
    if s.dtype == "f32":
        assert n_sure == N + 1
    if n_sure == 0:
        pytest.skip("the very first greedy token is a near-tie at this precision")
    assert root == o_seq[0]
    # plain decoding on the device, one token per step
    p1, d1 = fi.chain_tree(1)
    ar, tk = [], root
    for _ in range(N):
        a, acc, tk = g.verify_tree([tk], p1, d1)
        assert a == 0 and len(acc) == 0
        ar.append(tk)
    assert ar[:n_sure - 1] == [int(t) for t in o_seq[1:n_sure]]
    # the same tokens through tree verification; the drafter is fed the DEVICE's greedy sequence, so
    # that past a near-tie (where device and oracle may part ways) the loop is still checked against
    # the device's own one-token-at-a-time decoding
    g.rollback(L0, root)
    emitted, tk, step, accepted = [], root, 0, []
    while len(emitted) < N - 6:
        future = ar[len(emitted):]
        tokens, parent, depth, n_ok = fi.draft_tree(500 + step, tk, future, 24, [3, 3, 2, 2, 1], 0.75, s.vocab)
        a, acc, nxt = g.verify_tree(tokens, parent, depth)
        sure = len(emitted) + n_ok + 1 <= n_sure - 1
        if sure:
            assert a == n_ok, f"step {step}: accepted {a}, drafter got {n_ok} right"
        emitted += list(acc) + [nxt]
        accepted.append(a)
        tk = nxt
        step += 1
        assert g.state() == (L0 + len(emitted), tk)
        if emitted != ar[:len(emitted)]:
            # only a near-tie may make tree verification and single-token decoding disagree
            k = next(i for i in range(len(emitted)) if emitted[i] != ar[i])
            assert k + 1 >= n_sure, f"token {k} differs although its margin is clear"
            say("sequences part at token", k, "(near-tie): stop")
            break
    k = min(len(emitted), n_sure - 1)
    assert emitted[:k] == [int(t) for t in o_seq[1:1 + k]]
    say("steps", step, "tokens", len(emitted), "mean accepted length", float(np.mean(accepted)))
    g.close()


def test_a_partial_tile_that_never_arrives_ends_in_an_error_not_a_hang(fvmod, monkeypatch):
    """The GEMM workgroup that finishes a shared row group waits for the other workgroups' partial
    sums with a bounded number of looks.  FV_EXCHANGE_TEST=timeout (read when the context is created)
    makes the condition from the host: contributors leave their tiles unmarked and
    finishers give up after two looks.  Every kernel ends normally; the step reports
    FV_E_EXCHANGE_TIMEOUT, and so does every later step of that context."""
    name = "small-gqa"
    shape, weights = SHAPES[name], weights_of(name)
    monkeypatch.setenv("FV_EXCHANGE_TEST", "timeout")
    g = make_gpu(fvmod, shape, weights, 160, 64)
    monkeypatch.delenv("FV_EXCHANGE_TEST")
    prefix = fi.gen_prefix(3, 40, shape.vocab)
    with pytest.raises(fvmod.FvError) as e1:
        g.prefill(prefix)
    assert e1.value.status == -12, e1.value
    with pytest.raises(fvmod.FvError) as e2:
        g.prefill(prefix)
    assert e2.value.status == -12, e2.value
    g.close()
    # a context created without the switch is not affected
    g2 = make_gpu(fvmod, shape, weights, 160, 64)
    g2.prefill(prefix)
    g2.close()
