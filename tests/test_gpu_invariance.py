"""Row invariance on the GPU: a node's logits are bitwise the same whether the target verifies it
alone, one token per step (plain decoding), or as one node of a tree (paper, Abstract and section
"Custom-Designed Decoding Tree": what drafting plus verification emits is exactly what plain
decoding emits).  Both sides of every comparison are the library's own results, so these tests say
nothing about correctness against the oracle (tests/test_gpu_parity.py does); they pin the property
that makes the decoding loop lossless bit for bit instead of up to top-2 near-ties."""
import numpy as np
import pytest

import fv_inputs as fi

pytestmark = pytest.mark.gpu


def _verifier(shape, weights, max_seq, max_tree=64):
    import paper_2412_12639_amd as m
    g = m.FalconVerifier(shape, max_seq=max_seq, max_tree=max_tree, device="cuda:0")
    g.init_weights(weights)
    g.set_step_invariant(True)
    return g


def _alone(g, L, path_tokens):
    """Logits of the last token of `path_tokens`, decoded one token per step from a cache of L tokens."""
    out = None
    for d, tk in enumerate(path_tokens):
        g.rollback(L + d, int(tk))
        g.verify_tree(np.array([tk], dtype=np.int32), np.array([-1], dtype=np.int32), np.array([0], dtype=np.int32))
        out = g.logits(1)[0].copy()
    return out


def _paths(parent):
    paths = []
    for i in range(len(parent)):
        p, j = [], i
        while j >= 0:
            p.append(j)
            j = int(parent[j])
        paths.append(p[::-1])
    return paths


CASES = [
    # shape, layers (0: as defined), prefix length, nodes, branching
    ("small-gqa", 0, 70, 64, [8, 4, 2, 2, 1, 1]),
    ("small-gqa", 0, 5, 20, [3, 2, 2, 1]),            # window reaches position 0
    ("small-gqa", 0, 33, 40, [4, 3, 2, 1, 1, 1, 1]),  # one far block for the deeper nodes only
    ("small-gqa", 0, 130, 33, None),                  # a chain of 33: depth 32, the deepest the canonical form takes
    ("small-gqa-f32", 0, 70, 48, [6, 3, 2, 2, 1]),
    ("tiny-bf16", 0, 90, 64, [8, 4, 2, 2, 1, 1]),       # head size 64
    ("tiny", 0, 40, 30, [4, 2, 2, 1, 1]),
    ("7b", 2, 200, 64, [8, 4, 2, 2, 1, 1, 1, 1]),
    ("7b", 2, 700, 40, [5, 3, 2, 2, 1, 1]),           # several far parts with runs of two blocks
]


@pytest.mark.parametrize("name,layers,L,T,branching", CASES)
def test_tree_rows_equal_plain_decoding_bit_for_bit(name, layers, L, T, branching):
    if name not in fi.SHAPES:
        pytest.skip(f"no shape {name}")
    shape = fi.SHAPES[name]
    if layers:
        shape = shape.with_layers(layers)
    weights = fi.gen_weights(shape, seed=0, gain_jitter=0.1)
    g = _verifier(shape, weights, L + T + 8)
    try:
        prefix = fi.gen_prefix(11, L, shape.vocab)
        root = g.prefill(prefix)
        if branching is None:
            parent, depth = fi.chain_tree(T)
        else:
            parent, depth, _ = fi.gen_tree(7, T, branching, 0)
        rng = np.random.default_rng(5)
        tokens = np.concatenate([[root], rng.integers(0, shape.vocab, T - 1)]).astype(np.int32)
        g.rollback(L, root)
        g.verify_tree(tokens, parent, depth)
        tree_logits = g.logits(T).copy()
        assert np.all(np.isfinite(tree_logits))
        paths = _paths(parent)
        # every node of the small cases; at the 7B width a sample that holds the deepest nodes
        nodes = range(T) if shape.hidden <= 1024 else sorted(set([0, 1, T // 2, T - 1] + list(np.argsort(depth)[-4:])))
        bad = []
        for i in nodes:
            alone = _alone(g, L, tokens[paths[i]])
            if not np.array_equal(alone, tree_logits[i]):
                bad.append((i, int(depth[i]), float(np.max(np.abs(alone - tree_logits[i])) / np.max(np.abs(alone)))))
        assert not bad, f"rows that differ from plain decoding (node, depth, relative difference): {bad[:8]}"
    finally:
        g.close()


def test_decoding_with_trees_emits_plain_decodings_tokens_and_logits():
    """Several rounds of tree verification against the same number of one-token steps, from the same prompt:
    same tokens, and the cache rows and the features they leave behind are bitwise equal."""
    shape = fi.SHAPES["small-gqa"]
    weights = fi.gen_weights(shape, seed=0, gain_jitter=0.1)
    L, n_new = 50, 24
    prefix = fi.gen_prefix(3, L, shape.vocab)
    ga = _verifier(shape, weights, L + n_new + 80)
    gt = _verifier(shape, weights, L + n_new + 80)
    try:
        ra = ga.prefill(prefix)
        rt = gt.prefill(prefix)
        assert ra == rt
        plain = [ra]
        for _ in range(n_new):
            a, _, nxt = ga.verify_tree(np.array([plain[-1]], dtype=np.int32), np.array([-1], dtype=np.int32), np.array([0], dtype=np.int32))
            assert a == 0
            plain.append(nxt)
        emitted = [rt]
        step = 0
        from fv_inputs.drafter import draft_tree
        while len(emitted) <= n_new:
            future = plain[len(emitted):len(emitted) + 8]
            tokens, parent, depth, _ = draft_tree(100 + step, emitted[-1], future, 24, [3, 2, 2, 1, 1], 0.8, shape.vocab)
            a, acc, nxt = gt.verify_tree(tokens, parent, depth)
            emitted += list(acc) + [nxt]
            step += 1
        n = min(len(emitted), len(plain))
        assert emitted[:n] == plain[:n]
        # the caches agree bit for bit over what both have committed
        n_rows = min(ga.state()[0], gt.state()[0])
        for layer in range(shape.n_layers):
            ka, va = ga.read_kv(layer, 0, n_rows)
            kt, vt = gt.read_kv(layer, 0, n_rows)
            assert np.array_equal(ka, kt) and np.array_equal(va, vt), f"layer {layer}"
    finally:
        ga.close()
        gt.close()
