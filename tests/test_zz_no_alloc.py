"""fv_verify_tree_noalloc (scratch in the library's static device array) against fv_verify_tree,
through the C ABI: two calls in a row, the second with a smaller tree, and a last one that is
refused for its size.  Collected last (file name), so that a failure here hides no other test."""
import numpy as np
import pytest

import fv_inputs as fi
from fv_inputs.trees import fill_tokens

pytestmark = pytest.mark.gpu


def _tree(seed, n, vocab, root):
    parent, depth, _ = fi.gen_tree(seed, n, [6, 3, 2, 2, 1, 1])
    return fill_tokens(seed, parent, vocab, root), parent, depth


@pytest.mark.parametrize("invariant", [False, True])
@pytest.mark.parametrize("name", ["small-gqa", "small-gqa-f32", "7b-L2"])
def test_noalloc_entry_point_equals_the_arena_one(name, invariant):
    import torch
    assert torch.cuda.is_available(), "needs the GPU"
    import paper_2412_12639_amd as m
    m.load_library()
    s = fi.SHAPES["7b"].with_layers(2) if name == "7b-L2" else fi.SHAPES[name]
    w = fi.gen_weights(s, seed=0, gain_jitter=0.1)
    L = 150
    g = m.FalconVerifier(s, max_seq=L + 80, max_tree=64)
    g.init_weights(w)
    g.set_step_invariant(invariant)   # the attention's far-key parts and window live in the static array too
    root = g.prefill(fi.gen_prefix(9, L, s.vocab))
    for n in (61, 19):    # two calls in a row on the shared static array, the second one smaller
        tok, parent, depth = _tree(n, n, s.vocab, root)
        ref = g.verify_tree(tok, parent, depth)
        ref_logits, ref_mask, ref_moves = g.logits(n).copy(), g.tree_mask(n).copy(), g.kv_moves()
        ref_kv = [g.read_kv(l, L, ref[0] + 1) for l in range(s.n_layers)]
        ref_feat = g.features(ref[0] + 1).copy()
        assert g.state() == (L + ref[0] + 1, ref[2])
        g.rollback(L, root)
        got = g.verify_tree(tok, parent, depth, noalloc=True)
        assert got[0] == ref[0] and list(got[1]) == list(ref[1]) and got[2] == ref[2]
        assert g.state() == (L + ref[0] + 1, ref[2])
        assert np.array_equal(g.tree_mask(n), ref_mask)
        src, dst = g.kv_moves()
        assert list(src) == list(ref_moves[0]) and list(dst) == list(ref_moves[1])
        # same kernels, same split, same summation order: bit for bit
        assert np.array_equal(g.logits(n).view(np.uint32), ref_logits.view(np.uint32))
        assert np.array_equal(g.features(ref[0] + 1).view(np.uint32), ref_feat.view(np.uint32))
        for l in range(s.n_layers):
            k, v = g.read_kv(l, L, ref[0] + 1)
            assert np.array_equal(k, ref_kv[l][0]) and np.array_equal(v, ref_kv[l][1])
        g.rollback(L, root)
    g.close()


def test_noalloc_entry_point_refuses_what_exceeds_its_scratch():
    import paper_2412_12639_amd as m
    s = fi.SHAPES["small-gqa"]
    g = m.FalconVerifier(s, max_seq=400, max_tree=128)
    g.init_weights(fi.gen_weights(s, seed=0))
    root = g.prefill(fi.gen_prefix(9, 40, s.vocab))
    tok, parent, depth = _tree(3, 65, s.vocab, root)
    with pytest.raises(m.FvError) as ei:
        g.verify_tree(tok, parent, depth, noalloc=True)
    assert ei.value.status == -11 and g.state() == (40, root)
    a, acc, nxt = g.verify_tree(tok[:1], parent[:1], depth[:1], noalloc=True)   # and still works afterwards
    assert a == 0 and g.state() == (41, nxt)
    g.close()


def test_noalloc_entry_point_refuses_a_prefix_whose_far_key_parts_exceed_its_slots():
    """With step-invariant rows on, the far keys of a step are cut into parts at fixed positions, one slot each;
    the static array holds eight slots per item, which a prefix of 1500 tokens exceeds."""
    import paper_2412_12639_amd as m
    s = fi.SHAPES["small-gqa"]
    L = 1500
    g = m.FalconVerifier(s, max_seq=L + 80, max_tree=64)
    g.init_weights(fi.gen_weights(s, seed=0))
    g.set_step_invariant(True)
    root = g.prefill(fi.gen_prefix(9, L, s.vocab))
    tok, parent, depth = _tree(3, 20, s.vocab, root)
    with pytest.raises(m.FvError) as ei:
        g.verify_tree(tok, parent, depth, noalloc=True)
    assert ei.value.status == -11 and g.state() == (L, root)
    a, acc, nxt = g.verify_tree(tok, parent, depth)   # the arena's scratch takes it
    assert g.state() == (L + a + 1, nxt)
    g.close()
