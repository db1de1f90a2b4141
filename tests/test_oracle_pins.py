"""Pins for the CPU oracle: each check compares it with something it does not compute
itself -- a library implementation of the same decoder, closed forms, brute force,
or an invariant the method fixes."""
import math

import numpy as np
import pytest
import torch

import fv_inputs as fi
from fv_inputs.shapes import ModelShape
from fv_inputs.trees import fill_tokens
from oracle import falcon_oracle as fo


def _f32(shape, seed=0, jitter=0.1):
    return fi.gen_weights(shape, seed=seed, gain_jitter=jitter)


# ------------------------------------------------------------------ library pins

@pytest.mark.parametrize("hq,hkv", [(4, 4), (8, 2)])
def test_causal_forward_matches_library_llama(hq, hkv):
    """The decoder definition against the transformers Llama implementation (fp64),
    random weights, multi-head and grouped-query variants.  Pins RMSNorm (eps place,
    gain), rotate-half rotary pairing and angle, KV-head grouping, causal softmax
    scale, SwiGLU, residual order and the untied head."""
    from transformers import LlamaConfig, LlamaForCausalLM
    s = ModelShape("pin", 2, hq * 16, hq, hkv, 16, 160, 211, "f32")
    w = _f32(s, seed=11)
    cfg = LlamaConfig(vocab_size=s.vocab, hidden_size=s.hidden, intermediate_size=s.ffn,
                      num_hidden_layers=s.n_layers, num_attention_heads=hq, num_key_value_heads=hkv,
                      head_dim=s.head_dim, max_position_embeddings=256, rms_norm_eps=s.rms_eps,
                      rope_theta=s.rope_base, attention_bias=False, mlp_bias=False,
                      tie_word_embeddings=False, attn_implementation="eager")
    m = LlamaForCausalLM(cfg).double().eval()
    sd = {"model.embed_tokens.weight": w["embed"], "model.norm.weight": w["g_final"], "lm_head.weight": w["lm_head"]}
    names = dict(wq="self_attn.q_proj", wk="self_attn.k_proj", wv="self_attn.v_proj", wo="self_attn.o_proj",
                 wg="mlp.gate_proj", wu="mlp.up_proj", wd="mlp.down_proj",
                 g_attn="input_layernorm", g_mlp="post_attention_layernorm")
    for l in range(s.n_layers):
        for k, hf in names.items():
            sd[f"model.layers.{l}.{hf}.weight"] = w[f"l{l}.{k}"]
    missing = m.load_state_dict({k: torch.from_numpy(np.asarray(v, dtype=np.float64)) for k, v in sd.items()}, strict=False)
    assert not [k for k in missing.missing_keys if "rotary" not in k]
    toks = fi.gen_prefix(2, 23, s.vocab)
    with torch.no_grad():
        out = m(torch.from_numpy(toks.astype(np.int64))[None], output_hidden_states=True)
        ref = out.logits[0].numpy()
        ref_hidden = out.hidden_states[-1][0].numpy()   # the library's last hidden state: after its final norm
    got, hidden = fo.causal_forward(s, w, toks, return_hidden=True)
    assert got.shape == ref.shape
    assert np.max(np.abs(hidden - ref_hidden)) / np.max(np.abs(ref_hidden)) < 1e-6
    # the library builds its rotary tables in fp32, which caps the agreement near 1e-7
    assert np.max(np.abs(got - ref)) < 1e-6 * np.max(np.abs(ref))


def test_rmsnorm_silu_softmax_against_library():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((5, 64))
    g = rng.standard_normal(64)
    ref = torch.nn.functional.rms_norm(torch.from_numpy(x), (64,), torch.from_numpy(g), eps=1e-5).numpy()
    assert np.allclose(fo.rmsnorm(x, g, 1e-5), ref, rtol=0, atol=1e-13)
    assert np.allclose(fo.silu(x), torch.nn.functional.silu(torch.from_numpy(x)).numpy(), atol=1e-14)
    assert np.allclose(fo.softmax_lastaxis(x), torch.softmax(torch.from_numpy(x), -1).numpy(), atol=1e-15)


def test_rope_closed_forms():
    # d = 4: pairs (0,2) at angle pos, (1,3) at angle pos * base^(-1/2)
    x = np.array([[[1.0, 2.0, 3.0, 4.0]]])
    base, pos = 100.0, 3
    y = fo.rope(x, [pos], base)[0, 0]
    a0, a1 = pos * 1.0, pos * base ** -0.5
    want = [1 * math.cos(a0) - 3 * math.sin(a0), 2 * math.cos(a1) - 4 * math.sin(a1),
            3 * math.cos(a0) + 1 * math.sin(a0), 4 * math.cos(a1) + 2 * math.sin(a1)]
    assert np.allclose(y, want, atol=1e-14)
    rng = np.random.default_rng(3)
    q, k = rng.standard_normal((1, 2, 64)), rng.standard_normal((1, 2, 64))
    assert np.allclose(fo.rope(q, [0], 10000.0), q)                                    # position 0 is the identity
    assert np.allclose(np.linalg.norm(fo.rope(q, [977], 10000.0)), np.linalg.norm(q))  # a rotation
    d1 = np.sum(fo.rope(q, [40], 1e4) * fo.rope(k, [33], 1e4), -1)
    d2 = np.sum(fo.rope(q, [1007], 1e4) * fo.rope(k, [1000], 1e4), -1)
    assert np.allclose(d1, d2, atol=1e-10)                                             # only pos_q - pos_k matters


def test_first_argmax_ties_and_nan():
    assert fo.first_argmax(np.array([1.0, 5.0, 5.0, 2.0])) == 1
    with pytest.raises(FloatingPointError):
        fo.first_argmax(np.array([1.0, np.nan]))


# ------------------------------------------------------------------ mask closed forms (bit-exact)

def _bits(words):
    return [j for j in range(256) if (int(words[j // 64]) >> (j % 64)) & 1]


@pytest.mark.parametrize("n,br", [(16, [4, 2, 1, 1]), (64, [8, 4, 2, 2, 1, 1]), (256, [8, 8, 4, 2, 2, 2, 1, 1])])
def test_ancestor_mask_closed_forms(n, br):
    parent, depth, _ = fi.gen_tree(1, n, br)
    m = fo.ancestor_mask(parent)
    assert m.shape == (n, 4) and m.dtype == np.uint64
    for i in range(n):
        b = _bits(m[i])
        assert len(b) == depth[i] + 1                       # popcount = depth + 1
        assert [int(depth[j]) for j in b] == list(range(depth[i] + 1))  # one node per level, in order
        assert b[-1] == i
        for j in b:                                           # ancestors' sets are subsets
            assert all((int(m[j][w]) & ~int(m[i][w])) == 0 for w in range(4))
        if i:
            x = [int(m[i][w]) ^ int(m[parent[i]][w]) for w in range(4)]
            assert x[i // 64] == 1 << (i % 64) and sum(v != 0 for v in x) == 1
    # chain: mask[i] = all ones up to bit i
    cp, _ = fi.chain_tree(130)
    cm = fo.ancestor_mask(cp)
    assert _bits(cm[129]) == list(range(130)) and int(cm[63][0]) == 2 ** 64 - 1 and int(cm[63][1]) == 0


# ------------------------------------------------------------------ method invariants on the tiny config

TINY = fi.SHAPES["tiny"]
SMALL = ModelShape("pin-gqa", 2, 128, 4, 2, 32, 176, 300, "f32")


@pytest.fixture(scope="module")
def tiny():
    w = _f32(TINY, seed=0)
    prefix = fi.gen_prefix(0, 64, TINY.vocab)
    return TINY, w, prefix


@pytest.fixture(scope="module")
def small():
    w = _f32(SMALL, seed=5)
    prefix = fi.gen_prefix(5, 19, SMALL.vocab)
    return SMALL, w, prefix


def _planted_tree(s, w, prefix, seed, n, br, plant_len):
    o = fo.Oracle(s, w, max_seq=len(prefix) + n + 16)
    root = o.prefill(prefix)
    greedy = fo.greedy_decode(s, w, list(prefix) + [root], plant_len + 1)
    parent, depth, planted = fi.gen_tree(seed, n, br, plant_len)
    # keep non-planted children away from their parent's greedy token: needs the parent's
    # greedy choice, known here only along the planted path
    avoid = {i: set() for i in range(n)}
    for i in range(1, n):
        if parent[i] in list(planted):
            j = list(planted).index(parent[i])
            avoid[i].add(greedy[j])
    tok = fill_tokens(seed, parent, s.vocab, root, planted, greedy[:plant_len], avoid)
    return o, root, greedy, parent, depth, planted, tok


def test_prefill_equals_full_forward(tiny):
    s, w, prefix = tiny
    o = fo.Oracle(s, w, max_seq=80)
    nxt = o.prefill(prefix)
    ref = fo.causal_forward(s, w, prefix)
    assert np.max(np.abs(o.last_logits - ref)) < 1e-11
    assert nxt == int(np.argmax(ref[-1]))


@pytest.mark.parametrize("which", ["tiny", "small"])
def test_node_logits_equal_full_forward_over_root_path(which, tiny, small):
    """Brute force: each node's logits are the last row of a from-scratch causal
    forward over prefix ++ tokens on its root path."""
    s, w, prefix = tiny if which == "tiny" else small
    o, root, greedy, parent, depth, planted, tok = _planted_tree(s, w, prefix, 0, 16, [4, 2, 1, 1], 4)
    r = o.verify_tree(tok, parent, depth)
    for i in range(16):
        seq = list(prefix) + [int(tok[j]) for j in fo.root_path(parent, i)]
        ref = fo.causal_forward(s, w, seq)[-1]
        assert np.max(np.abs(r["logits"][i] - ref)) < 1e-10 * np.max(np.abs(ref))


def test_planted_path_is_accepted(tiny):
    s, w, prefix = tiny
    o, root, greedy, parent, depth, planted, tok = _planted_tree(s, w, prefix, 0, 16, [4, 2, 1, 1], 4)
    r = o.verify_tree(tok, parent, depth)
    assert r["accepted_len"] == 4
    assert list(r["accepted_tokens"]) == greedy[:4]
    assert r["next_token"] == greedy[4]
    assert list(r["path"]) == list(planted)
    assert list(r["src_slot"]) == list(planted) and list(r["dst_slot"]) == [64 + j for j in range(5)]
    assert o.L == 64 + 5 and o.pending == greedy[4]


def test_chain_reproduces_greedy_decoding(small):
    """A chain tree is plain speculative decoding with one candidate; root-only trees
    are vanilla decoding.  Both must emit the target's own greedy sequence."""
    s, w, prefix = small
    o = fo.Oracle(s, w, max_seq=64)
    root = o.prefill(prefix)
    greedy = fo.greedy_decode(s, w, list(prefix) + [root], 9)
    # (a) T = 1 steps: token-for-token
    out = []
    tokn = root
    for _ in range(6):
        p, d = fi.chain_tree(1)
        r = o.verify_tree(np.array([tokn]), p, d)
        assert r["accepted_len"] == 0 and len(r["accepted_tokens"]) == 0
        tokn = r["next_token"]
        out.append(tokn)
    assert out == greedy[:6]
    # (b) a fully correct chain is accepted whole
    o2 = fo.Oracle(s, w, max_seq=64)
    assert o2.prefill(prefix) == root
    p, d = fi.chain_tree(6)
    r = o2.verify_tree(np.array([root] + greedy[:5]), p, d)
    assert r["accepted_len"] == 5 and list(r["accepted_tokens"]) == greedy[:5] and r["next_token"] == greedy[5]
    # (c) a chain that goes wrong at draft position 3 is accepted up to there
    o3 = fo.Oracle(s, w, max_seq=64)
    o3.prefill(prefix)
    bad = [root] + greedy[:5]
    bad[3] = (bad[3] + 1) % s.vocab
    r = o3.verify_tree(np.array(bad), p, d)
    assert r["accepted_len"] == 2 and list(r["accepted_tokens"]) == greedy[:2] and r["next_token"] == greedy[2]


def test_accepted_tokens_are_prefix_of_greedy_for_random_trees(small):
    s, w, prefix = small
    o = fo.Oracle(s, w, max_seq=128)
    root = o.prefill(prefix)
    greedy = fo.greedy_decode(s, w, list(prefix) + [root], 8)
    rng = np.random.default_rng(0)
    for seed in range(6):
        parent, depth, planted = fi.gen_tree(seed, 24, [3, 3, 2, 2, 1, 1], plant_len=seed % 4)
        tok = fill_tokens(seed, parent, s.vocab, root, planted, greedy[:seed % 4])
        # sprinkle more greedy tokens at random nodes (some land on accepted paths, some not)
        for i in rng.integers(1, 24, size=6):
            tok[i] = greedy[depth[i] - 1]
        o.rollback(len(prefix), root)
        r = o.verify_tree(tok, parent, depth)
        emitted = list(r["accepted_tokens"]) + [r["next_token"]]
        assert emitted == greedy[:len(emitted)]
        assert r["accepted_len"] >= seed % 4


def test_cache_after_compaction_equals_fresh_prefill(small):
    s, w, prefix = small
    o, root, greedy, parent, depth, planted, tok = _planted_tree(s, w, prefix, 3, 20, [3, 2, 2, 1], 3)
    r = o.verify_tree(tok, parent, depth)
    assert r["accepted_len"] == 3
    n = len(prefix) + 4
    o2 = fo.Oracle(s, w, max_seq=64)
    nxt = o2.prefill(list(prefix) + [root] + greedy[:3])
    assert nxt == r["next_token"]
    assert np.max(np.abs(o.K[:, :n] - o2.K[:, :n])) < 1e-12
    assert np.max(np.abs(o.V[:, :n] - o2.V[:, :n])) < 1e-12
    # and decoding continues identically from the compacted cache
    p1, d1 = fi.chain_tree(1)
    a = o.verify_tree(np.array([r["next_token"]]), p1, d1)
    b = o2.verify_tree(np.array([nxt]), p1, d1)
    g5 = fo.greedy_decode(s, w, list(prefix) + [root], 5)
    assert g5[:4] == greedy and a["next_token"] == b["next_token"] == g5[4]
    assert np.max(np.abs(a["logits"] - b["logits"])) < 1e-11


def test_relabelling_and_pruning_leave_results_unchanged(small):
    s, w, prefix = small
    o, root, greedy, parent, depth, planted, tok = _planted_tree(s, w, prefix, 4, 20, [3, 2, 2, 1], 2)
    r = o.verify_tree(tok, parent, depth)
    # (a) another topological order: reverse the order inside every depth level
    order = sorted(range(20), key=lambda i: (depth[i], -i))
    new_of = {old: new for new, old in enumerate(order)}
    p2 = np.array([-1 if parent[old] < 0 else new_of[parent[old]] for old in order], dtype=np.int32)
    o.rollback(len(prefix), root)
    r2 = o.verify_tree(tok[order], p2, depth[order])
    assert np.max(np.abs(r2["logits"] - r["logits"][order])) < 1e-12
    assert list(r2["accepted_tokens"]) == list(r["accepted_tokens"]) and r2["next_token"] == r["next_token"]
    # (b) delete every node that is not on node 19's root path or the planted path
    keep = sorted(set(fo.root_path(parent, 19)) | set(int(i) for i in planted))
    new_of = {old: new for new, old in enumerate(keep)}
    p3 = np.array([-1 if parent[old] < 0 else new_of[parent[old]] for old in keep], dtype=np.int32)
    o.rollback(len(prefix), root)
    r3 = o.verify_tree(tok[keep], p3, depth[keep])
    # (the library matmul blocks differently for another row count: rounding-level only)
    assert np.max(np.abs(r3["logits"] - r["logits"][keep])) < 1e-12
    assert list(r3["accepted_tokens"]) == list(r["accepted_tokens"])


def test_single_node_and_empty_acceptance(tiny):
    s, w, prefix = tiny
    o = fo.Oracle(s, w, max_seq=96)
    root = o.prefill(prefix)
    ref = fo.causal_forward(s, w, list(prefix) + [root])[-1]
    p, d = fi.chain_tree(1)
    r = o.verify_tree(np.array([root]), p, d)
    assert r["accepted_len"] == 0 and r["next_token"] == int(np.argmax(ref)) and o.L == 65
    assert np.max(np.abs(r["logits"][0] - ref)) < 1e-11
    # all draft tokens wrong
    o.rollback(64, root)
    parent, depth, _ = fi.gen_tree(2, 16, [4, 2, 1, 1])
    wrong = (int(np.argmax(ref)) + 1 + np.arange(16)) % s.vocab
    wrong[0] = root
    r = o.verify_tree(wrong.astype(np.int32), parent, depth)
    assert r["accepted_len"] == 0 and r["next_token"] == int(np.argmax(ref)) and o.L == 65
    assert list(r["src_slot"]) == [0] and list(r["dst_slot"]) == [64]


def test_equal_siblings_get_equal_logits(tiny):
    s, w, prefix = tiny
    o = fo.Oracle(s, w, max_seq=96)
    root = o.prefill(prefix)
    parent = np.array([-1, 0, 0, 1, 2], dtype=np.int32)
    depth = fi.tree_depths(parent)
    tok = np.array([root, 5, 5, 9, 9], dtype=np.int32)
    r = o.verify_tree(tok, parent, depth)
    assert np.array_equal(r["logits"][1], r["logits"][2]) and np.array_equal(r["logits"][3], r["logits"][4])
    # a different position changes the logits: same token one level deeper
    assert not np.allclose(r["logits"][1], r["logits"][3])


def test_tie_between_equal_depth_paths_takes_lowest_index(tiny):
    s, w, prefix = tiny
    o = fo.Oracle(s, w, max_seq=96)
    root = o.prefill(prefix)
    g = fo.greedy_decode(s, w, list(prefix) + [root], 1)[0]
    parent = np.array([-1, 0, 0], dtype=np.int32)
    r = o.verify_tree(np.array([root, g, g], dtype=np.int32), parent, fi.tree_depths(parent))
    assert r["accepted_len"] == 1 and list(r["path"]) == [0, 1]


@pytest.mark.parametrize("bad", ["order", "depth", "token", "root", "full", "noroot"])
def test_invalid_trees_are_rejected_without_state_change(bad, tiny):
    s, w, prefix = tiny
    o = fo.Oracle(s, w, max_seq=70)
    root = o.prefill(prefix)
    parent = np.array([-1, 0, 1, 1], dtype=np.int32)
    depth = np.array([0, 1, 2, 2], dtype=np.int32)
    tok = np.array([root, 1, 2, 3], dtype=np.int32)
    if bad == "order":
        parent[2] = 3
    elif bad == "depth":
        depth[3] = 1
    elif bad == "token":
        tok[2] = s.vocab
    elif bad == "root":
        tok[0] = (root + 1) % s.vocab
    elif bad == "noroot":
        parent[0] = 0
    elif bad == "full":
        parent, depth = fi.chain_tree(7)
        tok = np.array([root] + [1] * 6, dtype=np.int32)
    with pytest.raises(fo.TreeVerifyError):
        o.verify_tree(tok, parent, depth)
    assert o.L == 64 and o.pending == root


def test_fp32_working_precision_stays_close(tiny):
    s, w, prefix = tiny
    a = fo.causal_forward(s, w, prefix[:20], dtype=np.float64)
    b = fo.causal_forward(s, w, prefix[:20], dtype=np.float32)
    assert np.max(np.abs(a - b)) < 1e-4 * np.max(np.abs(a))


def test_bf16_weights_are_consumed_bit_exactly():
    s16 = fi.SHAPES["tiny-bf16"]
    w16 = fi.gen_weights(s16, seed=0)
    w32 = {k: (fi.f32_from_bf16_bits(v) if v.dtype == np.uint16 else v) for k, v in w16.items()}
    toks = fi.gen_prefix(1, 9, s16.vocab)
    assert np.array_equal(fo.causal_forward(s16, w16, toks), fo.causal_forward(fi.SHAPES["tiny"], w32, toks))


def test_features_are_the_lm_head_input(small):
    """The features returned with the accepted tokens: multiplying them by the LM head gives the
    path nodes' logits back (closed form), and they equal the final hidden state of a from-scratch
    causal forward over prefix ++ root path (brute force)."""
    s, w, prefix = small
    o, root, greedy, parent, depth, planted, tok = _planted_tree(s, w, prefix, 0, 16, [4, 2, 1, 1], 3)
    r = o.verify_tree(tok, parent, depth)
    f = r["features"]
    assert f.shape == (r["accepted_len"] + 1, s.hidden) and r["accepted_len"] == 3
    back = f @ fo._up(w["lm_head"], np.float64).T
    assert np.max(np.abs(back - r["logits"][r["path"]])) < 1e-10
    for j, node in enumerate(r["path"]):
        seq = list(prefix) + [int(tok[k]) for k in fo.root_path(parent, int(node))]
        _, hid = fo.causal_forward(s, w, seq, return_hidden=True)
        assert np.max(np.abs(hid[-1] - f[j])) < 1e-10 * np.max(np.abs(hid[-1]))


# ------------------------------------------------------------------ the acceptance rule as a pure function

def _accept_by_enumeration(tokens, parent, depth, argmax):
    """Independent statement of the rule: enumerate every root path, keep those whose every
    non-root node carries the target's choice at its parent, take the longest (lowest end node
    among equally long ones)."""
    T = len(tokens)
    best_path = [0]
    for end in range(T):
        path, j = [], end
        while j >= 0:
            path.append(j)
            j = int(parent[j])
        path = path[::-1]
        ok = all(int(tokens[c]) == int(argmax[p]) for p, c in zip(path[:-1], path[1:]))
        if ok and len(path) > len(best_path):
            best_path = path
    return best_path


def test_greedy_accept_hand_made_cases():
    """Values worked out by hand.  Tree: 0 -> (1, 2); 1 -> (3, 4); 2 -> 5; 3 -> 6."""
    parent = np.array([-1, 0, 0, 1, 1, 2, 3], dtype=np.int32)
    depth = np.array([0, 1, 1, 2, 2, 2, 3], dtype=np.int32)
    tok = np.array([10, 11, 12, 13, 14, 15, 16], dtype=np.int32)
    # target picks 11 after the root, 14 after node 1, 99 after node 4: path 0 -> 1 -> 4
    am = np.array([11, 14, 15, 16, 99, 7, 7], dtype=np.int32)
    r = fo.greedy_accept(tok, parent, depth, am, L=100)
    assert r["accepted_len"] == 2 and list(r["path"]) == [0, 1, 4]
    assert list(r["accepted_tokens"]) == [11, 14] and r["next_token"] == 99
    assert list(r["src_slot"]) == [0, 1, 4] and list(r["dst_slot"]) == [100, 101, 102]
    # node 5 matches its parent's choice (15) but its parent (node 2) is not accepted: not taken
    assert 5 not in r["path"]
    # nothing matches: only the root, bonus token = the choice at the root
    am0 = np.array([77, 14, 15, 16, 99, 7, 7], dtype=np.int32)
    r = fo.greedy_accept(tok, parent, depth, am0, L=5)
    assert r["accepted_len"] == 0 and list(r["path"]) == [0] and r["next_token"] == 77
    assert len(r["accepted_tokens"]) == 0 and list(r["dst_slot"]) == [5]
    # a full-depth path: 0 -> 1 -> 3 -> 6
    am3 = np.array([11, 13, 0, 16, 0, 0, 42], dtype=np.int32)
    r = fo.greedy_accept(tok, parent, depth, am3, L=0)
    assert r["accepted_len"] == 3 and list(r["path"]) == [0, 1, 3, 6] and r["next_token"] == 42
    # a single node
    r = fo.greedy_accept(np.array([3]), np.array([-1]), np.array([0]), np.array([8]), L=9)
    assert r["accepted_len"] == 0 and r["next_token"] == 8 and list(r["dst_slot"]) == [9]
    # equal siblings, both matching: the lower index wins
    r = fo.greedy_accept(np.array([1, 2, 2]), np.array([-1, 0, 0]), np.array([0, 1, 1]), np.array([2, 5, 6]), L=0)
    assert list(r["path"]) == [0, 1] and r["next_token"] == 5


def test_greedy_accept_chains_and_random_trees_against_enumeration():
    rng = np.random.default_rng(7)
    # chain whose first m draft tokens are right
    for n, m in [(1, 0), (6, 0), (6, 3), (6, 5), (40, 17)]:
        parent, depth = fi.chain_tree(n)
        am = rng.integers(0, 50, size=n).astype(np.int32)
        tok = np.zeros(n, dtype=np.int32)
        tok[1:] = am[:-1]
        if m + 1 < n:
            tok[m + 1] = (am[m] + 1) % 50
        r = fo.greedy_accept(tok, parent, depth, am, L=3)
        assert r["accepted_len"] == min(m, n - 1) and list(r["path"]) == list(range(min(m, n - 1) + 1))
        assert r["next_token"] == am[min(m, n - 1)]
    # random trees with a small vocabulary, so that matches are frequent and paths branch
    for seed in range(40):
        n = int(rng.integers(2, 60))
        parent, depth, _ = fi.gen_tree(seed, n, [3, 3, 2, 2, 2, 1, 1, 1])
        tok = rng.integers(0, 3, size=n).astype(np.int32)
        am = rng.integers(0, 3, size=n).astype(np.int32)
        r = fo.greedy_accept(tok, parent, depth, am, L=11)
        want = _accept_by_enumeration(tok, parent, depth, am)
        assert list(r["path"]) == want, (seed, list(r["path"]), want)
        assert r["accepted_len"] == len(want) - 1 == depth[want[-1]]
        assert list(r["accepted_tokens"]) == [int(tok[j]) for j in want[1:]]
        assert r["next_token"] == am[want[-1]]
        assert list(r["src_slot"]) == want and list(r["dst_slot"]) == list(range(11, 11 + len(want)))
        # the set bits of the best node's ancestor mask are the path (what the library's scan uses)
        m = fo.ancestor_mask(parent)[want[-1]]
        assert _bits(m) == want


def test_greedy_accept_is_invariant_under_relabelling():
    rng = np.random.default_rng(3)
    for seed in range(10):
        parent, depth, _ = fi.gen_tree(seed, 30, [3, 2, 2, 2, 1, 1])
        tok = rng.integers(0, 3, size=30).astype(np.int32)
        am = rng.integers(0, 3, size=30).astype(np.int32)
        # siblings distinct, so that the accepted path is unique whatever the node order
        for i in range(1, 30):
            sib = [j for j in range(1, i) if parent[j] == parent[i]]
            while any(tok[j] == tok[i] for j in sib):
                tok[i] += 3
        r = fo.greedy_accept(tok, parent, depth, am, L=0)
        order = sorted(range(30), key=lambda i: (depth[i], -i))
        new_of = {old: new for new, old in enumerate(order)}
        p2 = np.array([-1 if parent[o] < 0 else new_of[parent[o]] for o in order], dtype=np.int32)
        r2 = fo.greedy_accept(tok[order], p2, depth[order], am[order], L=0)
        assert list(r2["accepted_tokens"]) == list(r["accepted_tokens"]) and r2["next_token"] == r["next_token"]
        assert [order[j] for j in r2["path"]] == list(r["path"])


def test_top2_margin_against_sorted_array():
    rng = np.random.default_rng(1)
    for _ in range(20):
        row = rng.standard_normal(int(rng.integers(2, 500)))
        srt = np.sort(row)
        assert fo.top2_margin(row) == float(srt[-1] - srt[-2])
    assert fo.top2_margin(np.array([1.0, 4.0, 4.0, -2.0])) == 0.0          # maximum attained twice
    assert fo.top2_margin(np.array([3.0, -1.0])) == 4.0
    assert fo.top2_margin(np.array([-5.0, -7.0, -6.0])) == 1.0              # all negative
    assert fo.top2_margin(np.array([2.0, 9.0, 9.0, 9.0])) == 0.0


def test_verify_tree_uses_the_acceptance_function(tiny):
    """verify_tree's decisions are greedy_accept of its own argmax; tree_logits leaves the state alone."""
    s, w, prefix = tiny
    o, root, greedy, parent, depth, planted, tok = _planted_tree(s, w, prefix, 0, 16, [4, 2, 1, 1], 2)
    lg, nk, nv = o.tree_logits(tok, parent, depth)
    assert o.L == 64 and o.pending == root
    r = o.verify_tree(tok, parent, depth)
    assert np.array_equal(lg, r["logits"]) and np.array_equal(nk, r["tree_k"])
    d = fo.greedy_accept(tok, parent, depth, r["argmax"], 64)
    for key in ("accepted_len", "next_token"):
        assert d[key] == r[key]
    for key in ("path", "accepted_tokens", "src_slot", "dst_slot"):
        assert list(d[key]) == list(r[key])
    for j, node in enumerate(r["path"]):
        assert np.array_equal(o.K[:, 64 + j], r["tree_k"][:, node]) and np.array_equal(o.V[:, 64 + j], r["tree_v"][:, node])


# ------------------------------------------------------------------ non-greedy acceptance (multi-step speculative sampling)

def _softmax(z):
    e = np.exp(z - np.max(z))
    return e / e.sum()


def _chi2_ok(counts, probs, alpha=1e-4):
    from scipy.stats import chisquare
    keep = probs > 0
    assert counts[~keep].sum() == 0
    return chisquare(counts[keep], probs[keep] * counts.sum()).pvalue > alpha


def test_sampled_accept_emits_the_target_distribution_for_deterministic_children():
    """Point-mass proposals (top-m children): whatever the children are, the first emitted token is
    distributed as the target's softmax at the root, and the token after an accepted child as the
    target's softmax at that child (the guarantee the method rests on).  Seeded Monte Carlo, chi-square."""
    rng = np.random.default_rng(11)
    V = 7
    #        0
    #     1  2  3        tokens 4, 0, 6
    #    4 5    6        tokens 2, 3 | 1
    parent = np.array([-1, 0, 0, 0, 1, 1, 3], dtype=np.int32)
    depth = np.array([0, 1, 1, 1, 2, 2, 2], dtype=np.int32)
    tok = np.array([5, 4, 0, 6, 2, 3, 1], dtype=np.int32)
    logits = rng.standard_normal((7, V)) * 1.5
    temp = 0.8
    N = 60000
    first = np.zeros(V)
    second = {c: np.zeros(V) for c in (1, 2, 3)}
    for _ in range(N):
        r = fo.sampled_accept(logits, tok, parent, depth, 0, temp, rng.random(7), rng.random(7))
        em = list(r["accepted_tokens"]) + [r["next_token"]]
        first[em[0]] += 1
        if r["accepted_len"] >= 1:
            second[int(r["path"][1])][em[1]] += 1
        assert [int(tok[j]) for j in r["path"][1:]] == em[:-1] and r["accepted_len"] == depth[r["path"][-1]]
    assert _chi2_ok(first, _softmax(logits[0] / temp))
    for c in (1, 2, 3):
        assert second[c].sum() > 800 and _chi2_ok(second[c], _softmax(logits[c] / temp))
    # and a wrong rule is caught by this check: accepting with p[x] but NOT striking x on rejection
    # would over-produce the children's tokens -- the exact first-token law of that variant differs
    p = _softmax(logits[0] / temp)
    wrong = p.copy()
    rej = 1.0
    for x in (4, 0, 6):
        rej *= 1 - p[x]
    wrong = np.array([p[v] * rej for v in range(V)])
    acc_mass = 1.0
    for x in (4, 0, 6):
        wrong[x] += acc_mass * p[x]
        acc_mass *= 1 - p[x]
    assert abs(wrong.sum() - 1) < 1e-12 and not _chi2_ok(first, wrong)


def test_sampled_accept_with_a_draft_distribution():
    """Children drawn i.i.d. from the drafter's q: first emitted token still follows the target's p
    (q far from p, three children), and q == p accepts the first child always."""
    rng = np.random.default_rng(5)
    V = 6
    parent = np.array([-1, 0, 0, 0], dtype=np.int32)
    depth = np.array([0, 1, 1, 1], dtype=np.int32)
    logits = rng.standard_normal((4, V)) * 2.0
    p = _softmax(logits[0])
    q = _softmax(rng.standard_normal(V) * 2.0)
    draft = np.zeros((4, V))
    draft[0] = q
    N = 60000
    first = np.zeros(V)
    n_acc = 0
    for _ in range(N):
        tok = np.concatenate([[0], rng.choice(V, size=3, p=q)]).astype(np.int32)
        r = fo.sampled_accept(logits, tok, parent, depth, 0, 1.0, rng.random(4), rng.random(4), draft_probs=draft)
        em = list(r["accepted_tokens"]) + [r["next_token"]]
        first[em[0]] += 1
        n_acc += r["accepted_len"]
    assert _chi2_ok(first, p)
    assert 0.2 * N < n_acc < N            # some accepted, some resampled: both branches exercised
    draft[0] = p
    for _ in range(200):
        tok = np.concatenate([[0], rng.choice(V, size=3, p=p)]).astype(np.int32)
        r = fo.sampled_accept(logits, tok, parent, depth, 0, 1.0, rng.random(4), rng.random(4), draft_probs=draft)
        assert r["accepted_len"] == 1 and list(r["path"]) == [0, 1]


def test_sampled_accept_limits_and_inputs():
    rng = np.random.default_rng(2)
    V = 50
    # temperature -> 0 with deterministic children is greedy acceptance, for any uniforms
    for seed in range(20):
        n = 25
        parent, depth, _ = fi.gen_tree(seed, n, [3, 2, 2, 2, 1])
        logits = rng.standard_normal((n, V))
        am = np.argmax(logits, axis=-1).astype(np.int32)
        tok = rng.integers(0, V, size=n).astype(np.int32)
        for i in range(1, n):                    # make some paths right
            if rng.random() < 0.5:
                tok[i] = am[parent[i]]
        for i in range(1, n):                    # siblings distinct
            sib = [j for j in range(1, i) if parent[j] == parent[i]]
            while any(tok[j] == tok[i] for j in sib):
                tok[i] = (tok[i] + 1) % V
        g = fo.greedy_accept(tok, parent, depth, am, L=9)
        r = fo.sampled_accept(logits, tok, parent, depth, 9, 1e-3, rng.random(n), rng.random(n))
        assert list(r["path"]) == list(g["path"]) and r["next_token"] == g["next_token"]
        assert list(r["dst_slot"]) == list(g["dst_slot"]) and list(r["accepted_tokens"]) == list(g["accepted_tokens"])
    # a token the target gives (numerically) no mass is never accepted, and never drawn
    parent = np.array([-1, 0], dtype=np.int32)
    depth = np.array([0, 1], dtype=np.int32)
    logits = np.zeros((2, 4))
    logits[0, 2] = -1e4
    for _ in range(50):
        r = fo.sampled_accept(logits, np.array([0, 2]), parent, depth, 0, 1.0, rng.random(2), rng.random(2))
        assert r["accepted_len"] == 0 and r["next_token"] != 2
    # only the uniforms of tested children and of the node where the draw happens matter; hand-computed draw:
    # root p = (0.1, 0.2, 0.3, 0.4), child token 3 rejected at u = 0.9 -> p' = (1/6, 2/6, 3/6, 0); u_sample 0.6 -> token 2
    logits = np.log(np.array([[0.1, 0.2, 0.3, 0.4], [0.25, 0.25, 0.25, 0.25]]))
    r = fo.sampled_accept(logits, np.array([1, 3]), parent, depth, 7, 1.0, [0.123, 0.9], [0.6, 0.999])
    assert r["accepted_len"] == 0 and r["next_token"] == 2 and list(r["dst_slot"]) == [7]
    assert abs(r["min_margin"] - min(0.9 - 0.4, 0.6 - 0.5) / 0.9) < 1e-9 or r["min_margin"] > 0.05
    r = fo.sampled_accept(logits, np.array([1, 3]), parent, depth, 7, 1.0, [0.123, 0.39], [0.6, 0.7])   # accepted at u = 0.39 < 0.4
    assert r["accepted_len"] == 1 and list(r["accepted_tokens"]) == [3] and r["next_token"] == 2      # leaf: draw from uniform p at 0.7 -> token 2
    with pytest.raises(FloatingPointError):
        fo.sampled_accept(np.array([[0.0, np.nan]]), np.array([0]), np.array([-1]), np.array([0]), 0, 1.0, [0.5], [0.5])
