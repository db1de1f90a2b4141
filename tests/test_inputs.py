"""The seeded generators: determinism, distribution, bf16 rounding, tree validity."""
import numpy as np
import torch

import fv_inputs as fi
from fv_inputs.trees import fill_tokens


def test_bf16_rounding_matches_library_rne():
    rng = np.random.default_rng(1)
    x = (rng.standard_normal(200000) * 0.02).astype(np.float32)
    # exact ties and values next to them
    ties = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -0.5 - 2.0 ** -9, 3.0e-3], dtype=np.float32)
    x = np.concatenate([x, ties])
    ours = fi.bf16_bits_from_f32(x)
    lib = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(ours, lib)
    back = fi.f32_from_bf16_bits(ours)
    assert np.all(np.abs(back - x) <= np.abs(x) * 2.0 ** -8)


def test_weights_deterministic_and_layer_stable():
    s = fi.SHAPES["small-gqa"]
    a = fi.gen_weights(s, seed=3)
    b = fi.gen_weights(s, seed=3)
    assert all(np.array_equal(a[k], b[k]) for k in a)
    c = fi.gen_weights(s.with_layers(1), seed=3)
    assert all(np.array_equal(a[k], c[k]) for k in c)
    assert a["l0.wq"].dtype == np.uint16 and a["l0.wq"].shape == (8 * 128, 512)
    assert a["l0.wk"].shape == (2 * 128, 512) and a["l1.wd"].shape == (512, 1376)
    w = fi.f32_from_bf16_bits(a["l1.wg"])
    assert abs(w.std() - 0.02) < 5e-4 and abs(w.mean()) < 2e-4
    d = fi.gen_weights(s, seed=4)
    assert not np.array_equal(a["l0.wq"], d["l0.wq"])
    assert np.all(a["g_final"] == 1.0)
    j = fi.gen_weights(s, seed=3, gain_jitter=0.1)
    assert j["g_final"].std() > 0.05 and np.array_equal(j["l0.wq"], a["l0.wq"])


def _check_topology(parent, depth):
    assert parent[0] == -1 and depth[0] == 0
    for i in range(1, len(parent)):
        assert 0 <= parent[i] < i
        assert depth[i] == depth[parent[i]] + 1
    assert np.all(np.diff(depth) >= 0)  # depth-major numbering


def test_tree_generator_configs():
    p, d, pl = fi.gen_tree(0, 16, [4, 2, 1, 1], plant_len=4)
    _check_topology(p, d)
    assert len(p) == 16 and d.max() == 4 and list(d[pl]) == [0, 1, 2, 3, 4]
    for j in range(1, 5):
        assert p[pl[j]] == pl[j - 1]
    p, d, pl = fi.gen_tree(0, 64, [8, 4, 2, 2, 1, 1], plant_len=3)
    _check_topology(p, d)
    assert len(p) == 64 and d.max() <= 6
    for n in (16, 32, 64, 128, 256):
        br = fi.random_branching(5, n)
        p, d, _ = fi.gen_tree(5, n, br)
        _check_topology(p, d)
        assert len(p) == n and d.max() <= 8
    # children per node never exceed the branching of the parent's depth
    br = [8, 4, 2, 2, 1, 1]
    p, d, _ = fi.gen_tree(9, 64, br, 3)
    for i in range(64):
        assert np.sum(p == i) <= (br[d[i]] if d[i] < len(br) else 0)


def test_fill_tokens_siblings_distinct_and_planted():
    p, d, pl = fi.gen_tree(0, 64, [8, 4, 2, 2, 1, 1], plant_len=3)
    tok = fill_tokens(0, p, 50, root_token=7, planted=pl, plant_tokens=[11, 12, 13])
    assert tok[0] == 7 and [tok[i] for i in pl[1:]] == [11, 12, 13]
    for i in range(64):
        kids = tok[p == i]
        assert len(set(kids.tolist())) == len(kids)
    assert tok.min() >= 0 and tok.max() < 50


def test_step_bytes_headline():
    # 7B shape, prefix 512, 64 nodes: 13.2 GB of weights + 0.3 GB of K/V
    s = fi.SHAPES["7b"]
    assert s.weight_params() * 2 == 13_214_154_752
    assert abs(s.step_bytes(512, 64) / 1e9 - 13.52) < 0.01


def test_synthetic_drafter_plants_the_drawn_number_of_greedy_tokens():
    future = [5, 9, 2, 7, 7, 1, 3, 8]
    lens = []
    for seed in range(200):
        tok, parent, depth, n_ok = fi.draft_tree(seed, 4, future, 24, [3, 3, 2, 2, 1], 0.75, 50)
        assert tok[0] == 4 and len(tok) == 24 and all(parent[i] < i for i in range(1, 24))
        # walk the greedy path through the tree: exactly n_ok tokens match, then none
        node, k = 0, 0
        while k < len(future):
            nxt = [j for j in range(1, 24) if parent[j] == node and tok[j] == future[k]]
            if not nxt:
                break
            node, k = nxt[0], k + 1
        assert k == n_ok and n_ok <= 5
        lens.append(n_ok)
    assert 2.0 < np.mean(lens) < 3.2   # geometric with p = 0.75 capped at depth 5: mean about 2.3-2.6
