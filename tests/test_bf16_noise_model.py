"""The bf16 rounding-noise model used by the full-depth parity test (tests/bf16_noise_model.py) is
itself checked here, on the CPU: its rounding against a library conversion, and that with every
rounding switched off it is the oracle, and with them on it still is the same method."""
import numpy as np
import pytest
import torch

import fv_inputs as fi
from fv_inputs.shapes import ModelShape
from fv_inputs.trees import fill_tokens
from oracle import falcon_oracle as fo
from tests import bf16_noise_model as nm

SMALL = ModelShape("pin-gqa", 2, 128, 4, 2, 32, 176, 300, "f32")


@pytest.fixture(scope="module")
def small():
    return SMALL, fi.gen_weights(SMALL, seed=5, gain_jitter=0.1), fi.gen_prefix(5, 19, SMALL.vocab)


def _tree(s, w, prefix, seed, n, br, plant_len):
    o = fo.Oracle(s, w, max_seq=len(prefix) + n + 16)
    root = o.prefill(prefix)
    greedy = fo.greedy_decode(s, w, list(prefix) + [root], plant_len + 1)
    parent, depth, planted = fi.gen_tree(seed, n, br, plant_len)
    tok = fill_tokens(seed, parent, s.vocab, root, planted, greedy[:plant_len])
    return o, root, parent, depth, tok


def test_round_bf16_matches_library_conversion():
    """Round-to-nearest-even to bf16, against torch's conversion: random values over many binades,
    exact ties in both directions, signed zeros, values that round up into the next binade."""
    rng = np.random.default_rng(0)
    x = (rng.standard_normal(20000) * np.exp(rng.uniform(-30, 30, 20000))).astype(np.float32)
    ties = np.array([0x3F808000, 0x3F818000, 0xBF808000, 0xBF818000, 0x3FFF8000, 0x3FFFFFFF, 0x00000000, 0x80000000,
                     0x3F807FFF, 0x3F808001], dtype=np.uint32).view(np.float32)
    x = np.concatenate([x, ties])
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    got = nm.round_bf16(x)
    assert got.dtype == np.float32 and np.array_equal(got.view(np.uint32), ref.view(np.uint32))
    got64 = nm.round_bf16(x.astype(np.float64))
    assert got64.dtype == np.float64 and np.array_equal(got64, ref.astype(np.float64))
    # the two tie cases by hand: 1 + 2^-8 is halfway between 1 and 1 + 2^-7 -> even mantissa (1.0);
    # 1 + 3*2^-8 is halfway between 1 + 2^-7 and 1 + 2^-6 -> even mantissa (1 + 2^-6)
    assert nm.round_bf16(np.float32(1 + 2.0 ** -8)) == 1.0
    assert nm.round_bf16(np.float32(1 + 3 * 2.0 ** -8)) == np.float32(1 + 2.0 ** -6)


def test_without_rounding_the_model_is_the_oracle(small):
    s, w, prefix = small
    o, root, parent, depth, tok = _tree(s, w, prefix, 0, 16, [4, 2, 1, 1], 3)
    m = nm.StorageNoiseModel(s, w, max_seq=len(prefix) + 40, rounded=())
    assert m.prefill(prefix) == root
    assert np.max(np.abs(m.last_logits - o.last_logits)) < 1e-11
    r, rm = o.verify_tree(tok, parent, depth), m.verify_tree(tok, parent, depth)
    assert np.max(np.abs(rm["logits"] - r["logits"])) < 1e-11 * np.max(np.abs(r["logits"]))
    assert rm["accepted_len"] == r["accepted_len"] == 3 and list(rm["path"]) == list(r["path"])
    with pytest.raises(ValueError):
        nm.StorageNoiseModel(s, w, max_seq=8, rounded=("fp8",))


def test_with_rounding_it_is_still_the_same_method(small):
    """Every node's logits are those of a plain prefill (same rounding) over prefix ++ root path, a
    chain reproduces single-token decoding, and the result sits at rounding distance from the exact
    one: not equal, not far.  Each tensor class on its own moves the logits, and less than all together."""
    s, w, prefix = small
    o, root, parent, depth, tok = _tree(s, w, prefix, 0, 16, [4, 2, 1, 1], 3)
    exact = o.tree_logits(tok, parent, depth)[0]
    mb = nm.StorageNoiseModel(s, w, max_seq=len(prefix) + 40)
    rootb = mb.prefill(prefix)
    tok_b = np.array(tok).copy()
    tok_b[0] = rootb
    rb = mb.verify_tree(tok_b, parent, depth)
    if rootb == root:
        err = np.max(np.abs(rb["logits"] - exact), axis=-1) / np.max(np.abs(exact), axis=-1)
        assert 1e-4 < err.max() < 2e-2
        for cls in nm.ALL_CLASSES:
            m1 = nm.StorageNoiseModel(s, w, max_seq=len(prefix) + 40, rounded=(cls,))
            m1.prefill(prefix)
            m1.rollback(len(prefix), root)
            e1 = np.max(np.abs(m1.tree_logits(tok, parent, depth)[0] - exact), axis=-1) / np.max(np.abs(exact), axis=-1)
            assert 1e-6 < e1.max() < err.max() * 1.5, cls
    for i in (0, 3, 9, 15):
        seq = list(prefix) + [int(tok_b[j]) for j in fo.root_path(parent, i)]
        m2 = nm.StorageNoiseModel(s, w, max_seq=len(seq) + 4)
        m2.prefill(seq)
        ref = m2.last_logits[-1]
        assert np.max(np.abs(rb["logits"][i] - ref)) < 1e-9 * np.max(np.abs(ref))
    m3 = nm.StorageNoiseModel(s, w, max_seq=len(prefix) + 40)
    t0 = m3.prefill(prefix)
    seq, tk = [], t0
    p1, d1 = fi.chain_tree(1)
    for _ in range(4):
        tk = m3.verify_tree(np.array([tk], dtype=np.int32), p1, d1)["next_token"]
        seq.append(tk)
    m3.rollback(len(prefix), t0)
    pc, dc = fi.chain_tree(4)
    rc = m3.verify_tree(np.array([t0] + seq[:3], dtype=np.int32), pc, dc)
    assert rc["accepted_len"] == 3 and rc["next_token"] == seq[3]
