"""The C-ABI library loads and exports every symbol include/falcon_verify.h declares;
host-only entry points behave (no GPU needed, no compute calls)."""
import ctypes
import os
import re

import numpy as np
import pytest

import fv_inputs as fi

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2412_12639_amd import build, binding
    build.build(force=False)
    return binding.load_library()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "falcon_verify.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fv_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert "fv_verify_tree" in names and "fv_prefill" in names and "fv_init_weights" in names and len(names) >= 15
    for n in names:
        assert hasattr(lib, n), n
    raw = ctypes.CDLL(os.path.join(ROOT, "paper_2412_12639_amd", "libfalcon_verify.so"))
    for n in names:
        getattr(raw, n)


def test_workspace_bytes_and_bad_configs(lib):
    from paper_2412_12639_amd import binding as b
    s = fi.SHAPES["7b"]
    n = b.workspace_bytes(s, 2048 + 256, 256)
    weights = s.weight_params() * 2
    assert weights < n < weights + 6e9
    from dataclasses import replace
    for bad in (replace(s, head_dim=96), replace(s, hidden=4100), replace(s, ffn=11009), replace(s, n_kv_heads=5)):
        with pytest.raises(b.FvError):
            b.workspace_bytes(bad, 1024, 64)
    with pytest.raises(b.FvError):
        b.workspace_bytes(s, 1024, 257)


def test_validate_tree_codes(lib):
    from paper_2412_12639_amd import binding as b
    s = fi.SHAPES["tiny"]
    ok = ([5, 1, 2, 3], [-1, 0, 1, 1], [0, 1, 2, 2])
    assert b.validate_tree(s, 128, 64, *ok, 5, 64) == 0
    assert b.validate_tree(s, 128, 64, ok[0], [-1, 0, 2, 1], ok[2], 5, 64) == -2
    assert b.validate_tree(s, 128, 64, ok[0], [0, 0, 1, 1], ok[2], 5, 64) == -2
    assert b.validate_tree(s, 128, 64, ok[0], ok[1], [0, 1, 2, 1], 5, 64) == -3
    assert b.validate_tree(s, 128, 64, [5, 1, 2, 1000], ok[1], ok[2], 5, 64) == -4
    assert b.validate_tree(s, 128, 64, [5, 1, -2, 3], ok[1], ok[2], 5, 64) == -4
    assert b.validate_tree(s, 128, 3, *ok, 5, 64) == -5
    assert b.validate_tree(s, 66, 64, *ok, 5, 64) == -6
    assert b.validate_tree(s, 128, 64, *ok, 6, 64) == -7
    # same verdicts as the oracle's own input rules on random mutations of a valid tree
    from oracle import falcon_oracle as fo
    rng = np.random.default_rng(0)
    parent, depth, _ = fi.gen_tree(0, 16, [4, 2, 1, 1])
    tok = rng.integers(0, s.vocab, 16).astype(np.int32)
    for _ in range(200):
        p, d, t = parent.copy(), depth.copy(), tok.copy()
        k = rng.integers(0, 4)
        i = rng.integers(0, 16)
        if k == 0:
            p[i] = rng.integers(-1, 16)
        elif k == 1:
            d[i] = rng.integers(0, 5)
        elif k == 2:
            t[i] = rng.integers(-1, s.vocab + 1)
        rc = b.validate_tree(s, 128, 64, t, p, d, int(tok[0]), 64)
        try:
            fo.Oracle.check_tree(t, p, d, s.vocab, int(tok[0]), 64, 128, 64)
            assert rc == 0
        except fo.TreeVerifyError:
            assert rc < 0


def test_no_gpu_means_loud_failure(lib):
    import torch
    if torch.cuda.is_available():
        pytest.skip("GPU present")
    import paper_2412_12639_amd as m
    with pytest.raises(RuntimeError):
        m.FalconVerifier(fi.SHAPES["tiny"], 128, 16)
