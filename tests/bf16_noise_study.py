"""CPU study (not a test; run as `python -m tests.bf16_noise_study [n_layers]` from the repo root, about 20 minutes and
30 GB of RAM at 32 layers): how far each tensor class that a bf16 configuration stores in bf16 moves the logits of the
7B-shaped model at depth, measured with the rounding-noise model of tests/bf16_noise_model.py against the oracle (fp32
working precision).  Prints max / median / rms over the 64 node rows of max_v|model - exact| / max_v|exact|."""
import sys, time, json
import os
sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
import numpy as np
import fv_inputs as fi
from fv_inputs.trees import fill_tokens
from oracle import falcon_oracle as fo
from tests import bf16_noise_model as nm
NL = int(sys.argv[1]) if len(sys.argv) > 1 else 32
s = fi.SHAPES["7b"].with_layers(NL) if NL != 32 else fi.SHAPES["7b"]
t0 = time.time(); w = fi.gen_weights(s, seed=0); print("weights", time.time() - t0, flush=True)
L, T = 512, 64
prefix = fi.gen_prefix(0, L, s.vocab)
o = fo.Oracle(s, w, max_seq=L + T + 8, dtype=np.float32)
t0 = time.time(); root = o.prefill(prefix); print("exact prefill", time.time() - t0, flush=True)
parent, depth, planted = fi.gen_tree(0, T, [8, 4, 2, 2, 1, 1], 0)
tok = fill_tokens(0, parent, s.vocab, root)
exact = o.tree_logits(tok, parent, depth)[0].astype(np.float64)
def err(lg):
    e = np.max(np.abs(lg.astype(np.float64) - exact), axis=-1) / np.max(np.abs(exact), axis=-1)
    return float(e.max()), float(np.median(e)), float(np.sqrt(np.mean(e * e)))
sets = [("all", nm.ALL_CLASSES), ("floor: GEMM inputs + K/V cache", nm.GEMM_INPUTS + nm.KV_CACHE),
        ("GEMM inputs only", nm.GEMM_INPUTS), ("K/V cache only", nm.KV_CACHE), ("q + p only", nm.OTHER)] + [(c, (c,)) for c in nm.ALL_CLASSES]
out = {}
for name, cls in sets:
    t0 = time.time()
    m = nm.StorageNoiseModel(s, w, max_seq=L + T + 8, dtype=np.float32, rounded=cls)
    m.prefill(prefix); m.rollback(L, root)
    out[name] = err(m.tree_logits(tok, parent, depth)[0])
    print(f"{name:34s} max {out[name][0]:.3e} median {out[name][1]:.3e} rms {out[name][2]:.3e}   ({time.time()-t0:.0f} s)", flush=True)
