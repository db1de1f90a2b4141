"""Random-init weights: every matrix i.i.d. N(0, 0.02), norm gains 1 (optionally
jittered so that a test notices a gain that is ignored or mis-indexed).

Each tensor has its own counter-based Philox stream keyed by (seed, tensor id), so
tensors can be generated in any order or in parallel and always come out the same.
For "bf16" shapes the fp32 draws are rounded once (round-to-nearest-even) to bf16
and returned as uint16 bit patterns; both the oracle and the HIP library consume
exactly these bits."""
from concurrent.futures import ThreadPoolExecutor
import os
import numpy as np

from .shapes import ModelShape

STD = 0.02


def bf16_bits_from_f32(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit pattern, round to nearest even (inputs are finite)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) >> np.uint32(16)
    return r.astype(np.uint16)


def f32_from_bf16_bits(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _tensor_ids(s: ModelShape):
    """(name, shape) for every tensor, in a fixed order that defines the stream ids."""
    qd, kvd = s.n_q_heads * s.head_dim, s.n_kv_heads * s.head_dim
    out = [("embed", (s.vocab, s.hidden))]
    for l in range(s.n_layers):
        out += [
            (f"l{l}.wq", (qd, s.hidden)), (f"l{l}.wk", (kvd, s.hidden)), (f"l{l}.wv", (kvd, s.hidden)),
            (f"l{l}.wo", (s.hidden, qd)),
            (f"l{l}.wg", (s.ffn, s.hidden)), (f"l{l}.wu", (s.ffn, s.hidden)), (f"l{l}.wd", (s.hidden, s.ffn)),
            (f"l{l}.g_attn", (s.hidden,)), (f"l{l}.g_mlp", (s.hidden,)),
        ]
    out += [("g_final", (s.hidden,)), ("lm_head", (s.vocab, s.hidden))]
    return out


def _tensor_key(name: str) -> int:
    """Stable per-tensor stream id, independent of the layer count (so that a model
    truncated to fewer layers shares its tensors with the full one)."""
    if name == "embed":
        return 1
    if name == "g_final":
        return 2
    if name == "lm_head":
        return 3
    lname, t = name.split(".")
    kinds = ["wq", "wk", "wv", "wo", "wg", "wu", "wd", "g_attn", "g_mlp"]
    return 16 + int(lname[1:]) * 16 + kinds.index(t)


def _gen_one(seed: int, name: str, shp, dtype: str, gain_jitter: float) -> np.ndarray:
    rng = np.random.Generator(np.random.Philox(key=[seed, _tensor_key(name)]))
    if len(shp) == 1:  # norm gain
        g = np.ones(shp, dtype=np.float32)
        if gain_jitter:
            g += np.float32(gain_jitter) * rng.standard_normal(shp, dtype=np.float32)
        return g
    rows, cols = shp
    if dtype == "f32":
        w = rng.standard_normal(shp, dtype=np.float32)
        w *= np.float32(STD)
        return w
    out = np.empty(shp, dtype=np.uint16)
    step = max(1, (1 << 24) // cols)
    for r0 in range(0, rows, step):  # chunked to bound the fp32 temporary
        blk = rng.standard_normal((min(step, rows - r0), cols), dtype=np.float32)
        blk *= np.float32(STD)
        out[r0:r0 + blk.shape[0]] = bf16_bits_from_f32(blk)
    return out


def gen_weights(shape: ModelShape, seed: int = 0, gain_jitter: float = 0.0, threads: int = 0) -> dict:
    """dict name -> array.  Matrices are [out_features, in_features] row-major:
    float32 for "f32" shapes, uint16 bf16 bits for "bf16" shapes.  Gains are float32."""
    items = _tensor_ids(shape)
    threads = threads or min(16, os.cpu_count() or 1)
    if threads > 1 and shape.weight_params() > (1 << 26):
        with ThreadPoolExecutor(threads) as ex:
            arrs = list(ex.map(lambda it: _gen_one(seed, it[0], it[1], shape.dtype, gain_jitter), items))
    else:
        arrs = [_gen_one(seed, n, s, shape.dtype, gain_jitter) for n, s in items]
    return {n: a for (n, _), a in zip(items, arrs)}


def sub_model(shape: ModelShape, weights: dict, n_layers: int):
    """The same model cut to its first n_layers layers (shares the arrays)."""
    sub = shape.with_layers(n_layers)
    keep = {k: v for k, v in weights.items()
            if not k.startswith("l") or k == "lm_head" or int(k.split(".")[0][1:]) < n_layers}
    return sub, keep


# ----------------------------------------------------------------------------- drafter (SAR head)

def drafter_tensor_ids(s: ModelShape):
    """(name, shape) of the drafter's own tensors: two LSTM layers (fused input 2h -> h, then
    h -> h; gate rows in the order input, forget, cell, output), one decoder layer of the target's
    geometry.  Embedding and LM head are the target's (section "Framework and Computational
    Process") and are not listed."""
    h, qd, kvd = s.hidden, s.n_q_heads * s.head_dim, s.n_kv_heads * s.head_dim
    return [
        ("lstm0.w_ih", (4 * h, 2 * h)), ("lstm0.w_hh", (4 * h, h)), ("lstm0.b", (4 * h,)),
        ("lstm1.w_ih", (4 * h, h)), ("lstm1.w_hh", (4 * h, h)), ("lstm1.b", (4 * h,)),
        ("d.wq", (qd, h)), ("d.wk", (kvd, h)), ("d.wv", (kvd, h)), ("d.wo", (h, qd)),
        ("d.wg", (s.ffn, h)), ("d.wu", (s.ffn, h)), ("d.wd", (h, s.ffn)),
        ("d.g_attn", (h,)), ("d.g_mlp", (h,)),
    ]


def gen_drafter_weights(shape: ModelShape, seed: int = 0, gain_jitter: float = 0.0, bias_std: float = 0.1) -> dict:
    """Random-init drafter tensors (the trained ones are not available): matrices N(0, 0.02) in the
    shape's storage type, LSTM biases N(0, bias_std) in float32 (non-zero so that a dropped or
    mis-indexed bias shows), gains 1 (+ jitter)."""
    out = {}
    for idx, (name, shp) in enumerate(drafter_tensor_ids(shape)):
        if name.endswith(".b"):
            rng = np.random.Generator(np.random.Philox(key=[seed, 4096 + idx]))
            out[name] = (np.float32(bias_std) * rng.standard_normal(shp, dtype=np.float32)).astype(np.float32)
            continue
        if len(shp) == 1:   # gains: same recipe as the target's
            rng = np.random.Generator(np.random.Philox(key=[seed, 4096 + idx]))
            g = np.ones(shp, dtype=np.float32)
            if gain_jitter:
                g += np.float32(gain_jitter) * rng.standard_normal(shp, dtype=np.float32)
            out[name] = g
            continue
        rng = np.random.Generator(np.random.Philox(key=[seed, 4096 + idx]))
        rows, cols = shp
        if shape.dtype == "f32":
            w = rng.standard_normal(shp, dtype=np.float32)
            w *= np.float32(STD)
            out[name] = w
        else:
            arr = np.empty(shp, dtype=np.uint16)
            step = max(1, (1 << 24) // cols)
            for r0 in range(0, rows, step):
                blk = rng.standard_normal((min(step, rows - r0), cols), dtype=np.float32)
                blk *= np.float32(STD)
                arr[r0:r0 + blk.shape[0]] = bf16_bits_from_f32(blk)
            out[name] = arr
    return out


def gen_features(seed: int, n: int, hidden: int) -> np.ndarray:
    """Stand-ins for target-model features (LM-head inputs after the final norm): N(0, 1) rows, float32."""
    rng = np.random.Generator(np.random.Philox(key=[seed, 7020]))
    return rng.standard_normal((n, hidden), dtype=np.float32)
