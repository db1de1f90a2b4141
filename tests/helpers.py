"""Shared by the GPU parity tests: builds seeded cases with the oracle (inputs and
expected values come from fv_inputs and oracle/ only) and compares results."""
import numpy as np

import fv_inputs as fi
from fv_inputs.trees import fill_tokens
from oracle import falcon_oracle as fo

TOL_BF16 = 2e-2    # max |gpu - oracle| per node row, relative to that row's max |oracle| (bf16 shapes)
TOL_F32 = 2e-4     # same for fp32 shapes: fp32 accumulation order and fast exp only


def tol_for(shape):
    return TOL_BF16 if shape.dtype == "bf16" else TOL_F32


def row_rel_err(got, ref):
    """Per-row max abs error relative to the row's max abs reference value."""
    return np.max(np.abs(got - ref), axis=-1) / np.max(np.abs(ref), axis=-1)


def decision_margins_ok(res, tokens, parent, tol):
    """True if every node whose argmax decides acceptance has a top-2 gap above 2*tol*max|row|:
    parents of children carrying their top-1 or top-2 token, and the best node (next_token)."""
    logits = res["logits"]
    deciders = {int(res["path"][-1])}
    for i in range(1, len(tokens)):
        p = int(parent[i])
        top2 = np.argsort(logits[p])[-2:]
        if int(tokens[i]) in top2:
            deciders.add(p)
    for p in deciders:
        if fo.top2_margin(logits[p]) <= 2 * tol * np.max(np.abs(logits[p])):
            return False
    return True


def planted_case(shape, weights, prefix_len, n_nodes, branching, plant_len, seed=0, max_tries=40, extra_seq=0,
                 odtype=np.float64):
    """Prefill + one planted tree whose decisive margins clear the tolerance.  Returns a dict
    with the inputs, the oracle object (state AFTER the verify) and the oracle's results."""
    tol = tol_for(shape)
    for attempt in range(max_tries):
        sd = seed + 1000 * attempt
        prefix = fi.gen_prefix(sd, prefix_len, shape.vocab)
        o = fo.Oracle(shape, weights, max_seq=prefix_len + n_nodes + 8 + extra_seq, dtype=odtype)
        root = o.prefill(prefix)
        prefill_logits = o.last_logits
        if fo.top2_margin(prefill_logits[-1]) <= 2 * tol * np.max(np.abs(prefill_logits[-1])):
            continue
        parent, depth, planted = fi.gen_tree(sd, n_nodes, branching, plant_len)
        # greedy tokens along the planted path, from cached single-node steps of a scratch oracle
        greedy = []
        tk = root
        for _ in range(plant_len):
            p1, d1 = fi.chain_tree(1)
            r1 = o.verify_tree(np.array([tk], dtype=np.int32), p1, d1)
            tk = r1["next_token"]
            greedy.append(tk)
        o.rollback(prefix_len, root)
        tokens = fill_tokens(sd, parent, shape.vocab, root, planted, greedy)
        res = o.verify_tree(tokens, parent, depth)
        if not decision_margins_ok(res, tokens, parent, tol):
            continue
        return dict(prefix=prefix, root=root, parent=parent, depth=depth, planted=planted, tokens=tokens,
                    greedy=greedy, oracle=o, res=res, prefill_logits=prefill_logits, seed=sd,
                    hidden=o.last_hidden.copy())
    raise RuntimeError("no instance with clear margins found")


def check_decisions(gpu, tokens, parent, depth, L, got):
    """Integer outputs of a verify step, bit-exact and unconditionally: the device's argmax is the
    first maximum of its own logits, and its accepted length, tokens, bonus token, compaction moves
    and state are the oracle's acceptance rule applied to that argmax.  Returns the decision."""
    a, acc_tokens, nxt = got
    T = len(parent)
    logits = gpu.logits(T)
    assert np.all(np.isfinite(logits)), "non-finite logits"
    am = gpu.argmax(T)
    assert np.array_equal(am, np.argmax(logits, axis=-1)), "device argmax vs its own logits"
    d = fo.greedy_accept(tokens, parent, depth, am, L)
    assert a == d["accepted_len"], f"accepted_len {a} vs {d['accepted_len']}"
    assert list(acc_tokens) == list(d["accepted_tokens"]), "accepted tokens"
    assert nxt == d["next_token"], "bonus token"
    src, dst = gpu.kv_moves()
    assert list(src) == list(d["src_slot"]) and list(dst) == list(d["dst_slot"]), "compaction moves"
    assert gpu.state() == (L + a + 1, nxt), "state after the step"
    return d


def check_path_cache(gpu, shape, L, path, tree_k, tree_v, tol):
    """Cache slots L .. L+a after compaction against the oracle's K/V of the nodes on `path` (the
    path the device took): holds whatever the acceptance decisions were."""
    n = len(path)
    worst = 0.0
    for l in range(shape.n_layers):
        k, v = gpu.read_kv(l, L, n)
        for got, ref in ((k, tree_k[l][path]), (v, tree_v[l][path])):
            e = np.max(np.abs(got - ref)) / np.max(np.abs(ref))
            worst = max(worst, e)
            assert e <= tol, f"layer {l}: compacted K/V rel err {e:.3e}"
    return worst


def check_step(gpu, case, got, tol, L=None, oracle_decisions=True):
    """Compare one verify step of the HIP path (already run) with the oracle's.  L = committed
    length before the step (default: the oracle's dst_slot[0]).  oracle_decisions=False drops only
    the demand that the decisions equal the ORACLE's (for instances whose deciding rows are near-ties);
    everything else -- mask, logits, argmax on clear rows, decisions as a function of the device's own
    argmax, compacted K/V of the path taken, features -- is always checked."""
    res, parent, tokens, depth = case["res"], case["parent"], case["tokens"], case["depth"]
    T = len(parent)
    if L is None:
        L = int(res["dst_slot"][0])
    assert np.array_equal(gpu.tree_mask(T), res["mask"]), "ancestor mask"
    logits = gpu.logits(T)
    err = row_rel_err(logits.astype(np.float64), res["logits"])
    assert err.max() <= tol, f"logits rel err {err.max():.3e} > {tol}"
    am = gpu.argmax(T)
    for i in range(T):
        row = res["logits"][i]
        if fo.top2_margin(row) > tol * np.max(np.abs(row)):
            assert am[i] == res["argmax"][i], f"argmax of node {i}"
    d = check_decisions(gpu, tokens, parent, depth, L, got)
    if oracle_decisions:
        assert d["accepted_len"] == res["accepted_len"], f"accepted_len {d['accepted_len']} vs oracle {res['accepted_len']}"
        assert list(d["accepted_tokens"]) == list(res["accepted_tokens"]) and d["next_token"] == res["next_token"]
        assert list(d["src_slot"]) == list(res["src_slot"]) and list(d["dst_slot"]) == list(res["dst_slot"])
    check_path_cache(gpu, gpu.shape, L, d["path"], res["tree_k"], res["tree_v"], tol)
    # features of the accepted path (the LM head's input), same relative bar as the logits
    feat = gpu.features(d["accepted_len"] + 1).astype(np.float64)
    ref = case["hidden"][d["path"]] if "hidden" in case else np.asarray(res["features"], dtype=np.float64)
    ferr = row_rel_err(feat, np.asarray(ref, dtype=np.float64))
    assert ferr.max() <= tol, f"features rel err {ferr.max():.3e} > {tol}"
    return err.max()


def check_cache(gpu, oracle, shape, n_slots, tol):
    """Cache slots [0, n_slots) of every layer against the oracle's cache."""
    worst = 0.0
    for l in range(shape.n_layers):
        k, v = gpu.read_kv(l, 0, n_slots)
        for got, ref in ((k, oracle.K[l, :n_slots]), (v, oracle.V[l, :n_slots])):
            scale = np.max(np.abs(ref))
            e = np.max(np.abs(got - ref)) / scale
            worst = max(worst, e)
            assert e <= tol, f"layer {l} cache rel err {e:.3e}"
    return worst
