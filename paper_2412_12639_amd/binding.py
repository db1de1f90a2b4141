"""ctypes marshalling for libfalcon_verify.so.  Function names and semantics are those
of include/falcon_verify.h; nothing here computes anything."""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

STATUS = {0: "FV_OK", -1: "FV_E_BAD_ARG", -2: "FV_E_TREE_ORDER", -3: "FV_E_TREE_DEPTH", -4: "FV_E_TOKEN_RANGE",
          -5: "FV_E_TREE_TOO_BIG", -6: "FV_E_CACHE_FULL", -7: "FV_E_ROOT_MISMATCH", -8: "FV_E_NO_PREFILL",
          -9: "FV_E_HIP", -10: "FV_E_NONFINITE", -11: "FV_E_SCRATCH_LIMIT", -12: "FV_E_EXCHANGE_TIMEOUT"}
PHASES = ("gemm", "fixup", "attn", "other")


class FvError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        msg = STATUS.get(status, str(status))
        if _LIB is not None:
            msg += ": " + _LIB.fv_status_str(status).decode()
        super().__init__(f"{where} -> {msg}")


class fv_cfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "hidden", "n_q_heads", "n_kv_heads", "head_dim", "ffn", "vocab",
                                         "dtype", "max_seq", "max_tree")] + [("rope_base", C.c_float), ("rms_eps", C.c_float)]


class fv_drafter_host_weights(C.Structure):
    _fields_ = [("lstm_w_ih", C.c_void_p * 2), ("lstm_w_hh", C.c_void_p * 2), ("lstm_b", C.c_void_p * 2)] + \
               [(n, C.c_void_p) for n in ("wq", "wk", "wv", "wo", "wg", "wu", "wd", "g_attn", "g_mlp")]


class fv_host_weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("lm_head", C.c_void_p), ("g_final", C.c_void_p)] + \
               [(n, C.POINTER(C.c_void_p)) for n in ("wq", "wk", "wv", "wo", "wg", "wu", "wd", "g_attn", "g_mlp")]


def lib_path() -> str:
    return os.path.join(_HERE, "libfalcon_verify.so")


def load_library():
    """Load the built library; there is no fallback of any kind."""
    global _LIB
    if _LIB is not None:
        return _LIB
    # torch ships its own HIP runtime; it must be the one already in the process when this
    # library is loaded, or two runtimes would coexist and not know each other's allocations
    import torch  # noqa: F401
    path = lib_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it first (python -m paper_2412_12639_amd.build, "
                          "or __graft_entry__.build())")
    lib = C.CDLL(path)
    i32p, vp = C.POINTER(C.c_int32), C.c_void_p
    lib.fv_status_str.restype = C.c_char_p
    lib.fv_status_str.argtypes = [C.c_int]
    sigs = {
        "fv_workspace_bytes": [C.POINTER(fv_cfg), C.POINTER(C.c_size_t)],
        "fv_validate_tree": [C.POINTER(fv_cfg), i32p, i32p, i32p, C.c_int32, C.c_int32, C.c_int32],
        "fv_create": [C.POINTER(fv_cfg), vp, C.c_size_t, vp, C.POINTER(vp)],
        "fv_init_weights": [vp, C.POINTER(fv_host_weights)],
        "fv_prefill": [vp, i32p, C.c_int32, i32p],
        "fv_verify_tree": [vp, i32p, i32p, i32p, C.c_int32, i32p, i32p, i32p],
        "fv_verify_tree_noalloc": [vp, i32p, i32p, i32p, C.c_int32, i32p, i32p, i32p],
        "fv_verify_tree_sampled": [vp, i32p, i32p, i32p, C.c_int32, C.c_float, vp, C.POINTER(C.c_double), C.POINTER(C.c_double),
                                   i32p, i32p, i32p],
        "fv_rollback": [vp, C.c_int32, C.c_int32],
        "fv_get_state": [vp, i32p, i32p],
        "fv_get_tree_mask": [vp, C.POINTER(C.c_uint64), C.c_int32],
        "fv_get_logits": [vp, C.POINTER(C.c_float), C.c_int32],
        "fv_get_argmax": [vp, i32p, C.c_int32],
        "fv_get_kv_moves": [vp, i32p, i32p, i32p],
        "fv_get_features": [vp, C.POINTER(C.c_float), C.c_int32],
        "fv_read_kv": [vp, C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_float), C.POINTER(C.c_float)],
        "fv_debug_read_activation": [vp, C.c_int32, C.c_int32, C.POINTER(C.c_float)],
        "fv_stream_read": [vp, C.c_int32, C.POINTER(C.c_float)],
        "fv_set_profiling": [vp, C.c_int32],
        "fv_set_step_invariant": [vp, C.c_int32],
        "fv_get_phase_times": [vp, C.POINTER(C.c_float), i32p],
        "fv_last_step_ms": [vp, C.POINTER(C.c_float)],
        "fv_drafter_workspace_bytes": [C.POINTER(fv_cfg), C.POINTER(C.c_size_t)],
        "fv_drafter_create": [vp, C.c_int32, vp, C.c_size_t, C.POINTER(vp)],
        "fv_drafter_init_weights": [vp, C.POINTER(fv_drafter_host_weights)],
        "fv_draft_reset": [vp],
        "fv_draft_commit": [vp, i32p, vp, C.c_int32],
        "fv_draft_tree": [vp, i32p, i32p, i32p, C.c_int32, C.c_int32, i32p],
        "fv_draft_get_state": [vp, i32p, i32p, i32p],
        "fv_draft_get_rows": [vp, C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_float)],
        "fv_draft_get_top": [vp, C.c_int32, C.c_int32, i32p],
        "fv_draft_read_kv": [vp, C.c_int32, C.c_int32, C.POINTER(C.c_float), C.POINTER(C.c_float)],
        "fv_draft_last_ms": [vp, C.POINTER(C.c_float)],
        "fv_features_device_ptr": [vp, C.POINTER(vp)],
    }
    for name, args in sigs.items():
        fn = getattr(lib, name)
        fn.argtypes = args
        fn.restype = C.c_int
    lib.fv_destroy.argtypes = [vp]
    lib.fv_destroy.restype = None
    lib.fv_drafter_destroy.argtypes = [vp]
    lib.fv_drafter_destroy.restype = None
    _LIB = lib
    return lib


def make_cfg(shape, max_seq: int, max_tree: int) -> fv_cfg:
    """`shape` is any object with n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab,
    dtype ("f32" | "bf16"), rope_base, rms_eps."""
    return fv_cfg(shape.n_layers, shape.hidden, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.ffn,
                  shape.vocab, 1 if shape.dtype == "bf16" else 0, max_seq, max_tree, shape.rope_base, shape.rms_eps)


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(C.POINTER(C.c_int32))


def validate_tree(shape, max_seq, max_tree, tokens, parent, depth, pending_root, cur_len) -> int:
    """Host-only tree check (no GPU needed); returns the status code."""
    lib = load_library()
    cfg = make_cfg(shape, max_seq, max_tree)
    t, tp = _i32(tokens)
    p, pp = _i32(parent)
    d, dp = _i32(depth)
    return lib.fv_validate_tree(C.byref(cfg), tp, pp, dp, len(t), int(pending_root), int(cur_len))


def workspace_bytes(shape, max_seq, max_tree) -> int:
    lib = load_library()
    cfg = make_cfg(shape, max_seq, max_tree)
    out = C.c_size_t(0)
    rc = lib.fv_workspace_bytes(C.byref(cfg), C.byref(out))
    if rc:
        raise FvError(rc, "fv_workspace_bytes")
    return out.value


class FalconVerifier:
    """One decoding session on one GPU: owns the torch arena and the fv_ctx."""

    def __init__(self, shape, max_seq: int, max_tree: int, device: str = "cuda:0", stream=None):
        import torch
        self.lib = load_library()
        self.shape, self.max_seq, self.max_tree = shape, max_seq, max_tree
        self.cfg = make_cfg(shape, max_seq, max_tree)
        self.bytes = workspace_bytes(shape, max_seq, max_tree)
        if not torch.cuda.is_available():
            raise RuntimeError("FalconVerifier needs a GPU: there is no CPU path")
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.arena = torch.empty(self.bytes + 256, dtype=torch.uint8, device=self.device)
        base = self.arena.data_ptr()
        self._ptr = (base + 255) // 256 * 256
        self.stream = stream if stream is not None else torch.cuda.current_stream(self.device)
        ctx = C.c_void_p()
        rc = self.lib.fv_create(C.byref(self.cfg), C.c_void_p(self._ptr), C.c_size_t(self.bytes),
                                C.c_void_p(self.stream.cuda_stream), C.byref(ctx))
        if rc:
            raise FvError(rc, "fv_create")
        self.ctx = ctx
        self.last_n = 0

    def close(self):
        if getattr(self, "ctx", None):
            self.lib.fv_destroy(self.ctx)
            self.ctx = None
        self.arena = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _chk(self, rc, where):
        if rc:
            raise FvError(rc, where)

    def init_weights(self, weights: dict):
        """weights: name -> numpy array as produced for the model shape (matrices float32 or
        uint16 bf16 bits, gains float32)."""
        s = self.shape
        want = np.uint16 if s.dtype == "bf16" else np.float32
        keep = []

        def ptr(a, dt):
            a = np.ascontiguousarray(a, dtype=dt)
            if a.dtype != dt:
                raise TypeError("weight dtype mismatch")
            keep.append(a)
            return a.ctypes.data

        def arr(kind, dt):
            v = (C.c_void_p * s.n_layers)(*[ptr(weights[f"l{l}.{kind}"], dt) for l in range(s.n_layers)])
            keep.append(v)
            return C.cast(v, C.POINTER(C.c_void_p))

        for k, v in weights.items():
            if v.ndim == 2 and v.dtype != want:
                raise TypeError(f"{k}: expected {want} for dtype {s.dtype}, got {v.dtype}")
        hw = fv_host_weights(ptr(weights["embed"], want), ptr(weights["lm_head"], want), ptr(weights["g_final"], np.float32),
                             arr("wq", want), arr("wk", want), arr("wv", want), arr("wo", want), arr("wg", want),
                             arr("wu", want), arr("wd", want), arr("g_attn", np.float32), arr("g_mlp", np.float32))
        self._chk(self.lib.fv_init_weights(self.ctx, C.byref(hw)), "fv_init_weights")

    def prefill(self, tokens) -> int:
        t, tp = _i32(tokens)
        nxt = C.c_int32(-1)
        self._chk(self.lib.fv_prefill(self.ctx, tp, len(t), C.byref(nxt)), "fv_prefill")
        self.last_n = len(t) - ((len(t) - 1) // self.max_tree) * self.max_tree   # rows of the last chunk
        return nxt.value

    def verify_tree(self, tokens, parent, depth, noalloc: bool = False):
        """noalloc=True calls fv_verify_tree_noalloc (scratch in the library's static device array)."""
        t, tp = _i32(tokens)
        p, pp = _i32(parent)
        d, dp = _i32(depth)
        if not (len(t) == len(p) == len(d)):
            raise ValueError("tokens, parent and depth must have the same length")
        a = C.c_int32(-1)
        nxt = C.c_int32(-1)
        acc = np.zeros(max(1, len(t)), dtype=np.int32)
        fn = self.lib.fv_verify_tree_noalloc if noalloc else self.lib.fv_verify_tree
        self._chk(fn(self.ctx, tp, pp, dp, len(t), C.byref(a), acc.ctypes.data_as(C.POINTER(C.c_int32)), C.byref(nxt)),
                  "fv_verify_tree_noalloc" if noalloc else "fv_verify_tree")
        self.last_n = len(t)
        return a.value, acc[:a.value].copy(), nxt.value

    def verify_tree_sampled(self, tokens, parent, depth, temperature, u_accept, u_sample, draft_probs=None):
        """Non-greedy step.  draft_probs: None, or a torch float32 tensor [n_nodes, vocab] on this device
        (only its data pointer is passed on)."""
        t, tp = _i32(tokens)
        p, pp = _i32(parent)
        d, dp = _i32(depth)
        ua = np.ascontiguousarray(u_accept, dtype=np.float64)
        us = np.ascontiguousarray(u_sample, dtype=np.float64)
        if not (len(t) == len(p) == len(d) == len(ua) == len(us)):
            raise ValueError("tokens, parent, depth, u_accept and u_sample must have the same length")
        qptr = None
        if draft_probs is not None:
            if not (draft_probs.is_cuda and draft_probs.is_contiguous() and tuple(draft_probs.shape) == (len(t), self.shape.vocab)
                    and str(draft_probs.dtype) == "torch.float32"):
                raise ValueError("draft_probs must be a contiguous float32 device tensor [n_nodes, vocab]")
            qptr = C.c_void_p(draft_probs.data_ptr())
        a, nxt = C.c_int32(-1), C.c_int32(-1)
        acc = np.zeros(max(1, len(t)), dtype=np.int32)
        self._chk(self.lib.fv_verify_tree_sampled(self.ctx, tp, pp, dp, len(t), C.c_float(temperature), qptr,
                                                  ua.ctypes.data_as(C.POINTER(C.c_double)), us.ctypes.data_as(C.POINTER(C.c_double)),
                                                  C.byref(a), acc.ctypes.data_as(C.POINTER(C.c_int32)), C.byref(nxt)),
                  "fv_verify_tree_sampled")
        self.last_n = len(t)
        return a.value, acc[:a.value].copy(), nxt.value

    def rollback(self, new_len: int, pending_root: int):
        self._chk(self.lib.fv_rollback(self.ctx, int(new_len), int(pending_root)), "fv_rollback")

    def state(self):
        a, b = C.c_int32(), C.c_int32()
        self._chk(self.lib.fv_get_state(self.ctx, C.byref(a), C.byref(b)), "fv_get_state")
        return a.value, b.value

    # ---- read-back of the last step
    def tree_mask(self, n=None):
        n = n or self.last_n
        out = np.zeros((n, 4), dtype=np.uint64)
        self._chk(self.lib.fv_get_tree_mask(self.ctx, out.ctypes.data_as(C.POINTER(C.c_uint64)), n), "fv_get_tree_mask")
        return out

    def logits(self, n=None):
        n = n or self.last_n
        out = np.zeros((n, self.shape.vocab), dtype=np.float32)
        self._chk(self.lib.fv_get_logits(self.ctx, out.ctypes.data_as(C.POINTER(C.c_float)), n), "fv_get_logits")
        return out

    def argmax(self, n=None):
        n = n or self.last_n
        out = np.zeros(n, dtype=np.int32)
        self._chk(self.lib.fv_get_argmax(self.ctx, out.ctypes.data_as(C.POINTER(C.c_int32)), n), "fv_get_argmax")
        return out

    def kv_moves(self):
        src = np.zeros(256, dtype=np.int32)
        dst = np.zeros(256, dtype=np.int32)
        cnt = C.c_int32()
        self._chk(self.lib.fv_get_kv_moves(self.ctx, src.ctypes.data_as(C.POINTER(C.c_int32)),
                                           dst.ctypes.data_as(C.POINTER(C.c_int32)), C.byref(cnt)), "fv_get_kv_moves")
        return src[:cnt.value].copy(), dst[:cnt.value].copy()

    def features(self, n_rows: int):
        """LM-head inputs (post final norm) of the first n_rows nodes of the accepted path -> [n_rows, hidden] float32."""
        out = np.zeros((n_rows, self.shape.hidden), dtype=np.float32)
        self._chk(self.lib.fv_get_features(self.ctx, out.ctypes.data_as(C.POINTER(C.c_float)), n_rows), "fv_get_features")
        return out

    def read_kv(self, layer: int, slot0: int, n: int):
        s = self.shape
        k = np.zeros((n, s.n_kv_heads, s.head_dim), dtype=np.float32)
        v = np.zeros_like(k)
        self._chk(self.lib.fv_read_kv(self.ctx, layer, slot0, n, k.ctypes.data_as(C.POINTER(C.c_float)),
                                      v.ctypes.data_as(C.POINTER(C.c_float))), "fv_read_kv")
        return k, v

    def activation(self, which: str, n=None):
        """Last layer's intermediate: which in x, xb, q, attn, ffn -> [n, features] float32."""
        s = self.shape
        idx = ("x", "xb", "q", "attn", "ffn").index(which)
        feats = (s.hidden, s.hidden, s.n_q_heads * s.head_dim, s.n_q_heads * s.head_dim, s.ffn)[idx]
        n = n or self.last_n
        out = np.zeros((n, feats), dtype=np.float32)
        self._chk(self.lib.fv_debug_read_activation(self.ctx, idx, n, out.ctypes.data_as(C.POINTER(C.c_float))),
                  "fv_debug_read_activation")
        return out

    def set_step_invariant(self, on: bool):
        """Rows bitwise independent of the step they are verified in (see fv_set_step_invariant)."""
        self._chk(self.lib.fv_set_step_invariant(self.ctx, 1 if on else 0), "fv_set_step_invariant")

    # ---- measurement
    def set_profiling(self, on: bool):
        self._chk(self.lib.fv_set_profiling(self.ctx, 1 if on else 0), "fv_set_profiling")

    def phase_times(self):
        ms = (C.c_float * len(PHASES))()
        n = (C.c_int32 * len(PHASES))()
        self._chk(self.lib.fv_get_phase_times(self.ctx, ms, n), "fv_get_phase_times")
        return {PHASES[i]: (ms[i], n[i]) for i in range(len(PHASES))}

    def stream_read_gbs(self, passes: int = 4) -> float:
        """GB/s of the library's plain streaming-read kernel over the tiled weights (roofline context)."""
        v = C.c_float()
        self._chk(self.lib.fv_stream_read(self.ctx, passes, C.byref(v)), "fv_stream_read")
        return v.value

    def last_step_ms(self) -> float:
        v = C.c_float()
        self._chk(self.lib.fv_last_step_ms(self.ctx, C.byref(v)), "fv_last_step_ms")
        return v.value


DRAFT_MAX_M = 32


class FalconDrafter:
    """The drafting phase next to a FalconVerifier (whose stream, embedding table and LM head it uses):
    owns its torch arena and the fv_drafter."""

    def __init__(self, target: FalconVerifier, k: int):
        import torch
        self.lib, self.target, self.k = target.lib, target, int(k)
        out = C.c_size_t(0)
        rc = self.lib.fv_drafter_workspace_bytes(C.byref(target.cfg), C.byref(out))
        if rc:
            raise FvError(rc, "fv_drafter_workspace_bytes")
        self.bytes = out.value
        self.arena = torch.empty(self.bytes + 256, dtype=torch.uint8, device=target.device)
        self._ptr = (self.arena.data_ptr() + 255) // 256 * 256
        h = C.c_void_p()
        rc = self.lib.fv_drafter_create(target.ctx, self.k, C.c_void_p(self._ptr), C.c_size_t(self.bytes), C.byref(h))
        if rc:
            raise FvError(rc, "fv_drafter_create")
        self.h = h

    def close(self):
        if getattr(self, "h", None):
            self.lib.fv_drafter_destroy(self.h)
            self.h = None
        self.arena = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _chk(self, rc, where):
        if rc:
            raise FvError(rc, where)

    def init_weights(self, weights: dict):
        """weights: the drafter's own tensors by name (lstm{0,1}.{w_ih,w_hh,b}, d.{wq,..,wd,g_attn,g_mlp})."""
        want = np.uint16 if self.target.shape.dtype == "bf16" else np.float32
        keep = []

        def ptr(name, dt):
            a = weights[name]
            if a.dtype != dt:
                raise TypeError(f"{name}: expected {dt}, got {a.dtype}")
            a = np.ascontiguousarray(a)
            keep.append(a)
            return a.ctypes.data

        hw = fv_drafter_host_weights(
            (C.c_void_p * 2)(ptr("lstm0.w_ih", want), ptr("lstm1.w_ih", want)),
            (C.c_void_p * 2)(ptr("lstm0.w_hh", want), ptr("lstm1.w_hh", want)),
            (C.c_void_p * 2)(ptr("lstm0.b", np.float32), ptr("lstm1.b", np.float32)),
            *[ptr(f"d.{n}", want) for n in ("wq", "wk", "wv", "wo", "wg", "wu", "wd")],
            ptr("d.g_attn", np.float32), ptr("d.g_mlp", np.float32))
        self._chk(self.lib.fv_drafter_init_weights(self.h, C.byref(hw)), "fv_drafter_init_weights")

    def reset(self):
        self._chk(self.lib.fv_draft_reset(self.h), "fv_draft_reset")

    def commit(self, tokens, features):
        """features: a torch float32 CUDA tensor [n, hidden] (or a raw device address) of the target's features."""
        t, tp = _i32(tokens)
        if hasattr(features, "data_ptr"):
            if features.dtype.__str__() != "torch.float32" or not features.is_contiguous() or features.shape[0] < len(t):
                raise TypeError("features: contiguous float32 [n, hidden] on the GPU")
            addr = features.data_ptr()
        else:
            addr = int(features)
        self._chk(self.lib.fv_draft_commit(self.h, tp, C.c_void_p(addr), len(t)), "fv_draft_commit")

    def draft_tree(self, parent, depth, rank, root_token: int):
        p, pp = _i32(parent)
        d, dp = _i32(depth)
        r, rp = _i32(rank)
        out = np.zeros(len(p), dtype=np.int32)
        self._chk(self.lib.fv_draft_tree(self.h, pp, dp, rp, len(p), int(root_token), out.ctypes.data_as(C.POINTER(C.c_int32))),
                  "fv_draft_tree")
        return out

    def state(self):
        a, b, c = C.c_int32(), C.c_int32(), C.c_int32()
        self._chk(self.lib.fv_draft_get_state(self.h, C.byref(a), C.byref(b), C.byref(c)), "fv_draft_get_state")
        return a.value, b.value, c.value

    def rows(self, what: str, row0: int, n: int):
        width = self.target.shape.hidden if what == "features" else self.target.shape.vocab
        out = np.zeros((n, width), dtype=np.float32)
        self._chk(self.lib.fv_draft_get_rows(self.h, 0 if what == "features" else 1, row0, n,
                                             out.ctypes.data_as(C.POINTER(C.c_float))), "fv_draft_get_rows")
        return out

    def top(self, row0: int, n: int):
        out = np.zeros((n, DRAFT_MAX_M), dtype=np.int32)
        self._chk(self.lib.fv_draft_get_top(self.h, row0, n, out.ctypes.data_as(C.POINTER(C.c_int32))), "fv_draft_get_top")
        return out

    def read_kv(self, slot0: int, n: int):
        s = self.target.shape
        k = np.zeros((n, s.n_kv_heads, s.head_dim), dtype=np.float32)
        v = np.zeros_like(k)
        self._chk(self.lib.fv_draft_read_kv(self.h, slot0, n, k.ctypes.data_as(C.POINTER(C.c_float)),
                                            v.ctypes.data_as(C.POINTER(C.c_float))), "fv_draft_read_kv")
        return k, v

    def last_ms(self) -> float:
        ms = C.c_float(0)
        self._chk(self.lib.fv_draft_last_ms(self.h, C.byref(ms)), "fv_draft_last_ms")
        return ms.value


def features_device_ptr(target: FalconVerifier) -> int:
    out = C.c_void_p()
    rc = target.lib.fv_features_device_ptr(target.ctx, C.byref(out))
    if rc:
        raise FvError(rc, "fv_features_device_ptr")
    return out.value
