"""ctypes binding of include/revffn.h.  Argument marshalling only."""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

EXPORTED_SYMBOLS = (
    "revffn_workspace_bytes", "revffn_create", "revffn_destroy", "revffn_set_inv_iters",
    "revffn_set_inverse_tolerance", "revffn_set_inverse_tolerance_blocked", "revffn_get_inverse_stats",
    "revffn_get_inverse_blocks",
    "revffn_merge_adapters", "revffn_forward_merged", "revffn_inverse_merged",
    "revffn_forward", "revffn_inverse", "revffn_backward", "revffn_backward_stored", "revffn_inverse_backward", "revffn_stack_forward",
    "revffn_stack_backward", "revffn_get_routing", "revffn_enable_taps", "revffn_get_branch",
    "revffn_set_kernel_mode", "revffn_set_helper_streams", "revffn_strerror", "revffn_profile_enable", "revffn_profile_read",
    "revffn_profile_kernel_name", "revffn_op_gemm", "revffn_op_attention_fwd", "revffn_op_attention_bwd",
    "revffn_op_attention_bwd_noalloc", "revffn_op_tile_placement",
)

WEIGHT_FIELDS = (
    "norm_a1", "norm_a2", "norm_m", "pup_a", "pdn_a", "pup_m", "pdn_m",
    "wq", "wk", "wv", "wo", "bq", "bk", "bv", "w_router", "b_router",
    "w_gate_up", "w_down", "ws_gate_up", "ws_down", "ws_gate",
)


class RevffnError(RuntimeError):
    pass


class Config(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "d_model", "n_heads", "head_dim", "n_experts", "top_k", "d_expert", "d_shared",
        "dtype", "causal", "use_rope", "norm_topk_prob", "n_inv_iters")] + [
        ("rope_theta", ctypes.c_float), ("rms_eps", ctypes.c_float), ("fp32_streams", ctypes.c_int32),
        ("symmetric", ctypes.c_int32), ("fp32_grads", ctypes.c_int32)]


class Weights(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in WEIGHT_FIELDS]


class Grads(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in WEIGHT_FIELDS]


MERGED_FIELDS = ("wq", "wk", "wv", "wo", "w_gate_up", "w_down", "ws_gate_up", "ws_down", "w_router")


class Merged(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in MERGED_FIELDS]


def library_path():
    return os.path.join(_HERE, "librevffn.so")


def load_library():
    """Load librevffn.so (built by __graft_entry__.build() or `make -C csrc`).  Raises if absent."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = library_path()
    if not os.path.exists(path):
        raise RevffnError(f"{path} is not built; run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(there is no CPU fallback)")
    lib = ctypes.CDLL(path)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    lib.revffn_workspace_bytes.restype = ctypes.c_size_t
    lib.revffn_workspace_bytes.argtypes = [ctypes.POINTER(Config), i32, i32]
    lib.revffn_create.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(Config), i32, i32]
    lib.revffn_destroy.argtypes = [vp]
    lib.revffn_destroy.restype = None
    lib.revffn_set_inv_iters.argtypes = [vp, i32]
    lib.revffn_set_inverse_tolerance.argtypes = [vp, ctypes.c_float, i32]
    lib.revffn_set_inverse_tolerance_blocked.argtypes = [vp, ctypes.c_float, i32, i32]
    lib.revffn_get_inverse_blocks.argtypes = [vp, vp, vp, i32, ctypes.POINTER(i32)]
    lib.revffn_get_inverse_stats.argtypes = [vp, ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int64),
                                             ctypes.POINTER(i32), ctypes.POINTER(ctypes.c_float)]
    lib.revffn_enable_taps.argtypes = [vp, i32]
    lib.revffn_set_kernel_mode.argtypes = [vp, i32]
    lib.revffn_set_helper_streams.argtypes = [vp, i32]
    lib.revffn_merge_adapters.argtypes = [vp, ctypes.POINTER(Weights), ctypes.POINTER(Merged), vp]
    lib.revffn_forward_merged.argtypes = [vp, ctypes.POINTER(Weights), ctypes.POINTER(Merged), vp, vp, vp, vp, i32, i32, i64, vp]
    lib.revffn_inverse_merged.argtypes = [vp, ctypes.POINTER(Weights), ctypes.POINTER(Merged), vp, vp, vp, vp, i32, i32, i64, vp, vp]
    lib.revffn_forward.argtypes = [vp, ctypes.POINTER(Weights), vp, vp, vp, vp, i32, i32, i64, vp]
    lib.revffn_inverse.argtypes = [vp, ctypes.POINTER(Weights), vp, vp, vp, vp, i32, i32, i64, vp, vp]
    lib.revffn_backward.argtypes = [vp, ctypes.POINTER(Weights), vp, vp, vp, vp, vp, vp, vp,
                                    ctypes.POINTER(Grads), i32, i32, i64, vp]
    lib.revffn_backward_stored.argtypes = lib.revffn_backward.argtypes
    lib.revffn_inverse_backward.argtypes = [vp, ctypes.POINTER(Weights), vp, vp, vp, vp, vp, vp, vp, vp,
                                            ctypes.POINTER(Grads), i32, i32, i64, vp, vp]
    lib.revffn_stack_forward.argtypes = [vp, ctypes.POINTER(Weights), i32, vp, vp, vp, vp, i32, i32, i64, vp]
    lib.revffn_stack_backward.argtypes = [vp, ctypes.POINTER(Weights), ctypes.POINTER(Grads), i32,
                                          vp, vp, vp, vp, i32, i32, i64, vp]
    lib.revffn_get_routing.argtypes = [vp, vp, vp, vp, vp, vp, vp]
    lib.revffn_get_branch.argtypes = [vp, i32, vp, vp]
    lib.revffn_op_gemm.argtypes = [i32, i32, vp, vp, vp, i32, i32, i32, i64, i64, i64, i32, i32, i32, vp]
    lib.revffn_op_attention_fwd.argtypes = [i32, i32, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, vp]
    lib.revffn_op_tile_placement.argtypes = [i32, i32, i32, i32, i32, i32, vp, i32, vp, i32]
    lib.revffn_op_attention_bwd.argtypes = [i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp,
                                            i32, i32, i32, i32, i32, vp]
    lib.revffn_op_attention_bwd_noalloc.argtypes = [i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp,
                                                    i32, i32, i32, i32, i32, vp]
    lib.revffn_profile_enable.argtypes = [vp, i32]
    lib.revffn_profile_read.argtypes = [vp, i32, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64),
                                        ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
    lib.revffn_profile_kernel_name.restype = ctypes.c_char_p
    lib.revffn_profile_kernel_name.argtypes = [i32]
    lib.revffn_strerror.restype = ctypes.c_char_p
    lib.revffn_strerror.argtypes = [ctypes.c_int]
    for name in EXPORTED_SYMBOLS:
        if name not in ("revffn_workspace_bytes", "revffn_destroy", "revffn_strerror",
                        "revffn_profile_kernel_name"):
            getattr(lib, name).restype = ctypes.c_int
    _LIB = lib
    return lib


def revffn_strerror(code):
    return load_library().revffn_strerror(int(code)).decode()


def _check(code):
    if code != 0:
        raise RevffnError(f"librevffn error {code}: {revffn_strerror(code)}")


def _ptr(t):
    """Device pointer of a torch tensor, a raw integer address, or None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _struct(cls, tensors):
    s = cls()
    for n in WEIGHT_FIELDS:
        setattr(s, n, _ptr(tensors.get(n)))
    return s


class Context:
    """Owns one revffn_ctx (the device workspace).  cfg: a Config or a dict of its fields."""

    def __init__(self, cfg, max_B, max_S):
        lib = load_library()
        self.cfg = cfg if isinstance(cfg, Config) else Config(**cfg)
        h = ctypes.c_void_p()
        _check(lib.revffn_create(ctypes.byref(h), ctypes.byref(self.cfg), max_B, max_S))
        self.handle = h
        self.lib = lib

    def close(self):
        if getattr(self, "handle", None):
            self.lib.revffn_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def workspace_bytes(self, max_B, max_S):
        return self.lib.revffn_workspace_bytes(ctypes.byref(self.cfg), max_B, max_S)

    def set_inv_iters(self, n):
        _check(self.lib.revffn_set_inv_iters(self.handle, n))

    def set_inverse_tolerance(self, tol, max_iters=16, block_positions=0):
        _check(self.lib.revffn_set_inverse_tolerance_blocked(self.handle, float(tol), int(max_iters),
                                                             int(block_positions)))

    def inverse_blocks(self):
        """(iterations, residuals) per block of the most recent tolerance-driven inverse, as numpy arrays."""
        import numpy as np
        n = ctypes.c_int32(0)
        _check(self.lib.revffn_get_inverse_blocks(self.handle, None, None, 0, ctypes.byref(n)))
        it = np.zeros(n.value, dtype=np.int32)
        rs = np.zeros(n.value, dtype=np.float32)
        if n.value:
            _check(self.lib.revffn_get_inverse_blocks(self.handle, it.ctypes.data, rs.ctypes.data, n.value,
                                                      ctypes.byref(n)))
        return it, rs

    def inverse_stats(self):
        """(inverses run, iterations summed, iterations of the last one, residual of the last one)."""
        calls, iters = ctypes.c_int64(0), ctypes.c_int64(0)
        last, res = ctypes.c_int32(0), ctypes.c_float(0.0)
        _check(self.lib.revffn_get_inverse_stats(self.handle, ctypes.byref(calls), ctypes.byref(iters),
                                                 ctypes.byref(last), ctypes.byref(res)))
        return calls.value, iters.value, last.value, res.value

    def enable_taps(self, on=True):
        _check(self.lib.revffn_enable_taps(self.handle, 1 if on else 0))

    def set_kernel_mode(self, mode):
        _check(self.lib.revffn_set_kernel_mode(self.handle, mode))

    def set_helper_streams(self, on=True):
        _check(self.lib.revffn_set_helper_streams(self.handle, 1 if on else 0))

    def profile_enable(self, on=True):
        _check(self.lib.revffn_profile_enable(self.handle, 1 if on else 0))

    def profile_read(self):
        """{kernel family: dict(ms, launches, flops, bytes)} summed since profile_enable (blocks)."""
        out, kid = {}, 0
        while True:
            name = self.lib.revffn_profile_kernel_name(kid)
            if name is None:
                return out
            ms, n, fl, by = ctypes.c_double(), ctypes.c_int64(), ctypes.c_double(), ctypes.c_double()
            _check(self.lib.revffn_profile_read(self.handle, kid, ctypes.byref(ms), ctypes.byref(n),
                                                ctypes.byref(fl), ctypes.byref(by)))
            if n.value:
                out[name.decode()] = dict(ms=ms.value, launches=n.value, flops=fl.value, bytes=by.value)
            kid += 1


def _w(weights):
    return weights if isinstance(weights, Weights) else _struct(Weights, weights)


def _g(grads):
    if grads is None:
        return None
    return grads if isinstance(grads, Grads) else _struct(Grads, grads)


def revffn_forward(ctx, weights, x1, x2, y1, y2, B, S, ld, stream=None):
    w = _w(weights)
    _check(ctx.lib.revffn_forward(ctx.handle, ctypes.byref(w), _ptr(x1), _ptr(x2), _ptr(y1), _ptr(y2),
                                  B, S, ld, _stream(stream)))


def revffn_inverse(ctx, weights, y1, y2, x1, x2, B, S, ld, residual=None, stream=None):
    w = _w(weights)
    _check(ctx.lib.revffn_inverse(ctx.handle, ctypes.byref(w), _ptr(y1), _ptr(y2), _ptr(x1), _ptr(x2),
                                  B, S, ld, _ptr(residual), _stream(stream)))


def revffn_backward(ctx, weights, x1, x2, y1, dy1, dy2, dx1, dx2, grads, B, S, ld, stream=None):
    w, g = _w(weights), _g(grads)
    _check(ctx.lib.revffn_backward(ctx.handle, ctypes.byref(w), _ptr(x1), _ptr(x2), _ptr(y1), _ptr(dy1),
                                   _ptr(dy2), _ptr(dx1), _ptr(dx2), ctypes.byref(g) if g is not None else None,
                                   B, S, ld, _stream(stream)))


def revffn_backward_stored(ctx, weights, x1, x2, y1, dy1, dy2, dx1, dx2, grads, B, S, ld, stream=None):
    w, g = _w(weights), _g(grads)
    _check(ctx.lib.revffn_backward_stored(ctx.handle, ctypes.byref(w), _ptr(x1), _ptr(x2), _ptr(y1), _ptr(dy1),
                                          _ptr(dy2), _ptr(dx1), _ptr(dx2),
                                          ctypes.byref(g) if g is not None else None, B, S, ld, _stream(stream)))


def revffn_inverse_backward(ctx, weights, y1, y2, x1, x2, dy1, dy2, dx1, dx2, grads, B, S, ld, residual=None,
                            stream=None):
    w, g = _w(weights), _g(grads)
    _check(ctx.lib.revffn_inverse_backward(ctx.handle, ctypes.byref(w), _ptr(y1), _ptr(y2), _ptr(x1), _ptr(x2),
                                           _ptr(dy1), _ptr(dy2), _ptr(dx1), _ptr(dx2),
                                           ctypes.byref(g) if g is not None else None, B, S, ld, _ptr(residual),
                                           _stream(stream)))


def revffn_stack_forward(ctx, weights_list, x1, x2, y1, y2, B, S, ld, stream=None):
    arr = (Weights * len(weights_list))(*[_w(w) for w in weights_list])
    _check(ctx.lib.revffn_stack_forward(ctx.handle, arr, len(weights_list), _ptr(x1), _ptr(x2), _ptr(y1),
                                        _ptr(y2), B, S, ld, _stream(stream)))


def revffn_stack_backward(ctx, weights_list, grads_list, y1, y2, dy1, dy2, B, S, ld, stream=None):
    arr = (Weights * len(weights_list))(*[_w(w) for w in weights_list])
    garr = None
    if grads_list is not None:
        garr = (Grads * len(grads_list))(*[_g(g) for g in grads_list])
    _check(ctx.lib.revffn_stack_backward(ctx.handle, arr, garr, len(weights_list), _ptr(y1), _ptr(y2),
                                         _ptr(dy1), _ptr(dy2), B, S, ld, _stream(stream)))


def revffn_get_routing(ctx, idx=None, wts=None, counts=None, offsets=None, row_map=None, stream=None):
    _check(ctx.lib.revffn_get_routing(ctx.handle, _ptr(idx), _ptr(wts), _ptr(counts), _ptr(offsets),
                                      _ptr(row_map), _stream(stream)))


def revffn_get_branch(ctx, which, dst, stream=None):
    _check(ctx.lib.revffn_get_branch(ctx.handle, which, _ptr(dst), _stream(stream)))


def revffn_op_gemm(dtype, kernel_mode, a, b, c, M, N, K, lda, ldb, ldc, a_trans, b_trans, out_f32=False, stream=None):
    _check(load_library().revffn_op_gemm(dtype, kernel_mode, _ptr(a), _ptr(b), _ptr(c), M, N, K, lda, ldb, ldc,
                                         int(a_trans), int(b_trans), int(out_f32), _stream(stream)))


def revffn_op_tile_placement(group_mode, tiles_m, tiles_n, bm, bn, n_groups=1, tile_first=None, n_used=0):
    """Host-only: (n-tile, m-tile, group) of every workgroup of the launch, -1s for workgroups without a tile.
    Returns an int32 numpy array [workgroups, 3]."""
    import numpy as np
    cap = 8 * (tiles_m + 8) * (tiles_n + 8) * (n_groups + 8 if group_mode == 2 else 1)
    out = np.empty((cap, 3), dtype=np.int32)
    tf = None
    if tile_first is not None:
        tf = np.ascontiguousarray(tile_first, dtype=np.int32)
    n = load_library().revffn_op_tile_placement(group_mode, tiles_m, tiles_n, bm, bn, n_groups,
                                                tf.ctypes.data if tf is not None else None, n_used,
                                                out.ctypes.data, cap)
    if n < 0:
        _check(n)
    return out[:n].copy()


def revffn_op_attention_fwd(dtype, kernel_mode, q, k, v, o, lse, B, S, H, dh, causal, stream=None):
    _check(load_library().revffn_op_attention_fwd(dtype, kernel_mode, _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse),
                                                  B, S, H, dh, int(causal), _stream(stream)))


def revffn_op_attention_bwd(dtype, kernel_mode, q, k, v, o, d_o, lse, dvec, dq, dk, dv, B, S, H, dh, causal,
                            stream=None):
    _check(load_library().revffn_op_attention_bwd(dtype, kernel_mode, _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(d_o),
                                                  _ptr(lse), _ptr(dvec), _ptr(dq), _ptr(dk), _ptr(dv), B, S, H, dh,
                                                  int(causal), _stream(stream)))


def revffn_op_attention_bwd_noalloc(dtype, kernel_mode, q, k, v, o, d_o, lse, dq, dk, dv, B, S, H, dh, causal,
                                    stream=None):
    _check(load_library().revffn_op_attention_bwd_noalloc(dtype, kernel_mode, _ptr(q), _ptr(k), _ptr(v), _ptr(o),
                                                          _ptr(d_o), _ptr(lse), _ptr(dq), _ptr(dk), _ptr(dv), B, S, H,
                                                          dh, int(causal), _stream(stream)))


def _m(merged):
    if isinstance(merged, Merged):
        return merged
    s = Merged()
    for n in MERGED_FIELDS:
        setattr(s, n, _ptr(merged.get(n)))
    return s


def revffn_merge_adapters(ctx, weights, merged, stream=None):
    w, m = _w(weights), _m(merged)
    _check(ctx.lib.revffn_merge_adapters(ctx.handle, ctypes.byref(w), ctypes.byref(m), _stream(stream)))


def revffn_forward_merged(ctx, weights, merged, x1, x2, y1, y2, B, S, ld, stream=None):
    w, m = _w(weights), _m(merged)
    _check(ctx.lib.revffn_forward_merged(ctx.handle, ctypes.byref(w), ctypes.byref(m), _ptr(x1), _ptr(x2), _ptr(y1),
                                         _ptr(y2), B, S, ld, _stream(stream)))


def revffn_inverse_merged(ctx, weights, merged, y1, y2, x1, x2, B, S, ld, residual=None, stream=None):
    w, m = _w(weights), _m(merged)
    _check(ctx.lib.revffn_inverse_merged(ctx.handle, ctypes.byref(w), ctypes.byref(m), _ptr(y1), _ptr(y2), _ptr(x1),
                                         _ptr(x2), B, S, ld, _ptr(residual), _stream(stream)))
