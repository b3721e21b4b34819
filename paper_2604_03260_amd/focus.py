"""Thin ctypes binding of libfocus.so: argument marshalling only.

The functions mirror include/focus.h one to one (focus_workspace_size,
focus_assign, focus_attn_fwd, focus_workspace_views, focus_route_workspace_size,
focus_route, focus_assign_tokens, focus_attn_fwd_set, focus_attn_merge, focus_attn_fwd_two_call,
focus_decode_state_size, focus_decode_prefill, focus_decode_step, focus_decode_state_views, focus_last_error, focus_version).  Tensors are torch CUDA tensors used purely as device buffers;
the calls are enqueued on torch's current stream.  There is no CPU fallback: a
missing library is an error.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfocus.so")

FOCUS_OK, FOCUS_EINVAL, FOCUS_EUNSUPPORTED, FOCUS_EWORKSPACE, FOCUS_EHIP = 0, -1, -2, -3, -4
FOCUS_F32, FOCUS_BF16, FOCUS_F16 = 0, 1, 2
DTYPES = {"f32": FOCUS_F32, "bf16": FOCUS_BF16, "f16": FOCUS_F16}
TORCH_DTYPE_CODES = {torch.float32: FOCUS_F32, torch.bfloat16: FOCUS_BF16, torch.float16: FOCUS_F16}

EXPORTS = ("focus_workspace_size", "focus_assign", "focus_attn_fwd", "focus_workspace_views",
           "focus_route_workspace_size", "focus_route", "focus_route_noalloc", "focus_assign_tokens",
           "focus_attn_fwd_set", "focus_attn_merge", "focus_attn_fwd_two_call",
           "focus_decode_state_size", "focus_decode_prefill", "focus_decode_step",
           "focus_decode_state_views", "focus_decode_step_at",
           "focus_decode_prefill_tokens", "focus_decode_step_tokens",
           "focus_soft_workspace_size", "focus_attn_soft_fwd",
           "focus_attn_fwd_vector", "focus_attn_soft_fwd_vector",
           "focus_last_error", "focus_version", "focus_build_id")


class FocusRouteParams(ctypes.Structure):
    _fields_ = [
        ("B", ctypes.c_int32), ("n", ctypes.c_int32), ("d_model", ctypes.c_int32), ("d_g", ctypes.c_int32),
        ("K", ctypes.c_int32), ("topk", ctypes.c_int32), ("dtype", ctypes.c_int32),
        ("sinkhorn_iters", ctypes.c_int32), ("tau", ctypes.c_double),
    ]


class FocusParams(ctypes.Structure):
    _fields_ = [
        ("B", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32),
        ("n", ctypes.c_int32), ("d", ctypes.c_int32),
        ("K", ctypes.c_int32), ("topk", ctypes.c_int32),
        ("window", ctypes.c_int32), ("causal", ctypes.c_int32), ("dtype", ctypes.c_int32),
        ("scale", ctypes.c_float), ("softcap", ctypes.c_float),
        ("head_map", ctypes.POINTER(ctypes.c_int32)),
        ("q_strides", ctypes.c_int64 * 3), ("kv_strides", ctypes.c_int64 * 3), ("o_strides", ctypes.c_int64 * 3),
    ]


class FocusError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("libfocus status %d: %s" % (status, message))
        self.status = status


_lib = None


def load_library():
    """Loads libfocus.so; builds it first when no built library is present, or when the one present was
    compiled from other sources than those on disk (a stale library must never pass for the current code)."""
    global _lib
    if _lib is not None:
        return _lib
    from . import build as _build
    if not os.path.exists(LIB_PATH):
        _build.build_library()
    lib = ctypes.CDLL(LIB_PATH)
    want = _build.source_id()
    try:
        lib.focus_build_id.restype = ctypes.c_char_p
        have = lib.focus_build_id().decode()
    except AttributeError:
        have = "none"
    if have != want:
        import sys
        sys.stderr.write("libfocus.so was built from other sources (%s, now %s): rebuilding\n" % (have, want))
        del lib
        _build.build_library()
        lib = ctypes.CDLL(LIB_PATH)
        lib.focus_build_id.restype = ctypes.c_char_p
        if lib.focus_build_id().decode() != want:
            raise RuntimeError("libfocus.so does not match its sources after a rebuild")
    vp, sz = ctypes.c_void_p, ctypes.c_size_t
    pp = ctypes.POINTER(FocusParams)
    lib.focus_workspace_size.argtypes = [pp, ctypes.POINTER(sz)]
    lib.focus_workspace_size.restype = ctypes.c_int
    lib.focus_assign.argtypes = [pp, vp, vp, vp, vp, sz, vp]
    lib.focus_assign.restype = ctypes.c_int
    lib.focus_attn_fwd.argtypes = [pp, vp, vp, vp, vp, sz, vp, vp, vp, vp]
    lib.focus_attn_fwd.restype = ctypes.c_int
    lib.focus_attn_fwd_vector.argtypes = [pp, vp, vp, vp, vp, sz, vp, vp, vp, vp]
    lib.focus_attn_fwd_vector.restype = ctypes.c_int
    lib.focus_workspace_views.argtypes = [pp, vp] + [ctypes.POINTER(vp)] * 6
    lib.focus_workspace_views.restype = ctypes.c_int
    lib.focus_attn_fwd_set.argtypes = [pp, ctypes.c_int32, vp, vp, vp, vp, sz, vp, vp, vp, vp]
    lib.focus_attn_fwd_set.restype = ctypes.c_int
    lib.focus_attn_merge.argtypes = [ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, vp, vp, vp, vp, vp, vp, vp]
    lib.focus_attn_merge.restype = ctypes.c_int
    lib.focus_attn_fwd_two_call.argtypes = [pp, vp, vp, vp, vp, sz, vp, vp, vp, vp, vp]
    lib.focus_attn_fwd_two_call.restype = ctypes.c_int
    lib.focus_soft_workspace_size.argtypes = [pp, ctypes.POINTER(sz)]
    lib.focus_soft_workspace_size.restype = ctypes.c_int
    for fn in (lib.focus_attn_soft_fwd, lib.focus_attn_soft_fwd_vector):
        fn.argtypes = [pp, ctypes.c_float, vp, vp, vp, vp, vp, sz, vp, vp, vp]
        fn.restype = ctypes.c_int
    lib.focus_decode_state_size.argtypes = [pp, ctypes.POINTER(sz)]
    lib.focus_decode_state_size.restype = ctypes.c_int
    lib.focus_decode_prefill.argtypes = [pp, ctypes.c_int32, vp, vp, vp, sz, vp]
    lib.focus_decode_prefill.restype = ctypes.c_int
    lib.focus_decode_step.argtypes = [pp, ctypes.c_int32, vp, vp, vp, vp, vp, vp, vp, sz, vp, vp, vp, vp]
    lib.focus_decode_step.restype = ctypes.c_int
    lib.focus_decode_prefill_tokens.argtypes = [pp, ctypes.c_int32, vp, vp, sz, vp]
    lib.focus_decode_prefill_tokens.restype = ctypes.c_int
    lib.focus_decode_step_tokens.argtypes = [pp, ctypes.c_int32, vp, vp, vp, vp, vp, vp, vp, sz, vp, vp, vp, vp]
    lib.focus_decode_step_tokens.restype = ctypes.c_int
    lib.focus_decode_step_at.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp, vp, vp, vp]
    lib.focus_decode_step_at.restype = ctypes.c_int
    lib.focus_decode_state_views.argtypes = [pp, vp] + [ctypes.POINTER(vp)] * 4
    lib.focus_decode_state_views.restype = ctypes.c_int
    rp = ctypes.POINTER(FocusRouteParams)
    lib.focus_route_workspace_size.argtypes = [rp, ctypes.POINTER(sz)]
    lib.focus_route_workspace_size.restype = ctypes.c_int
    lib.focus_route.argtypes = [rp, vp, vp, vp, vp, sz, vp, vp, vp]
    lib.focus_route.restype = ctypes.c_int
    lib.focus_route_noalloc.argtypes = [rp, vp, vp, vp, vp, vp, vp]
    lib.focus_route_noalloc.restype = ctypes.c_int
    lib.focus_assign_tokens.argtypes = [pp, vp, vp, vp, sz, vp, vp]
    lib.focus_assign_tokens.restype = ctypes.c_int
    lib.focus_last_error.argtypes = []
    lib.focus_last_error.restype = ctypes.c_char_p
    lib.focus_version.argtypes = []
    lib.focus_version.restype = ctypes.c_int
    lib.focus_build_id.argtypes = []
    _lib = lib
    return lib


def strides_of(t):
    """(batch, head, position) strides in elements of a torch tensor indexed [B,H,n,d] (any view whose last
    dimension is contiguous, e.g. x.view(B, n, H, d).permute(0, 2, 1, 3))."""
    assert t.dim() == 4 and t.stride(3) == 1
    return tuple(int(x) for x in t.stride()[:3])


def make_params(B, Hq, Hkv, n, d, K, topk, window, causal=True, dtype="bf16", scale=0.0, softcap=0.0,
                head_map=None, q_strides=None, kv_strides=None, o_strides=None):
    """Returns FocusParams (it keeps the host head_map array alive).  Strides: None = contiguous [B,H,n,d]."""
    keep = None
    hm = None
    if head_map is not None:
        keep = (ctypes.c_int32 * len(head_map))(*[int(x) for x in head_map])
        hm = ctypes.cast(keep, ctypes.POINTER(ctypes.c_int32))
    arr = lambda st: (ctypes.c_int64 * 3)(*(st if st is not None else (0, 0, 0)))
    p = FocusParams(B, Hq, Hkv, n, d, K, topk, window, 1 if causal else 0,
                    DTYPES[dtype], scale, softcap, hm, arr(q_strides), arr(kv_strides), arr(o_strides))
    p._keep = keep
    return p


def _check(st):
    if st != FOCUS_OK:
        raise FocusError(st, load_library().focus_last_error().decode())


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else ctypes.c_void_p(0)


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def focus_version():
    return load_library().focus_version()


def focus_last_error():
    return load_library().focus_last_error().decode()


def focus_workspace_size(p):
    out = ctypes.c_size_t(0)
    _check(load_library().focus_workspace_size(ctypes.byref(p), ctypes.byref(out)))
    return out.value


def focus_assign(p, q, k, centroids, workspace):
    _check(load_library().focus_assign(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(centroids), _ptr(workspace),
                                       workspace.numel() * workspace.element_size(), _stream()))


def focus_attn_fwd(p, q, k, v, workspace, out, lse=None, row_pairs=None, vector=False):
    fn = load_library().focus_attn_fwd_vector if vector else load_library().focus_attn_fwd
    _check(fn(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(workspace),
              workspace.numel() * workspace.element_size(), _ptr(out), _ptr(lse), _ptr(row_pairs), _stream()))


FOCUS_PAIRS_ALL, FOCUS_PAIRS_SHARED, FOCUS_PAIRS_CROSS_LOCAL = 0, 1, 2


def focus_soft_workspace_size(p):
    out = ctypes.c_size_t(0)
    _check(load_library().focus_soft_workspace_size(ctypes.byref(p), ctypes.byref(out)))
    return out.value


def alloc_soft_workspace(p, device="cuda"):
    nbytes = focus_soft_workspace_size(p)
    return torch.empty(((nbytes + 255) // 256) * 256, dtype=torch.uint8, device=device)


def focus_attn_soft_fwd(p, lam, g, q, k, v, workspace, out, lse=None, vector=False):
    """Sec. 2 Eq. 2: g [B,n,K] float32 on the device, lam the slope of the gate."""
    assert g.dtype == torch.float32 and g.is_contiguous()
    fn = load_library().focus_attn_soft_fwd_vector if vector else load_library().focus_attn_soft_fwd
    _check(fn(ctypes.byref(p), float(lam), _ptr(g), _ptr(q), _ptr(k), _ptr(v), _ptr(workspace),
              workspace.numel() * workspace.element_size(), _ptr(out), _ptr(lse), _stream()))


def focus_attn_fwd_set(p, pair_set, q, k, v, workspace, out, lse=None, row_pairs=None):
    _check(load_library().focus_attn_fwd_set(ctypes.byref(p), pair_set, _ptr(q), _ptr(k), _ptr(v), _ptr(workspace),
                                             workspace.numel() * workspace.element_size(), _ptr(out), _ptr(lse),
                                             _ptr(row_pairs), _stream()))


def focus_attn_merge(out_a, lse_a, out_b, lse_b, out, lse=None):
    d = out_a.shape[-1]
    rows = out_a.numel() // d
    dtype = TORCH_DTYPE_CODES[out_a.dtype]
    _check(load_library().focus_attn_merge(rows, d, dtype, _ptr(out_a), _ptr(lse_a), _ptr(out_b), _ptr(lse_b),
                                           _ptr(out), _ptr(lse), _stream()))


def focus_attn_fwd_two_call(p, q, k, v, workspace, out, lse, part_out, part_lse):
    _check(load_library().focus_attn_fwd_two_call(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(workspace),
                                                  workspace.numel() * workspace.element_size(), _ptr(out), _ptr(lse),
                                                  _ptr(part_out), _ptr(part_lse), _stream()))


def focus_decode_state_size(p):
    out = ctypes.c_size_t(0)
    _check(load_library().focus_decode_state_size(ctypes.byref(p), ctypes.byref(out)))
    return out.value


def alloc_decode_state(p, device="cuda"):
    nbytes = focus_decode_state_size(p)
    return torch.empty(((nbytes + 255) // 256) * 256, dtype=torch.uint8, device=device)


def focus_decode_prefill(p, n_ctx, k_cache, centroids, state):
    _check(load_library().focus_decode_prefill(ctypes.byref(p), n_ctx, _ptr(k_cache), _ptr(centroids), _ptr(state),
                                               state.numel() * state.element_size(), _stream()))


def focus_decode_step(p, pos, q_new, k_new, v_new, centroids, k_cache, v_cache, state, out, lse=None, row_pairs=None):
    _check(load_library().focus_decode_step(ctypes.byref(p), pos, _ptr(q_new), _ptr(k_new), _ptr(v_new),
                                            _ptr(centroids), _ptr(k_cache), _ptr(v_cache), _ptr(state),
                                            state.numel() * state.element_size(), _ptr(out), _ptr(lse),
                                            _ptr(row_pairs), _stream()))


def focus_decode_prefill_tokens(p, n_ctx, token_masks, state):
    _check(load_library().focus_decode_prefill_tokens(ctypes.byref(p), n_ctx, _ptr(token_masks), _ptr(state),
                                                      state.numel() * state.element_size(), _stream()))


def focus_decode_step_tokens(p, pos, token_mask, q_new, k_new, v_new, k_cache, v_cache, state, out, lse=None,
                             row_pairs=None):
    _check(load_library().focus_decode_step_tokens(ctypes.byref(p), pos, _ptr(token_mask), _ptr(q_new), _ptr(k_new),
                                                   _ptr(v_new), _ptr(k_cache), _ptr(v_cache), _ptr(state),
                                                   state.numel() * state.element_size(), _ptr(out), _ptr(lse),
                                                   _ptr(row_pairs), _stream()))


def focus_decode_step_at(p, pos_dev, q_new, k_new, v_new, centroids, k_cache, v_cache, state, out, lse=None,
                         row_pairs=None):
    """The step with the positions in device memory (int32 [B], one per sequence; outside [0, n) = skip the
    sequence): capturable once, and the sequences of a batch may stand at different positions."""
    assert pos_dev.dtype == torch.int32 and pos_dev.is_cuda and pos_dev.numel() == p.B
    _check(load_library().focus_decode_step_at(ctypes.byref(p), _ptr(pos_dev), _ptr(q_new), _ptr(k_new), _ptr(v_new),
                                               _ptr(centroids), _ptr(k_cache), _ptr(v_cache), _ptr(state),
                                               state.numel() * state.element_size(), _ptr(out), _ptr(lse),
                                               _ptr(row_pairs), _stream()))


def focus_decode_state_views(p, state):
    """Returns dict of torch int32 tensors aliasing the decode state (no copies)."""
    ptrs = [ctypes.c_void_p(0) for _ in range(4)]
    _check(load_library().focus_decode_state_views(ctypes.byref(p), _ptr(state), *[ctypes.byref(x) for x in ptrs]))
    base = state.data_ptr()
    raw = state.view(torch.uint8).reshape(-1)

    def view(ptr, shape):
        count = 1
        for x in shape:
            count *= x
        off = ptr.value - base
        return raw[off:off + 4 * count].view(torch.int32).view(*shape)
    B, Hq, Hkv, n, K = p.B, p.Hq, p.Hkv, p.n, p.K
    return {"mk": view(ptrs[0], (B, Hkv, n)), "lists": view(ptrs[1], (B, Hkv, K, n)),
            "counts": view(ptrs[2], (B, Hkv, K)), "mq": view(ptrs[3], (B, Hq))}


def make_route_params(B, n, d_model, d_g, K, topk, dtype="bf16", sinkhorn_iters=10, tau=0.1):
    return FocusRouteParams(B, n, d_model, d_g, K, topk, DTYPES[dtype],
                            sinkhorn_iters, tau)


def focus_route_workspace_size(rp):
    out = ctypes.c_size_t(0)
    _check(load_library().focus_route_workspace_size(ctypes.byref(rp), ctypes.byref(out)))
    return out.value


def alloc_route_workspace(rp, device="cuda"):
    nbytes = focus_route_workspace_size(rp)
    return torch.empty(((nbytes + 255) // 256) * 256, dtype=torch.uint8, device=device)


def focus_route(rp, hidden, w_g, centroids, route_workspace, token_masks, soft=None):
    _check(load_library().focus_route(ctypes.byref(rp), _ptr(hidden), _ptr(w_g), _ptr(centroids),
                                      _ptr(route_workspace),
                                      route_workspace.numel() * route_workspace.element_size(),
                                      _ptr(token_masks), _ptr(soft), _stream()))


def focus_route_noalloc(rp, hidden, w_g, centroids, token_masks, soft=None):
    """focus_route with the library's static scratch instead of a workspace (no allocation anywhere)."""
    _check(load_library().focus_route_noalloc(ctypes.byref(rp), _ptr(hidden), _ptr(w_g), _ptr(centroids),
                                              _ptr(token_masks), _ptr(soft), _stream()))


def focus_assign_tokens(p, token_masks, k, workspace, invalid_count=None):
    _check(load_library().focus_assign_tokens(ctypes.byref(p), _ptr(token_masks), _ptr(k), _ptr(workspace),
                                              workspace.numel() * workspace.element_size(),
                                              _ptr(invalid_count), _stream()))


def focus_workspace_views(p, workspace):
    """Returns dict of torch tensors aliasing the workspace (no copies)."""
    lib = load_library()
    ptrs = [ctypes.c_void_p(0) for _ in range(6)]
    _check(lib.focus_workspace_views(ctypes.byref(p), _ptr(workspace), *[ctypes.byref(x) for x in ptrs]))
    base = workspace.data_ptr()
    raw = workspace.view(torch.uint8).reshape(-1)

    def view(ptr, count):
        off = ptr.value - base
        return raw[off:off + 4 * count].view(torch.int32)
    B, Hq, Hkv, n, K, topk = p.B, p.Hq, p.Hkv, p.n, p.K, p.topk
    return {
        "mq": view(ptrs[0], B * Hq * n).view(B, Hq, n),
        "mk": view(ptrs[1], B * Hkv * n).view(B, Hkv, n),
        "q_group_counts": view(ptrs[2], B * Hq * K).view(B, Hq, K),
        "k_group_counts": view(ptrs[3], B * Hkv * K).view(B, Hkv, K),
        "q_group_lists": view(ptrs[4], B * Hq * topk * n).view(B, Hq, topk * n),
        "k_group_lists": view(ptrs[5], B * Hkv * topk * n).view(B, Hkv, topk * n),
    }


def alloc_workspace(p, device="cuda"):
    nbytes = focus_workspace_size(p)
    return torch.empty(((nbytes + 255) // 256) * 256, dtype=torch.uint8, device=device)
