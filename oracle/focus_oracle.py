"""ctypes front-end of the fp64 CPU oracle (oracle/focus_oracle.c).

TEST INFRASTRUCTURE: only tests, the smoke check and the benchmark's
cpu_baseline leg import this.  It holds no arithmetic of the method: it
marshals numpy arrays into the C routines and builds the shared object with
gcc when it is missing.  It never imports the HIP package.

Arrays: q [B,Hq,n,d], k/v [B,Hkv,n,d] as float32, or as uint16 holding bf16 bit
patterns; centroids [Hkv,K,d] float32.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "focus_oracle.c")
_LIB = os.path.join(_HERE, "libfocus_oracle.so")


def build(force=False):
    """Compile the oracle with gcc (-O2, OpenMP, IEEE semantics)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-Wall", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


class _Params(ctypes.Structure):
    _fields_ = [
        ("B", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32),
        ("n", ctypes.c_int32), ("d", ctypes.c_int32),
        ("K", ctypes.c_int32), ("topk", ctypes.c_int32), ("window", ctypes.c_int32),
        ("causal", ctypes.c_int32), ("dtype", ctypes.c_int32),
        ("scale", ctypes.c_double), ("softcap", ctypes.c_double),
        ("head_map", ctypes.c_void_p),
    ]


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        for name in ("focus_oracle_scores", "focus_oracle_topk_masks", "focus_oracle_membership",
                     "focus_oracle_group_lists", "focus_oracle_attn_rows",
                     "focus_oracle_pair_counts", "focus_oracle_num_threads"):
            getattr(lib, name).restype = ctypes.c_int
        _lib = lib
    return _lib


def num_threads():
    return int(_load().focus_oracle_num_threads())


DTYPES = {"f32": 0, "bf16": 1, "f16": 2}      # 16-bit types travel as uint16 bit patterns


def _ptr(a):
    return ctypes.c_void_p(a.ctypes.data) if a is not None else ctypes.c_void_p(0)


class Problem:
    """Shape and parameters of one Focus attention problem (host side)."""

    def __init__(self, B, Hq, Hkv, n, d, K, topk, window, causal=True, dtype="f32",
                 scale=0.0, softcap=0.0, head_map=None):
        self.B, self.Hq, self.Hkv, self.n, self.d = B, Hq, Hkv, n, d
        self.K, self.topk, self.window = K, topk, window
        self.causal = bool(causal)
        self.dtype = dtype
        self.scale, self.softcap = float(scale), float(softcap)
        self.head_map = None if head_map is None else np.ascontiguousarray(head_map, dtype=np.int32)

    def _c(self):
        p = _Params(self.B, self.Hq, self.Hkv, self.n, self.d, self.K, self.topk, self.window,
                    1 if self.causal else 0, DTYPES[self.dtype],
                    self.scale, self.softcap,
                    self.head_map.ctypes.data if self.head_map is not None else None)
        return p

    def _check_tensor(self, x, H):
        want = np.float32 if self.dtype == "f32" else np.uint16
        assert x.dtype == want, (x.dtype, want)
        assert x.shape == (self.B, H, self.n, self.d), x.shape
        assert x.flags["C_CONTIGUOUS"]


def _rc(rc, what):
    if rc != 0:
        raise RuntimeError("oracle %s failed with code %d" % (what, rc))


def scores(pb, x, centroids, is_query):
    H = pb.Hq if is_query else pb.Hkv
    pb._check_tensor(x, H)
    c = np.ascontiguousarray(centroids, dtype=np.float32)
    assert c.shape == (pb.Hkv, pb.K, pb.d)
    out = np.empty((pb.B, H, pb.n, pb.K), dtype=np.float64)
    p = pb._c()
    _rc(_load().focus_oracle_scores(ctypes.byref(p), _ptr(x), int(is_query), _ptr(c), _ptr(out)),
        "scores")
    return out


def topk_masks(pb, sc):
    sc = np.ascontiguousarray(sc, dtype=np.float64)
    B, H, n, K = sc.shape
    out = np.empty((B, H, n), dtype=np.uint32)
    p = pb._c()
    _rc(_load().focus_oracle_topk_masks(ctypes.byref(p), _ptr(sc), int(H), _ptr(out)), "topk")
    return out


def membership(pb, x, centroids, is_query):
    H = pb.Hq if is_query else pb.Hkv
    pb._check_tensor(x, H)
    c = np.ascontiguousarray(centroids, dtype=np.float32)
    assert c.shape == (pb.Hkv, pb.K, pb.d)
    out = np.empty((pb.B, H, pb.n), dtype=np.uint32)
    p = pb._c()
    _rc(_load().focus_oracle_membership(ctypes.byref(p), _ptr(x), int(is_query), _ptr(c), _ptr(out)),
        "membership")
    return out


def group_lists(pb, masks):
    masks = np.ascontiguousarray(masks, dtype=np.uint32)
    B, H, n = masks.shape
    counts = np.empty((B, H, pb.K), dtype=np.int32)
    lists = np.full((B, H, pb.topk * n), -1, dtype=np.int32)
    p = pb._c()
    _rc(_load().focus_oracle_group_lists(ctypes.byref(p), _ptr(masks), int(H), _ptr(counts),
                                         _ptr(lists)), "group_lists")
    return counts, lists


PAIR_SETS = {"all": 0, "A": 1, "B": 2}


def attn_rows(pb, q, k, v, mq, mk, rows=None, want_probs=False, pair_set="all"):
    """rows: int array [nrows,3] of (b,h,i) or None for every row.  pair_set: "all" (the whole mask),
    "A" (pairs that share a group) or "B" (window pairs that share none), App. D.
    Returns out [nrows,d] f64, lse [nrows] f64, row_pairs [nrows] i64 (and probs [nrows,n])."""
    pb._check_tensor(q, pb.Hq)
    pb._check_tensor(k, pb.Hkv)
    pb._check_tensor(v, pb.Hkv)
    mq = np.ascontiguousarray(mq, dtype=np.uint32)
    mk = np.ascontiguousarray(mk, dtype=np.uint32)
    assert mq.shape == (pb.B, pb.Hq, pb.n) and mk.shape == (pb.B, pb.Hkv, pb.n)
    if rows is None:
        nrows = pb.B * pb.Hq * pb.n
        rows_arr = None
    else:
        rows_arr = np.ascontiguousarray(rows, dtype=np.int32).reshape(-1, 3)
        nrows = rows_arr.shape[0]
    out = np.empty((nrows, pb.d), dtype=np.float64)
    lse = np.empty((nrows,), dtype=np.float64)
    pairs = np.empty((nrows,), dtype=np.int64)
    probs = np.zeros((nrows, pb.n), dtype=np.float64) if want_probs else None
    p = pb._c()
    lib = _load()
    lib.focus_oracle_attn_rows_set.restype = ctypes.c_int
    _rc(lib.focus_oracle_attn_rows_set(ctypes.byref(p), ctypes.c_int32(PAIR_SETS[pair_set]), _ptr(q), _ptr(k),
                                       _ptr(v), _ptr(mq), _ptr(mk), ctypes.c_int64(nrows), _ptr(rows_arr),
                                       _ptr(out), _ptr(lse), _ptr(pairs), _ptr(probs)), "attn_rows")
    if want_probs:
        return out, lse, pairs, probs
    return out, lse, pairs


def soft_rows(pb, lam, g, q, k, v, rows=None, want_probs=False):
    """Sec. 2 Eq. 2 (soft-gated attention of training).  g [B,n,K] float32, lam the gate's slope.
    rows as in attn_rows.  Returns out [nrows,d] f64, lse [nrows] f64 (and probs [nrows,n])."""
    pb._check_tensor(q, pb.Hq)
    pb._check_tensor(k, pb.Hkv)
    pb._check_tensor(v, pb.Hkv)
    g = np.ascontiguousarray(g, dtype=np.float32)
    assert g.shape == (pb.B, pb.n, pb.K), g.shape
    if rows is None:
        nrows = pb.B * pb.Hq * pb.n
        rows_arr = None
    else:
        rows_arr = np.ascontiguousarray(rows, dtype=np.int32).reshape(-1, 3)
        nrows = rows_arr.shape[0]
    out = np.empty((nrows, pb.d), dtype=np.float64)
    lse = np.empty((nrows,), dtype=np.float64)
    probs = np.zeros((nrows, pb.n), dtype=np.float64) if want_probs else None
    p = pb._c()
    lib = _load()
    lib.focus_oracle_soft_rows.restype = ctypes.c_int
    _rc(lib.focus_oracle_soft_rows(ctypes.byref(p), ctypes.c_double(float(lam)), _ptr(g), _ptr(q), _ptr(k), _ptr(v),
                                   ctypes.c_int64(nrows), _ptr(rows_arr), _ptr(out), _ptr(lse), _ptr(probs)),
        "soft_rows")
    if want_probs:
        return out, lse, probs
    return out, lse


def merge(oa, la, ob, lb):
    """App. D merge of two disjoint partial attentions: returns (out [nrows,d], lse [nrows])."""
    lib = _load()
    lib.focus_oracle_merge.restype = ctypes.c_int
    oa, ob = (np.ascontiguousarray(x, dtype=np.float64) for x in (oa, ob))
    la, lb = (np.ascontiguousarray(x, dtype=np.float64) for x in (la, lb))
    nrows, d = oa.shape
    assert ob.shape == (nrows, d) and la.shape == (nrows,) and lb.shape == (nrows,)
    out = np.empty((nrows, d), dtype=np.float64)
    lse = np.empty((nrows,), dtype=np.float64)
    _rc(lib.focus_oracle_merge(ctypes.c_int64(nrows), ctypes.c_int32(d), _ptr(oa), _ptr(la), _ptr(ob), _ptr(lb),
                               _ptr(out), _ptr(lse)), "merge")
    return out, lse


def pair_counts(pb, mq, mk):
    """Closed-form (inclusion-exclusion) counts: allowed [B,Hq] u64, group_pairs [B,Hq,K] u64."""
    mq = np.ascontiguousarray(mq, dtype=np.uint32)
    mk = np.ascontiguousarray(mk, dtype=np.uint32)
    allowed = np.zeros((pb.B, pb.Hq), dtype=np.uint64)
    gp = np.zeros((pb.B, pb.Hq, pb.K), dtype=np.uint64)
    p = pb._c()
    _rc(_load().focus_oracle_pair_counts(ctypes.byref(p), _ptr(mq), _ptr(mk), _ptr(allowed), _ptr(gp)),
        "pair_counts")
    return allowed, gp


def route(hidden, wg, cent, topk, tau=0.1, iters=10, dtype="f32", want_soft=False):
    """The paper's router (Sec. 2 Eq. 1 + Sinkhorn).  hidden [B,n,dm] (float32, or uint16 bf16 bits),
    wg [dm,dg] f32, cent [K,dg] f32.  Returns masks [B,n] u32 (and z [B,n,dg], g [B,n,K] f64)."""
    lib = _load()
    lib.focus_oracle_route.restype = ctypes.c_int
    want = np.float32 if dtype == "f32" else np.uint16
    hidden = np.ascontiguousarray(hidden)
    assert hidden.dtype == want and hidden.ndim == 3
    B, n, dm = hidden.shape
    wg = np.ascontiguousarray(wg, dtype=np.float32)
    cent = np.ascontiguousarray(cent, dtype=np.float32)
    dg, K = wg.shape[1], cent.shape[0]
    assert wg.shape == (dm, dg) and cent.shape == (K, dg) and dg <= 256
    masks = np.empty((B, n), dtype=np.uint32)
    z = np.empty((B, n, dg), dtype=np.float64) if want_soft else None
    g = np.empty((B, n, K), dtype=np.float64) if want_soft else None
    _rc(lib.focus_oracle_route(ctypes.c_int32(B), ctypes.c_int32(n), ctypes.c_int32(dm), ctypes.c_int32(dg),
                               ctypes.c_int32(K), ctypes.c_int32(topk),
                               ctypes.c_int32(DTYPES[dtype]), _ptr(hidden), _ptr(wg), _ptr(cent),
                               ctypes.c_double(tau), ctypes.c_int32(iters), _ptr(z), _ptr(g), _ptr(masks)),
        "route")
    if want_soft:
        return masks, z, g
    return masks


def broadcast_masks(pb, token_masks):
    """One mask per token -> (mq [B,Hq,n], mk [B,Hkv,n])."""
    lib = _load()
    lib.focus_oracle_broadcast_masks.restype = ctypes.c_int
    tm = np.ascontiguousarray(token_masks, dtype=np.uint32)
    assert tm.shape == (pb.B, pb.n)
    mq = np.empty((pb.B, pb.Hq, pb.n), dtype=np.uint32)
    mk = np.empty((pb.B, pb.Hkv, pb.n), dtype=np.uint32)
    p = pb._c()
    _rc(lib.focus_oracle_broadcast_masks(ctypes.byref(p), _ptr(tm), _ptr(mq), _ptr(mk)), "broadcast_masks")
    return mq, mk
