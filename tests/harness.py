"""Shared helpers of the GPU parity tests: run the HIP path through the C ABI
binding and the CPU oracle on the same bytes."""
import numpy as np
import torch

from oracle import focus_oracle as fo
from paper_2604_03260_amd import focus, workloads

# stated tolerances of the benchmark spec: bf16 max-abs 2e-2 / mean-abs 2e-3, fp32 1e-5; fp16 (three more
# fraction bits than bf16 in the inputs' storage, the rounded probabilities and the output) a fifth of bf16's
TOL = {"bf16": dict(out_max=2e-2, out_mean=2e-3, lse=1e-2), "f32": dict(out_max=1e-5, out_mean=1e-6, lse=1e-5),
       "f16": dict(out_max=4e-3, out_mean=4e-4, lse=2e-3)}


def params_of(wl, head_map=None, scale=0.0):
    return focus.make_params(wl.B, wl.Hq, wl.Hkv, wl.n, wl.d, wl.K, wl.topk, wl.window, causal=wl.causal,
                             dtype=wl.dtype, scale=scale, softcap=wl.softcap, head_map=head_map)


def problem_of(wl, head_map=None, scale=0.0):
    return fo.Problem(wl.B, wl.Hq, wl.Hkv, wl.n, wl.d, wl.K, wl.topk, wl.window, causal=wl.causal,
                      dtype=wl.dtype, scale=scale, softcap=wl.softcap, head_map=head_map)


def run_gpu(wl, inp, head_map=None, scale=0.0, vector=False, want_pairs=True, want_lse=True):
    p = params_of(wl, head_map, scale)
    ws = focus.alloc_workspace(p)
    focus.focus_assign(p, inp["q"], inp["k"], inp["centroids"], ws)
    out = torch.empty_like(inp["q"])
    lse = torch.empty((wl.B, wl.Hq, wl.n), dtype=torch.float32, device="cuda") if want_lse else None
    rp = torch.empty((wl.B, wl.Hq, wl.n), dtype=torch.int32, device="cuda") if want_pairs else None
    focus.focus_attn_fwd(p, inp["q"], inp["k"], inp["v"], ws, out, lse, rp, vector=vector)
    torch.cuda.synchronize()
    views = focus.focus_workspace_views(p, ws)
    return dict(out=out, lse=lse, row_pairs=rp, views=views, ws=ws, params=p)


def oracle_membership(wl, inp, head_map=None):
    pb = problem_of(wl, head_map)
    qh, kh = workloads.to_host_bits(inp["q"]), workloads.to_host_bits(inp["k"])
    c = inp["centroids"].cpu().numpy()
    return fo.membership(pb, qh, c, True), fo.membership(pb, kh, c, False)


def check_assign(wl, inp, res, head_map=None):
    """Membership masks, group counts and lists: bit-exact."""
    pb = problem_of(wl, head_map)
    mq, mk = oracle_membership(wl, inp, head_map)
    v = res["views"]
    got_mq = v["mq"].cpu().numpy().view(np.uint32)
    got_mk = v["mk"].cpu().numpy().view(np.uint32)
    assert np.array_equal(got_mq, mq), "query membership differs in %d places" % int((got_mq != mq).sum())
    assert np.array_equal(got_mk, mk), "key membership differs in %d places" % int((got_mk != mk).sum())
    for side, m in (("q", mq), ("k", mk)):
        counts, lists = fo.group_lists(pb, m)
        assert np.array_equal(v[side + "_group_counts"].cpu().numpy(), counts)
        assert np.array_equal(v[side + "_group_lists"].cpu().numpy(), lists)
    return mq, mk


def host_inputs(inp):
    """q, k, v as the host arrays the oracle takes (the same bytes)."""
    return tuple(workloads.to_host_bits(inp[x]) for x in ("q", "k", "v"))


def check_attn(wl, inp, res, mq, mk, rows=None, head_map=None, scale=0.0, tol=None, host=None):
    """Outputs against the oracle on `rows` ((b,h,i) triples) or every row.  host: host_inputs(inp), when
    a caller checks several slices of rows and wants the device-to-host copies made once."""
    pb = problem_of(wl, head_map, scale)
    qh, kh, vh = host if host is not None else host_inputs(inp)
    o_ref, lse_ref, pairs_ref = fo.attn_rows(pb, qh, kh, vh, mq, mk, rows=rows)
    if rows is None:
        sel = lambda t: t.reshape((-1,) + tuple(t.shape[3:]))
    else:
        ridx = torch.from_numpy(rows.astype(np.int64)).to(res["out"].device)
        sel = lambda t: t[ridx[:, 0], ridx[:, 1], ridx[:, 2]]       # gather on the device first
    o_got = sel(res["out"]).float().cpu().numpy().astype(np.float64)
    lse_got = sel(res["lse"]).cpu().numpy().astype(np.float64) if res["lse"] is not None else None
    rp_got = sel(res["row_pairs"]).cpu().numpy() if res["row_pairs"] is not None else None
    t = dict(TOL[wl.dtype])
    if tol:
        t.update(tol)
    err = np.abs(o_got - o_ref)
    stats = dict(max_abs=float(err.max()), mean_abs=float(err.mean()))
    assert np.isfinite(o_got).all(), "non-finite outputs"
    assert stats["max_abs"] <= t["out_max"], stats
    assert stats["mean_abs"] <= t["out_mean"], stats
    if lse_got is not None:
        stats["lse_max"] = float(np.abs(lse_got - lse_ref).max())
        assert stats["lse_max"] <= t["lse"], stats
    if rp_got is not None:
        assert np.array_equal(rp_got.astype(np.int64), pairs_ref), "row pair counts differ"
    num = (o_got * o_ref).sum()
    stats["cos"] = float(num / (np.linalg.norm(o_got) * np.linalg.norm(o_ref) + 1e-300))
    return stats


def check_pair_totals(wl, res, mq, mk, head_map=None):
    """Sum of the GPU's per-row pair counts equals the closed-form count, exactly."""
    pb = problem_of(wl, head_map)
    allowed, gp = fo.pair_counts(pb, mq, mk)
    got = res["row_pairs"].to(torch.int64).sum(dim=2).cpu().numpy().astype(np.uint64)
    assert np.array_equal(got, allowed), (got, allowed)
    return allowed, gp
