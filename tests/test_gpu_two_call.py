"""GPU parity of the paper's two-call evaluation (App. D) built from this library's kernels:
attention restricted to set A (pairs that share a group) and to set B (window pairs that share
none), the log-sum-exp merge, and the three together against the oracle and against the fused
single-softmax kernel.  Same tolerances as the fused path; pair counts bit-exact."""
import numpy as np
import pytest
import torch

from oracle import focus_oracle as fo
from paper_2604_03260_amd import focus, workloads
from tests import harness

pytestmark = pytest.mark.gpu


def run_sets(wl, inp, head_map=None):
    p = harness.params_of(wl, head_map)
    ws = focus.alloc_workspace(p)
    focus.focus_assign(p, inp["q"], inp["k"], inp["centroids"], ws)
    shape = (wl.B, wl.Hq, wl.n)
    res = {}
    for name, ps in (("all", focus.FOCUS_PAIRS_ALL), ("A", focus.FOCUS_PAIRS_SHARED), ("B", focus.FOCUS_PAIRS_CROSS_LOCAL)):
        out = torch.full_like(inp["q"], float("nan"))
        lse = torch.full(shape, float("nan"), dtype=torch.float32, device="cuda")
        rp = torch.full(shape, -7, dtype=torch.int32, device="cuda")
        focus.focus_attn_fwd_set(p, ps, inp["q"], inp["k"], inp["v"], ws, out, lse, rp)
        res[name] = dict(out=out, lse=lse, row_pairs=rp)
    merged = torch.full_like(inp["q"], float("nan"))
    mlse = torch.full(shape, float("nan"), dtype=torch.float32, device="cuda")
    focus.focus_attn_merge(res["A"]["out"], res["A"]["lse"], res["B"]["out"], res["B"]["lse"], merged, mlse)
    res["merged"] = dict(out=merged, lse=mlse, row_pairs=None)
    two = torch.full_like(inp["q"], float("nan"))
    tlse = torch.full(shape, float("nan"), dtype=torch.float32, device="cuda")
    part_out = torch.empty((2,) + tuple(inp["q"].shape), dtype=inp["q"].dtype, device="cuda")
    part_lse = torch.empty((2,) + shape, dtype=torch.float32, device="cuda")
    focus.focus_attn_fwd_two_call(p, inp["q"], inp["k"], inp["v"], ws, two, tlse, part_out, part_lse)
    torch.cuda.synchronize()
    res["two_call"] = dict(out=two, lse=tlse, row_pairs=None)
    res["views"] = focus.focus_workspace_views(p, ws)
    return res


def check_set(wl, inp, got, mq, mk, pair_set, head_map=None, rows=None):
    """One restricted launch against the oracle's same set: outputs, lse (empty rows: -inf), pair counts."""
    pb = harness.problem_of(wl, head_map)
    qh, kh, vh = (workloads.to_host_bits(inp[x]) for x in ("q", "k", "v"))
    o_ref, l_ref, p_ref = fo.attn_rows(pb, qh, kh, vh, mq, mk, rows=rows, pair_set=pair_set)
    if rows is None:
        sel = lambda t: t.reshape((-1,) + tuple(t.shape[3:]))
    else:
        ridx = torch.from_numpy(rows.astype(np.int64)).cuda()
        sel = lambda t: t[ridx[:, 0], ridx[:, 1], ridx[:, 2]]
    o = sel(got["out"]).float().cpu().numpy().astype(np.float64)
    l = sel(got["lse"]).cpu().numpy().astype(np.float64)
    tol = harness.TOL[wl.dtype]
    assert np.isfinite(o).all()
    err = np.abs(o - o_ref)
    assert err.max() <= tol["out_max"] and err.mean() <= tol["out_mean"], (pair_set, err.max(), err.mean())
    empty = ~np.isfinite(l_ref)
    assert np.array_equal(np.isneginf(l), empty), "empty rows differ"
    assert (o[empty] == 0).all()
    if (~empty).any():
        assert np.abs(l[~empty] - l_ref[~empty]).max() <= tol["lse"]
    if got["row_pairs"] is not None:
        assert np.array_equal(sel(got["row_pairs"]).cpu().numpy().astype(np.int64), p_ref)
    return int(empty.sum())


CASES = [
    # B, Hq, Hkv, n, d, dtype, K, topk, window, softcap
    (1, 2, 2, 300, 64, "f32", 4, 1, 16, 0.0),
    (2, 4, 2, 777, 64, "bf16", 4, 1, 32, 0.0),
    (1, 4, 1, 1500, 128, "bf16", 8, 1, 64, 50.0),
    (1, 2, 2, 900, 128, "bf16", 6, 2, 40, 0.0),
    (1, 2, 1, 513, 64, "f32", 8, 3, 1, 0.0),
    (1, 2, 2, 260, 128, "bf16", 1, 1, 8, 0.0),         # one group: B is empty everywhere
    (1, 2, 2, 3, 64, "bf16", 4, 1, 2, 0.0),
    (1, 4, 2, 800, 96, "f16", 4, 2, 50, 0.0),          # half precision, a head dim inside 128-wide copies
    (1, 2, 1, 600, 256, "bf16", 8, 1, 30, 0.0),
    (1, 4, 2, 900, 128, "bf16", 4, 1, 40, 0.0, False), # keys on both sides of the query
    (1, 2, 2, 500, 64, "f32", 8, 2, 9, 0.0, False),
    (1, 4, 2, 1300, 128, "bf16", 32, 2, 40, 0.0),      # 496 membership sets on classes of super-groups
    (1, 2, 2, 700, 64, "f32", 16, 3, 12, 0.0),
    (1, 2, 1, 900, 96, "f16", 32, 2, 25, 0.0, False),  # ... non-causal
]


@pytest.mark.parametrize("case", CASES, ids=[str(i) for i in range(len(CASES))])
def test_sets_merge_and_two_call_small(case):
    B, Hq, Hkv, n, d, dtype, K, topk, w, cap = case[:10]
    causal = case[10] if len(case) > 10 else True
    wl = workloads.Workload("t", 70 + K + topk, B, Hq, Hkv, n, d, dtype, K, topk, w, causal=causal, softcap=cap,
                            mixture=3)
    inp = workloads.make_inputs(wl, "cuda")
    res = run_sets(wl, inp)
    mq, mk = harness.oracle_membership(wl, inp)
    assert np.array_equal(res["views"]["mq"].cpu().numpy().view(np.uint32), mq)
    nA = check_set(wl, inp, res["A"], mq, mk, "A")
    nB = check_set(wl, inp, res["B"], mq, mk, "B")
    check_set(wl, inp, res["all"], mq, mk, "all")
    if K == 1:
        assert nB == B * Hq * n and nA == 0
    # the two sets partition the mask: counts add up, row by row
    tot = res["A"]["row_pairs"].to(torch.int64) + res["B"]["row_pairs"].to(torch.int64)
    assert torch.equal(tot, res["all"]["row_pairs"].to(torch.int64))
    # merged parts and the convenience call: the oracle's whole-mask attention, and each other bit for bit
    for name in ("merged", "two_call"):
        harness.check_attn(wl, inp, dict(out=res[name]["out"], lse=res[name]["lse"], row_pairs=None), mq, mk)
    assert torch.equal(res["merged"]["out"], res["two_call"]["out"])
    assert torch.equal(res["merged"]["lse"], res["two_call"]["lse"])
    # against the fused kernel: the same function, two roundings of the partial outputs apart
    diff = (res["two_call"]["out"].float() - res["all"]["out"].float()).abs().max().item()
    assert diff <= harness.TOL[dtype]["out_max"]


def test_merge_edge_cases():
    rows, d = 5, 64
    oa = torch.randn((rows, d), device="cuda").to(torch.bfloat16)
    ob = torch.randn((rows, d), device="cuda").to(torch.bfloat16)
    inf = float("inf")
    la = torch.tensor([0.0, -inf, 3.0, 80.0, -inf], dtype=torch.float32, device="cuda")
    lb = torch.tensor([0.0, 1.0, -inf, 80.0 + float(np.log(3.0)), -inf], dtype=torch.float32, device="cuda")
    out = torch.empty_like(oa)
    lse = torch.empty((rows,), dtype=torch.float32, device="cuda")
    focus.focus_attn_merge(oa, la, ob, lb, out, lse)
    torch.cuda.synchronize()
    o_ref, l_ref = fo.merge(oa.float().cpu().numpy(), la.cpu().numpy(), ob.float().cpu().numpy(), lb.cpu().numpy())
    assert np.abs(out.float().cpu().numpy() - o_ref).max() <= 2e-2
    assert torch.equal(out[1], ob[1]) and torch.equal(out[2], oa[2])      # an empty part weighs nothing
    assert (out[4] == 0).all() and lse[4].item() == -inf
    fin = np.isfinite(l_ref)
    assert np.abs(lse.cpu().numpy()[fin] - l_ref[fin]).max() <= 1e-5


def test_restricted_set_is_refused_when_the_window_covers_the_sequence():
    wl = workloads.CONFIGS["cfg1"].scaled(n=128, window=128, Hq=2, Hkv=2)
    inp = workloads.make_inputs(wl, "cuda")
    p = harness.params_of(wl)
    ws = focus.alloc_workspace(p)
    focus.focus_assign(p, inp["q"], inp["k"], inp["centroids"], ws)
    out = torch.empty_like(inp["q"])
    with pytest.raises(focus.FocusError) as e:
        focus.focus_attn_fwd_set(p, focus.FOCUS_PAIRS_SHARED, inp["q"], inp["k"], inp["v"], ws, out)
    assert e.value.status == focus.FOCUS_EUNSUPPORTED
    focus.focus_attn_fwd_set(p, focus.FOCUS_PAIRS_ALL, inp["q"], inp["k"], inp["v"], ws, out)
    torch.cuda.synchronize()


@pytest.mark.parametrize("name", ["cfg4a"])
def test_two_call_full_size_sampled(name):
    """The hard-assignment configuration at full size: sets and two-call result on sampled rows, counts in full."""
    wl = workloads.CONFIGS[name]
    inp = workloads.make_inputs(wl, "cuda")
    res = run_sets(wl, inp)
    mq, mk = harness.oracle_membership(wl, inp)          # the oracle's own membership, not the device's
    assert np.array_equal(res["views"]["mq"].cpu().numpy().view(np.uint32), mq)
    assert np.array_equal(res["views"]["mk"].cpu().numpy().view(np.uint32), mk)
    rows = workloads.sample_rows(wl, 768)
    check_set(wl, inp, res["A"], mq, mk, "A", rows=rows)
    check_set(wl, inp, res["B"], mq, mk, "B", rows=rows)
    tot = res["A"]["row_pairs"].to(torch.int64) + res["B"]["row_pairs"].to(torch.int64)
    assert torch.equal(tot, res["all"]["row_pairs"].to(torch.int64))
    harness.check_attn(wl, inp, dict(out=res["two_call"]["out"], lse=res["two_call"]["lse"], row_pairs=None),
                       mq, mk, rows=rows)
