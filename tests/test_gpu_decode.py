"""GPU parity of the incremental path (focus_decode_prefill / focus_decode_step) against the oracle.

A synthetic sequence of n tokens is split into a cached prefix (n0 tokens, state built by
focus_decode_prefill) and steps n0 .. n-1 (focus_decode_step, one token each).  The output of the step at
position i is row i of the oracle's attention over the whole sequence (the mask is causal, so row i sees
keys 0..i only); memberships of cached keys and group lists are checked bit for bit, outputs to the
tolerances of the prefill path, the number of attended keys exactly."""
import numpy as np
import pytest
import torch

from oracle import focus_oracle as fo
from paper_2604_03260_amd import focus, workloads
from tests import harness

pytestmark = pytest.mark.gpu


def run_decode(wl, inp, n0, steps, head_map=None):
    """Caches hold the first n0 tokens; then `steps` tokens are decoded.  Returns per-step outputs."""
    p = harness.params_of(wl, head_map)
    state = focus.alloc_decode_state(p)
    kc = torch.zeros_like(inp["k"])
    vc = torch.zeros_like(inp["v"])
    kc[:, :, :n0] = inp["k"][:, :, :n0]
    vc[:, :, :n0] = inp["v"][:, :, :n0]
    focus.focus_decode_prefill(p, n0, kc, inp["centroids"], state)
    outs, lses, pairs = [], [], []
    for i in range(n0, n0 + steps):
        q_new = inp["q"][:, :, i].contiguous()
        k_new = inp["k"][:, :, i].contiguous()
        v_new = inp["v"][:, :, i].contiguous()
        out = torch.full_like(q_new, float("nan"))
        lse = torch.full((wl.B, wl.Hq), float("nan"), dtype=torch.float32, device="cuda")
        rp = torch.full((wl.B, wl.Hq), -1, dtype=torch.int32, device="cuda")
        focus.focus_decode_step(p, i, q_new, k_new, v_new, inp["centroids"], kc, vc, state, out, lse, rp)
        outs.append(out); lses.append(lse); pairs.append(rp)
    torch.cuda.synchronize()
    return dict(out=torch.stack(outs, 2), lse=torch.stack(lses, 2), row_pairs=torch.stack(pairs, 2), kc=kc, vc=vc,
                state=state, params=p)


def check_decode(wl, inp, res, n0, steps, head_map=None):
    pb = harness.problem_of(wl, head_map)
    qh, kh, vh = (workloads.to_host_bits(inp[x]) for x in ("q", "k", "v"))
    mq, mk = harness.oracle_membership(wl, inp, head_map)
    rows = np.array([(b, h, i) for b in range(wl.B) for h in range(wl.Hq) for i in range(n0, n0 + steps)], dtype=np.int32)
    o_ref, l_ref, p_ref = fo.attn_rows(pb, qh, kh, vh, mq, mk, rows=rows)
    o = res["out"].float().cpu().numpy().astype(np.float64).reshape(-1, wl.d)       # [B,Hq,steps,d] in the same order
    l = res["lse"].cpu().numpy().astype(np.float64).reshape(-1)
    rp = res["row_pairs"].cpu().numpy().astype(np.int64).reshape(-1)
    tol = harness.TOL[wl.dtype]
    assert np.isfinite(o).all()
    err = np.abs(o - o_ref)
    assert err.max() <= tol["out_max"] and err.mean() <= tol["out_mean"], (err.max(), err.mean())
    assert np.abs(l - l_ref).max() <= tol["lse"]
    assert np.array_equal(rp, p_ref), "attended key counts differ"
    # the caches now hold the whole prefix + decoded tokens
    n1 = n0 + steps
    assert torch.equal(res["kc"][:, :, :n1], inp["k"][:, :, :n1]) and torch.equal(res["vc"][:, :, :n1], inp["v"][:, :, :n1])
    return mk


CASES = [
    # B, Hq, Hkv, n, d, dtype, K, topk, window, softcap, n0, steps
    (1, 2, 2, 300, 64, "f32", 4, 2, 16, 0.0, 250, 50),
    (2, 4, 2, 1500, 128, "bf16", 4, 2, 64, 0.0, 1490, 10),
    (1, 8, 2, 3000, 128, "bf16", 8, 1, 100, 50.0, 2990, 10),
    (1, 2, 1, 40, 64, "bf16", 4, 2, 8, 0.0, 0, 40),              # from an empty cache, token by token
    (1, 2, 2, 700, 64, "f32", 32, 4, 5, 0.0, 690, 10),           # C(32,4) classes: beyond the prefill path's limit
    (1, 4, 4, 2500, 128, "bf16", 4, 3, 3000, 0.0, 2495, 5),      # window wider than the sequence
    (1, 2, 2, 520, 64, "bf16", 1, 1, 4, 0.0, 515, 5),
    (1, 8, 1, 600, 64, "bf16", 8, 2, 16, 0.0, 590, 10),         # 8 query heads on one KV head
    (2, 16, 2, 900, 128, "f32", 6, 2, 30, 0.0, 880, 8),
    (1, 6, 2, 400, 64, "bf16", 4, 2, 10, 0.0, 390, 10),          # 3 query heads per KV head (matrix cores)
    (1, 6, 2, 400, 64, "f32", 4, 2, 10, 0.0, 390, 10),           # ... in fp32: per-head kernel
    (2, 14, 2, 900, 128, "f16", 8, 2, 50, 0.0, 893, 7),          # 7 query heads per KV head
    (1, 5, 1, 700, 96, "bf16", 4, 1, 30, 0.0, 695, 5),           # 5 query heads per KV head, d = 96
    (1, 16, 1, 900, 128, "bf16", 4, 2, 40, 0.0, 894, 6),         # 16 query heads on one KV head: every column of the products
    (1, 24, 2, 800, 64, "f16", 8, 1, 30, 0.0, 795, 5),           # 12 per KV head
    (1, 40, 1, 1100, 128, "bf16", 8, 2, 64, 0.0, 1095, 5),       # 40 on one KV head: sub-groups of 16, 16 and 8
    (1, 16, 1, 900, 128, "f32", 4, 2, 40, 0.0, 896, 4),          # ... in fp32: per-head kernel
    (1, 2, 1, 60000, 64, "bf16", 4, 2, 300, 0.0, 59996, 4),      # long context: several chunks per work-group
    (1, 3, 1, 60000, 64, "f32", 4, 2, 300, 0.0, 59997, 3),       # ... in the per-head kernel
    (1, 4, 2, 1500, 128, "f16", 4, 2, 64, 0.0, 1490, 10),        # IEEE half precision
    (1, 3, 1, 900, 64, "f16", 8, 2, 20, 30.0, 892, 8),           # ... three heads on one KV head, softcap
    (1, 8, 2, 1200, 80, "bf16", 4, 2, 40, 0.0, 1192, 8),         # head dims inside 16 lanes per key: 10 of them hold data
    (2, 4, 4, 800, 96, "f32", 8, 2, 25, 0.0, 792, 8),
    (1, 6, 2, 700, 96, "f16", 4, 2, 30, 0.0, 694, 6),            # 3 heads per KV head at d = 96
    (1, 4, 2, 1000, 256, "bf16", 4, 2, 50, 0.0, 992, 8),         # 32 lanes per key
    (1, 2, 2, 600, 256, "f32", 8, 1, 16, 0.0, 594, 6),
    (1, 3, 1, 40000, 256, "f16", 4, 2, 200, 0.0, 39997, 3),      # long context, three heads on one KV head, d = 256
    (1, 2, 1, 250000, 64, "bf16", 4, 2, 300, 0.0, 249997, 3),    # work-groups that walk two chunks, positions walked (matrix cores)
    (1, 3, 1, 250000, 64, "f32", 4, 2, 300, 0.0, 249998, 2),     # ... in the per-head kernel
    (1, 4, 2, 300000, 128, "bf16", 16, 1, 512, 0.0, 299997, 3),  # ... group lists walked: they are the shorter walk
    (1, 4, 1, 262144, 128, "f16", 4, 2, 1024, 30.0, 262141, 3),  # ... four heads per KV head, half precision, softcap
    (1, 8, 1, 5000, 128, "f32", 4, 2, 100, 0.0, 4996, 4),        # eight fp32 heads on one KV head (vector kernel)
]


@pytest.mark.parametrize("B,Hq,Hkv,n,d,dtype,K,topk,w,cap,n0,steps", CASES)
def test_decode_steps_small(B, Hq, Hkv, n, d, dtype, K, topk, w, cap, n0, steps):
    wl = workloads.Workload("dec", 80 + K + topk, B, Hq, Hkv, n, d, dtype, K, topk, w, softcap=cap, mixture=3)
    inp = workloads.make_inputs(wl, "cuda")
    res = run_decode(wl, inp, n0, steps)
    check_decode(wl, inp, res, n0, steps)


def test_decode_state_matches_oracle_lists():
    wl = workloads.Workload("dec", 95, 2, 4, 2, 900, 64, "bf16", 6, 2, 32, mixture=3)
    inp = workloads.make_inputs(wl, "cuda")
    n0, steps = 600, 300
    res = run_decode(wl, inp, n0, steps)
    mk = check_decode(wl, inp, res, n0, steps)
    views = focus.focus_decode_state_views(res["params"], res["state"])
    got_mk = views["mk"].cpu().numpy().view(np.uint32)
    assert np.array_equal(got_mk, mk)
    lists = views["lists"].cpu().numpy()
    counts = views["counts"].cpu().numpy()
    for b in range(wl.B):
        for h in range(wl.Hkv):
            for g in range(wl.K):
                want = np.nonzero((mk[b, h] >> g) & 1)[0]
                assert counts[b, h, g] == len(want)
                assert np.array_equal(lists[b, h, g, :len(want)], want)


def test_decode_with_head_map():
    wl = workloads.Workload("dec", 96, 1, 6, 3, 800, 64, "bf16", 4, 2, 20, mixture=3)
    inp = workloads.make_inputs(wl, "cuda")
    hm = [2, 0, 1, 1, 2, 0]
    res = run_decode(wl, inp, 780, 20, head_map=hm)
    check_decode(wl, inp, res, 780, 20, head_map=hm)


def test_decode_agrees_with_prefill_kernel_long_context():
    """cfg3's shape: the last rows of the prefill kernel's output against decode steps at the same positions."""
    wl = workloads.CONFIGS["cfg3"]
    inp = workloads.make_inputs(wl, "cuda")
    steps = 4
    n0 = wl.n - steps
    res = run_decode(wl, inp, n0, steps)
    full = harness.run_gpu(wl, inp)
    a = res["out"].float()
    b = full["out"][:, :, n0:].float()
    assert (a - b).abs().max().item() <= 2e-2
    assert torch.equal(res["row_pairs"], full["row_pairs"][:, :, n0:])
    assert (res["lse"] - full["lse"][:, :, n0:]).abs().max().item() <= 1e-2
    check_decode(wl, inp, res, n0, steps)


@pytest.mark.parametrize("kw", [dict(Hq=8, Hkv=2, d=128, dtype="bf16", K=4, topk=2),
                                dict(Hq=3, Hkv=1, d=96, dtype="f16", K=8, topk=2),
                                dict(Hq=4, Hkv=4, d=64, dtype="f32", K=4, topk=1)])
def test_decode_step_with_the_position_on_the_device_replays_from_one_graph(kw):
    # A generation loop as a serving stack would run it: one HIP graph captured around focus_decode_step_at,
    # replayed once per token; the new token's q, k, v are written into the captured buffers and the position
    # advances on the device.  Every step is checked against the oracle, the state against the host-position path.
    wl = workloads.Workload("dec_graph", 45, 2, kw["Hq"], kw["Hkv"], 1300, kw["d"], kw["dtype"], kw["K"], kw["topk"], 48)
    n0, steps = 1200, 40
    inp = workloads.make_inputs(wl, "cuda")
    p = harness.params_of(wl)
    state = focus.alloc_decode_state(p)
    kc = torch.zeros_like(inp["k"]); vc = torch.zeros_like(inp["v"])
    kc[:, :, :n0] = inp["k"][:, :, :n0]; vc[:, :, :n0] = inp["v"][:, :, :n0]
    focus.focus_decode_prefill(p, n0, kc, inp["centroids"], state)
    q_new = inp["q"][:, :, n0].contiguous(); k_new = inp["k"][:, :, n0].contiguous(); v_new = inp["v"][:, :, n0].contiguous()
    out = torch.empty_like(q_new)
    lse = torch.empty((wl.B, wl.Hq), dtype=torch.float32, device="cuda")
    rp = torch.empty((wl.B, wl.Hq), dtype=torch.int32, device="cuda")
    pos = torch.full((wl.B,), n0, dtype=torch.int32, device="cuda")

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        focus.focus_decode_step_at(p, pos, q_new, k_new, v_new, inp["centroids"], kc, vc, state, out, lse, rp)
        pos.add_(1)                                   # the position advances inside the graph
    outs, lses, pairs = [], [], []
    for i in range(n0, n0 + steps):
        q_new.copy_(inp["q"][:, :, i]); k_new.copy_(inp["k"][:, :, i]); v_new.copy_(inp["v"][:, :, i])
        out.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        outs.append(out.clone()); lses.append(lse.clone()); pairs.append(rp.clone())
    assert pos.tolist() == [n0 + steps] * wl.B
    res = dict(out=torch.stack(outs, 2), lse=torch.stack(lses, 2), row_pairs=torch.stack(pairs, 2), kc=kc, vc=vc)
    check_decode(wl, inp, res, n0, steps)
    # the same steps with the position as a host argument: identical state, outputs equal up to the
    # grouping of the partial sums (the launch shapes differ)
    ref = run_decode(wl, inp, n0, steps)
    va = focus.focus_decode_state_views(p, state)
    vb = focus.focus_decode_state_views(ref["params"], ref["state"])
    assert torch.equal(va["mk"][:, :, :n0 + steps], vb["mk"][:, :, :n0 + steps])
    assert torch.equal(va["counts"], vb["counts"])
    cnt = va["counts"].cpu().numpy()
    la, lb = va["lists"].cpu().numpy(), vb["lists"].cpu().numpy()
    for b in range(cnt.shape[0]):
        for h in range(cnt.shape[1]):
            for g in range(cnt.shape[2]):
                assert np.array_equal(la[b, h, g, :cnt[b, h, g]], lb[b, h, g, :cnt[b, h, g]])
    assert torch.equal(res["row_pairs"], ref["row_pairs"])
    tol = harness.TOL[wl.dtype]
    assert (res["out"].float() - ref["out"].float()).abs().max().item() <= tol["out_max"]


def test_decode_step_with_a_device_position_outside_the_caches_does_nothing():
    wl = workloads.Workload("dec_oob", 46, 1, 4, 2, 256, 64, "bf16", 4, 2, 16)
    inp = workloads.make_inputs(wl, "cuda")
    p = harness.params_of(wl)
    state = focus.alloc_decode_state(p)
    kc = inp["k"].clone(); vc = inp["v"].clone()
    focus.focus_decode_prefill(p, 200, kc, inp["centroids"], state)
    torch.cuda.synchronize()
    before = (kc.clone(), vc.clone(), state.clone())
    out = torch.full((wl.B, wl.Hq, wl.d), 7.0, dtype=torch.bfloat16, device="cuda")
    for bad in (-1, 256, 1 << 30):
        pos = torch.full((wl.B,), bad, dtype=torch.int32, device="cuda")
        focus.focus_decode_step_at(p, pos, inp["q"][:, :, 0].contiguous(), inp["k"][:, :, 0].contiguous(),
                                   inp["v"][:, :, 0].contiguous(), inp["centroids"], kc, vc, state, out)
        torch.cuda.synchronize()
        assert torch.equal(kc, before[0]) and torch.equal(vc, before[1]) and torch.equal(state, before[2])
        assert bool((out == 7.0).all())


@pytest.mark.parametrize("kw", [dict(Hq=8, Hkv=2, d=128, dtype="bf16", K=4, topk=2, n0=1188),
                                dict(Hq=3, Hkv=1, d=64, dtype="f32", K=8, topk=1, n0=0),
                                dict(Hq=4, Hkv=4, d=96, dtype="f16", K=32, topk=3, n0=1100)])
def test_decode_with_memberships_from_the_router(kw):
    # The paper's flow at inference: one routing per token from the layer's hidden state (no Sinkhorn rounds at
    # decode time), the token's membership for all its heads as query and as key.  The state is built from the
    # routed masks of the cached prefix, every step gets the new token's mask from focus_route on one token.
    n, n0 = 1200, kw["n0"]
    steps = 12 if n0 else 30
    wl = workloads.Workload("dec_routed", 47, 2, kw["Hq"], kw["Hkv"], n if n0 else steps, kw["d"], kw["dtype"], kw["K"], kw["topk"], 40)
    n = wl.n
    inp = workloads.make_inputs(wl, "cuda")
    rin = workloads.make_router_inputs(wl, "cuda", d_model=128)
    m_ref = fo.route(workloads.to_host_bits(rin["hidden"]), rin["w_g"].cpu().numpy(), rin["router_centroids"].cpu().numpy(),
                     wl.topk, tau=0.1, iters=0, dtype=wl.dtype)
    # the prefix routed in one call, the new tokens one call each (n = 1 per sequence)
    rp_all = focus.make_route_params(wl.B, n, 128, workloads.ROUTER_DG, wl.K, wl.topk, dtype=wl.dtype, sinkhorn_iters=0, tau=0.1)
    masks_all = torch.empty((wl.B, n), dtype=torch.int32, device="cuda")
    focus.focus_route(rp_all, rin["hidden"], rin["w_g"], rin["router_centroids"], focus.alloc_route_workspace(rp_all), masks_all)
    assert np.array_equal(masks_all.cpu().numpy().view(np.uint32), m_ref)
    rp_one = focus.make_route_params(wl.B, 1, 128, workloads.ROUTER_DG, wl.K, wl.topk, dtype=wl.dtype, sinkhorn_iters=0, tau=0.1)
    rws_one = focus.alloc_route_workspace(rp_one)
    p = harness.params_of(wl)
    state = focus.alloc_decode_state(p)
    kc = torch.zeros_like(inp["k"]); vc = torch.zeros_like(inp["v"])
    kc[:, :, :n0] = inp["k"][:, :, :n0]; vc[:, :, :n0] = inp["v"][:, :, :n0]
    focus.focus_decode_prefill_tokens(p, n0, masks_all[:, :n0].contiguous() if n0 else None, state)
    outs, lses, pairs = [], [], []
    for i in range(n0, n0 + steps):
        tmask = torch.empty((wl.B, 1), dtype=torch.int32, device="cuda")
        focus.focus_route(rp_one, rin["hidden"][:, i:i + 1].contiguous(), rin["w_g"], rin["router_centroids"], rws_one, tmask)
        out = torch.full((wl.B, wl.Hq, wl.d), float("nan"), dtype=inp["q"].dtype, device="cuda")
        lse = torch.empty((wl.B, wl.Hq), dtype=torch.float32, device="cuda")
        rp = torch.empty((wl.B, wl.Hq), dtype=torch.int32, device="cuda")
        focus.focus_decode_step_tokens(p, i, tmask, inp["q"][:, :, i].contiguous(), inp["k"][:, :, i].contiguous(),
                                       inp["v"][:, :, i].contiguous(), kc, vc, state, out, lse, rp)
        outs.append(out); lses.append(lse); pairs.append(rp)
    torch.cuda.synchronize()
    # oracle: the whole sequence with the routed membership broadcast to every head
    pb = harness.problem_of(wl)
    mq, mk = fo.broadcast_masks(pb, m_ref)
    qh, kh, vh = (workloads.to_host_bits(inp[x]) for x in ("q", "k", "v"))
    rows = np.array([(b, h, i) for b in range(wl.B) for h in range(wl.Hq) for i in range(n0, n0 + steps)], dtype=np.int32)
    o_ref, l_ref, p_ref = fo.attn_rows(pb, qh, kh, vh, mq, mk, rows=rows)
    o = torch.stack(outs, 2).float().cpu().numpy().astype(np.float64).reshape(-1, wl.d)
    l = torch.stack(lses, 2).cpu().numpy().astype(np.float64).reshape(-1)
    tol = harness.TOL[wl.dtype]
    err = np.abs(o - o_ref)
    assert np.isfinite(o).all() and err.max() <= tol["out_max"] and err.mean() <= tol["out_mean"], (err.max(), err.mean())
    assert np.abs(l - l_ref).max() <= tol["lse"]
    assert np.array_equal(torch.stack(pairs, 2).cpu().numpy().astype(np.int64).reshape(-1), p_ref)
    views = focus.focus_decode_state_views(p, state)
    n1 = n0 + steps
    assert np.array_equal(views["mk"][:, :, :n1].cpu().numpy().view(np.uint32), mk[:, :, :n1])


def test_decode_token_masks_that_are_no_topk_subset_are_replaced():
    wl = workloads.Workload("dec_badmask", 48, 1, 2, 2, 64, 64, "bf16", 4, 2, 8)
    inp = workloads.make_inputs(wl, "cuda")
    p = harness.params_of(wl)
    state = focus.alloc_decode_state(p)
    bad = torch.tensor([[0b1111, 0b0001, 0b10000, 0b0110]], dtype=torch.int32, device="cuda")    # only the last is valid
    focus.focus_decode_prefill_tokens(p, 4, bad, state)
    torch.cuda.synchronize()
    mk = focus.focus_decode_state_views(p, state)["mk"][:, :, :4].cpu().numpy()
    assert (mk == np.array([0b0011, 0b0011, 0b0011, 0b0110])).all()


def decode_sweep_cases(count, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for _ in range(count):
        K = int(rng.choice([1, 2, 4, 6, 8, 16, 32]))
        Hkv = int(rng.choice([1, 2, 3]))
        n = int(rng.integers(40, 1500))
        steps = int(rng.integers(2, 9))
        cases.append((int(rng.choice([1, 2])), Hkv * int(rng.choice([1, 2, 3, 4, 8])), Hkv, n, int(rng.choice([64, 80, 96, 128, 256])),
                      str(rng.choice(["bf16", "f16", "f32"])), K, int(rng.integers(1, min(K, 4) + 1)),
                      int(rng.choice([1, 3, 16, 100, n + 7])), float(rng.choice([0.0, 0.0, 20.0])),
                      int(rng.integers(0, n - steps + 1)), steps))
    return cases


@pytest.mark.parametrize("B,Hq,Hkv,n,d,dtype,K,topk,w,cap,n0,steps", decode_sweep_cases(24, 20260404))
def test_decode_random_parameter_sweep(B, Hq, Hkv, n, d, dtype, K, topk, w, cap, n0, steps):
    wl = workloads.Workload("dsweep", 49, B, Hq, Hkv, n, d, dtype, K, topk, w, softcap=cap, mixture=3 if K > 2 else 0)
    inp = workloads.make_inputs(wl, "cuda")
    res = run_decode(wl, inp, n0, steps)
    check_decode(wl, inp, res, n0, steps)


def test_decode_sequences_of_a_batch_at_different_positions():
    # continuous batching: three sequences with prefixes of different lengths share one step call; a sequence
    # that has not started or has finished is skipped by giving it a position outside the caches
    wl = workloads.Workload("dec_ragged", 44, 3, 8, 2, 900, 128, "bf16", 4, 2, 32)
    inp = workloads.make_inputs(wl, "cuda")
    p = harness.params_of(wl)
    state = focus.alloc_decode_state(p)
    starts = [300, 640, 880]                                          # first decoded position of every sequence
    ends = [330, 660, 900]
    n0 = min(starts)
    kc = torch.zeros_like(inp["k"]); vc = torch.zeros_like(inp["v"])
    kc[:, :, :n0] = inp["k"][:, :, :n0]; vc[:, :, :n0] = inp["v"][:, :, :n0]
    focus.focus_decode_prefill(p, n0, kc, inp["centroids"], state)
    # bring the longer prefixes in token by token (the shorter sequences sit out), then decode all three
    outs = {}
    cur = [n0] * wl.B
    q_new = torch.empty((wl.B, wl.Hq, wl.d), dtype=torch.bfloat16, device="cuda")
    k_new = torch.empty((wl.B, wl.Hkv, wl.d), dtype=torch.bfloat16, device="cuda")
    v_new = torch.empty_like(k_new)
    out = torch.empty_like(q_new)
    rp = torch.empty((wl.B, wl.Hq), dtype=torch.int32, device="cuda")
    while any(c < e for c, e in zip(cur, ends)):
        # a sequence takes part while it is below its end; sequence b decodes "for real" from starts[b] on
        active = [c < e for c, e in zip(cur, ends)]
        pos = torch.tensor([c if a else -1 for c, a in zip(cur, active)], dtype=torch.int32, device="cuda")
        for b in range(wl.B):
            i = min(cur[b], wl.n - 1)
            q_new[b] = inp["q"][b, :, i]; k_new[b] = inp["k"][b, :, i]; v_new[b] = inp["v"][b, :, i]
        out.fill_(float("nan")); rp.fill_(-5)
        focus.focus_decode_step_at(p, pos, q_new, k_new, v_new, inp["centroids"], kc, vc, state, out, None, rp)
        torch.cuda.synchronize()
        for b in range(wl.B):
            if active[b]:
                if cur[b] >= starts[b]:
                    outs[(b, cur[b])] = (out[b].clone(), rp[b].clone())
                cur[b] += 1
            else:
                assert bool(torch.isnan(out[b].float()).all()) and bool((rp[b] == -5).all())   # skipped: untouched
    pb = harness.problem_of(wl)
    qh, kh, vh = (workloads.to_host_bits(inp[x]) for x in ("q", "k", "v"))
    mq, mk = harness.oracle_membership(wl, inp)
    keys = sorted(outs)
    rows = np.array([(b, h, i) for (b, i) in keys for h in range(wl.Hq)], dtype=np.int32)
    o_ref, _, p_ref = fo.attn_rows(pb, qh, kh, vh, mq, mk, rows=rows)
    o = torch.stack([outs[k][0] for k in keys]).float().cpu().numpy().astype(np.float64).reshape(-1, wl.d)
    rpg = torch.stack([outs[k][1] for k in keys]).cpu().numpy().astype(np.int64).reshape(-1)
    err = np.abs(o - o_ref)
    tol = harness.TOL[wl.dtype]
    assert err.max() <= tol["out_max"] and err.mean() <= tol["out_mean"], (err.max(), err.mean())
    assert np.array_equal(rpg, p_ref)
