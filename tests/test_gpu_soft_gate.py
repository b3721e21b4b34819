"""GPU parity of the soft-gated attention of training (Sec. 2 Eq. 2) through the C ABI against the
fp64 oracle on the same bytes: outputs and lse within the stated tolerances of the I/O type."""
import numpy as np
import pytest
import torch

from oracle import focus_oracle as fo
from paper_2604_03260_amd import focus, workloads
from tests import harness

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)


def soft_assignment(wl, device, sharp=4.0):
    """Seeded soft assignments [B,n,K] fp32, rows on the simplex (a softmax of random scores; larger
    `sharp` = closer to one-hot).  Tensor id 11 of the workload's seed family."""
    gen = torch.Generator(device=device)
    gen.manual_seed(1000 * wl.config_id + 11)
    s = torch.randn((wl.B, wl.n, wl.K), generator=gen, device=device, dtype=torch.float32) * sharp
    return torch.softmax(s, dim=-1).contiguous()


def run_soft(wl, inp, g, lam, vector=False):
    p = harness.params_of(wl)
    ws = focus.alloc_soft_workspace(p)
    out = torch.full_like(inp["q"], float("nan"))
    lse = torch.full((wl.B, wl.Hq, wl.n), float("nan"), dtype=torch.float32, device="cuda")
    focus.focus_attn_soft_fwd(p, lam, g, inp["q"], inp["k"], inp["v"], ws, out, lse, vector=vector)
    torch.cuda.synchronize()
    return out, lse


def check_soft(wl, inp, g, lam, out, lse, rows=None):
    pb = harness.problem_of(wl)
    qh, kh, vh = (workloads.to_host_bits(inp[x]) for x in ("q", "k", "v"))
    o_ref, l_ref = fo.soft_rows(pb, lam, g.cpu().numpy(), qh, kh, vh, rows=rows)
    if rows is None:
        sel = lambda t: t.reshape((-1,) + tuple(t.shape[3:]))
    else:
        ridx = torch.from_numpy(rows.astype(np.int64)).cuda()
        sel = lambda t: t[ridx[:, 0], ridx[:, 1], ridx[:, 2]]
    o = sel(out).float().cpu().numpy().astype(np.float64)
    l = sel(lse).cpu().numpy().astype(np.float64)
    tol = harness.TOL[wl.dtype]
    assert np.isfinite(o).all() and np.isfinite(l).all()
    err = np.abs(o - o_ref)
    stats = dict(max_abs=float(err.max()), mean_abs=float(err.mean()), lse_max=float(np.abs(l - l_ref).max()))
    assert stats["max_abs"] <= tol["out_max"] and stats["mean_abs"] <= tol["out_mean"], stats
    assert stats["lse_max"] <= tol["lse"], stats
    return stats


def case(name, **kw):
    base = dict(name=name, config_id=95, B=1, Hq=4, Hkv=2, n=600, d=64, dtype="bf16", K=4, topk=1, window=32)
    base.update(kw)
    return workloads.Workload(**base)


CASES = [
    (case("bf16_d64"), 5.0),
    (case("bf16_d128_k8", n=1400, d=128, K=8, window=64, mixture=8), 8.0),
    (case("f16_d128", n=777, d=128, dtype="f16", K=4, window=50), 3.0),
    (case("bf16_d96_k16", n=900, d=96, K=16, window=20), 10.0),
    (case("bf16_d80_k32", n=700, d=80, K=32, window=16, Hq=2, Hkv=2), 12.0),       # two k-steps of groups
    (case("f32_d64", n=500, dtype="f32", K=4, window=24), 6.0),
    (case("f32_d256_k2", n=300, d=256, dtype="f32", K=2, window=8, Hq=2, Hkv=1), 2.0),
    (case("bf16_d256_vector_path", n=400, d=256, K=4, window=20, Hq=2, Hkv=1), 6.0),   # 16-bit d = 256: vector kernel
    (case("lambda_zero", n=520, d=128), 0.0),                                      # every distant logit halved
    (case("negative_slope", n=640, d=64, K=8), -7.0),
    (case("window_covers", n=300, d=128, window=300), 9.0),                        # plain causal attention
    (case("window_one", n=513, d=64, window=1, K=2), 4.0),
    (case("batch_gqa", B=3, Hq=8, Hkv=2, n=400, d=128, K=4), 5.0),
    (case("one_token", n=1, d=64), 5.0),
    (case("tile_multiple", n=512, d=128, K=8, window=64), 20.0),
]


@pytest.mark.parametrize("wl,lam", CASES, ids=[c[0].name for c in CASES])
def test_soft_gate_small_cases_all_rows(wl, lam):
    say("case", wl, lam)
    inp = workloads.make_inputs(wl, "cuda")
    g = soft_assignment(wl, "cuda")
    out, lse = run_soft(wl, inp, g, lam)
    say(wl.name, check_soft(wl, inp, g, lam, out, lse))


def test_soft_gate_one_hot_assignments():
    # hard (one-hot) assignments and a steep gate: same-group pairs at full strength, the others halved
    wl = case("one_hot", n=1000, d=128, K=8, window=40)
    inp = workloads.make_inputs(wl, "cuda")
    gen = torch.Generator(device="cuda")
    gen.manual_seed(77)
    grp = torch.randint(0, wl.K, (wl.B, wl.n), generator=gen, device="cuda")
    g = torch.nn.functional.one_hot(grp, wl.K).float().contiguous()
    out, lse = run_soft(wl, inp, g, 60.0)
    say(check_soft(wl, inp, g, 60.0, out, lse))


def test_soft_gate_matrix_core_and_vector_kernels_agree_mid_size():
    wl = case("mid", n=12000 + 5, d=128, K=4, window=700, Hq=4, Hkv=1)
    inp = workloads.make_inputs(wl, "cuda")
    g = soft_assignment(wl, "cuda", sharp=2.0)
    out, lse = run_soft(wl, inp, g, 6.0)
    rows = workloads.sample_rows(wl, 512)
    say("mid", check_soft(wl, inp, g, 6.0, out, lse, rows=rows))
    out_v, lse_v = run_soft(wl, inp, g, 6.0, vector=True)
    diff = (out.float() - out_v.float()).abs()
    assert diff.max().item() <= 2e-2 and diff.mean().item() <= 2e-3
    assert (lse - lse_v).abs().max().item() <= 1e-2


def test_soft_gate_full_size_sampled_rows():
    # the shape and inputs of bench.py's soft_gate leg (cfg3's q, k, v; seeded soft assignments; slope 8)
    wl = workloads.CONFIGS["cfg3"]
    inp = workloads.make_inputs(wl, "cuda")
    g = soft_assignment(wl, "cuda")
    out, lse = run_soft(wl, inp, g, 8.0)
    rows = workloads.sample_rows(wl, 512)
    say("cfg3 soft gate", check_soft(wl, inp, g, 8.0, out, lse, rows=rows))


def test_soft_gate_with_the_router_output():
    # the router's Sinkhorn-normalised soft assignment (fp64) rounded to fp32 feeds the gate
    wl = case("routed", n=1500, d=128, K=4, window=64, Hq=8, Hkv=2)
    inp = workloads.make_inputs(wl, "cuda")
    rin = workloads.make_router_inputs(wl, "cuda", d_model=256)
    rp = focus.make_route_params(wl.B, wl.n, 256, workloads.ROUTER_DG, wl.K, 2, dtype=wl.dtype, sinkhorn_iters=10, tau=0.1)
    rws = focus.alloc_route_workspace(rp)
    masks = torch.empty((wl.B, wl.n), dtype=torch.int32, device="cuda")
    soft = torch.empty((wl.B, wl.n, wl.K), dtype=torch.float64, device="cuda")
    focus.focus_route(rp, rin["hidden"], rin["w_g"], rin["router_centroids"], rws, masks, soft)
    g = soft.float().contiguous()
    out, lse = run_soft(wl, inp, g, 8.0)
    say("routed", check_soft(wl, inp, g, 8.0, out, lse))


def test_soft_gate_refusals():
    p = focus.make_params(1, 2, 2, 256, 64, 4, 1, 16, causal=False)
    with pytest.raises(focus.FocusError) as e:
        focus.focus_soft_workspace_size(p)
    assert e.value.status == focus.FOCUS_EUNSUPPORTED
    p = focus.make_params(1, 2, 2, 256, 64, 4, 1, 16, softcap=30.0)
    with pytest.raises(focus.FocusError) as e:
        focus.focus_soft_workspace_size(p)
    assert e.value.status == focus.FOCUS_EUNSUPPORTED
