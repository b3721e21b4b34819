"""Strided q, k, v and out: the three tensors as views of ONE packed projection output
[B, n, (Hq + 2 Hkv) d] (position-major, heads side by side), out as [B, n, Hq, d].  The kernels read
rows through the strides in focus_params; results must equal the contiguous run's bytes and the oracle."""
import numpy as np
import pytest
import torch

from paper_2604_03260_amd import focus, workloads
from tests import harness

pytestmark = pytest.mark.gpu


def packed_views(wl, inp):
    """q, k, v copied into one [B, n, W] buffer; returns [B,H,n,d] views of it and an out view of a [B,n,Hq,d] buffer."""
    W = (wl.Hq + 2 * wl.Hkv) * wl.d
    buf = torch.empty((wl.B, wl.n, W), dtype=inp["q"].dtype, device="cuda")
    hq, hk = wl.Hq * wl.d, wl.Hkv * wl.d
    buf[:, :, :hq] = inp["q"].permute(0, 2, 1, 3).reshape(wl.B, wl.n, hq)
    buf[:, :, hq:hq + hk] = inp["k"].permute(0, 2, 1, 3).reshape(wl.B, wl.n, hk)
    buf[:, :, hq + hk:] = inp["v"].permute(0, 2, 1, 3).reshape(wl.B, wl.n, hk)
    q = buf[:, :, :hq].view(wl.B, wl.n, wl.Hq, wl.d).permute(0, 2, 1, 3)
    k = buf[:, :, hq:hq + hk].view(wl.B, wl.n, wl.Hkv, wl.d).permute(0, 2, 1, 3)
    v = buf[:, :, hq + hk:].view(wl.B, wl.n, wl.Hkv, wl.d).permute(0, 2, 1, 3)
    out_buf = torch.full((wl.B, wl.n, wl.Hq, wl.d), float("nan"), dtype=inp["q"].dtype, device="cuda")
    return buf, q, k, v, out_buf, out_buf.permute(0, 2, 1, 3)


CASES = [
    dict(dtype="bf16", d=128, Hq=8, Hkv=2, n=1500, K=4, topk=2, window=64),
    dict(dtype="f32", d=64, Hq=4, Hkv=4, n=700, K=8, topk=2, window=20),
    dict(dtype="f16", d=80, Hq=6, Hkv=2, n=900, K=4, topk=2, window=33),
    dict(dtype="bf16", d=256, Hq=2, Hkv=1, n=640, K=4, topk=1, window=16, B=2),
    dict(dtype="bf16", d=64, Hq=4, Hkv=2, n=1100, K=32, topk=2, window=25, causal=False),
]


@pytest.mark.parametrize("kw", CASES, ids=[str(i) for i in range(len(CASES))])
def test_strided_tensors_give_the_contiguous_result(kw):
    base = dict(name="strided", config_id=52, B=1, softcap=0.0)
    base.update(kw)
    wl = workloads.Workload(**base)
    inp = workloads.make_inputs(wl, "cuda")
    ref = harness.run_gpu(wl, inp)                                   # contiguous tensors
    buf, q, k, v, out_buf, out = packed_views(wl, inp)
    assert k.data_ptr() == v.data_ptr() - wl.Hkv * wl.d * q.element_size()
    assert focus.strides_of(k) == focus.strides_of(v)
    p = focus.make_params(wl.B, wl.Hq, wl.Hkv, wl.n, wl.d, wl.K, wl.topk, wl.window, causal=wl.causal, dtype=wl.dtype,
                          q_strides=focus.strides_of(q), kv_strides=focus.strides_of(k), o_strides=focus.strides_of(out))
    ws = focus.alloc_workspace(p)
    lse = torch.empty((wl.B, wl.Hq, wl.n), dtype=torch.float32, device="cuda")
    rp = torch.empty((wl.B, wl.Hq, wl.n), dtype=torch.int32, device="cuda")
    keep = buf.clone()
    focus.focus_assign(p, q, k, inp["centroids"], ws)
    focus.focus_attn_fwd(p, q, k, v, ws, out, lse, rp)
    torch.cuda.synchronize()
    assert torch.equal(buf, keep), "inputs were modified"
    views = focus.focus_workspace_views(p, ws)
    for key in ("mq", "mk", "q_group_counts", "k_group_counts", "q_group_lists", "k_group_lists"):
        assert torch.equal(views[key], ref["views"][key]), key
    assert torch.equal(out_buf.permute(0, 2, 1, 3), ref["out"])
    assert torch.equal(lse, ref["lse"]) and torch.equal(rp, ref["row_pairs"])
    # and against the oracle (through the contiguous copies)
    res = dict(out=out_buf.permute(0, 2, 1, 3).contiguous(), lse=lse, row_pairs=rp, views=views)
    mq, mk = harness.check_assign(wl, inp, res)
    harness.check_attn(wl, inp, res, mq, mk)
    # the fp32 vector kernel reads the same strides
    out_buf.fill_(float("nan"))
    focus.focus_attn_fwd(p, q, k, v, ws, out, lse, rp, vector=True)
    torch.cuda.synchronize()
    vec = harness.run_gpu(wl, inp, vector=True)
    assert torch.equal(out_buf.permute(0, 2, 1, 3), vec["out"])


def test_strided_soft_gate_and_token_membership():
    wl = workloads.Workload("strided_soft", 53, 1, 4, 2, 800, 128, "bf16", 4, 2, 40)
    inp = workloads.make_inputs(wl, "cuda")
    buf, q, k, v, out_buf, out = packed_views(wl, inp)
    kw = dict(q_strides=focus.strides_of(q), kv_strides=focus.strides_of(k), o_strides=focus.strides_of(out))
    gen = torch.Generator(device="cuda")
    gen.manual_seed(9)
    g = torch.softmax(torch.randn((wl.B, wl.n, wl.K), generator=gen, device="cuda") * 3, dim=-1).contiguous()
    pc = harness.params_of(wl)
    ps = focus.make_params(wl.B, wl.Hq, wl.Hkv, wl.n, wl.d, wl.K, wl.topk, wl.window, dtype=wl.dtype, **kw)
    o_ref = torch.empty_like(inp["q"])
    focus.focus_attn_soft_fwd(pc, 5.0, g, inp["q"], inp["k"], inp["v"], focus.alloc_soft_workspace(pc), o_ref)
    focus.focus_attn_soft_fwd(ps, 5.0, g, q, k, v, focus.alloc_soft_workspace(ps), out)
    torch.cuda.synchronize()
    assert torch.equal(out_buf.permute(0, 2, 1, 3), o_ref)
    # membership given per token: only k is read by the bucketing
    masks = torch.randint(0, 2, (wl.B, wl.n), generator=gen, device="cuda", dtype=torch.int32) * 2 + 5   # {0,2} or {0,1,2}->invalid
    masks = torch.where(masks == 7, torch.full_like(masks, 6), masks)                                      # {1,2} or {0,2}
    wsc, wss = focus.alloc_workspace(pc), focus.alloc_workspace(ps)
    focus.focus_assign_tokens(pc, masks, inp["k"], wsc)
    focus.focus_attn_fwd(pc, inp["q"], inp["k"], inp["v"], wsc, o_ref)
    out_buf.fill_(float("nan"))
    focus.focus_assign_tokens(ps, masks, k, wss)
    focus.focus_attn_fwd(ps, q, k, v, wss, out)
    torch.cuda.synchronize()
    assert torch.equal(out_buf.permute(0, 2, 1, 3), o_ref)
