"""focus_route_noalloc (the router with the library's static scratch, for callers that cannot allocate)
against focus_route on the same inputs: the same kernels on another buffer, so masks and soft assignments
must be bit-identical; and both against the oracle at the router's bars.  Two calls in a row, the second
on a smaller input, so leftovers of the first call in the shared scratch would show."""
import numpy as np
import pytest
import torch

from paper_2604_03260_amd import focus, workloads
from tests import test_gpu_router as tr

pytestmark = pytest.mark.gpu


def route_both(wl, rin, iters):
    hidden = rin["hidden"]
    dm, dg = hidden.shape[-1], rin["w_g"].shape[1]
    rp = focus.make_route_params(wl.B, wl.n, dm, dg, wl.K, wl.topk, dtype=wl.dtype, sinkhorn_iters=iters, tau=0.1)
    out = {}
    for name in ("workspace", "noalloc"):
        masks = torch.full((wl.B, wl.n), -1, dtype=torch.int32, device="cuda")
        soft = torch.full((wl.B, wl.n, wl.K), float("nan"), dtype=torch.float64, device="cuda")
        if name == "workspace":
            rws = focus.alloc_route_workspace(rp)
            focus.focus_route(rp, hidden, rin["w_g"], rin["router_centroids"], rws, masks, soft)
        else:
            focus.focus_route_noalloc(rp, hidden, rin["w_g"], rin["router_centroids"], masks, soft)
        torch.cuda.synchronize()
        out[name] = (masks, soft)
    return out


CASES = [
    # B, n, d_model, d_g, K, topk, dtype, Sinkhorn rounds -- each followed by a smaller call
    ((2, 9000, 512, 16, 8, 2, "bf16", 10), (1, 700, 264, 16, 4, 2, "bf16", 10)),
    ((1, 20000, 256, 32, 16, 3, "f32", 3), (3, 130, 64, 8, 8, 1, "f32", 0)),
    ((1, 32768, 1024, 16, 4, 2, "f16", 0), (1, 1, 64, 16, 4, 2, "f16", 10)),
]


@pytest.mark.parametrize("first,second", CASES)
def test_noalloc_router_matches_the_workspace_router(first, second):
    for case_no, (B, n, dm, dg, K, topk, dtype, iters) in enumerate((first, second)):
        print("case", case_no, (B, n, dm, dg, K, topk, dtype, iters), flush=True)
        wl = workloads.Workload("r", 70 + case_no, B, 1, 1, n, 64, dtype, K, topk, 16, mixture=3 if K > 4 else 0)
        rin = workloads.make_router_inputs(wl, "cuda", d_model=dm, d_g=dg)
        got = route_both(wl, rin, iters)
        assert torch.equal(got["noalloc"][0], got["workspace"][0]), "masks differ"
        assert torch.equal(got["noalloc"][1], got["workspace"][1]), "soft assignments differ"
        # and the router's own bars against the oracle (bit-exact without Sinkhorn, 1e-9 relative with it)
        m_ref, _, g_ref = tr.oracle_route(wl, rin, iters)
        masks = got["noalloc"][0].cpu().numpy().view(np.uint32)
        g_got = got["noalloc"][1].cpu().numpy()
        if iters == 0:
            assert np.array_equal(g_got, g_ref) and np.array_equal(masks, m_ref)
        else:
            rel = np.abs(g_got - g_ref) / np.maximum(np.abs(g_ref), 1e-300)
            assert rel.max() <= tr.SOFT_RTOL
            if n > 1:
                assert (masks == m_ref).mean() > 0.999
