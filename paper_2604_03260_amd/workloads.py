"""Seeded synthetic workloads: the five benchmark shapes and their generators.

This module holds no arithmetic of the method (no scoring, top-k, masking or
softmax): it only draws inputs.  Both the HIP path and the CPU oracle are fed
the bytes produced here, so the generator need not be portable between CPU and
GPU.

Recipe (stands in for the paper's PG-19 activations of GPT-2 124M, Mistral 7B
and LLaMA-2 70B, Sec. 3 / Table 2 / Table 7, which are not available offline):
  seed(tensor) = 1000 * config_id + tensor_id, tensor ids q=0 k=1 v=2
  centroids=3 cluster-ids=4 means=5 row-sample=6.
  q, k, v ~ N(0, 1) drawn in fp32, then (mixture configs) a per-token mean is
  added, then rounded to the config dtype.
  Mixture: each (batch, token) draws one cluster id z in [0, M) with Zipf
  weights 1/(m+1), shared by all heads and by q, k, v; every (tensor, head, m)
  has a mean mu ~ N(0, sigma^2 I_d); x = eps + mu[z].
  Centroids [Hkv, K, d] ~ N(0, 1), each row L2-normalised in fp64, stored fp32.
"""
from dataclasses import dataclass, replace

import numpy as np
import torch

TORCH_DTYPES = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}


@dataclass(frozen=True)
class Workload:
    name: str
    config_id: int
    B: int
    Hq: int
    Hkv: int
    n: int
    d: int
    dtype: str          # "f32" | "bf16" | "f16"
    K: int
    topk: int
    window: int
    causal: bool = True
    softcap: float = 0.0
    mixture: int = 0    # number of cluster means, 0 = none
    sigma: float = 0.5

    def scaled(self, **kw):
        """A smaller problem of the same structure (for oracle-sized parity cases)."""
        return replace(self, **kw)


CONFIGS = {
    "cfg1": Workload("cfg1", 1, 1, 12, 12, 1024, 64, "f32", 4, 2, 128),
    "cfg2": Workload("cfg2", 2, 8, 12, 12, 4096, 64, "bf16", 4, 2, 256, mixture=4),
    "cfg3": Workload("cfg3", 3, 1, 32, 8, 32768, 128, "bf16", 4, 2, 1024),
    "cfg4a": Workload("cfg4a", 4, 1, 64, 8, 131072, 128, "bf16", 8, 1, 4096, softcap=50.0, mixture=8),
    "cfg4b": Workload("cfg4b", 4, 1, 64, 8, 131072, 128, "bf16", 8, 2, 4096, softcap=50.0, mixture=8),
    "cfg5": Workload("cfg5", 5, 1, 32, 8, 1048576, 128, "bf16", 4, 2, 4096),
}


def _gen(device, seed):
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def _draw_tensor(wl, H, tensor_id, device, z, out_dtype):
    """[B,H,n,d] drawn head by head so the fp32 staging stays small."""
    base = 1000 * wl.config_id
    g = _gen(device, base + tensor_id)
    out = torch.empty((wl.B, H, wl.n, wl.d), dtype=out_dtype, device=device)
    mu = None
    if wl.mixture > 0:
        gm = _gen(device, base + 5 + 100 * (tensor_id + 1))
        mu = torch.randn((H, wl.mixture, wl.d), generator=gm, device=device,
                         dtype=torch.float32) * wl.sigma
    for b in range(wl.B):
        for h in range(H):
            x = torch.randn((wl.n, wl.d), generator=g, device=device, dtype=torch.float32)
            if mu is not None:
                x += mu[h][z[b]]
            out[b, h] = x.to(out_dtype)
    return out


def make_inputs(wl, device="cpu"):
    """Returns dict(q, k, v, centroids) of torch tensors on `device`."""
    device = torch.device(device)
    tdt = TORCH_DTYPES[wl.dtype]
    base = 1000 * wl.config_id
    z = None
    if wl.mixture > 0:
        gz = _gen(device, base + 4)
        wts = 1.0 / torch.arange(1, wl.mixture + 1, device=device, dtype=torch.float32)
        z = torch.multinomial(wts.expand(wl.B, -1), wl.n, replacement=True, generator=gz)
    q = _draw_tensor(wl, wl.Hq, 0, device, z, tdt)
    k = _draw_tensor(wl, wl.Hkv, 1, device, z, tdt)
    v = _draw_tensor(wl, wl.Hkv, 2, device, z, tdt)
    gc = _gen(device, base + 3)
    c = torch.randn((wl.Hkv, wl.K, wl.d), generator=gc, device=device, dtype=torch.float32)
    c64 = c.double()
    c64 = c64 / c64.norm(dim=-1, keepdim=True)
    return {"q": q, "k": k, "v": v, "centroids": c64.float().contiguous()}


ROUTER_DG = 16          # the paper's router width (Sec. 3.1: a 16-dimensional projection suffices)


def make_router_inputs(wl, device="cpu", d_model=None, d_g=ROUTER_DG):
    """Inputs of the per-layer router for the same shape: hidden [B,n,d_model] with
    d_model = Hq*d unless given, W_g [d_model,d_g] ~ N(0, 1/d_model), router centroids
    [K,d_g] ~ N(0,1) rows L2-normalised (so scores have unit scale and scores/tau at the
    paper's tau = 0.1 stay far inside the range of exp).  Tensor ids hidden=7 W_g=8
    router-centroids=9 router-means=10; the mixture configs add the same per-token cluster
    mean (cluster ids as for q, k, v) in hidden space."""
    device = torch.device(device)
    tdt = TORCH_DTYPES[wl.dtype]
    base = 1000 * wl.config_id
    dm = d_model if d_model is not None else wl.Hq * wl.d
    g = _gen(device, base + 7)
    hidden = torch.empty((wl.B, wl.n, dm), dtype=tdt, device=device)
    mu = z = None
    if wl.mixture > 0:
        gz = _gen(device, base + 4)
        wts = 1.0 / torch.arange(1, wl.mixture + 1, device=device, dtype=torch.float32)
        z = torch.multinomial(wts.expand(wl.B, -1), wl.n, replacement=True, generator=gz)
        mu = torch.randn((wl.mixture, dm), generator=_gen(device, base + 10), device=device,
                         dtype=torch.float32) * wl.sigma
    rows = max(1, min(wl.n, (1 << 24) // dm))
    for b in range(wl.B):
        for r0 in range(0, wl.n, rows):
            r1 = min(wl.n, r0 + rows)
            x = torch.randn((r1 - r0, dm), generator=g, device=device, dtype=torch.float32)
            if mu is not None:
                x += mu[z[b, r0:r1]]
            hidden[b, r0:r1] = x.to(tdt)
    w_g = torch.randn((dm, d_g), generator=_gen(device, base + 8), device=device, dtype=torch.float32) / dm ** 0.5
    c = torch.randn((wl.K, d_g), generator=_gen(device, base + 9), device=device, dtype=torch.float64)
    c = c / c.norm(dim=-1, keepdim=True)
    return {"hidden": hidden, "w_g": w_g.contiguous(), "router_centroids": c.float().contiguous()}


def sample_rows(wl, count, device="cpu"):
    """Seeded (b,h,i) triples: the window/sequence edge rows of every head first,
    then uniform draws.  Returns an int32 numpy array [count,3]."""
    g = torch.Generator(device="cpu")
    g.manual_seed(1000 * wl.config_id + 6)
    edges = sorted({0, 1, max(wl.window - 1, 0), wl.window, wl.window + 1, wl.n - 1})
    edges = [e for e in edges if 0 <= e < wl.n]
    rows = []
    for b in range(wl.B):
        for h in range(wl.Hq):
            for e in edges:
                rows.append((b, h, e))
    rows = rows[:count]
    rest = count - len(rows)
    if rest > 0:
        bb = torch.randint(0, wl.B, (rest,), generator=g)
        hh = torch.arange(rest) % wl.Hq            # every head covered evenly
        ii = torch.randint(0, wl.n, (rest,), generator=g)
        extra = torch.stack([bb, hh, ii], dim=1).numpy()
        rows = np.concatenate([np.asarray(rows, dtype=np.int64).reshape(-1, 3), extra], axis=0)
    return np.ascontiguousarray(np.asarray(rows, dtype=np.int32).reshape(-1, 3))


def to_host_bits(t):
    """Torch tensor -> numpy array the oracle accepts (fp32, or uint16 bit patterns of bf16 / fp16)."""
    t = t.detach().cpu().contiguous()
    if t.dtype in (torch.bfloat16, torch.float16):
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()
