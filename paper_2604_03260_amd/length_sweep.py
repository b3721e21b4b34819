"""Speed-up of the Focus mask over dense causal attention as the sequence grows (the shape of the paper's
wall-clock table, Sec. 3.6: K = 4 with top-2 and K = 8 with hard assignment, 1K to 1M tokens), measured with
this library on synthetic N(0,1) inputs: 32 query heads on 8 KV heads, d = 128, bf16, one sequence.

    python -m paper_2604_03260_amd.length_sweep [--window 1024] [--max-n 1048576]
    python -m paper_2604_03260_amd.length_sweep --decode          # one generated token against n cached tokens

Dense = the same kernel with window = n.  One JSON line per point, then a table.  Times are HIP-event means of
focus_attn_fwd (the bucketing, focus_assign, is timed separately); with --decode the median focus_decode_step
time, the K and V rows the step has to read (rows at least one query head of their KV head attends) and the
rate at which it reads them."""
import argparse
import json

import torch

from paper_2604_03260_amd import focus, workloads


def timed(fn, reps):
    fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def unit_centroids(Hkv, K, d):
    """Seeded N(0,1) rows of unit length, [Hkv, K, d] fp32 (the recipe of the workloads module)."""
    gen = torch.Generator(device="cuda").manual_seed(3003 + K)
    c = torch.randn((Hkv, K, d), generator=gen, device="cuda", dtype=torch.float32).double()
    return (c / c.norm(dim=-1, keepdim=True)).float().contiguous()


def decode_sweep(args):
    base = workloads.CONFIGS["cfg3"]
    steps = 24
    print("%9s | %28s | %28s" % ("n", "K=4 top-2: us, rows, TB/s", "K=8 top-1: us, rows, TB/s"))
    n = max(args.min_n, 4096)
    while n <= args.max_n:
        wl0 = base.scaled(n=n, window=min(args.window, n))
        inp = workloads.make_inputs(wl0, "cuda")
        point = {"n": n}
        cells = []
        for (K, topk) in ((4, 2), (8, 1)):
            wl = wl0.scaled(K=K, topk=topk)
            cents = unit_centroids(wl.Hkv, K, wl.d)
            p = focus.make_params(wl.B, wl.Hq, wl.Hkv, n, wl.d, K, topk, wl.window, dtype=wl.dtype)
            state = focus.alloc_decode_state(p)
            kc, vc = inp["k"].clone(), inp["v"].clone()
            n0 = n - steps
            focus.focus_decode_prefill(p, n0, kc, cents, state)
            qs = [inp["q"][:, :, i].contiguous() for i in range(n0, n)]
            ks = [inp["k"][:, :, i].contiguous() for i in range(n0, n)]
            vs = [inp["v"][:, :, i].contiguous() for i in range(n0, n)]
            out = torch.empty_like(qs[0])
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
            for s in range(steps):
                ev[s].record()
                focus.focus_decode_step(p, n0 + s, qs[s], ks[s], vs[s], cents, kc, vc, state, out)
            ev[steps].record()
            torch.cuda.synchronize()
            ts = sorted(ev[s].elapsed_time(ev[s + 1]) for s in range(4, steps))
            t = ts[len(ts) // 2]
            views = focus.focus_decode_state_views(p, state)
            G = wl.Hq // wl.Hkv
            gu = torch.zeros((wl.B, wl.Hkv), dtype=torch.int32, device="cuda")
            for g_ in range(G):
                gu |= views["mq"].view(wl.B, wl.Hkv, G)[:, :, g_]
            jj = torch.arange(n, device="cuda")
            att = ((views["mk"] & gu[:, :, None]) != 0) | (jj[None, None, :] > n - 1 - wl.window)
            rows = int(att.sum().item())
            nbytes = 2.0 * rows * wl.d * 2
            point["K%d_top%d" % (K, topk)] = {"us_per_step": 1e3 * t, "rows_read": rows, "rows_cached": wl.B * wl.Hkv * n,
                                              "TB_per_s": nbytes / (t * 1e-3) / 1e12}
            cells.append("%9.1f %10d %6.2f" % (1e3 * t, rows, nbytes / (t * 1e-3) / 1e12))
            del state, kc, vc
        print(json.dumps(point), flush=True)
        print("%9d | %28s | %28s" % (n, cells[0], cells[1]), flush=True)
        del inp
        torch.cuda.empty_cache()
        n *= 4


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--window", type=int, default=1024)
    ap.add_argument("--max-n", type=int, default=1 << 20)
    ap.add_argument("--min-n", type=int, default=1 << 10)
    ap.add_argument("--decode", action="store_true", help="time one generated token against n cached tokens instead")
    args = ap.parse_args()
    if args.decode:
        decode_sweep(args)
        return
    base = workloads.CONFIGS["cfg3"]
    rows = []
    n = args.min_n
    while n <= args.max_n:
        wl0 = base.scaled(n=n, window=min(args.window, n))
        inp = workloads.make_inputs(wl0, "cuda")
        q, k, v = inp["q"], inp["k"], inp["v"]
        out = torch.empty_like(q)
        reps = max(1, min(20, (1 << 17) // n))
        point = {"n": n}
        for (K, topk) in ((4, 2), (8, 1), (0, 0)):           # (0, 0): dense
            if K:
                wl = wl0.scaled(K=K, topk=topk)
                cents = unit_centroids(wl.Hkv, K, wl.d)
                p = focus.make_params(wl.B, wl.Hq, wl.Hkv, n, wl.d, K, topk, wl.window, dtype=wl.dtype)
            else:
                wl = wl0.scaled(K=4, topk=2, window=n)
                cents = inp["centroids"]
                p = focus.make_params(wl.B, wl.Hq, wl.Hkv, n, wl.d, 4, 2, n, dtype=wl.dtype)
            ws = focus.alloc_workspace(p)
            rp = torch.empty((wl.B, wl.Hq, n), dtype=torch.int32, device="cuda")
            t_assign = timed(lambda: focus.focus_assign(p, q, k, cents, ws), max(1, reps))
            focus.focus_attn_fwd(p, q, k, v, ws, out, None, rp)
            pairs = int(rp.to(torch.int64).sum().item())
            t_attn = timed(lambda: focus.focus_attn_fwd(p, q, k, v, ws, out, None, None), reps)
            key = "dense" if not K else "K%d_top%d" % (K, topk)
            point[key] = {"ms_assign": t_assign, "ms_attn": t_attn, "allowed_pairs": pairs,
                          "tflops": 4.0 * wl.d * pairs / (t_attn * 1e-3) / 1e12}
            del ws, rp
        for key in ("K4_top2", "K8_top1"):
            point[key]["speedup_vs_dense"] = point["dense"]["ms_attn"] / point[key]["ms_attn"]
            point[key]["allowed_fraction"] = point[key]["allowed_pairs"] / point["dense"]["allowed_pairs"]
        print(json.dumps(point), flush=True)
        rows.append(point)
        del inp, q, k, v, out
        torch.cuda.empty_cache()
        n *= 4
    print("%9s | %10s | %22s | %22s" % ("n", "dense ms", "K=4 top-2: ms, x, frac", "K=8 top-1: ms, x, frac"))
    for r in rows:
        a, b = r["K4_top2"], r["K8_top1"]
        print("%9d | %10.3f | %9.3f %5.2fx %5.1f%% | %9.3f %5.2fx %5.1f%%" % (
            r["n"], r["dense"]["ms_attn"], a["ms_attn"], a["speedup_vs_dense"], 100 * a["allowed_fraction"],
            b["ms_attn"], b["speedup_vs_dense"], 100 * b["allowed_fraction"]))


if __name__ == "__main__":
    main()
