#!/usr/bin/env python3
"""Benchmark of the Focus attention forward (focus_assign + focus_attn_fwd) on one MI355X.

One step = one pass of the whole hot path over one synthetic batch that is
already resident in HBM.  Prints ONE JSON line: useful TFLOP/s (4*d FLOPs per
allowed pair, exact pair count) of the whole step, with tokens/s, the MFMA
roofline of the attention kernel, the speed-up over the same library in dense
(plain causal) mode, and the CPU oracle timed on a bounded sample of the same
workload on this machine's host cores.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg3]
"""
import argparse
import json
import os
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

BF16_MFMA_PEAK_TFLOPS = 2516.6      # 256 CU x 2.4 GHz x 4096 FLOP/clk/CU (dense)
FP32_VECTOR_PEAK_TFLOPS = 157.3
FP64_VECTOR_PEAK_TFLOPS = 78.6
# HBM bytes per launch of the attention kernel from rocprofv3 FETCH_SIZE + WRITE_SIZE runs of this
# command (profiles/attn_mfma_kernel_cfg3_counters.txt); None where no counter run was made
MEASURED_TRAFFIC_BYTES = {"cfg3": 5.88e9}
# ... and of the three kernels of one incremental step (profiles/decode_step_cfg3_kernel_trace.txt)
MEASURED_DECODE_TRAFFIC_BYTES = {"cfg3": 1.38e8}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="cfg3")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--no-router", action="store_true")
    ap.add_argument("--no-two-call", action="store_true")
    ap.add_argument("--no-decode", action="store_true")
    ap.add_argument("--no-sdpa", action="store_true", help="skip torch's own causal attention (outside sanity number)")
    ap.add_argument("--no-soft", action="store_true", help="skip the soft-gated training attention leg")
    ap.add_argument("--no-wider", action="store_true", help="skip the half-precision / other-head-dim variants of cfg3")
    ap.add_argument("--cpu-seconds", type=float, default=15.0)
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one plain device copy of q (known size) so a counter run can be calibrated")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (every config is single-GPU); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2604_03260_amd import focus, workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    wl = workloads.CONFIGS[args.workload]
    default_steps = {"cfg1": 50, "cfg2": 50, "cfg3": 20, "cfg4a": 5, "cfg4b": 5, "cfg5": 2}
    steps = args.steps if args.steps is not None else default_steps[wl.name]
    warmup = args.warmup if args.warmup is not None else (1 if wl.name == "cfg5" else 3)

    inp = workloads.make_inputs(wl, "cuda")
    q, k, v, cents = inp["q"], inp["k"], inp["v"], inp["centroids"]

    def make(window):
        p = focus.make_params(wl.B, wl.Hq, wl.Hkv, wl.n, wl.d, wl.K, wl.topk, window, causal=True,
                              dtype=wl.dtype, softcap=wl.softcap)
        return p, focus.alloc_workspace(p)

    p, ws = make(wl.window)
    out = torch.empty_like(q)
    lse = torch.empty((wl.B, wl.Hq, wl.n), dtype=torch.float32, device="cuda")

    # exact allowed-pair count (untimed): the kernel's own per-row counts
    rp = torch.empty((wl.B, wl.Hq, wl.n), dtype=torch.int32, device="cuda")
    focus.focus_assign(p, q, k, cents, ws)
    focus.focus_attn_fwd(p, q, k, v, ws, out, lse, rp)
    torch.cuda.synchronize()
    allowed = int(rp.to(torch.int64).sum().item())
    views = focus.focus_workspace_views(p, ws)
    kcounts = views["k_group_counts"].to(torch.float64)
    dominance = float((kcounts.max(dim=-1).values / wl.n).mean().item())
    del rp
    causal_pairs = wl.B * wl.Hq * (wl.n * (wl.n + 1) // 2)
    useful_flop = 4.0 * wl.d * allowed

    def timed(pp, wws, nsteps, nwarm):
        for _ in range(nwarm):
            focus.focus_assign(pp, q, k, cents, wws)
            focus.focus_attn_fwd(pp, q, k, v, wws, out, lse, None)
        torch.cuda.synchronize()
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(nsteps)]
        t0 = time.perf_counter()
        for s in range(nsteps):
            ev[s][0].record()
            focus.focus_assign(pp, q, k, cents, wws)
            ev[s][1].record()
            focus.focus_attn_fwd(pp, q, k, v, wws, out, lse, None)
            ev[s][2].record()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        t_assign = sum(e[0].elapsed_time(e[1]) for e in ev) / nsteps
        t_attn = sum(e[1].elapsed_time(e[2]) for e in ev) / nsteps
        return wall * 1e3 / nsteps, t_assign, t_attn

    if args.calib_copy:
        calib = q.clone()                 # reads and writes q.numel()*elem bytes once
        torch.cuda.synchronize()
        del calib
    ms_step, ms_assign, ms_attn = timed(p, ws, steps, warmup)
    out_focus = out
    out = torch.empty_like(q)          # later runs (dense mode) must not overwrite the checked output
    tflops_step = useful_flop / (ms_step * 1e-3) / 1e12
    tflops_attn = useful_flop / (ms_attn * 1e-3) / 1e12
    half = wl.dtype in ("bf16", "f16")          # both 16-bit types run on the matrix cores at the same peak
    peak = BF16_MFMA_PEAK_TFLOPS if half else FP32_VECTOR_PEAK_TFLOPS

    result = {
        "metric": "useful TFLOP/s of Focus attention fwd (assign + attention, 4*d FLOP per allowed pair)",
        "value": tflops_step,
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": ms_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": wl.dtype,
        "data": "synthetic",
        "config": {"workload": "%s: B=%d Hq=%d Hkv=%d n=%d d=%d K=%d topk=%d window=%d softcap=%g %s"
                   % (wl.name, wl.B, wl.Hq, wl.Hkv, wl.n, wl.d, wl.K, wl.topk, wl.window, wl.softcap, wl.dtype),
                   "mixture": wl.mixture},
        "tokens_per_s": wl.B * wl.n / (ms_step * 1e-3),
        "ms_assign": ms_assign,
        "ms_attn": ms_attn,
        "allowed_pairs": allowed,
        "allowed_fraction": allowed / causal_pairs,
        "largest_group_fraction": dominance,
        "pct_of_peak_step": 100.0 * tflops_step / peak,
        "roofline": {
            "bound": "mfma" if half else "alu",
            "kernel": "attn_mfma_kernel" if half else "attn_simple_kernel",
            "achieved": tflops_attn,
            "peak": peak,
            "unit": "TFLOP/s",
            "frac": tflops_attn / peak,
            "traffic": MEASURED_TRAFFIC_BYTES.get(wl.name),
            "note": "achieved = 4*d*allowed_pairs / mean focus_attn_fwd time (HIP events; includes the V staging kernel)",
        },
        "paper_context": "paper reports 2.0x (K=4, top-2) and 8.6x (K=8, 1M tokens) over dense FlashAttention on H100-80GB",
    }

    # the matrix-core rate this machine sustains in a register-only MFMA loop (the stand-alone probe the build
    # leaves beside the library), as a second denominator next to the nominal peak
    probe = os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_2604_03260_amd", "_build", "mfma_peak")
    if half and os.path.exists(probe):
        try:
            got = subprocess.run([probe], capture_output=True, text=True, timeout=120)
            fields = got.stdout.strip().split()
            measured_peak = float(fields[0])              # constant operands
            result["measured_mfma_peak_tflops"] = measured_peak
            result["pct_of_measured_mfma_peak_attn"] = 100.0 * tflops_attn / measured_peak
            if len(fields) > 1:                           # operands that change from one MFMA to the next
                result["measured_mfma_peak_random_operands_tflops"] = float(fields[1])
                result["pct_of_measured_mfma_peak_random_operands_attn"] = 100.0 * tflops_attn / float(fields[1])
        except Exception as exc:              # the probe is optional: its absence or failure changes no figure above
            result["measured_mfma_peak_tflops"] = None
            print("bench.py: MFMA peak probe failed: %r" % (exc,), file=sys.stderr)

    if not args.no_dense:
        pd, wsd = make(wl.n)
        dsteps = max(2, steps // 2)
        ms_step_d, _, ms_attn_d = timed(pd, wsd, dsteps, 1)
        result["dense_ms_attn"] = ms_attn_d
        result["dense_tflops_attn"] = 4.0 * wl.d * causal_pairs / (ms_attn_d * 1e-3) / 1e12
        result["speedup_vs_dense_attn"] = ms_attn_d / ms_attn
        result["speedup_vs_dense_step"] = ms_step_d / ms_step
        del wsd
        # an outside sanity number for the dense comparator: torch's own causal attention on the same tensors
        # (harness only; never part of the library or of `value`)
        if half and not args.no_sdpa:
            try:
                import torch.nn.functional as F
                with torch.no_grad():
                    for _ in range(2):
                        o_sd = F.scaled_dot_product_attention(q, k, v, is_causal=True, enable_gqa=(wl.Hq != wl.Hkv))
                    torch.cuda.synchronize()
                    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
                    nsd = max(2, steps // 4)
                    ev[0].record()
                    for _ in range(nsd):
                        o_sd = F.scaled_dot_product_attention(q, k, v, is_causal=True, enable_gqa=(wl.Hq != wl.Hkv))
                    ev[1].record()
                    torch.cuda.synchronize()
                ms_sd = ev[0].elapsed_time(ev[1]) / nsd
                result["torch_sdpa_dense"] = {"ms": ms_sd, "tflops": 4.0 * wl.d * causal_pairs / (ms_sd * 1e-3) / 1e12,
                                              "what": "torch.nn.functional.scaled_dot_product_attention, causal, same q/k/v"}
                del o_sd
            except Exception as exc:
                print("bench.py: torch SDPA sanity run skipped: %r" % (exc,), file=sys.stderr)
            # ... and what the vendor's GEMM library sustains on N(0,1) operands of this dtype on this machine: the
            # rate a dense bf16/fp16 contraction on real data reaches here (the chip's clock follows the data)
            try:
                gen = torch.Generator(device="cuda").manual_seed(4242)
                ga = torch.randn((8192, 8192), generator=gen, device="cuda", dtype=torch.float32).to(q.dtype)
                gb = torch.randn((8192, 8192), generator=gen, device="cuda", dtype=torch.float32).to(q.dtype)
                for _ in range(3):
                    gc = ga @ gb
                torch.cuda.synchronize()
                ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
                ev[0].record()
                for _ in range(20):
                    gc = ga @ gb
                ev[1].record()
                torch.cuda.synchronize()
                ms_mm = ev[0].elapsed_time(ev[1]) / 20
                result["torch_matmul_8192"] = {"ms": ms_mm, "tflops": 2.0 * 8192.0 ** 3 / (ms_mm * 1e-3) / 1e12,
                                               "what": "torch.matmul of two 8192 x 8192 N(0,1) matrices of the workload's dtype"}
                del ga, gb, gc
            except Exception as exc:
                print("bench.py: torch matmul sanity run skipped: %r" % (exc,), file=sys.stderr)

    # context: other shapes through the same step (assign + attention), reported beside the headline workload:
    # the GPT-2 124M shape (short sequences), and the headline shape in half precision and at other head dims
    # (query heads scaled so that Hq*d stays 4096)
    def quick(w2, label, nrep):
        i2 = workloads.make_inputs(w2, "cuda")
        p2 = focus.make_params(w2.B, w2.Hq, w2.Hkv, w2.n, w2.d, w2.K, w2.topk, w2.window, causal=True,
                               dtype=w2.dtype, softcap=w2.softcap)
        ws2 = focus.alloc_workspace(p2)
        o2 = torch.empty_like(i2["q"])
        rp2 = torch.empty((w2.B, w2.Hq, w2.n), dtype=torch.int32, device="cuda")
        focus.focus_assign(p2, i2["q"], i2["k"], i2["centroids"], ws2)
        focus.focus_attn_fwd(p2, i2["q"], i2["k"], i2["v"], ws2, o2, None, rp2)
        torch.cuda.synchronize()
        allowed2 = int(rp2.to(torch.int64).sum().item())
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        ev[0].record()
        for _ in range(nrep):
            focus.focus_assign(p2, i2["q"], i2["k"], i2["centroids"], ws2)
            focus.focus_attn_fwd(p2, i2["q"], i2["k"], i2["v"], ws2, o2, None, None)
        ev[1].record()
        torch.cuda.synchronize()
        ms2 = ev[0].elapsed_time(ev[1]) / nrep
        return {"workload": label, "ms_per_step": ms2, "tokens_per_s": w2.B * w2.n / (ms2 * 1e-3),
                "useful_tflops_step": 4.0 * w2.d * allowed2 / (ms2 * 1e-3) / 1e12,
                "allowed_fraction": allowed2 / (w2.B * w2.Hq * (w2.n * (w2.n + 1) // 2))}

    if wl.name == "cfg3" and not args.no_dense:
        result["other_workloads"] = {"cfg2": quick(
            workloads.CONFIGS["cfg2"], "cfg2: B=8 H=12 n=4096 d=64 K=4 topk=2 window=256 bf16 (4-cluster mixture)", 20)}
    if wl.name == "cfg3" and not args.no_wider:
        from dataclasses import replace
        wider = result.setdefault("other_workloads", {})
        for tag, kw in (("cfg3_f16", dict(dtype="f16")), ("cfg3_d256", dict(d=256, Hq=16, Hkv=4)),
                        ("cfg3_d96", dict(d=96, Hq=40, Hkv=8)), ("cfg3_d80", dict(d=80, Hq=48, Hkv=8)),
                        ("cfg3_d64", dict(d=64, Hq=64, Hkv=16))):
            w2 = replace(wl, name=tag, **kw)
            wider[tag] = quick(w2, "%s: B=%d Hq=%d Hkv=%d n=%d d=%d K=%d topk=%d window=%d %s" % (
                tag, w2.B, w2.Hq, w2.Hkv, w2.n, w2.d, w2.K, w2.topk, w2.window, w2.dtype), 5)

    # the paper's own evaluation order (App. D): the set of pairs that share a group, the set of window pairs
    # that share none, one softmax each, merged through their log-sum-exp -- built from the same kernels, on
    # the same membership, as a comparator of the fused single-softmax launch
    if not args.no_two_call and wl.window < wl.n:
        part_out = torch.empty((2,) + tuple(q.shape), dtype=q.dtype, device="cuda")
        part_lse = torch.empty((2, wl.B, wl.Hq, wl.n), dtype=torch.float32, device="cuda")
        focus.focus_assign(p, q, k, cents, ws)
        tsteps = max(2, steps // 2)
        for _ in range(1):
            focus.focus_attn_fwd_two_call(p, q, k, v, ws, out, lse, part_out, part_lse)
        torch.cuda.synchronize()
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(tsteps)]
        for s in range(tsteps):
            ev[s][0].record()
            focus.focus_attn_fwd_set(p, focus.FOCUS_PAIRS_SHARED, q, k, v, ws, part_out[0], part_lse[0], None)
            ev[s][1].record()
            focus.focus_attn_fwd_set(p, focus.FOCUS_PAIRS_CROSS_LOCAL, q, k, v, ws, part_out[1], part_lse[1], None)
            ev[s][2].record()
            focus.focus_attn_merge(part_out[0], part_lse[0], part_out[1], part_lse[1], out, lse)
            ev[s][3].record()
        torch.cuda.synchronize()
        t_a, t_b, t_m = (sum(e[i].elapsed_time(e[i + 1]) for e in ev) / tsteps for i in range(3))
        result["two_call"] = {
            "what": "App. D: set A (shared group, causal) + set B (window, no shared group) + log-sum-exp merge, "
                    "same kernels and membership; the fused launch is ms_attn",
            "ms_set_a": t_a, "ms_set_b": t_b, "ms_merge": t_m, "ms_attn_two_call": t_a + t_b + t_m,
            "fused_speedup": (t_a + t_b + t_m) / ms_attn,
            "max_abs_diff_vs_fused": float((out.float() - out_focus.float()).abs().max().item()),
        }
        del part_out, part_lse

    # the soft-gated attention of training (Sec. 2 Eq. 2) on the same q, k, v: every causal pair, gate from
    # seeded soft assignments (a softmax of N(0, 4^2) scores per token), slope 8
    if not args.no_soft and wl.softcap == 0.0 and not (wl.d == 256 and half):
        ps = focus.make_params(wl.B, wl.Hq, wl.Hkv, wl.n, wl.d, wl.K, 1, wl.window, causal=True, dtype=wl.dtype)
        wss = focus.alloc_soft_workspace(ps)
        gen = torch.Generator(device="cuda")
        gen.manual_seed(1000 * wl.config_id + 11)
        gsoft = torch.softmax(torch.randn((wl.B, wl.n, wl.K), generator=gen, device="cuda") * 4.0, dim=-1).contiguous()
        focus.focus_attn_soft_fwd(ps, 8.0, gsoft, q, k, v, wss, out)
        torch.cuda.synchronize()
        nsoft = max(2, steps // 4)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        ev[0].record()
        for _ in range(nsoft):
            focus.focus_attn_soft_fwd(ps, 8.0, gsoft, q, k, v, wss, out)
        ev[1].record()
        torch.cuda.synchronize()
        ms_soft = ev[0].elapsed_time(ev[1]) / nsoft
        tf_soft = 4.0 * wl.d * causal_pairs / (ms_soft * 1e-3) / 1e12
        result["soft_gate"] = {
            "what": "focus_attn_soft_fwd (Sec. 2 Eq. 2, forward only): staging + attention over every causal pair",
            "ms": ms_soft, "tflops_qk_pv": tf_soft,
            "roofline": {"bound": "mfma" if half else "alu", "kernel": "attn_mfma_kernel (soft gate)" if half else "attn_simple_kernel",
                         "achieved": tf_soft, "peak": peak, "unit": "TFLOP/s", "frac": tf_soft / peak, "traffic": None,
                         "note": "4*d FLOP per causal pair; the affinity products (3 or 6 MFMAs per 32 keys) are not counted"}}
        del wss, gsoft

    # incremental inference: one token per sequence against the cached K/V of this workload (memory-bound)
    if not args.no_decode:
        dsteps = 32
        n0 = wl.n - dsteps
        state = focus.alloc_decode_state(p)
        kc, vc = k.clone(), v.clone()
        focus.focus_decode_prefill(p, n0, kc, cents, state)
        qs = [q[:, :, i].contiguous() for i in range(n0, wl.n)]
        ks = [k[:, :, i].contiguous() for i in range(n0, wl.n)]
        vs = [v[:, :, i].contiguous() for i in range(n0, wl.n)]
        dout = torch.empty_like(qs[0])
        drp = torch.empty((wl.B, wl.Hq), dtype=torch.int32, device="cuda")
        for s in range(4):                               # warm-up steps (they also advance the cache)
            focus.focus_decode_step(p, n0 + s, qs[s], ks[s], vs[s], cents, kc, vc, state, dout, None, drp)
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(dsteps - 4 + 1)]
        for s in range(4, dsteps):
            ev[s - 4].record()
            focus.focus_decode_step(p, n0 + s, qs[s], ks[s], vs[s], cents, kc, vc, state, dout, None, drp)
        ev[dsteps - 4].record()
        torch.cuda.synchronize()
        ts = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(dsteps - 4))
        t_dec = ts[len(ts) // 2]
        # the same steps replayed from ONE captured HIP graph (position in device memory, advanced inside the
        # graph): what a generation loop pays per token without per-step launch work on the host
        focus.focus_decode_prefill(p, n0, kc, cents, state)          # lists back to n0; the caches keep their rows
        posd = torch.full((wl.B,), n0, dtype=torch.int32, device="cuda")
        qb, kb, vb = qs[0].clone(), ks[0].clone(), vs[0].clone()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        dgraph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(dgraph, stream=side):
            focus.focus_decode_step_at(p, posd, qb, kb, vb, cents, kc, vc, state, dout, None, drp)
            posd.add_(1)
        for s in range(4):                               # warm-up replays
            qb.copy_(qs[s]); kb.copy_(ks[s]); vb.copy_(vs[s])
            dgraph.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for s in range(4, dsteps):                       # the whole loop enqueued, as a generation loop would
            qb.copy_(qs[s]); kb.copy_(ks[s]); vb.copy_(vs[s])
            dgraph.replay()
        e1.record()
        torch.cuda.synchronize()
        t_dec_graph = e0.elapsed_time(e1) / (dsteps - 4)
        # rows of K and V the last step had to read: per KV head the union over its query heads of
        # {window} + {keys whose group set meets the head's}; membership read back from the state
        dviews = focus.focus_decode_state_views(p, state)
        mk_t, mq_t = dviews["mk"], dviews["mq"]
        Gq = wl.Hq // wl.Hkv
        gu = torch.zeros((wl.B, wl.Hkv), dtype=torch.int32, device="cuda")
        for g_ in range(Gq):
            gu |= mq_t.view(wl.B, wl.Hkv, Gq)[:, :, g_]
        pos_last = wl.n - 1
        jj = torch.arange(wl.n, device="cuda")
        att = ((mk_t & gu[:, :, None]) != 0) | (jj[None, None, :] > pos_last - wl.window)
        unique_rows = int(att.sum().item())
        elem = 2 if wl.dtype in ("bf16", "f16") else 4
        dec_bytes = 2.0 * unique_rows * wl.d * elem
        per_head_rows = int(drp.to(torch.int64).sum().item())
        result["decode"] = {
            "what": "focus_decode_step at context n (route + append + attention + merge), median of %d steps" % (dsteps - 4),
            "ms_per_step": t_dec, "tokens_per_s": wl.B / (t_dec * 1e-3),
            "ms_per_token_graph_loop": t_dec_graph,      # three input copies + one graph replay per token, enqueued back to back
            "attended_keys_all_heads": per_head_rows,
            "roofline": {"bound": "hbm", "kernel": "decode_attn (whole step timed)", "achieved": dec_bytes / (t_dec * 1e-3) / 1e9,
                         "peak": 8000.0, "unit": "GB/s", "frac": dec_bytes / (t_dec * 1e-3) / 1e9 / 8000.0,
                         "traffic": MEASURED_DECODE_TRAFFIC_BYTES.get(wl.name),
                         "note": "algorithmic bytes = K and V rows of the keys at least one query head of the KV head "
                                 "attends, read once (%d rows, %.1f MB); per-head reads would be %.1f MB"
                                 % (unique_rows, dec_bytes / 1e6, 2.0 * per_head_rows * wl.d * elem / 1e6)},
        }
        del state, kc, vc, qs, ks, vs

    mq_host = mk_host = None
    if not args.no_cpu_baseline:       # the router leg below reuses the workspace: keep the per-head membership
        mq_host = views["mq"].cpu().numpy().view(np.uint32).copy()
        mk_host = views["mk"].cpu().numpy().view(np.uint32).copy()

    # the paper's own front-end: one routing per token from the layer's hidden state (Sec. 2), then the same
    # bucketing and attention; reported beside the headline path, never part of `value`
    if not args.no_router:
        rin = workloads.make_router_inputs(wl, "cuda")
        dm, dg = rin["hidden"].shape[-1], rin["w_g"].shape[1]
        tmasks = torch.empty((wl.B, wl.n), dtype=torch.int32, device="cuda")
        rp10 = focus.make_route_params(wl.B, wl.n, dm, dg, wl.K, wl.topk, dtype=wl.dtype, sinkhorn_iters=10, tau=0.1)
        rp0 = focus.make_route_params(wl.B, wl.n, dm, dg, wl.K, wl.topk, dtype=wl.dtype, sinkhorn_iters=0, tau=0.1)
        rws = focus.alloc_route_workspace(rp10)
        rpairs = torch.empty((wl.B, wl.Hq, wl.n), dtype=torch.int32, device="cuda")
        focus.focus_route(rp10, rin["hidden"], rin["w_g"], rin["router_centroids"], rws, tmasks)
        focus.focus_assign_tokens(p, tmasks, k, ws)
        focus.focus_attn_fwd(p, q, k, v, ws, out, None, rpairs)
        torch.cuda.synchronize()
        r_allowed = int(rpairs.to(torch.int64).sum().item())
        del rpairs
        rsteps = max(3, steps // 2)
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(rsteps)]
        for s in range(rsteps):
            ev[s][0].record()
            focus.focus_route(rp0, rin["hidden"], rin["w_g"], rin["router_centroids"], rws, tmasks)
            ev[s][1].record()
            focus.focus_route(rp10, rin["hidden"], rin["w_g"], rin["router_centroids"], rws, tmasks)
            ev[s][2].record()
            focus.focus_assign_tokens(p, tmasks, k, ws)
            ev[s][3].record()
            focus.focus_attn_fwd(p, q, k, v, ws, out, None, None)
            ev[s][4].record()
        torch.cuda.synchronize()
        t_proj, t_route, t_tok, t_rattn = (sum(e[i].elapsed_time(e[i + 1]) for e in ev) / rsteps for i in range(4))
        proj_flop = 2.0 * wl.B * wl.n * dm * dg
        result["router_path"] = {
            "workload": "hidden [B=%d, n=%d, d_model=%d] %s, d_g=%d, K=%d, top-%d, tau=0.1, 10 Sinkhorn rounds"
                        % (wl.B, wl.n, dm, wl.dtype, dg, wl.K, wl.topk),
            "ms_route": t_route, "ms_route_no_sinkhorn": t_proj, "ms_assign_tokens": t_tok, "ms_attn": t_rattn,
            "ms_per_step": t_route + t_tok + t_rattn,
            "tokens_per_s": wl.B * wl.n / ((t_route + t_tok + t_rattn) * 1e-3),
            "allowed_fraction": r_allowed / causal_pairs,
            "useful_tflops_step": 4.0 * wl.d * r_allowed / ((t_route + t_tok + t_rattn) * 1e-3) / 1e12,
            "roofline": {"bound": "alu", "kernel": "route_project_kernel", "achieved": proj_flop / (t_proj * 1e-3) / 1e12,
                         "peak": FP64_VECTOR_PEAK_TFLOPS, "unit": "TFLOP/s",
                         "frac": proj_flop / (t_proj * 1e-3) / 1e12 / FP64_VECTOR_PEAK_TFLOPS, "traffic": None,
                         "note": "achieved = 2*B*n*d_model*d_g fp64 FLOP / mean focus_route time without Sinkhorn "
                                 "(projection + two table conversions)"},
        }
        del rin, rws, tmasks

    if not args.no_cpu_baseline:
        from oracle import focus_oracle as fo
        pb = fo.Problem(wl.B, wl.Hq, wl.Hkv, wl.n, wl.d, wl.K, wl.topk, wl.window, causal=True,
                        dtype=wl.dtype, softcap=wl.softcap)
        mq, mk = mq_host, mk_host
        qh, kh, vh = (workloads.to_host_bits(t) for t in (q, k, v))
        rows_all = workloads.sample_rows(wl, min(wl.B * wl.Hq * wl.n, 1 << 20))
        # calibrate on a few rows, then size the sample to about cpu_seconds
        t0 = time.perf_counter()
        _, _, pr = fo.attn_rows(pb, qh, kh, vh, mq, mk, rows=rows_all[:64])
        dt = time.perf_counter() - t0
        nrows = int(min(len(rows_all), max(64, 64 * args.cpu_seconds / max(dt, 1e-3))))
        t0 = time.perf_counter()
        o_ref, _, pr = fo.attn_rows(pb, qh, kh, vh, mq, mk, rows=rows_all[:nrows])
        dt = time.perf_counter() - t0
        sample_flop = 4.0 * wl.d * float(pr.sum())
        rr = rows_all[:nrows]
        got = out_focus[rr[:, 0], rr[:, 1], rr[:, 2]].float().cpu().numpy().astype(np.float64)
        result["cpu_baseline"] = {
            "value": sample_flop / dt / 1e12,
            "unit": "TFLOP/s",
            "cores": fo.num_threads(),
            "kind": "oracle",
            "sample": "%d seeded query rows (all heads) of %s, attention rows only, %.1f s" % (nrows, wl.name, dt),
            "max_abs_err_vs_gpu": float(np.abs(got - o_ref).max()),
        }
    print(json.dumps(result))


if __name__ == "__main__":
    main()
