#!/usr/bin/env python3
"""Benchmark of the Focus attention forward (focus_assign + focus_attn_fwd) on one MI355X.

One step = one pass of the whole hot path over one synthetic batch that is already resident in HBM.
Prints ONE JSON line.  The headline workload is the largest single-GPU configuration, cfg5 (1M tokens);
`value` is its useful TFLOP/s (4*d FLOP per allowed pair, exact pair count) over the whole step.  The same
line carries the MFMA roofline of the attention kernel and the HBM roofline of the assignment pass for the
headline and for every other configuration (`other_workloads`), the speed-up over this library's own dense
(plain causal) mode, the CPU oracle timed on a bounded sample on this machine's host cores, and the side legs
(two-call comparator, router front-end, incremental step, soft gate, other head dims and types).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg5] [--only-headline]
    python bench.py --sweep lengths | decode      # Focus against dense from 1K to 1M tokens (a table, no JSON line)

Progress goes to stderr, the JSON line to stdout.
"""
import argparse
import json
import os
import re
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

BF16_MFMA_PEAK_TFLOPS = 2516.6      # 256 CU x 2.4 GHz x 4096 FLOP/clk/CU (dense)
FP32_VECTOR_PEAK_TFLOPS = 157.3
FP64_VECTOR_PEAK_TFLOPS = 78.6
HBM_PEAK_GBS = 8000.0
DEFAULT_STEPS = {"cfg1": (50, 5), "cfg2": (50, 5), "cfg3": (20, 5), "cfg4a": (5, 2), "cfg4b": (5, 2), "cfg5": (5, 1)}
PAPER_CONTEXT = ("paper reports 2.0x (K=4, top-2) and 8.6x (K=8, 1M tokens) over dense FlashAttention, "
                 "two FlashAttention calls + PyTorch on one H100-80GB; ratios only, another machine")


def note(*a):
    print("[bench]", *a, file=sys.stderr, flush=True)


class ClockSampler:
    """Samples the GPU core clock with `rocm-smi -c --json` (a child process about every 0.3 s; reads sysfs, touches no
    HIP state) while timed steps run: the clock the chip actually holds under this kernel on this data."""

    def __init__(self):
        import threading
        self.samples, self.stop, self.thread = [], False, threading.Thread(target=self._run, daemon=True)

    def _run(self):
        while not self.stop:
            try:
                r = subprocess.run(["rocm-smi", "-c", "--json"], capture_output=True, text=True, timeout=10)
                card = json.loads(r.stdout)
                card = card[sorted(card.keys())[0]]
                m = re.search(r"(\d+)\s*Mhz", card.get("sclk clock speed:", ""), re.I)
                if m:
                    self.samples.append((time.perf_counter(), int(m.group(1))))
            except Exception:
                return
            time.sleep(0.05)

    def __enter__(self):
        self.thread.start()
        return self

    def __exit__(self, *a):
        self.stop = True
        self.thread.join(timeout=15)

    def summary(self, t0, t1):
        xs = [v for t, v in self.samples if t0 <= t <= t1]
        if not xs:
            return None
        return {"mean": sum(xs) / len(xs), "min": min(xs), "max": max(xs), "samples": len(xs),
                "what": "sclk from rocm-smi -c while the timed steps ran (nominal 2400 MHz)"}


def measured_traffic(kernel, workload):
    """HBM bytes per launch from the committed counter summary of that kernel and workload
    (profiles/<kernel>_<workload>_counters.txt, a line `traffic_bytes_per_launch = <number>`), else None:
    counters cannot be read from inside this process, so the figure lives in the summary of the rocprofv3
    --pmc runs of this same command and nowhere else."""
    path = os.path.join(ROOT, "profiles", "%s_%s_counters.txt" % (kernel, workload))
    try:
        m = re.search(r"^\s*traffic_bytes_per_launch\s*=\s*([0-9.eE+]+)", open(path).read(), re.M)
        return float(m.group(1)) if m else None
    except OSError:
        return None


def describe(wl):
    return "%s: B=%d Hq=%d Hkv=%d n=%d d=%d K=%d topk=%d window=%d softcap=%g %s%s" % (
        wl.name, wl.B, wl.Hq, wl.Hkv, wl.n, wl.d, wl.K, wl.topk, wl.window, wl.softcap, wl.dtype,
        " (%d-cluster mixture)" % wl.mixture if wl.mixture else "")


def assign_bytes(wl):
    """Algorithmic bytes of the assignment pass: every query and key row read once (d * elemsize), one 4-byte
    membership mask and topk 4-byte list entries written per token-head."""
    elem = 4 if wl.dtype == "f32" else 2
    token_heads = wl.B * (wl.Hq + wl.Hkv) * wl.n
    return float(token_heads) * (wl.d * elem + 4 + 4 * wl.topk)


class Runner:
    """One workload resident on the device: inputs, params, workspace, outputs."""

    def __init__(self, torch, focus, workloads, wl, window=None, zero_inputs=False):
        self.torch, self.focus, self.wl = torch, focus, wl
        self.inp = workloads.make_inputs(wl, "cuda")
        if zero_inputs:                         # same launches, no switching activity in the multipliers
            for name in ("q", "k", "v"):
                self.inp[name].zero_()
        self.t_timed = (0.0, 0.0)
        self.p = self.params(wl.window if window is None else window)
        self.ws = focus.alloc_workspace(self.p)
        self.out = torch.empty_like(self.inp["q"])
        self.lse = torch.empty((wl.B, wl.Hq, wl.n), dtype=torch.float32, device="cuda")

    def params(self, window):
        wl = self.wl
        return self.focus.make_params(wl.B, wl.Hq, wl.Hkv, wl.n, wl.d, wl.K, wl.topk, window, causal=True,
                                      dtype=wl.dtype, softcap=wl.softcap)

    def step(self, p=None, ws=None, row_pairs=None):
        i, f = self.inp, self.focus
        p = self.p if p is None else p
        ws = self.ws if ws is None else ws
        f.focus_assign(p, i["q"], i["k"], i["centroids"], ws)
        f.focus_attn_fwd(p, i["q"], i["k"], i["v"], ws, self.out, self.lse, row_pairs)

    def count_pairs(self):
        """Exact allowed-pair count (untimed): the kernel's own per-row counts."""
        torch, wl = self.torch, self.wl
        rp = torch.empty((wl.B, wl.Hq, wl.n), dtype=torch.int32, device="cuda")
        self.step(row_pairs=rp)
        torch.cuda.synchronize()
        return int(rp.to(torch.int64).sum().item())

    def timed(self, steps, warmup, p=None, ws=None, label=None):
        """`warmup` untimed steps, then exactly `steps` steps between two device synchronisations.  Per step, HIP
        events on the launch stream split the assignment pass from the attention launch.  Returns
        (wall ms per step, mean focus_assign ms, mean focus_attn_fwd ms)."""
        torch, i, f = self.torch, self.inp, self.focus
        p = self.p if p is None else p
        ws = self.ws if ws is None else ws
        for _ in range(warmup):
            self.step(p, ws)
        torch.cuda.synchronize()
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
        t0 = time.perf_counter()
        for s in range(steps):
            ev[s][0].record()
            f.focus_assign(p, i["q"], i["k"], i["centroids"], ws)
            ev[s][1].record()
            f.focus_attn_fwd(p, i["q"], i["k"], i["v"], ws, self.out, self.lse, None)
            ev[s][2].record()
        if label:                               # everything is enqueued: waiting step by step costs the GPU nothing
            for s in range(steps):
                ev[s][2].synchronize()
                if time.perf_counter() - t0 > 5.0:
                    note("%s: step %d of %d done" % (label, s + 1, steps))
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        self.t_timed = (t0, t0 + wall)
        t_assign = sum(e[0].elapsed_time(e[1]) for e in ev) / steps
        t_attn = sum(e[1].elapsed_time(e[2]) for e in ev) / steps
        return wall * 1e3 / steps, t_assign, t_attn


def measure(torch, focus, workloads, wl, steps, warmup, dense_steps, keep=False, clock=None, zero_inputs=False):
    """The step on one workload: times, exact pair count, the two rooflines, the dense comparator."""
    note("workload", describe(wl) + (" (q, k, v zeroed)" if zero_inputs else ""))
    r = Runner(torch, focus, workloads, wl, zero_inputs=zero_inputs)
    allowed = r.count_pairs()
    kcounts = focus.focus_workspace_views(r.p, r.ws)["k_group_counts"].to(torch.float64)
    dominance = float((kcounts.max(dim=-1).values / wl.n).mean().item())
    causal_pairs = wl.B * wl.Hq * (wl.n * (wl.n + 1) // 2)
    useful_flop = 4.0 * wl.d * allowed
    ms_step, ms_assign, ms_attn = r.timed(steps, warmup, label=wl.name)
    sclk = clock.summary(*r.t_timed) if clock else None
    half = wl.dtype in ("bf16", "f16")          # both 16-bit types run on the matrix cores at the same peak
    peak = BF16_MFMA_PEAK_TFLOPS if half else FP32_VECTOR_PEAK_TFLOPS
    kernel = "attn_mfma_kernel" if half else "attn_simple_kernel"
    tflops_attn = useful_flop / (ms_attn * 1e-3) / 1e12
    gbs_assign = assign_bytes(wl) / (ms_assign * 1e-3) / 1e9
    res = {
        "workload": describe(wl),
        "steps": steps, "warmup": warmup,
        "ms_per_step": ms_step, "ms_assign": ms_assign, "ms_attn": ms_attn,
        "useful_tflops_step": useful_flop / (ms_step * 1e-3) / 1e12,
        "tokens_per_s": wl.B * wl.n / (ms_step * 1e-3),
        "allowed_pairs": allowed, "allowed_fraction": allowed / causal_pairs,
        "largest_group_fraction": dominance,
        "sclk_mhz": sclk,
        "roofline": {
            "bound": "mfma" if half else "alu", "kernel": kernel,
            "achieved": tflops_attn, "peak": peak, "unit": "TFLOP/s", "frac": tflops_attn / peak,
            "traffic": measured_traffic(kernel, wl.name),
            "note": "achieved = 4*d*allowed_pairs / mean focus_attn_fwd time (HIP events on the launch stream; "
                    "the launch includes the V staging kernel, about 1 %)",
        },
        "roofline_assign": {
            "bound": "hbm", "kernel": "focus_assign (all its launches)",
            "achieved": gbs_assign, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs_assign / HBM_PEAK_GBS,
            "traffic": measured_traffic("focus_assign", wl.name),
            "note": "algorithmic bytes = (q + k rows read once) + 4 B mask + 4*topk B list entries per token-head "
                    "= %.1f MB, over the mean focus_assign time" % (assign_bytes(wl) / 1e6),
        },
    }
    if dense_steps > 0 and wl.window < wl.n:
        pd = r.params(wl.n)
        wsd = focus.alloc_workspace(pd)
        keep_out = r.out
        r.out = torch.empty_like(keep_out)      # the dense run must not overwrite the checked output
        ms_step_d, _, ms_attn_d = r.timed(dense_steps, 1, pd, wsd, label=wl.name + " dense")
        r.out = keep_out
        res["dense"] = {"ms_attn": ms_attn_d, "ms_per_step": ms_step_d,
                        "sclk_mhz": clock.summary(*r.t_timed) if clock else None,
                        "tflops_attn": 4.0 * wl.d * causal_pairs / (ms_attn_d * 1e-3) / 1e12,
                        "frac_of_peak": 4.0 * wl.d * causal_pairs / (ms_attn_d * 1e-3) / 1e12 / peak,
                        "what": "this library with window = n (plain causal attention through the same kernel)"}
        res["speedup_vs_dense_attn"] = ms_attn_d / ms_attn
        res["speedup_vs_dense_step"] = ms_step_d / ms_step
        del wsd
    if keep:
        return res, r
    del r
    torch.cuda.empty_cache()
    return res


def leg_mfma_probe(result, tflops_attn):
    """The matrix-core rate this machine sustains in a register-only MFMA loop (the stand-alone program the build
    leaves beside the library), as a second denominator next to the nominal peak."""
    probe = os.path.join(ROOT, "paper_2604_03260_amd", "_build", "mfma_peak")
    if not os.path.exists(probe):
        return
    try:
        got = subprocess.run([probe], capture_output=True, text=True, timeout=120)
        fields = got.stdout.strip().split()
        result["measured_mfma_peak_tflops"] = float(fields[0])               # constant operands
        result["pct_of_measured_mfma_peak_attn"] = 100.0 * tflops_attn / float(fields[0])
        result["measured_mfma_peak_random_operands_tflops"] = float(fields[1])   # operands that change every MFMA
        result["pct_of_measured_mfma_peak_random_operands_attn"] = 100.0 * tflops_attn / float(fields[1])
    except Exception as exc:                  # optional: its absence or failure changes no figure above
        result["measured_mfma_peak_tflops"] = None
        note("MFMA peak probe failed: %r" % (exc,))


def leg_outside_numbers(torch, r, result, steps):
    """Harness-only sanity numbers from torch itself on the same box: its causal attention on the same q, k, v,
    and its bf16 GEMM on N(0,1) operands (what a plain dense contraction on real data reaches here)."""
    wl, i = r.wl, r.inp
    causal_pairs = wl.B * wl.Hq * (wl.n * (wl.n + 1) // 2)
    try:
        import torch.nn.functional as F
        with torch.no_grad():
            for _ in range(2):
                o_sd = F.scaled_dot_product_attention(i["q"], i["k"], i["v"], is_causal=True, enable_gqa=(wl.Hq != wl.Hkv))
            torch.cuda.synchronize()
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
            nsd = max(2, steps // 4)
            ev[0].record()
            for _ in range(nsd):
                o_sd = F.scaled_dot_product_attention(i["q"], i["k"], i["v"], is_causal=True, enable_gqa=(wl.Hq != wl.Hkv))
            ev[1].record()
            torch.cuda.synchronize()
        ms_sd = ev[0].elapsed_time(ev[1]) / nsd
        result["torch_sdpa_dense"] = {"workload": wl.name, "ms": ms_sd,
                                      "tflops": 4.0 * wl.d * causal_pairs / (ms_sd * 1e-3) / 1e12,
                                      "what": "torch.nn.functional.scaled_dot_product_attention, causal, same q/k/v"}
        del o_sd
    except Exception as exc:
        note("torch SDPA sanity run skipped: %r" % (exc,))
    try:
        gen = torch.Generator(device="cuda").manual_seed(4242)
        ga = torch.randn((8192, 8192), generator=gen, device="cuda", dtype=torch.float32).to(i["q"].dtype)
        gb = torch.randn((8192, 8192), generator=gen, device="cuda", dtype=torch.float32).to(i["q"].dtype)
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
        note("torch matmul sanity run skipped: %r" % (exc,))


def leg_two_call(torch, focus, r, ms_attn, out_focus, tsteps):
    """The paper's own evaluation order (App. D): the pairs that share a group, the window pairs that share none,
    one softmax each, merged through their log-sum-exp; same kernels and membership as the fused launch."""
    wl, i, p, ws = r.wl, r.inp, r.p, r.ws
    q, k, v = i["q"], i["k"], i["v"]
    part_out = torch.empty((2,) + tuple(q.shape), dtype=q.dtype, device="cuda")
    part_lse = torch.empty((2, wl.B, wl.Hq, wl.n), dtype=torch.float32, device="cuda")
    out = torch.empty_like(q)
    focus.focus_assign(p, q, k, i["centroids"], ws)
    focus.focus_attn_fwd_two_call(p, q, k, v, ws, out, r.lse, part_out, part_lse)
    torch.cuda.synchronize()
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(tsteps)]
    for s in range(tsteps):
        ev[s][0].record()
        focus.focus_attn_fwd_set(p, focus.FOCUS_PAIRS_SHARED, q, k, v, ws, part_out[0], part_lse[0], None)
        ev[s][1].record()
        focus.focus_attn_fwd_set(p, focus.FOCUS_PAIRS_CROSS_LOCAL, q, k, v, ws, part_out[1], part_lse[1], None)
        ev[s][2].record()
        focus.focus_attn_merge(part_out[0], part_lse[0], part_out[1], part_lse[1], out, r.lse)
        ev[s][3].record()
    torch.cuda.synchronize()
    t_a, t_b, t_m = (sum(e[j].elapsed_time(e[j + 1]) for e in ev) / tsteps for j in range(3))
    return {
        "workload": wl.name,
        "what": "App. D: set A (shared group, causal) + set B (window, no shared group) + log-sum-exp merge, "
                "same kernels and membership; the fused launch is ms_attn_fused",
        "ms_set_a": t_a, "ms_set_b": t_b, "ms_merge": t_m, "ms_attn_two_call": t_a + t_b + t_m,
        "ms_attn_fused": ms_attn, "fused_speedup": (t_a + t_b + t_m) / ms_attn,
        "max_abs_diff_vs_fused": float((out.float() - out_focus.float()).abs().max().item()),
    }


def leg_soft_gate(torch, focus, r, steps):
    """The soft-gated attention of training (Sec. 2 Eq. 2) on the same q, k, v: every causal pair, gate from seeded
    soft assignments (a softmax of N(0, 4^2) scores per token), slope 8."""
    wl, i = r.wl, r.inp
    half = wl.dtype in ("bf16", "f16")
    peak = BF16_MFMA_PEAK_TFLOPS if half else FP32_VECTOR_PEAK_TFLOPS
    causal_pairs = wl.B * wl.Hq * (wl.n * (wl.n + 1) // 2)
    ps = focus.make_params(wl.B, wl.Hq, wl.Hkv, wl.n, wl.d, wl.K, 1, wl.window, causal=True, dtype=wl.dtype)
    wss = focus.alloc_soft_workspace(ps)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(1000 * wl.config_id + 11)
    gsoft = torch.softmax(torch.randn((wl.B, wl.n, wl.K), generator=gen, device="cuda") * 4.0, dim=-1).contiguous()
    out = torch.empty_like(i["q"])
    focus.focus_attn_soft_fwd(ps, 8.0, gsoft, i["q"], i["k"], i["v"], wss, out)
    torch.cuda.synchronize()
    nsoft = max(2, steps // 4)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    ev[0].record()
    for _ in range(nsoft):
        focus.focus_attn_soft_fwd(ps, 8.0, gsoft, i["q"], i["k"], i["v"], wss, out)
    ev[1].record()
    torch.cuda.synchronize()
    ms_soft = ev[0].elapsed_time(ev[1]) / nsoft
    tf_soft = 4.0 * wl.d * causal_pairs / (ms_soft * 1e-3) / 1e12
    return {
        "workload": wl.name,
        "what": "focus_attn_soft_fwd (Sec. 2 Eq. 2, forward only): staging + attention over every causal pair",
        "ms": ms_soft, "tflops_qk_pv": tf_soft,
        "roofline": {"bound": "mfma" if half else "alu", "kernel": "attn_mfma_kernel (soft gate)" if half else "attn_simple_kernel",
                     "achieved": tf_soft, "peak": peak, "unit": "TFLOP/s", "frac": tf_soft / peak, "traffic": None,
                     "note": "4*d FLOP per causal pair; the affinity products (3 or 6 MFMAs per 32 keys) are not counted"}}


def leg_decode(torch, focus, r):
    """Incremental inference: one token per sequence against the cached K/V of this workload (memory-bound)."""
    wl, i, p = r.wl, r.inp, r.p
    q, k, v, cents = i["q"], i["k"], i["v"], i["centroids"]
    dsteps = 32
    n0 = wl.n - dsteps
    state = focus.alloc_decode_state(p)
    kc, vc = k.clone(), v.clone()
    focus.focus_decode_prefill(p, n0, kc, cents, state)
    qs = [q[:, :, j].contiguous() for j in range(n0, wl.n)]
    ks = [k[:, :, j].contiguous() for j in range(n0, wl.n)]
    vs = [v[:, :, j].contiguous() for j in range(n0, wl.n)]
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
    ts = sorted(ev[j].elapsed_time(ev[j + 1]) for j in range(dsteps - 4))
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
    jj = torch.arange(wl.n, device="cuda")
    att = ((mk_t & gu[:, :, None]) != 0) | (jj[None, None, :] > wl.n - 1 - wl.window)
    unique_rows = int(att.sum().item())
    elem = 2 if wl.dtype in ("bf16", "f16") else 4
    dec_bytes = 2.0 * unique_rows * wl.d * elem
    per_head_rows = int(drp.to(torch.int64).sum().item())
    res = {
        "workload": wl.name,
        "what": "focus_decode_step at context n (route + append + attention + merge), median of %d steps" % (dsteps - 4),
        "ms_per_step": t_dec, "tokens_per_s": wl.B / (t_dec * 1e-3),
        "ms_per_token_graph_loop": t_dec_graph,      # three input copies + one graph replay per token, enqueued back to back
        "attended_keys_all_heads": per_head_rows,
        "roofline": {"bound": "hbm", "kernel": "decode_attn (whole step timed)", "achieved": dec_bytes / (t_dec * 1e-3) / 1e9,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": dec_bytes / (t_dec * 1e-3) / 1e9 / HBM_PEAK_GBS,
                     "traffic": measured_traffic("decode_step", wl.name),
                     "note": "algorithmic bytes = K and V rows of the keys at least one query head of the KV head "
                             "attends, read once (%d rows, %.1f MB); per-head reads would be %.1f MB"
                             % (unique_rows, dec_bytes / 1e6, 2.0 * per_head_rows * wl.d * elem / 1e6)},
    }
    del state, kc, vc
    return res


def leg_router(torch, focus, workloads, r, steps):
    """The paper's own front-end: one routing per token from the layer's hidden state (Sec. 2), then the same
    bucketing and attention on the routed membership.  Leaves the workspace holding the ROUTED membership."""
    wl, i, p, ws = r.wl, r.inp, r.p, r.ws
    q, k, v = i["q"], i["k"], i["v"]
    causal_pairs = wl.B * wl.Hq * (wl.n * (wl.n + 1) // 2)
    rin = workloads.make_router_inputs(wl, "cuda")
    dm, dg = rin["hidden"].shape[-1], rin["w_g"].shape[1]
    tmasks = torch.empty((wl.B, wl.n), dtype=torch.int32, device="cuda")
    rp10 = focus.make_route_params(wl.B, wl.n, dm, dg, wl.K, wl.topk, dtype=wl.dtype, sinkhorn_iters=10, tau=0.1)
    rp0 = focus.make_route_params(wl.B, wl.n, dm, dg, wl.K, wl.topk, dtype=wl.dtype, sinkhorn_iters=0, tau=0.1)
    rws = focus.alloc_route_workspace(rp10)
    rpairs = torch.empty((wl.B, wl.Hq, wl.n), dtype=torch.int32, device="cuda")
    out = torch.empty_like(q)
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
    t_proj, t_route, t_tok, t_rattn = (sum(e[j].elapsed_time(e[j + 1]) for e in ev) / rsteps for j in range(4))
    proj_flop = 2.0 * wl.B * wl.n * dm * dg
    return {
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


def leg_cpu_baseline(np, workloads, r, out_focus, cpu_seconds):
    """The CPU oracle on a bounded seeded sample of the same workload, on this machine's host cores.  The oracle
    computes its own membership from the input bytes: nothing it is fed comes from the device path."""
    from oracle import focus_oracle as fo
    wl, i = r.wl, r.inp
    pb = fo.Problem(wl.B, wl.Hq, wl.Hkv, wl.n, wl.d, wl.K, wl.topk, wl.window, causal=True,
                    dtype=wl.dtype, softcap=wl.softcap)
    qh, kh, vh = (workloads.to_host_bits(t) for t in (i["q"], i["k"], i["v"]))
    cents = i["centroids"].cpu().numpy()
    t0 = time.perf_counter()
    mq = fo.membership(pb, qh, cents, True)
    mk = fo.membership(pb, kh, cents, False)
    t_member = time.perf_counter() - t0
    note("cpu_baseline: oracle membership of every token in %.1f s" % t_member)
    rows_all = workloads.sample_rows(wl, min(wl.B * wl.Hq * wl.n, 1 << 20))
    # calibrate on a few rows, then size the sample to about cpu_seconds
    t0 = time.perf_counter()
    fo.attn_rows(pb, qh, kh, vh, mq, mk, rows=rows_all[:32])
    dt = time.perf_counter() - t0
    nrows = int(min(len(rows_all), max(32, 32 * cpu_seconds / max(dt, 1e-3))))
    t0 = time.perf_counter()
    o_ref, _, pr = fo.attn_rows(pb, qh, kh, vh, mq, mk, rows=rows_all[:nrows])
    dt = time.perf_counter() - t0
    sample_flop = 4.0 * wl.d * float(pr.sum())
    rr = rows_all[:nrows]
    got = out_focus[rr[:, 0], rr[:, 1], rr[:, 2]].float().cpu().numpy().astype(np.float64)
    return {
        "value": sample_flop / dt / 1e12,
        "unit": "TFLOP/s",
        "cores": fo.num_threads(),
        "kind": "oracle",
        "sample": "%d seeded query rows (all heads) of %s, attention rows only (4*d FLOP per allowed pair of the "
                  "sampled rows), %.1f s; oracle membership of all tokens before it: %.1f s, not counted"
                  % (nrows, wl.name, dt, t_member),
        "max_abs_err_vs_gpu": float(np.abs(got - o_ref).max()),
    }


def quick_variant(torch, focus, workloads, w2, nrep):
    """A shape outside the five configurations through the same step (assign + attention)."""
    r = Runner(torch, focus, workloads, w2)
    allowed = r.count_pairs()
    ms, ms_assign, ms_attn = r.timed(nrep, 1)
    tf = 4.0 * w2.d * allowed / (ms_attn * 1e-3) / 1e12
    res = {"workload": describe(w2), "ms_per_step": ms, "ms_attn": ms_attn, "tokens_per_s": w2.B * w2.n / (ms * 1e-3),
           "useful_tflops_step": 4.0 * w2.d * allowed / (ms * 1e-3) / 1e12,
           "allowed_fraction": allowed / (w2.B * w2.Hq * (w2.n * (w2.n + 1) // 2)),
           "roofline": {"bound": "mfma", "kernel": "attn_mfma_kernel", "achieved": tf, "peak": BF16_MFMA_PEAK_TFLOPS,
                        "unit": "TFLOP/s", "frac": tf / BF16_MFMA_PEAK_TFLOPS, "traffic": None}}
    del r
    torch.cuda.empty_cache()
    return res


# ------------------------------------------------------------------------------------------ sweeps (tables)
def sweep_lengths(torch, focus, workloads, args):
    """Speed-up of the Focus mask over dense causal attention as the sequence grows: the shape of the paper's
    wall-clock table (Sec. 3.6): K = 4 with top-2 and K = 8 with hard assignment, 1K to 1M tokens; 32 query heads
    on 8 KV heads, d = 128, bf16, N(0,1) inputs, one sequence.  Dense = the same kernel with window = n."""
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
        gen = torch.Generator(device="cuda").manual_seed(3003 + K)
        c = torch.randn((Hkv, K, d), generator=gen, device="cuda", dtype=torch.float32).double()
        return (c / c.norm(dim=-1, keepdim=True)).float().contiguous()

    base = workloads.CONFIGS["cfg3"]
    rows = []
    n = args.min_n
    while n <= args.max_n:
        wl0 = base.scaled(n=n, window=min(args.sweep_window, n))
        inp = workloads.make_inputs(wl0, "cuda")
        q, k, v = inp["q"], inp["k"], inp["v"]
        out = torch.empty_like(q)
        reps = max(1, min(20, (1 << 17) // n))
        point = {"n": n}
        for (K, topk) in ((4, 2), (8, 1), (0, 0)):           # (0, 0): dense
            if K:
                cents = unit_centroids(wl0.Hkv, K, wl0.d)
                p = focus.make_params(wl0.B, wl0.Hq, wl0.Hkv, n, wl0.d, K, topk, wl0.window, dtype=wl0.dtype)
            else:
                cents = inp["centroids"]
                p = focus.make_params(wl0.B, wl0.Hq, wl0.Hkv, n, wl0.d, 4, 2, n, dtype=wl0.dtype)
            ws = focus.alloc_workspace(p)
            rp = torch.empty((wl0.B, wl0.Hq, n), dtype=torch.int32, device="cuda")
            t_assign = timed(lambda: focus.focus_assign(p, q, k, cents, ws), max(1, reps))
            focus.focus_attn_fwd(p, q, k, v, ws, out, None, rp)
            pairs = int(rp.to(torch.int64).sum().item())
            t_attn = timed(lambda: focus.focus_attn_fwd(p, q, k, v, ws, out, None, None), reps)
            key = "dense" if not K else "K%d_top%d" % (K, topk)
            point[key] = {"ms_assign": t_assign, "ms_attn": t_attn, "allowed_pairs": pairs,
                          "tflops": 4.0 * wl0.d * pairs / (t_attn * 1e-3) / 1e12}
            del ws, rp
        for key in ("K4_top2", "K8_top1"):
            point[key]["speedup_vs_dense_attn"] = point["dense"]["ms_attn"] / point[key]["ms_attn"]
            point[key]["speedup_vs_dense_step"] = (point["dense"]["ms_attn"] + point["dense"]["ms_assign"]) / (
                point[key]["ms_attn"] + point[key]["ms_assign"])
            point[key]["allowed_fraction"] = point[key]["allowed_pairs"] / point["dense"]["allowed_pairs"]
        print(json.dumps(point), flush=True)
        rows.append(point)
        del inp, q, k, v, out
        torch.cuda.empty_cache()
        n *= 4
    print("%9s | %10s | %30s | %30s" % ("n", "dense ms", "K=4 top-2: ms, x attn, x step, frac", "K=8 top-1: ms, x attn, x step, frac"))
    for r in rows:
        a, b = r["K4_top2"], r["K8_top1"]
        print("%9d | %10.3f | %9.3f %5.2fx %5.2fx %5.1f%% | %9.3f %5.2fx %5.2fx %5.1f%%" % (
            r["n"], r["dense"]["ms_attn"], a["ms_attn"], a["speedup_vs_dense_attn"], a["speedup_vs_dense_step"],
            100 * a["allowed_fraction"], b["ms_attn"], b["speedup_vs_dense_attn"], b["speedup_vs_dense_step"],
            100 * b["allowed_fraction"]))


def sweep_decode(torch, focus, workloads, args):
    """One generated token against n cached tokens, 4K to 1M: median focus_decode_step time, the K and V rows the
    step has to read and the rate at which it reads them (K = 4 top-2 and K = 8 top-1)."""
    base = workloads.CONFIGS["cfg3"]
    steps = 24
    print("%9s | %28s | %28s" % ("n", "K=4 top-2: us, rows, TB/s", "K=8 top-1: us, rows, TB/s"))
    n = max(args.min_n, 4096)
    while n <= args.max_n:
        wl0 = base.scaled(n=n, window=min(args.sweep_window, n))
        inp = workloads.make_inputs(wl0, "cuda")
        cells = []
        for (K, topk) in ((4, 2), (8, 1)):
            gen = torch.Generator(device="cuda").manual_seed(3003 + K)
            c = torch.randn((wl0.Hkv, K, wl0.d), generator=gen, device="cuda", dtype=torch.float32).double()
            cents = (c / c.norm(dim=-1, keepdim=True)).float().contiguous()
            p = focus.make_params(wl0.B, wl0.Hq, wl0.Hkv, n, wl0.d, K, topk, wl0.window, dtype=wl0.dtype)
            state = focus.alloc_decode_state(p)
            kc, vc = inp["k"].clone(), inp["v"].clone()
            n0 = n - steps
            focus.focus_decode_prefill(p, n0, kc, cents, state)
            qs = [inp["q"][:, :, j].contiguous() for j in range(n0, n)]
            ks = [inp["k"][:, :, j].contiguous() for j in range(n0, n)]
            vs = [inp["v"][:, :, j].contiguous() for j in range(n0, n)]
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
            G = wl0.Hq // wl0.Hkv
            gu = torch.zeros((wl0.B, wl0.Hkv), dtype=torch.int32, device="cuda")
            for g_ in range(G):
                gu |= views["mq"].view(wl0.B, wl0.Hkv, G)[:, :, g_]
            jj = torch.arange(n, device="cuda")
            att = ((views["mk"] & gu[:, :, None]) != 0) | (jj[None, None, :] > n - 1 - wl0.window)
            nrows = int(att.sum().item())
            nbytes = 2.0 * nrows * wl0.d * 2
            cells.append("%9.1f %10d %6.2f" % (1e3 * t, nrows, nbytes / (t * 1e-3) / 1e12))
            del state, kc, vc
        print("%9d | %28s | %28s" % (n, cells[0], cells[1]), flush=True)
        del inp
        torch.cuda.empty_cache()
        n *= 4


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="cfg5", help="headline workload (default cfg5, the largest configuration)")
    ap.add_argument("--legs-workload", default="cfg3",
                    help="workload of the side legs (two-call, router, soft gate, other head dims and types)")
    ap.add_argument("--only-headline", action="store_true",
                    help="the headline step and its dense comparator only (profiling runs; add --no-dense to drop the latter)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--no-others", action="store_true", help="skip the other configurations")
    ap.add_argument("--no-legs", action="store_true", help="skip the side legs")
    ap.add_argument("--cpu-seconds", type=float, default=15.0)
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one plain device copy of q (known size) so a counter run can be calibrated")
    ap.add_argument("--no-clock", action="store_true", help="do not sample the core clock with rocm-smi during the steps")
    ap.add_argument("--zero-inputs", action="store_true",
                    help="zero q, k, v of the headline workload: the same launches without switching activity in the "
                         "multipliers (what the chip's clock does to the timings; every token then ties into one class)")
    ap.add_argument("--lib", default=None,
                    help="time another build of the library (a timing-only ablation build, build.py --ablate): headline "
                         "step only, no parity-dependent legs; the line says so and its numbers are not results")
    ap.add_argument("--sweep", choices=["lengths", "decode"], default=None)
    ap.add_argument("--sweep-window", type=int, default=1024)
    ap.add_argument("--min-n", type=int, default=1 << 10)
    ap.add_argument("--max-n", type=int, default=1 << 20)
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
    if args.lib:
        focus.LIB_PATH = os.path.abspath(args.lib)
        args.only_headline = True
        args.no_cpu_baseline = True
    if args.sweep == "lengths":
        return sweep_lengths(torch, focus, workloads, args)
    if args.sweep == "decode":
        return sweep_decode(torch, focus, workloads, args)

    wl = workloads.CONFIGS[args.workload]
    steps = args.steps if args.steps is not None else DEFAULT_STEPS[wl.name][0]
    warmup = args.warmup if args.warmup is not None else DEFAULT_STEPS[wl.name][1]
    only = args.only_headline
    t_start = time.perf_counter()

    if args.calib_copy:
        cal = torch.empty((64 << 20,), dtype=torch.float32, device="cuda")      # 256 MiB read + 256 MiB written
        cal2 = cal.clone()
        torch.cuda.synchronize()
        del cal, cal2
    dense_steps = 0 if args.no_dense else max(1 if only else 2, min(steps // 4, 5))
    clock = None if args.no_clock else ClockSampler()
    if clock:
        clock.__enter__()
    head, r = measure(torch, focus, workloads, wl, steps, warmup, dense_steps, keep=True, clock=clock,
                      zero_inputs=args.zero_inputs)
    if clock:
        clock.__exit__()
    out_focus = r.out
    half = wl.dtype in ("bf16", "f16")
    result = {
        "metric": "useful TFLOP/s of Focus attention fwd (assign + attention, 4*d FLOP per allowed pair)",
        "value": head["useful_tflops_step"],
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": wl.dtype,
        "data": "synthetic",
        "config": {"workload": describe(wl) + (" (q, k, v zeroed)" if args.zero_inputs else "")},
        "tokens_per_s": head["tokens_per_s"],
        "ms_assign": head["ms_assign"],
        "ms_attn": head["ms_attn"],
        "allowed_pairs": head["allowed_pairs"],
        "allowed_fraction": head["allowed_fraction"],
        "largest_group_fraction": head["largest_group_fraction"],
        "sclk_mhz": head["sclk_mhz"],
        "pct_of_peak_step": 100.0 * head["useful_tflops_step"] / head["roofline"]["peak"],
        "roofline": head["roofline"],
        "roofline_assign": head["roofline_assign"],
        "paper_context": PAPER_CONTEXT,
    }
    for key in ("dense", "speedup_vs_dense_attn", "speedup_vs_dense_step"):
        if key in head:
            result[key] = head[key]
    if args.lib:
        result["library"] = args.lib
        result["note"] = "timing of another build of the library (loop ablation): not a result of the method"
    if half and not only:
        leg_mfma_probe(result, head["roofline"]["achieved"])

    if not args.no_cpu_baseline and not only:
        result["cpu_baseline"] = leg_cpu_baseline(np, workloads, r, out_focus, args.cpu_seconds)

    if not args.no_legs and not only and wl.window < wl.n and wl.n > 131072:
        # at the headline's own size only the cheap or essential legs: two-call on the same membership, one decode step
        note("two-call comparator and decode step at", wl.name)
        result["two_call_headline"] = leg_two_call(torch, focus, r, head["ms_attn"], out_focus, 2)
        result["decode_headline"] = leg_decode(torch, focus, r)
    del r, out_focus
    torch.cuda.empty_cache()

    # every other configuration through the same step, each with its own rooflines
    if not args.no_others and not only:
        others = {}
        for name in ("cfg1", "cfg2", "cfg3", "cfg4a", "cfg4b", "cfg5"):
            if name == wl.name:
                continue
            if name == "cfg5" and wl.name != "cfg5":
                continue                                  # the 1M-token configuration is measured as a headline only
            w2 = workloads.CONFIGS[name]
            s2, u2 = DEFAULT_STEPS[name]
            others[name] = measure(torch, focus, workloads, w2, s2, u2, 0 if args.no_dense else 2)
        result["other_workloads"] = others

    # the side legs on a mid-size configuration
    if not args.no_legs and not only:
        lw = workloads.CONFIGS[args.legs_workload]
        note("side legs on", describe(lw))
        lsteps = DEFAULT_STEPS[lw.name][0]
        lres, lr = measure(torch, focus, workloads, lw, lsteps, 3, 0, keep=True)
        lhalf = lw.dtype in ("bf16", "f16")
        if lhalf:
            leg_outside_numbers(torch, lr, result, lsteps)
        if lw.window < lw.n:
            result["two_call"] = leg_two_call(torch, focus, lr, lres["ms_attn"], lr.out.clone(), max(2, lsteps // 2))
        if lw.softcap == 0.0 and not (lw.d == 256 and lhalf):
            result["soft_gate"] = leg_soft_gate(torch, focus, lr, lsteps)
        result["decode"] = leg_decode(torch, focus, lr)
        result["router_path"] = leg_router(torch, focus, workloads, lr, lsteps)
        del lr
        torch.cuda.empty_cache()
        if lw.name == "cfg3":
            from dataclasses import replace
            wider = {}
            for tag, kw in (("cfg3_f16", dict(dtype="f16")), ("cfg3_d256", dict(d=256, Hq=16, Hkv=4)),
                            ("cfg3_d96", dict(d=96, Hq=40, Hkv=8)), ("cfg3_d80", dict(d=80, Hq=48, Hkv=8)),
                            ("cfg3_d64", dict(d=64, Hq=64, Hkv=16))):
                wider[tag] = quick_variant(torch, focus, workloads, replace(lw, name=tag, **kw), 5)
            result["wider_variants"] = wider
    result["bench_wall_s"] = time.perf_counter() - t_start
    print(json.dumps(result))


if __name__ == "__main__":
    main()
