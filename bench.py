#!/usr/bin/env python3
"""Benchmark of the tensor-network linear forward on one MI355X.

A step is one tn_linear_forward of the TT-factorised query projection
(in 5120 = 8x10x8x8, out 8192 = 8x16x8x8, TT ranks 64, bf16) over 8192 tokens
already resident in HBM. Prints one JSON line: whole-job tokens/s, the roofline
figures of the dominant contraction kernel measured with HIP events on the
launch stream, the 1-, 8- and 64-token latencies, and the CPU oracle timed on a
bounded sample of the same workload (a baseline only).

With no --workload / --custom the same line also carries, under "configs", one
record each for the Tucker up_proj, the tensor-ring down_proj, a dense
5120 -> 8192 matrix and the mixed 64-layer stack (448 matrices), every one with
its own 8192-, 64- and 1-token figures, roofline and cpu_baseline.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "TN-linear tokens/s at 8192-tok prefill & 1-tok decode; % of MFMA/HBM peak"
PEAK_BF16_TFLOPS = 2500.0      # dense bf16 MFMA peak of MI355X
PEAK_HBM_GBS = 8000.0
RIDGE = PEAK_BF16_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9)
PAPER_CONTEXT = ("paper reports ~40 -> ~50 -> ~75 tokens/s end-to-end decode on Qwen3-32B, 8K context, "
                 "1x A100 80GB (whole model with healing and speculative decoding; not this kernel)")


def blas_threads():
    try:
        from threadpoolctl import threadpool_info
        return int(max([p.get("num_threads", 1) for p in threadpool_info()] or [1]))
    except Exception:
        return int(os.cpu_count() or 1)


def cpu_baseline(spec, tensors, sample_tokens, transpose=False, x_used=None, y_gpu=None):
    """The fp64 oracle as it stands: rebuild dense W once, multiply a sample of tokens. When the rows the GPU
    consumed (x_used, float64) and what it produced for them (y_gpu) are given, the oracle's product of those
    very rows is also compared with the GPU's and the error reported."""
    import numpy as np
    import oracle as O
    import workloads as wl
    x = wl.make_x(spec, sample_tokens, 1, instance=7) if x_used is None else x_used[:sample_tokens]
    if transpose and x_used is None:
        x = np.random.Generator(np.random.PCG64([wl.SEED_BASE, 7, 1])).standard_normal((sample_tokens, spec.M))
    t0 = time.perf_counter()
    w = O.dense_weight(spec.format, tensors, len(spec.out_modes))
    t1 = time.perf_counter()
    y = O.apply_linear(w.T if transpose else w, x)
    t2 = time.perf_counter()
    n = x.shape[0]
    out = {
        "value": n / (t2 - t0),
        "unit": "tokens/s",
        "cores": blas_threads(),
        "kind": "oracle",
        "sample": f"dense rebuild of W once ({t1 - t0:.2f} s) + fp64 multiply of {n} tokens "
                  f"({t2 - t1:.2f} s); multiply-only {n / (t2 - t1):.0f} tokens/s",
    }
    if y_gpu is not None:
        out["gpu_rel_max_err_on_these_rows"] = O.rel_max_err(y_gpu[:n], y)
    return out


def measured_traffic(workload, flags, tokens, fused):
    """HBM-side bytes per launch of the dominant kernel of workloads 1 to 3 and of the dense matrix (4) at their default settings, as
    measured in separate rocprofv3 counter runs (FETCH_SIZE, WRITE_SIZE, calibrated on a copy kernel) and
    recorded in profiles/: counters cannot be read from inside this process. Returns (bytes, file) or (None, None)."""
    if flags or tokens != 8192 or fused != (workload in (1, 3)):
        return None, None
    name, key = {1: ("tt_q_proj_prefill8192_hbm_traffic.txt", "pair"),
                 2: ("tucker_up_proj_prefill8192_hbm_traffic.txt", "core"),
                 3: ("tr_down_proj_prefill8192_hbm_traffic.txt", "kronsum"),
                 4: ("dense_q_proj_prefill8192_hbm_traffic.txt", "gemm")}.get(workload, (None, None))
    if name is None:
        return None, None
    try:
        m = re.search(rf"TRAFFIC_BYTES_PER_LAUNCH {key} = (\d+)", open(os.path.join(ROOT, "profiles", name)).read())
        return (int(m.group(1)), "profiles/" + name) if m else (None, None)
    except OSError:
        return None, None


class LayerBench:
    """One layer resident on the GPU and the measurements taken on it."""

    def __init__(self, spec, config_id, tokens, flags=0, workspace_mb=0, transpose=False):
        import numpy as np
        import torch
        import workloads as wl
        import paper_2602_01613_amd as tn
        self.tn, self.torch, self.wl = tn, torch, wl
        self.spec, self.tokens, self.flags, self.transpose = spec, tokens, flags, transpose
        self.tensors = wl.make_tensors(spec, config_id)
        x64 = wl.make_x(spec, tokens, config_id)
        if transpose:
            x64 = np.random.Generator(np.random.PCG64([wl.SEED_BASE, config_id, 99])).standard_normal((tokens, spec.M))
        self.tdt = torch.bfloat16 if spec.dtype == "bf16" else torch.float32
        self.code = tn.TN_DTYPE_BF16 if spec.dtype == "bf16" else tn.TN_DTYPE_F32
        self.esize = 2 if spec.dtype == "bf16" else 4
        self.dev = [torch.from_numpy(t).to(torch.float32).to(self.tdt).cuda() for t in self.tensors]
        self.x = torch.from_numpy(x64).to(torch.float32).to(self.tdt).cuda()
        self.x_head = self.x[:256].to(torch.float64).cpu().numpy()       # what the GPU consumed, for the oracle
        del x64
        self.layer = tn.TNLinear(spec.format, self.code, spec.out_modes, spec.in_modes, spec.ranks, self.dev,
                                 tokens, workspace_mb << 20, flags=flags)
        self.y = torch.empty((tokens, self.layer.M), dtype=self.tdt, device="cuda")
        self.lazy_min = self.layer.query(tn.TN_QUERY_LAZY_MIN_TOKENS)

    def close(self):
        self.layer.close()

    def plan_view(self, t):
        """Steps, FLOPs and algorithmic bytes of the plan a call of t tokens executes. Calls of at least lazy_min
        tokens (0: never) run on a plan whose merged tensors are rebuilt in the workspace per call: its steps, not
        the compact plan's, are the work such a call does."""
        tn, spec, layer, esize = self.tn, self.spec, self.layer, self.esize
        if self.lazy_min and t >= self.lazy_min:
            pq = lambda what: tn.plan_query(spec.format, self.code, spec.out_modes, spec.in_modes, spec.ranks, what,
                                            flags=self.flags | tn.TN_FLAG_MERGE_HALVES)
            qq = lambda s, f: 20 if f == 5 else pq(tn.TN_QUERY_STEP_BASE + 10 * s + f)
            n = pq(tn.TN_QUERY_NUM_STEPS)
            fl = pq(tn.TN_QUERY_FLOPS_PER_TOKEN)
        else:
            qq = lambda s, f: layer.query(tn.TN_QUERY_STEP_BASE + 10 * s + f)
            n = layer.query(tn.TN_QUERY_NUM_STEPS)
            fl = layer.query(tn.TN_QUERY_FLOPS_PER_TOKEN)
        return {"n_steps": n, "flops_tok": fl, "q": qq,
                "step_flops": [qq(s, 3) for s in range(n)],
                # algorithmic bytes of a step per token: read its [rows, K] input, write its [rows, cols]
                # output (bf16), plus its packed parameter tensor once per launch
                "step_io_bytes": [esize * qq(s, 0) * (qq(s, 1) + qq(s, 2)) for s in range(n)],
                "step_param_bytes": [esize * qq(s, 1) * qq(s, 2) for s in range(n)]}

    def prefill(self, steps, warmup, workload_id=None):
        """First a loop of K steps in which the library brackets every kernel launch with a HIP event pair on the stream
        the kernels run on (the per-kernel durations the roofline entry uses); then W untimed steps and exactly K
        timed steps between two synchronisations, with profiling off: nothing but kernel launches inside the timed
        region. A forward that is a single launch takes its roofline duration from the timed region itself."""
        torch, tn, layer, tokens, esize = self.torch, self.tn, self.layer, self.tokens, self.esize
        x, y = self.x, self.y
        stream = torch.cuda.current_stream()
        view = self.plan_view(tokens)
        flops_tok, n_steps, q = view["flops_tok"], view["n_steps"], view["q"]
        step_flops, step_io_bytes, step_param_bytes = view["step_flops"], view["step_io_bytes"], view["step_param_bytes"]
        # per-kernel durations first: the same steps with events around every launch
        layer.profile(True)
        for _ in range(steps):
            layer.forward(x, out=y)
        torch.cuda.synchronize()
        layer.profile(False)
        # the timed region
        for _ in range(warmup):
            layer.forward(x, out=y)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record(stream)
        for _ in range(steps):
            layer.forward(x, out=y)
        e1.record(stream)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        ms_events = e0.elapsed_time(e1) / steps
        tokens_per_s = tokens * steps / wall
        self.y_head = y[:256].to(torch.float64).cpu().numpy()
        reads = [layer.profile_read(s) for s in range(n_steps)]
        per_step = []
        for s in range(n_steps):
            ms, launches = reads[s]
            if launches == 0:            # ran inside the previous step's launch
                per_step.append({"step": s, "rows_per_token": q(s, 0), "K": q(s, 1), "cols": q(s, 2),
                                 "ms_per_forward": 0.0, "launches_per_forward": 0, "fused_into_previous": True})
                continue
            sec = ms * 1e-3
            # steps without launches of their own ran inside this step's launch: it reads this step's input
            # and writes the last of those steps' output; the intermediates never reach memory
            last = s
            while last + 1 < n_steps and reads[last + 1][1] == 0:
                last += 1
            fused = last > s
            flops_s = sum(step_flops[s:last + 1])
            io_s = esize * (q(s, 0) * q(s, 1) + q(last, 0) * q(last, 2)) if fused else step_io_bytes[s]
            par_s = sum(step_param_bytes[s:last + 1])
            nbytes = (io_s * tokens + par_s * (launches // steps)) * steps
            per_step.append({
                "step": s, "rows_per_token": q(s, 0), "K": q(s, 1), "cols": q(s, 2), "kernel_variant": q(s, 5),
                "ms_per_forward": ms / steps, "launches_per_forward": launches // steps,
                "avg_launch_us": 1e3 * ms / max(1, launches),
                "tflops": flops_s * tokens * steps / sec / 1e12 if sec > 0 else 0.0,
                "algorithmic_GBps": nbytes / sec / 1e9 if sec > 0 else 0.0,
                "algorithmic_bytes_per_forward": nbytes // steps,
                "flop_per_byte": flops_s / io_s,
                "fused_with_next": fused, "steps_in_launch": last - s + 1})
        dom = max(range(n_steps), key=lambda s: per_step[s]["ms_per_forward"])
        d = per_step[dom]
        if sum(p["launches_per_forward"] for p in per_step) == 1:
            # one launch per forward: the K timed steps are K back-to-back launches of this kernel, and the events
            # around them give its average duration (gaps between launches included) without per-launch events
            scale = d["ms_per_forward"] / ms_events
            d["avg_launch_us_profiled_loop"] = d["avg_launch_us"]
            d["avg_launch_us"] = 1e3 * ms_events
            d["ms_per_forward"] = ms_events
            d["tflops"] *= scale
            d["algorithmic_GBps"] *= scale
        if d["flop_per_byte"] >= RIDGE:
            roof = {"bound": "mfma", "achieved": d["tflops"], "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s"}
        else:
            roof = {"bound": "hbm", "achieved": d["algorithmic_GBps"], "peak": PEAK_HBM_GBS, "unit": "GB/s"}
        roof["frac"] = roof["achieved"] / roof["peak"]
        roof["traffic"], src = measured_traffic(workload_id, self.flags, tokens, d["fused_with_next"])
        if src:
            roof["traffic_source"] = src + " (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this workload, per launch)"
        if d["fused_with_next"]:
            n_in = d["steps_in_launch"]
            shapes = ", then ".join(f"rows {q(j, 0)} x K {q(j, 1)} x cols {q(j, 2)}" for j in range(dom, dom + n_in))
            roof["kernel"] = (f"contraction steps {dom}..{dom + n_in - 1} in one launch ({shapes} per token; intermediates "
                              f"on chip), {d['flop_per_byte']:.0f} FLOP/B against a ridge of {RIDGE:.0f}")
        else:
            roof["kernel"] = (f"contraction step {dom}: rows {q(dom, 0)} x K {q(dom, 1)} x cols {q(dom, 2)} per token, "
                              f"{d['flop_per_byte']:.0f} FLOP/B against a ridge of {RIDGE:.0f}")
        roof["avg_launch_us"] = d["avg_launch_us"]
        roof["launches_per_forward"] = d["launches_per_forward"]
        roof["also_tflops"] = d["tflops"]
        roof["also_GBps"] = d["algorithmic_GBps"]
        return {"tokens": tokens, "tokens_per_s": tokens_per_s, "ms_per_step": 1e3 * wall / steps,
                "gpu_ms_per_step_events": ms_events, "flops_per_token": flops_tok,
                "tflops_factorised": flops_tok * tokens_per_s / 1e12,
                "whole_chain_frac_of_mfma_peak": flops_tok * tokens_per_s / 1e12 / PEAK_BF16_TFLOPS,
                "roofline": roof, "per_step": per_step}

    def small_call(self, t, reps=200, detail=True):
        """Latency of calls of t tokens: back-to-back eager calls on one stream (profiling off), then the
        per-kernel durations of the same calls from the library's HIP events in a separate loop."""
        torch, layer = self.torch, self.layer
        t = min(t, self.tokens)
        v = self.plan_view(t)
        n_steps, flops_tok = v["n_steps"], v["flops_tok"]
        xt = self.x[:t].contiguous()
        yt = torch.empty((t, layer.M), dtype=self.tdt, device="cuda")
        for _ in range(20):
            layer.forward(xt, out=yt)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            layer.forward(xt, out=yt)
        torch.cuda.synchronize()
        us = (time.perf_counter() - t0) / reps * 1e6
        out = {"tokens": t, "us_per_call": us, "tokens_per_s": t * 1e6 / us, "tflops": flops_tok * t / us / 1e6,
               "frac_of_mfma_peak": flops_tok * t / us / 1e6 / PEAK_BF16_TFLOPS}
        if not detail:
            return out
        layer.profile(True)
        for _ in range(50):
            layer.forward(xt, out=yt)
        torch.cuda.synchronize()
        layer.profile(False)
        steps = []
        for s in range(n_steps):
            ms, launches = layer.profile_read(s)
            k_us = 1e3 * ms / max(1, launches)
            nbytes = v["step_io_bytes"][s] * t + v["step_param_bytes"][s]
            if launches == 0:        # runs inside the previous step's fused launch
                steps.append({"step": s, "kernel_us": 0.0, "fused_into_previous": True})
                continue
            steps.append({"step": s, "kernel_us": k_us, "launches": launches // 50, "GBps": nbytes / k_us / 1e3,
                          "param_GBps": v["step_param_bytes"][s] / k_us / 1e3,
                          "tflops": v["step_flops"][s] * t / k_us / 1e6})
        out["sum_kernel_us"] = sum(p["kernel_us"] * p.get("launches", 0) for p in steps)
        out["per_step"] = steps
        return out

    def decode_graph(self, t, instances):
        """Steady-state decode: `instances` distinct copies of the layer (own packed tensors, so the
        parameter stream cannot sit in the 256 MB last-level cache from one call to the next when their
        sum exceeds it) run back to back inside one captured HIP graph, replayed many times; time per
        layer call. This takes the host's launch cost out of the figure, which a serving loop does by
        capturing its decode step the same way."""
        torch, tn, spec, layer = self.torch, self.tn, self.spec, self.layer
        copies = [layer]
        for _ in range(instances - 1):
            copies.append(tn.TNLinear(spec.format, self.code, spec.out_modes, spec.in_modes, spec.ranks, self.dev,
                                      max(t, 1), flags=self.flags))
        xt = self.x[:t].contiguous()
        yt = torch.empty((t, layer.M), dtype=self.tdt, device="cuda")
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for c in copies:
                c.forward(xt, out=yt)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for c in copies:
                c.forward(xt, out=yt)
        for _ in range(5):
            graph.replay()
        torch.cuda.synchronize()
        reps = 50
        t0 = time.perf_counter()
        for _ in range(reps):
            graph.replay()
        torch.cuda.synchronize()
        us = (time.perf_counter() - t0) / reps / instances * 1e6
        # every replay must give what the eager call gives
        y_eager = torch.empty_like(yt)
        copies[-1].forward(xt, out=y_eager)
        torch.cuda.synchronize()
        ok = bool(torch.equal(y_eager, yt))
        packed = layer.query(tn.TN_QUERY_PACKED_BYTES)
        params = spec.n_params * self.esize
        for c in copies[1:]:
            c.close()
        flops = self.plan_view(t)["flops_tok"] * t
        out = {"tokens": t, "instances": instances, "us_per_layer_call": us, "tokens_per_s": t * 1e6 / us,
               "param_GBps": packed / us / 1e3, "caller_param_GBps": params / us / 1e3,
               "tflops": flops / us / 1e6, "param_MB_all_instances": packed * instances / 1e6,
               "replay_equals_eager": ok}
        # which roofline binds a call this small: the parameter stream or the matrix cores
        if flops / max(1, packed) < RIDGE:
            out["roofline"] = {"bound": "hbm", "achieved": packed / us / 1e3, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                               "frac": packed / us / 1e3 / PEAK_HBM_GBS,
                               "note": "packed parameter bytes per call / time per call; the copies' parameters "
                                       f"total {packed * instances / 1e6:.0f} MB per replay"}
        else:
            out["roofline"] = {"bound": "mfma", "achieved": flops / us / 1e6, "peak": PEAK_BF16_TFLOPS,
                               "unit": "TFLOP/s", "frac": flops / us / 1e6 / PEAK_BF16_TFLOPS,
                               "note": "parameters are a few MB: the HBM bound lies below the MFMA bound and "
                                       "both below launch latency"}
        return out


def layer_record(spec, config_id, args, flags, steps, warmup, workload_id=None, cpu_tokens=1024, detail=False):
    """All figures of one single-layer workload: 8192-token prefill, 64-, 8- and 1-token calls, the decode graph."""
    import workloads as wl
    lb = LayerBench(spec, config_id, args.tokens, flags=flags, workspace_mb=args.workspace_mb,
                    transpose=args.transpose and detail)
    # small calls first: by the time the prefill steps are timed the GPU has been awake for some tens of
    # milliseconds of light load
    dec1 = lb.small_call(1, detail=detail)
    dec1_graph = lb.decode_graph(1, args.graph_instances)
    dec8 = lb.small_call(8, detail=detail)          # the size a speculative-decoding verifier sends (Section 3.6)
    dec64 = lb.small_call(64, detail=detail)
    pre = lb.prefill(steps, warmup, workload_id)
    rec = {
        "workload": f"{spec.name}: {wl.FORMAT_NAMES[spec.format]} in {spec.N}={'x'.join(map(str, spec.in_modes))} "
                    f"out {spec.M}={'x'.join(map(str, spec.out_modes))} ranks {list(spec.ranks)}, "
                    f"{spec.dtype} storage, fp32 accumulate",
        "steps": steps, "warmup": warmup,
        "prefill": pre if detail else {k: v for k, v in pre.items() if k != "per_step"},
        "roofline": pre["roofline"],
        "decode_1tok": dec1,
        "decode_1tok_graph": dec1_graph,
        "verify_8tok": dec8,
        "decode_64tok": dec64,
        "create_time_merges": lb.layer.query(lb.tn.TN_QUERY_NUM_MERGES),
        "lazy_merge_from_tokens": lb.lazy_min,
        "chunk_tokens": lb.layer.query(lb.tn.TN_QUERY_CHUNK_TOKENS),
    }
    keep = (lb.spec, lb.tensors, lb.x_head, lb.y_head)
    lb.close()
    return rec, keep


def pair_record(spec, config_id, args, instances=8):
    """Two layers of one shape applied to the same activations (the gate and up projections of an MLP block):
    tn_linear_forward2 against two tn_linear_forward calls, as a captured decode graph over `instances` distinct
    pairs (time per pair) and at 8192 tokens."""
    import torch
    import workloads as wl
    import paper_2602_01613_amd as tn
    ts = [wl.make_tensors(spec, config_id, instance=i) for i in range(2)]
    dev = [[torch.from_numpy(t).to(torch.float32).to(torch.bfloat16).cuda() for t in tt] for tt in ts]
    pairs = [(tn.TNLinear(spec.format, tn.TN_DTYPE_BF16, spec.out_modes, spec.in_modes, spec.ranks, dev[0], args.tokens),
              tn.TNLinear(spec.format, tn.TN_DTYPE_BF16, spec.out_modes, spec.in_modes, spec.ranks, dev[1], args.tokens))
             for _ in range(instances)]
    x = torch.from_numpy(wl.make_x(spec, args.tokens, config_id)).to(torch.float32).to(torch.bfloat16).cuda()
    out = {"workload": f"two {wl.FORMAT_NAMES[spec.format]} layers {spec.N}->{spec.M} ranks {list(spec.ranks)} on the same activations",
           "instances": instances}
    packed = 2 * pairs[0][0].query(tn.TN_QUERY_PACKED_BYTES)
    for t in (1, args.tokens):
        xt = x[:t].contiguous()
        ya = torch.empty((t, spec.M), dtype=torch.bfloat16, device="cuda")
        yb = torch.empty_like(ya)
        res = {}
        for mode in ("forward2", "separate"):
            def run():
                for a, b in (pairs if t == 1 else pairs[:1]):
                    if mode == "forward2":
                        tn.forward2(a, b, xt, ya, yb)
                    else:
                        a.forward(xt, out=ya)
                        b.forward(xt, out=yb)
            n_pairs = len(pairs) if t == 1 else 1
            if t == 1:
                side = torch.cuda.Stream()
                side.wait_stream(torch.cuda.current_stream())
                with torch.cuda.stream(side):
                    run()
                torch.cuda.synchronize()
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph, stream=side):
                    run()
                go, reps = graph.replay, 50
            else:
                go, reps = run, max(3, args.steps // 2)
            for _ in range(3):
                go()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                go()
            torch.cuda.synchronize()
            res[mode] = (time.perf_counter() - t0) / reps / n_pairs * 1e6
            res[mode + "_ya"] = ya.clone()
        rec = {"us_per_pair_forward2": res["forward2"], "us_per_pair_two_calls": res["separate"],
               "speedup": res["separate"] / res["forward2"], "same_bits": bool(torch.equal(res["forward2_ya"], res["separate_ya"]))}
        if t == 1:
            rec["param_GBps_forward2"] = packed / res["forward2"] / 1e3
            rec["frac_of_hbm_peak"] = packed / res["forward2"] / 1e3 / PEAK_HBM_GBS
        else:
            rec["tokens_per_s_forward2"] = t * 1e6 / res["forward2"]
        out["decode_1tok_graph" if t == 1 else f"prefill_{t}tok"] = rec
    for a, b in pairs:
        a.close()
        b.close()
    return out


def quant_record(spec, config_id, args):
    """A layer with 4-bit tensors (TN_FLAG_QUANT_MXFP4) at decode sizes: one-token calls as a captured graph over
    distinct copies and eight-token calls, reading the 4-bit stream, next to the same quantised layer made to
    multiply with its bf16 copies (TN_FLAG_NO_Q4_STREAM); both checked against the oracle applied to the
    dequantised tensors."""
    import oracle as O
    import paper_2602_01613_amd as tn
    out = {"workload": f"{spec.name} with 4-bit tensors (blocks of 32, power-of-two scale, E2M1)"}
    w_q = None
    for name, flags in (("stream_4bit", tn.TN_FLAG_QUANT_MXFP4), ("bf16_copies", tn.TN_FLAG_QUANT_MXFP4 | tn.TN_FLAG_NO_Q4_STREAM)):
        lb = LayerBench(spec, config_id, 64, flags=flags)
        g = lb.decode_graph(1, args.graph_instances)
        rec = {"decode_1tok_graph_us_per_layer": g["us_per_layer_call"], "replay_equals_eager": g["replay_equals_eager"],
               "verify_8tok_us": lb.small_call(8, detail=False)["us_per_call"],
               "stream_bytes": lb.layer.query(tn.TN_QUERY_QUANT_STREAM_BYTES)}
        if rec["stream_bytes"]:
            rec["stream_GBps"] = rec["stream_bytes"] / g["us_per_layer_call"] / 1e3
        if w_q is None:
            w_q = O.dense_weight(spec.format, O.mxfp4_dequantized(lb.tensors), len(spec.out_modes))
        x8 = lb.x[:8].contiguous()
        y8 = lb.layer.forward(x8).float().cpu().numpy().astype("float64")
        rec["rel_max_err_vs_oracle_8tok"] = O.rel_max_err(y8, O.apply_linear(w_q, x8.float().cpu().numpy().astype("float64")))
        out[name] = rec
        lb.close()
    out["speedup_1tok"] = out["bf16_copies"]["decode_1tok_graph_us_per_layer"] / out["stream_4bit"]["decode_1tok_graph_us_per_layer"]
    return out


def gradient_record(spec, config_id, tokens, reps=3):
    """tn_linear_param_gradients (gradients of a loss with respect to every parameter tensor, Section 3.4) on a
    trainable copy of the layer: tokens/s of one call (forward with saved intermediates + backward) and the FLOP/s of
    its executed contractions (per step: the forward product, the parameter gradient and, except for the first step,
    the input gradient)."""
    import torch
    import workloads as wl
    import paper_2602_01613_amd as tn
    ts = wl.make_tensors(spec, config_id)
    tdt = torch.bfloat16 if spec.dtype == "bf16" else torch.float32
    code = tn.TN_DTYPE_BF16 if spec.dtype == "bf16" else tn.TN_DTYPE_F32
    dev = [torch.from_numpy(t).to(torch.float32).to(tdt).cuda() for t in ts]
    layer = tn.TNLinear(spec.format, code, spec.out_modes, spec.in_modes, spec.ranks, dev, tokens, flags=tn.TN_FLAG_TRAINABLE)
    x = torch.from_numpy(wl.make_x(spec, tokens, config_id)).to(torch.float32).to(tdt).cuda()
    dy = torch.from_numpy(wl.make_x(wl.TNSpec(spec.format, spec.dtype, spec.in_modes, spec.out_modes, spec.ranks), tokens,
                                    config_id, instance=3)).to(torch.float32).to(tdt).cuda()
    grads = layer.param_gradients(x, dy)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        layer.param_gradients(x, dy, out=grads)
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t0) / reps
    n = layer.query(tn.TN_QUERY_NUM_STEPS)
    step_flops = [layer.query(tn.TN_QUERY_STEP_BASE + 10 * s + 3) for s in range(n)]
    flops = sum(step_flops[:-1]) + sum(step_flops) + sum(step_flops[1:])
    out = {"workload": f"{spec.name}: parameter gradients, {tokens} tokens, {n} steps (no create-time merges)",
           "tokens": tokens, "ms_per_call": 1e3 * sec, "tokens_per_s": tokens / sec,
           "flops_per_token": flops, "tflops": flops * tokens / sec / 1e12,
           "backward_chunk_tokens": layer.query(tn.TN_QUERY_BACKWARD_CHUNK_TOKENS),
           "backward_workspace_MB": layer.query(tn.TN_QUERY_BACKWARD_WORKSPACE_BYTES) / 1e6,
           "roofline": {"bound": "mfma", "achieved": flops * tokens / sec / 1e12, "peak": 2500.0, "unit": "TFLOP/s",
                        "frac": flops * tokens / sec / 1e12 / 2500.0,
                        "kernel": "whole call: forward and input-gradient steps on the MFMA step kernels, parameter-gradient "
                                  "contractions on grad_param_mfma_kernel (128 x 128 tiles; both operands transposed through LDS, "
                                  "loaded in 16-byte pieces where their layout allows) or, for tensors under 8 wide or not bf16, on "
                                  "plain fp32 FMA"}}
    layer.close()
    return out


def draw_on_device(spec, gen):
    """Parameter tensors of one stack matrix drawn on the GPU (the stack holds 60 GB of them), same
    distributions as workloads.make_tensors, rounded to bf16: these are the inputs of both sides."""
    import torch
    import workloads as wl
    shapes = spec.tensor_shapes()
    if spec.format == wl.FORMAT_DENSE:
        return [(torch.randn(shapes[0], generator=gen, device="cuda") / spec.N ** 0.5).to(torch.bfloat16)]
    if spec.format in (wl.FORMAT_TT, wl.FORMAT_TR):
        return [(torch.randn(shp, generator=gen, device="cuda") / (shp[0] * shp[2]) ** 0.5).to(torch.bfloat16)
                for shp in shapes]
    p = len(spec.out_modes)
    core = torch.randn(shapes[0], generator=gen, device="cuda")
    flat = core.reshape(int(torch.tensor(shapes[0][:p]).prod()), -1)
    core = (flat / flat.norm(dim=1, keepdim=True)).reshape(shapes[0])
    out = [core.to(torch.bfloat16)]
    for shp in shapes[1:]:
        q, r = torch.linalg.qr(torch.randn(shp, generator=gen, device="cuda"))
        out.append((q * torch.sign(torch.diagonal(r))[None, :]).to(torch.bfloat16).contiguous())
    return out


def run_stack(args, verify=True, cpu=True):
    """The mixed 64-layer projection stack: 448 layers (format and rank drawn per matrix) run
    back to back on one stream, sharing one workspace block; 1-token decode and an 8192-token prefill pass.
    Returns the record (tokens/s is that of the prefill pass)."""
    import numpy as np
    import torch
    import oracle as O
    import workloads as wl
    import paper_2602_01613_amd as tn

    specs = wl.qwen3_32b_stack(args.layers)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(wl.SEED_BASE + 4)
    ws = torch.empty(args.stack_workspace_gb << 30, dtype=torch.uint8, device="cuda")
    tokens = args.tokens

    # one matrix per format is kept on the host for the oracle: the first drawn of the classes named here
    check_classes = {(wl.FORMAT_DENSE, 5120, 1024): None, (wl.FORMAT_TT, 5120, 1024): None,
                     (wl.FORMAT_TUCKER, 5120, 1024): None, (wl.FORMAT_TR, 25600, 5120): None}
    t0 = time.perf_counter()
    layers, flops, flops_prefill, flops_decode, params, packed = [], [], [], [], [], []
    for n, spec in enumerate(specs):
        ts = draw_on_device(spec, gen)
        layer = tn.TNLinear(spec.format, tn.TN_DTYPE_BF16, spec.out_modes, spec.in_modes, spec.ranks, ts,
                            tokens, flags=args.flags, workspace=ws)
        layers.append(layer)
        flops.append(layer.query(tn.TN_QUERY_FLOPS_PER_TOKEN))
        # large calls of some layers run on a cheaper plan rebuilt per call: count the work actually done
        lazy_min = layer.query(tn.TN_QUERY_LAZY_MIN_TOKENS)
        flops_prefill.append(layer.query(tn.TN_QUERY_LAZY_FLOPS_PER_TOKEN) if lazy_min and tokens >= lazy_min
                             else flops[-1])
        flops_decode.append(layer.query(tn.TN_QUERY_LAZY_FLOPS_PER_TOKEN) if lazy_min and 1 >= lazy_min else flops[-1])
        params.append(spec.n_params)
        packed.append(layer.query(tn.TN_QUERY_PACKED_BYTES))
        key = (spec.format, spec.N, spec.M)
        if verify and key in check_classes and check_classes[key] is None and \
                (spec.format != wl.FORMAT_TR or max(spec.ranks) == 96):
            check_classes[key] = (n, [t.to(torch.float64).cpu().numpy() for t in ts])
        del ts
    torch.cuda.synchronize()
    create_s = time.perf_counter() - t0
    xs = {n: torch.randn((tokens, n), generator=gen, device="cuda").to(torch.bfloat16) for n in {s.N for s in specs}}
    ys = {m: torch.empty((tokens, m), dtype=torch.bfloat16, device="cuda") for m in {s.M for s in specs}}
    stream = torch.cuda.current_stream()

    def one_pass(t, timed_events=False):
        evs = []
        for spec, layer in zip(specs, layers):
            if timed_events:
                e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
                e0.record(stream)
            layer.forward(xs[spec.N][:t], out=ys[spec.M][:t])
            if timed_events:
                e1.record(stream)
                evs.append((e0, e1))
        return evs

    def timed(t, reps):
        # reps == 0: one pass only, timed as it runs (the prefill pass of the full stack takes
        # seconds; the decode passes before it have already loaded the kernels)
        wall = None
        if reps > 0:
            one_pass(t)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                one_pass(t)
            torch.cuda.synchronize()
            wall = (time.perf_counter() - t0) / reps
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        evs = one_pass(t, timed_events=True)
        torch.cuda.synchronize()
        if wall is None:
            wall = time.perf_counter() - t0
        by_fmt, by_shape = {}, {}
        for spec, (e0, e1) in zip(specs, evs):
            k = wl.FORMAT_NAMES[spec.format]
            ms = e0.elapsed_time(e1)
            by_fmt[k] = by_fmt.get(k, 0.0) + ms
            k2 = f"{k} {spec.N}->{spec.M}" + (f" r{max(spec.ranks)}" if spec.ranks else "")
            n, tot, fl, pk = by_shape.get(k2, (0, 0.0, 0, 0))
            i = len(by_shape) if k2 not in by_shape else None
            by_shape[k2] = (n + 1, tot + ms, fl, pk)
        return wall, by_fmt, by_shape

    dec_wall, dec_fmt, dec_shape = timed(1, max(1, min(args.steps, 10)))
    # the same pass as one captured HIP graph (what a serving loop replays per token: no host launch cost between the
    # 448 forwards); every replay is checked against the eager pass's last output
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for spec, layer in zip(specs, layers):
            layer.forward(xs[spec.N][:1], out=ys[spec.M][:1])
    torch.cuda.synchronize()
    y_eager = {m: y[:1].clone() for m, y in ys.items()}
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        for spec, layer in zip(specs, layers):
            layer.forward(xs[spec.N][:1], out=ys[spec.M][:1])
    for _ in range(2):
        graph.replay()
    torch.cuda.synchronize()
    reps = max(3, min(args.steps, 10))
    t0 = time.perf_counter()
    for _ in range(reps):
        graph.replay()
    torch.cuda.synchronize()
    dec_graph_wall = (time.perf_counter() - t0) / reps
    dec_graph_ok = all(bool(torch.equal(y_eager[m], ys[m][:1])) for m in ys)
    del graph
    pre_wall, pre_fmt, pre_shape = timed(tokens, 0)

    # parity of what was just computed: for one matrix per format (the ring at rank 96 on the widest shape, which
    # alone is a quarter of the pass), the oracle's rows of W against the outputs the passes left behind would
    # need the outputs kept; instead those matrices are run once more on their own at both token counts
    parity = {}
    if verify:
        for key, kept in check_classes.items():
            if kept is None:
                continue
            n, ts64 = kept
            spec, layer = specs[n], layers[n]
            if spec.format == wl.FORMAT_TR:
                rows = np.unique(np.random.default_rng(n).choice(spec.M, size=12, replace=False))
                w = O.tr_dense_rows(ts64, rows)
            else:
                rows, w = None, O.dense_weight(spec.format, ts64, len(spec.out_modes))
            name = f"{wl.FORMAT_NAMES[spec.format]} {spec.N}->{spec.M}" + (f" r{max(spec.ranks)}" if spec.ranks else "")
            for t in (1, tokens):
                yd = layer.forward(xs[spec.N][:t], out=ys[spec.M][:t])
                torch.cuda.synchronize()
                tok = np.unique(np.concatenate([[0, t - 1], np.random.default_rng(t).choice(t, size=min(t, 30), replace=False)]))
                ti = torch.from_numpy(tok).cuda()
                y = yd[ti].to(torch.float64).cpu().numpy()
                if rows is not None:
                    y = y[:, rows]
                ref = O.apply_linear(w, xs[spec.N][ti].to(torch.float64).cpu().numpy())
                parity[f"{name} T={t}"] = O.rel_max_err(y, ref)
        assert all(v <= 2e-2 for v in parity.values()), parity

    counts = {}
    for spec in specs:
        k = f"{wl.FORMAT_NAMES[spec.format]}"
        counts[k] = counts.get(k, 0) + 1
    total_flops = sum(flops_prefill)
    # per-format roofline of the prefill pass: executed FLOPs of the format's matrices over their summed time
    fl_fmt, pk_fmt = {}, {}
    for spec, f, pk in zip(specs, flops_prefill, packed):
        k = wl.FORMAT_NAMES[spec.format]
        fl_fmt[k] = fl_fmt.get(k, 0) + f
        pk_fmt[k] = pk_fmt.get(k, 0) + pk
    roof_fmt = {k: {"tflops": fl_fmt[k] * tokens / (pre_fmt[k] * 1e-3) / 1e12,
                    "frac_of_mfma_peak": fl_fmt[k] * tokens / (pre_fmt[k] * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
                    "share_of_pass": pre_fmt[k] * 1e-3 / pre_wall} for k in pre_fmt}
    dom_fmt = max(pre_fmt, key=lambda k: pre_fmt[k])
    roofline = {"bound": "mfma", "achieved": roof_fmt[dom_fmt]["tflops"], "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": roof_fmt[dom_fmt]["frac_of_mfma_peak"], "traffic": None,
                "kernel": f"the {counts[dom_fmt]} {dom_fmt} matrices of the prefill pass ({100 * roof_fmt[dom_fmt]['share_of_pass']:.0f} % "
                          f"of its time; executed FLOPs of their plans over the sum of their HIP-event times): the "
                          f"Kronecker-sum kernel on half-ring slices rebuilt per call",
                "whole_pass_tflops": total_flops * tokens / pre_wall / 1e12,
                "whole_pass_frac": total_flops * tokens / pre_wall / 1e12 / PEAK_BF16_TFLOPS,
                "by_format": roof_fmt}
    dec_roof = {k: {"packed_GB": pk_fmt[k] / 1e9, "GBps": pk_fmt[k] / (dec_fmt[k] * 1e-3) / 1e9,
                    "frac_of_hbm_peak": pk_fmt[k] / (dec_fmt[k] * 1e-3) / 1e9 / PEAK_HBM_GBS,
                    "tflops": sum(f for s, f in zip(specs, flops_decode) if wl.FORMAT_NAMES[s.format] == k) / (dec_fmt[k] * 1e-3) / 1e12}
                for k in dec_fmt}
    top = sorted(pre_shape.items(), key=lambda kv: -kv[1][1])[:10]
    result = {
        "workload": f"mixed-format projection stack, {len(specs)} matrices ({args.layers} layers x 7), "
                    f"formats {counts}, ranks drawn from {{32,64,96}}; one token passes through every matrix once "
                    f"(a projection stack, not a transformer); weights drawn on the GPU from a seeded generator",
        "tokens": tokens, "matrices": len(specs),
        "prefill": {"tokens_per_s": tokens / pre_wall, "ms_per_pass": 1e3 * pre_wall,
                    "flops_per_token_all_matrices": total_flops,
                    "tflops_factorised": total_flops * tokens / pre_wall / 1e12,
                    "ms_by_format": pre_fmt,
                    "top10_classes_ms": {k: {"matrices": v[0], "ms_each": v[1] / v[0]} for k, v in top}},
        "roofline": roofline,
        "decode_1tok": {"ms_per_token_all_matrices": 1e3 * dec_wall, "tokens_per_s": 1.0 / dec_wall,
                        "graph_ms_per_token_all_matrices": 1e3 * dec_graph_wall, "graph_tokens_per_s": 1.0 / dec_graph_wall,
                        "graph_replay_equals_eager": dec_graph_ok,
                        "ms_by_format": dec_fmt, "by_format": dec_roof,
                        "top10_classes_us": {k: {"matrices": v[0], "us_each": 1e3 * v[1] / v[0]}
                                             for k, v in sorted(dec_shape.items(), key=lambda kv: -kv[1][1])[:10]},
                        "packed_GB": sum(packed) / 1e9, "packed_GBps": sum(packed) / dec_wall / 1e9,
                        "frac_of_hbm_peak": sum(packed) / dec_wall / 1e9 / PEAK_HBM_GBS},
        "parameters": sum(params), "create_seconds": create_s,
        "parity_rel_max_err": parity,
    }
    for layer in layers:
        layer.close()
    del ws, xs, ys
    torch.cuda.empty_cache()
    if cpu:
        result["cpu_baseline"] = stack_cpu_baseline(specs, tokens)
    return result


def stack_cpu_baseline(specs, tokens):
    """The oracle on the stack, extrapolated: one matrix per format (the 5120 -> 1024 class at rank 96) is timed
    in full - rebuild of W, product of 256 tokens - and the cost of
    every other matrix follows from its size: rebuild time scales with M N r^2 (ring), M N r (train) or M N (Tucker,
    dense), the product with M N."""
    import numpy as np
    import oracle as O
    import workloads as wl
    n_tok = 256
    unit = {}
    detail = {}
    for fmt in (wl.FORMAT_DENSE, wl.FORMAT_TT, wl.FORMAT_TR, wl.FORMAT_TUCKER):
        spec = wl.stack_spec(fmt, 5120, 1024, 96)
        ts = wl.make_tensors(spec, 4, instance=500 + fmt)
        x = wl.make_x(spec, n_tok, 4, instance=500 + fmt)
        t0 = time.perf_counter()
        w = O.dense_weight(fmt, ts, len(spec.out_modes))
        rebuild = time.perf_counter() - t0
        t1 = time.perf_counter()
        O.apply_linear(w, x)
        mult = (time.perf_counter() - t1) / n_tok
        scale = {wl.FORMAT_TR: 96.0 ** 2, wl.FORMAT_TT: 96.0}.get(fmt, 1.0)
        unit[fmt] = (rebuild / (spec.M * spec.N * scale), mult / (spec.M * spec.N))
        detail[wl.FORMAT_NAMES[fmt]] = {"rebuild_s_5120x1024_r96": rebuild, "multiply_s_per_token": mult}
    rebuild_total, mult_total = 0.0, 0.0
    for s in specs:
        r = max(s.ranks) if s.ranks else 1
        scale = {wl.FORMAT_TR: float(r) ** 2, wl.FORMAT_TT: float(r)}.get(s.format, 1.0)
        rebuild_total += unit[s.format][0] * s.M * s.N * scale
        mult_total += unit[s.format][1] * s.M * s.N
    return {"value": tokens / (rebuild_total + mult_total * tokens), "unit": "tokens/s", "cores": blas_threads(),
            "kind": "oracle",
            "sample": f"extrapolated: one 5120->1024 rank-96 matrix per format timed (rebuild, product of {n_tok} tokens), "
                      f"scaled by M N (r^2 ring, r train) to the {len(specs)} matrices: rebuild {rebuild_total:.0f} s once + "
                      f"{mult_total * tokens:.0f} s for {tokens} tokens; multiply-only {1.0 / mult_total:.1f} tokens/s",
            "timed": detail}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=50,
                    help="untimed steps first; the shader clock needs some tens of milliseconds of load to settle")
    ap.add_argument("--tokens", type=int, default=8192)
    ap.add_argument("--workload", type=int, default=-1,
                    help="one workload only, in detail: 0 (small fp32 TT; use --tokens 16), 1 (TT), 2 (Tucker), 3 (TR), "
                         "4 (the mixed 64-layer stack). Default: workload 1 as the headline plus one record per other "
                         "workload under \"configs\"")
    ap.add_argument("--calib-copy-mb", type=int, default=0,
                    help="also run one device-to-device copy of this many MiB (a kernel of known traffic, to "
                         "calibrate the profiler's FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--custom", type=str, default="",
                    help="one matrix of the stack instead of a numbered workload: format,in,out,rank "
                         "(e.g. tr,25600,5120,96)")
    ap.add_argument("--layers", type=int, default=64, help="layers of the stack (workload 4)")
    ap.add_argument("--stack-workspace-gb", type=int, default=64, help="shared workspace of the stack in GiB")
    ap.add_argument("--workspace-mb", type=int, default=0, help="workspace limit in MiB (0 = library default)")
    ap.add_argument("--variant", type=int, default=0, help="tuning override: kernel variant id of the wide steps")
    ap.add_argument("--no-merge", action="store_true",
                    help="keep the chain as given (no create-time merging of parameter tensors)")
    ap.add_argument("--shortk-mode", type=int, default=0, help="tuning override of the short-K kernel (0 = library choice, 1..3 = form 0..2)")
    ap.add_argument("--merge-grow", action="store_true",
                    help="allow create-time merges that add parameters (up to a quarter of the dense matrix)")
    ap.add_argument("--transpose", action="store_true",
                    help="apply W^T (TN_FLAG_TRANSPOSE): the gradient of the forward with respect to its input")
    ap.add_argument("--graph-instances", type=int, default=16,
                    help="distinct layer copies in the captured decode graph")
    ap.add_argument("--flags", type=int, default=0, help="extra TN_FLAG_* bits for the layer (e.g. 64: one launch per step)")
    ap.add_argument("--no-pair-chain", action="store_true",
                    help="run a two-step train as two launches (intermediate in the workspace)")
    ap.add_argument("--cpu-sample-tokens", type=int, default=8192)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-stack", action="store_true", help="default run: leave the 64-layer stack out")
    ap.add_argument("--time-budget-s", type=float, default=150.0,
                    help="default run: records that would start after this many seconds are skipped (and say so)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        return 2

    import torch
    import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    t_start = time.perf_counter()
    layer_flags = ((args.variant << 8) | (2 if args.no_merge else 0) | (16 if args.merge_grow else 0)
                   | (args.shortk_mode << 16) | (32 if args.no_pair_chain else 0) | args.flags | (128 if args.transpose else 0))
    args.flags = layer_flags
    everything = args.workload < 0 and not args.custom
    workload = 1 if args.workload < 0 else args.workload

    if workload == 4 and not args.custom:
        rec = run_stack(args, cpu=not args.no_cpu_baseline)
        result = {"metric": METRIC, "value": rec["prefill"]["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": 1,
                  "warmup": 0, "ms_per_step": rec["prefill"]["ms_per_pass"], "higher_is_better": True, "scaling": "weak",
                  "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
                  "config": {"workload": rec["workload"], "tokens": rec["tokens"], "matrices": rec["matrices"]}}
        result.update({k: v for k, v in rec.items() if k not in ("workload", "tokens", "matrices")})
        print(json.dumps(result))
        return 0

    if args.custom:
        f, n_in, n_out, r = args.custom.split(",")
        fmt = {"dense": wl.FORMAT_DENSE, "tt": wl.FORMAT_TT, "tr": wl.FORMAT_TR, "tucker": wl.FORMAT_TUCKER}[f]
        spec = wl.stack_spec(fmt, int(n_in), int(n_out), int(r), f"{f}_{n_in}_{n_out}_r{r}")
    else:
        spec, _ = wl.baseline_spec(workload)
    rec, keep = layer_record(spec, workload, args, layer_flags, args.steps, args.warmup,
                             workload_id=None if args.custom else workload, detail=True)
    # The headline workload is measured first, on a GPU that has not yet been heated by the long launches of the
    # other workloads (measured: after them the same kernel runs 7 % slower); the CPU oracle legs, during which the
    # GPU idles, all come after the last GPU measurement.
    configs, pending_cpu = {}, []
    if everything:
        subs = [("tucker_up_proj", wl.baseline_spec(2)[0], 2, 2, args.steps),
                ("tr_down_proj", wl.baseline_spec(3)[0], 3, 3, max(3, args.steps // 4)),
                ("dense_q_proj", wl.stack_spec(wl.FORMAT_DENSE, 5120, 8192, 0, "dense_q_proj"), 4, 4, args.steps)]
        for name, sub_spec, cid, wid, steps in subs:
            if time.perf_counter() - t_start > args.time_budget_s:
                configs[name] = {"skipped": "time budget of the default run exhausted"}
                continue
            sub_rec, sub_keep = layer_record(sub_spec, cid, args, 0, steps, min(args.warmup, steps), workload_id=wid)
            configs[name] = sub_rec
            pending_cpu.append((name, sub_keep))
        if time.perf_counter() - t_start <= args.time_budget_s:
            configs["tucker_gate_up_pair"] = pair_record(wl.baseline_spec(2)[0], 2, args)
        if time.perf_counter() - t_start <= args.time_budget_s:
            configs["quantised_4bit_decode"] = {
                "tucker_up_proj": quant_record(wl.baseline_spec(2)[0], 2, args),
                "dense_q_proj": quant_record(wl.stack_spec(wl.FORMAT_DENSE, 5120, 8192, 0, "dense_q_proj"), 4, args)}
        if time.perf_counter() - t_start <= args.time_budget_s:
            configs["param_gradients"] = {"tt_q_proj": gradient_record(wl.baseline_spec(1)[0], 1, 1024),
                                          "tucker_up_proj": gradient_record(wl.baseline_spec(2)[0], 2, 1024)}

    pre = rec["prefill"]
    result = {
        "metric": METRIC,
        "value": pre["tokens_per_s"],
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": pre["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": spec.dtype,
        "data": "synthetic",
        "config": {"workload": rec["workload"] + f", {args.tokens} tokens"
                               + (", applied transposed (Y = X W)" if args.transpose else ""),
                   "tokens": args.tokens, "chunk_tokens": rec["chunk_tokens"],
                   "create_time_merges": rec["create_time_merges"],
                   "lazy_merge_from_tokens": rec["lazy_merge_from_tokens"]},
        "flops_per_token": pre["flops_per_token"],
        "tflops_factorised": pre["tflops_factorised"],
        "gpu_ms_per_step_events": pre["gpu_ms_per_step_events"],
        "roofline": rec["roofline"],
        "whole_chain_frac_of_mfma_peak": pre["whole_chain_frac_of_mfma_peak"],
        "per_step": pre["per_step"],
        "decode_1tok": rec["decode_1tok"],
        "decode_1tok_graph": rec["decode_1tok_graph"],
        "verify_8tok": rec["verify_8tok"],
        "decode_64tok": rec["decode_64tok"],
        "paper_context": PAPER_CONTEXT,
    }
    # the stack runs after the headline workload: its parity check keeps the host busy and the GPU idle for seconds
    if everything and not args.no_stack:
        if time.perf_counter() - t_start > args.time_budget_s:
            configs["mixed_stack"] = {"skipped": "time budget of the default run exhausted"}
        else:
            configs["mixed_stack"] = run_stack(args, cpu=False)
    if args.calib_copy_mb > 0:
        src = torch.ones(args.calib_copy_mb << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        result["calib_copy_bytes"] = args.calib_copy_mb << 20
        del src, dst
    # ---- CPU legs (the GPU idles from here on)
    if not args.no_cpu_baseline:
        kspec, ktensors, x_head, y_head = keep
        if args.transpose:
            result["cpu_baseline"] = cpu_baseline(kspec, ktensors, min(args.cpu_sample_tokens, args.tokens), True)
        else:
            # the oracle runs on the rows the GPU consumed, and its product is compared with what the GPU wrote
            import numpy as np
            base = cpu_baseline(kspec, ktensors, args.cpu_sample_tokens)
            chk = cpu_baseline(kspec, ktensors, x_head.shape[0], x_used=x_head, y_gpu=y_head)
            base["gpu_rel_max_err_first_rows"] = chk["gpu_rel_max_err_on_these_rows"]
            base["rows_compared"] = int(x_head.shape[0])
            result["cpu_baseline"] = base
        for name, (kspec, ktensors, x_head, y_head) in pending_cpu:
            configs[name]["cpu_baseline"] = cpu_baseline(kspec, ktensors, x_head.shape[0], x_used=x_head, y_gpu=y_head)
        if "mixed_stack" in configs and "skipped" not in configs["mixed_stack"]:
            configs["mixed_stack"]["cpu_baseline"] = stack_cpu_baseline(wl.qwen3_32b_stack(args.layers), args.tokens)
    if everything:
        result["configs"] = configs
    result["bench_wall_s"] = time.perf_counter() - t_start
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
