#!/usr/bin/env python3
"""Benchmark of the Based sequence-mixer hot path on one MI355X.

One "step" is one pass of the whole hot path over one batch of the 1.3B-layer-shaped prefill
workload, the largest single-GPU prefill configuration (batch 16, 2048 tokens, 16 heads; d' = 16,
d_v = 128; window 64, head dim 128; bf16 in, fp32 accumulate): the chunked Taylor linear-attention
prefill, the sliding-window prefill, and then one fused decode step (state update/readout + ring
attention) for the next token of every sequence.  Inputs are seeded synthetic tensors already
resident in HBM; several distinct buffer sets are rotated so that no step finds its inputs in the
256 MB last-level cache.

Prints ONE JSON line.  ``value`` is tokens/s over the timed steps (B * (N + 1) tokens per step).
``roofline`` is the dominant kernel of that step (the linear-attention prefill), timed with events on
its own stream inside the timed region.  ``prefill_legs`` times the same step on the 360M-layer-shaped
and on the long-sequence (d' = 32) prefill workloads, each with the rooflines of both of its prefill
calls; ``decode`` is the 1.3B-shaped decode workload (batch 128, 1024 sequential steps) with the
roofline of the state update in its loop and over rotating state buffers (cold); ``cpu_baseline`` is
the CPU oracle timed on a bounded sample of the headline workload.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import math
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# Published MI355X peaks used as roofline denominators
PEAK_BF16_TFLOPS = 2500.0
PEAK_HBM_GBS = 8000.0

# HBM bytes per launch from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs summarised under
# profiles/ (counters scaled by what they read for a plain 1 GiB copy: fetch x 2.000, write x 1.000).
# Each figure belongs to the kernel sources it was measured on: it is reported only while the hash
# of those sources is the one recorded here, and as null after any change to them.
MEASURED_TRAFFIC = {
    # key: (entry point, workload) -> (bytes per launch, source files the kernel is built from, their hash)
    ("based_prefill", "prefill_1p3b"): (338599539, ("linattn_prefill_mfma.hip",), "a11fb2150fe2"),
    ("based_prefill", "prefill_360m"): (110228369, ("linattn_prefill_mfma.hip",), "a11fb2150fe2"),
    ("based_swa_prefill", "prefill_1p3b"): (553817107, ("swa_prefill_mfma16.hip",), "6d81285cd196"),
    ("based_swa_prefill", "prefill_360m"): (142845731, ("swa_prefill_mfma.hip",), "268b1a0162b0"),
    ("based_decode_step", "decode_1p3b"): (579192285, ("decode.hip",), "0e4b071cdd26"),
    ("based_decode_step_packed", "decode_1p3b"): (325422966, ("decode.hip",), "0e4b071cdd26"),
}


def progress(msg: str) -> None:
    """Progress lines go to stderr (stdout carries the one JSON line)."""
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def source_hash(files) -> str:
    h = hashlib.sha256()
    for f in files:
        with open(os.path.join(ROOT, "paper_2402_18668_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:12]


def measured_traffic(entry: str, workload: str):
    rec = MEASURED_TRAFFIC.get((entry, workload))
    if rec is None:
        return None
    nbytes, files, want = rec
    try:
        return nbytes if source_hash(files) == want else None
    except OSError:
        return None


def lin_prefill_flops_per_token_head(dp: int, dv: int, C: int = 64, packed: bool = True) -> int:
    """Credited work: readout + update against the state, the K-state, the causal half of the
    intra-chunk block.  The bf16 kernels carry one state row per unordered feature pair
    (D_sym = 1 + d' + d'(d'+1)/2 rows instead of D = 1 + d' + d'^2), so they are credited with D_sym;
    ``packed=False`` gives the figure of the full D-row formulation for comparison."""
    D = 1 + dp + (dp * (dp + 1) // 2 if packed else dp * dp)
    return 4 * D * dv + 4 * D + (C + 1) * (dp + dv + 1)


PREFILL_KERNEL = {
    16: "based_prefill (prefill_mfma_kernel: producer and consumer waves; segment increments and main chunked "
        "pass in one launch)",
    32: "based_prefill (dp32::prefill_kernel: increment launch + main launch, both inside the bracket)",
}


class StepRunner:
    """The step of one prefill workload over rotating buffer sets."""

    def __init__(self, torch, based, synth, dev, name: str, nsets: int):
        self.torch, self.based, self.name = torch, based, name
        wl = synth.WORKLOADS[name]
        self.wl = wl
        B, H, N, dp, dv, dh, w = wl.B, wl.H, wl.N, wl.d_feat, wl.d_v, wl.d_h, wl.w
        bf = torch.bfloat16
        self.scale = 1.0 / math.sqrt(dh)
        self.host = dict(zip(("q", "k", "v"), synth.linattn_inputs(wl)))
        self.host.update(zip(("sq", "sk", "sv"), synth.swa_inputs(wl)))
        dec = synth.decode_inputs(wl, 1)

        def up(a, shape):
            return torch.from_numpy(np.ascontiguousarray(a)).reshape(shape).to(bf).to(dev).contiguous()

        h = self.host
        base = dict(q=up(h["q"], (B, H, N, dp)), k=up(h["k"], (B, H, N, dp)), v=up(h["v"], (B, H, N, dv)),
                    sq=up(h["sq"], (B, H, N, dh)), sk=up(h["sk"], (B, H, N, dh)), sv=up(h["sv"], (B, H, N, dh)),
                    dq=up(dec["q"][0], (B, H, dp)), dk=up(dec["k"][0], (B, H, dp)), dv=up(dec["v"][0], (B, H, dv)),
                    dsq=up(dec["swa_q"][0], (B, H, dh)), dsk=up(dec["swa_k"][0], (B, H, dh)),
                    dsv=up(dec["swa_v"][0], (B, H, dh)))
        self.sets = []
        for i in range(nsets):
            s = {n: (t if i == 0 else t.clone()) for n, t in base.items()}
            s["y"] = torch.empty((B, H, N, dv), dtype=bf, device=dev)
            s["sy"] = torch.empty((B, H, N, dh), dtype=bf, device=dev)
            s["state"] = based.alloc_state(B, H, dp, dv, dev)
            s["ring"] = based.alloc_swa_ring(B, H, w, dh, bf, dev)
            s["yl"] = torch.empty((B, H, dv), dtype=bf, device=dev)
            s["ys"] = torch.empty((B, H, dh), dtype=bf, device=dev)
            self.sets.append(s)
        self.workspace = based.alloc_prefill_workspace(B, H, N, dp, dv, based.BF16, dev)
        self.tokens_per_step = B * (N + 1)

    def step(self, i, ev=None):
        based, wl = self.based, self.wl
        s = self.sets[i % len(self.sets)]
        if ev is not None:
            ev[0].record()
        based.prefill(s["q"], s["k"], s["v"], y=s["y"], state=s["state"], has_init=False, workspace=self.workspace)
        if ev is not None:
            ev[1].record()
        based.swa_prefill(s["sq"], s["sk"], s["sv"], wl.w, self.scale, y=s["sy"], ring=s["ring"])
        if ev is not None:
            ev[2].record()
        based.decode_fused(s["dq"], s["dk"], s["dv"], s["state"], s["dsq"], s["dsk"], s["dsv"], s["ring"],
                           wl.N + 1, wl.w, self.scale, y_lin=s["yl"], y_swa=s["ys"])

    def run(self, steps: int, warmup: int, ev_every: int = 4):
        """Warm up, then time exactly `steps` steps; events bracket the two prefill calls on every
        ev_every-th timed step (an event is a marker between two launches that costs about 3 us of GPU
        time, which the step time includes)."""
        torch = self.torch
        n_ev = (steps + ev_every - 1) // ev_every
        evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(n_ev)]
        for i in range(warmup):
            self.step(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            self.step(warmup + i, evs[i // ev_every] if i % ev_every == 0 else None)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ms_per_step = (t1 - t0) * 1e3 / steps
        prefill_ms = float(np.mean([e[0].elapsed_time(e[1]) for e in evs]))
        swa_ms = float(np.mean([e[1].elapsed_time(e[2]) for e in evs]))
        return ms_per_step, prefill_ms, swa_ms, n_ev

    def rooflines(self, prefill_ms: float, swa_ms: float):
        wl = self.wl
        U, N, dp, dv, dh = wl.units, wl.N, wl.d_feat, wl.d_v, wl.d_h
        flops = lin_prefill_flops_per_token_head(dp, dv) * U * N
        flops_full_d = lin_prefill_flops_per_token_head(dp, dv, packed=False) * U * N
        achieved = flops / (prefill_ms * 1e-3) / 1e12
        lin_bytes = (2 * dp + 2 * dv) * 2 * U * N
        lin = {
            "kernel": PREFILL_KERNEL[dp], "bound": "mfma", "achieved": round(achieved, 2),
            "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
            "traffic": measured_traffic("based_prefill", wl.name),
            "avg_ms": round(prefill_ms, 4), "flops_per_launch": flops,
            # the same duration priced with the unpacked (1 + d' + d'^2 rows) formulation's flop count
            "flops_per_launch_unpacked_state": flops_full_d,
            "achieved_unpacked_state_tflops": round(flops_full_d / (prefill_ms * 1e-3) / 1e12, 2),
            "algorithmic_bytes_per_launch": lin_bytes,
            # the same call against the HBM roof: with d' = 16 the packed-state work is 141-153 flop per
            # byte, below the ridge of 312, so bandwidth bounds the achievable MFMA fraction
            "algorithmic_gbs": round(lin_bytes / (prefill_ms * 1e-3) / 1e9, 1),
            "frac_of_hbm_peak": round(lin_bytes / (prefill_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
        }
        swa_bytes = 4 * dh * 2 * U * N
        gbs = swa_bytes / (swa_ms * 1e-3) / 1e9
        swa = {
            "kernel": "based_swa_prefill (" + ("swa_prefill_mfma16_kernel: 16 queries to a wave" if dh == 128 and wl.w in (32, 64)
                                               else "swa_prefill_mfma_kernel: 32 queries to a wave") + ")", "bound": "hbm", "achieved": round(gbs, 1),
            "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": round(gbs / PEAK_HBM_GBS, 4), "avg_ms": round(swa_ms, 4),
            "algorithmic_bytes_per_launch": swa_bytes, "traffic": measured_traffic("based_swa_prefill", wl.name),
        }
        return lin, swa

    def describe(self):
        wl = self.wl
        return (f"{wl.name}: B{wl.B} N{wl.N} H{wl.H} d'{wl.d_feat} d_v{wl.d_v} + window-{wl.w} attention d_h{wl.d_h}, "
                "then one fused decode step per sequence")


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--decode-steps", type=int, default=1024, help="steps of the batch-128 decode leg")
    ap.add_argument("--workload", default="prefill_1p3b", choices=["prefill_360m", "prefill_1p3b", "prefill_long"],
                    help="prefill workload of the step; the metric is quoted on the default (the largest single-GPU "
                         "prefill configuration), the others are also timed as legs of the default run")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-decode-leg", action="store_true")
    ap.add_argument("--no-graph-leg", action="store_true", help="skip the graph-replay legs")
    ap.add_argument("--no-projection-leg", action="store_true", help="skip the timing of the projection GEMMs")
    ap.add_argument("--no-prefill-legs", action="store_true", help="skip the other prefill workloads")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run three plain device copies of 1 GiB (not timed): the known traffic that "
                         "scales the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        return 2

    import torch
    from paper_2402_18668_amd import based, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if args.copy_probe:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)   # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # 3 sets x 0.3-0.85 GB of q/k/v/y traffic per step: every step reads data the caches no longer hold
    NSETS = 3
    progress(f"inputs of {args.workload}")
    runner = StepRunner(torch, based, synth, dev, args.workload, NSETS)
    wl = runner.wl
    progress("timed steps")
    ms_per_step, prefill_ms, swa_ms, n_ev = runner.run(args.steps, args.warmup)
    value = runner.tokens_per_step / (ms_per_step * 1e-3)
    roofline, swa_roofline = runner.rooflines(prefill_ms, swa_ms)

    out = {
        "metric": "prefill tokens/s + decode tokens/s per layer; % MFMA / % HBM peak",
        "value": round(value, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": runner.describe(), "tokens_per_step": runner.tokens_per_step,
                   "buffer_sets": NSETS, "steps_with_events": n_ev},
        "prefill_tokens_per_s_linear_attention_only": round(wl.B * wl.N / (prefill_ms * 1e-3), 1),
        "roofline": roofline,
        "swa_prefill": {"tokens_per_s": round(wl.B * wl.N / (swa_ms * 1e-3), 1), "roofline": swa_roofline},
    }

    def optional(name, fn):
        """Legs beside the timed step: a failure in one is reported in its place, the line is still printed."""
        progress(name)
        try:
            out[name] = fn()
        except Exception as e:   # noqa: BLE001
            out[name] = {"error": f"{type(e).__name__}: {e}"}

    # ---- the same step as captured graphs (one per buffer set), replayed: launch gaps and event markers gone
    def step_graph_leg():
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for i in range(NSETS):
                runner.step(i)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graphs = []
        for i in range(NSETS):
            gr = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gr, stream=side):
                runner.step(i)
            graphs.append(gr)
        for i in range(args.warmup):
            graphs[i % NSETS].replay()
        torch.cuda.synchronize()
        g0 = time.perf_counter()
        for i in range(args.steps):
            graphs[(args.warmup + i) % NSETS].replay()
        torch.cuda.synchronize()
        g_ms = (time.perf_counter() - g0) * 1e3 / args.steps
        del graphs
        return {"ms_per_step": round(g_ms, 4), "tokens_per_s": round(runner.tokens_per_step / (g_ms * 1e-3), 1)}

    if not args.no_graph_leg:
        optional("step_graph_replay", step_graph_leg)

    # ---- CPU oracle on a bounded sample of the headline workload -----------------------------------
    if not args.no_cpu_baseline:
        h = runner.host
        optional("cpu_baseline", lambda: cpu_baseline(wl, h["q"], h["k"], h["v"], h["sq"], h["sk"], h["sv"], runner.scale))

    # ---- the projections around the mixers (not part of the step or of `value`) ---------------------
    if not args.no_projection_leg:
        # model widths of the two trained sizes (training-settings table): 1024 and 1792
        optional("projection", lambda: projection_leg(torch, based, dev, wl.B, wl.N, 1024 if wl.d_v == 64 else 1792,
                                                      wl.H, wl.d_feat, wl.d_v))
    del runner
    torch.cuda.empty_cache()

    # ---- the other prefill workloads, timed the same way (fewer steps) ------------------------------
    def prefill_leg(name):
        r = StepRunner(torch, based, synth, dev, name, NSETS)
        steps = max(10, args.steps // 2)
        ms, p_ms, s_ms, _ = r.run(steps, max(2, args.warmup // 2))
        lin, swa = r.rooflines(p_ms, s_ms)
        res = {"workload": r.describe(), "steps": steps, "ms_per_step": round(ms, 4),
               "tokens_per_s": round(r.tokens_per_step / (ms * 1e-3), 1),
               "prefill_tokens_per_s_linear_attention_only": round(r.wl.B * r.wl.N / (p_ms * 1e-3), 1),
               "roofline": lin, "swa_prefill_roofline": swa}
        del r
        torch.cuda.empty_cache()
        return res

    if not args.no_prefill_legs:
        legs = {}
        for name in ("prefill_360m", "prefill_1p3b", "prefill_long"):
            if name == args.workload:
                continue
            progress(f"prefill leg {name}")
            try:
                legs[name] = prefill_leg(name)
            except Exception as e:   # noqa: BLE001
                legs[name] = {"error": f"{type(e).__name__}: {e}"}
        out["prefill_legs"] = legs

    # ---- decode leg: 1.3B-shaped, batch 128, fused state update/readout + ring attention ---------
    if not args.no_decode_leg:
        optional("decode", lambda: decode_leg(torch, based, synth, dev, args.decode_steps, not args.no_graph_leg))

    print(json.dumps(out))
    return 0


def decode_leg(torch, based, synth, dev, steps: int, with_graph: bool = True):
    wl = synth.WORKLOADS["decode_1p3b"]
    B, H, dp, dv, dh, w = wl.B, wl.H, wl.d_feat, wl.d_v, wl.d_h, wl.w
    U = B * H
    bf = torch.bfloat16
    scale = 1.0 / math.sqrt(dh)
    N0 = wl.N
    # state and ring from a 512-token seeded prefill (generated on the host in slabs of heads)
    q, k, v = synth.linattn_inputs(wl)
    sq, sk, sv = synth.swa_inputs(wl)

    def up(a, shape):
        return torch.from_numpy(np.ascontiguousarray(a)).reshape(shape).to(bf).to(dev).contiguous()

    state = based.alloc_state(B, H, dp, dv, dev)
    ring = based.alloc_swa_ring(B, H, w, dh, bf, dev)
    based.prefill(up(q, (B, H, N0, dp)), up(k, (B, H, N0, dp)), up(v, (B, H, N0, dv)), state=state)
    based.swa_prefill(up(sq, (B, H, N0, dh)), up(sk, (B, H, N0, dh)), up(sv, (B, H, N0, dh)), w, scale, ring=ring)
    del q, k, v, sq, sk, sv
    # a short cycle of decode tokens, reused round-robin (values do not affect the timing)
    CYC = 8
    d = synth.decode_inputs(wl, CYC)
    tq = up(d["q"], (CYC, B, H, dp)); tk = up(d["k"], (CYC, B, H, dp)); tv = up(d["v"], (CYC, B, H, dv))
    tsq = up(d["swa_q"], (CYC, B, H, dh)); tsk = up(d["swa_k"], (CYC, B, H, dh)); tsv = up(d["swa_v"], (CYC, B, H, dh))
    yl = torch.empty((B, H, dv), dtype=bf, device=dev)
    ys = torch.empty((B, H, dh), dtype=bf, device=dev)

    # the same state in the packed layout (one row per unordered feature pair): the variant
    # benchmarked beside the 273-row contract
    packed = based.alloc_packed_state(B, H, dp, dv, dev)
    based.state_pack(state, packed, B, H, dp, dv)

    def run(n, fused, lin_only=False, use_packed=False, states=None):
        a = torch.cuda.Event(enable_timing=True); b = torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        for t in range(n):
            c = t % CYC
            st = states[t % len(states)] if states else (packed if use_packed else state)
            if lin_only:
                based.decode_step(tq[c], tk[c], tv[c], st, y=yl, packed=use_packed)
            elif fused:
                based.decode_fused(tq[c], tk[c], tv[c], st, tsq[c], tsk[c], tsv[c], ring, N0 + t + 1, w, scale,
                                   y_lin=yl, y_swa=ys, packed=use_packed)
            else:
                based.decode_step(tq[c], tk[c], tv[c], state, y=yl)
                based.swa_decode(tsq[c], tsk[c], tsv[c], ring, N0 + t + 1, w, scale, y=ys)
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / n   # ms per step

    run(20, True)
    ms_fused = run(steps, True)
    ms_lin = run(steps, False, lin_only=True)
    run(20, True, use_packed=True)
    ms_fused_p = run(steps, True, use_packed=True)
    ms_lin_p = run(steps, False, lin_only=True, use_packed=True)
    # cold: the same launch over four rotating copies of the state (1.15 GB), so that no step finds any of
    # its state in the 256 MB last-level cache (a decode loop as the workload defines it re-reads one state)
    rot = [state] + [state.clone() for _ in range(3)]
    run(8, False, lin_only=True, states=rot)
    ms_lin_cold = run(max(64, steps // 4), False, lin_only=True, states=rot)
    del rot
    graph = graph_replay_leg(torch, based, synth, dev, steps) if with_graph else None
    D = 1 + dp + dp * dp
    Dp = 1 + dp + dp * (dp + 1) // 2
    lin_bytes = (2 * (D * dv + D) * 4 + (2 * dp + dv) * 2 + dv * 2) * U
    lin_bytes_p = (2 * (Dp * dv + Dp) * 4 + (2 * dp + dv) * 2 + dv * 2) * U
    swa_bytes = (2 * w * dh * 2 + 2 * dh * 2 + 3 * dh * 2 + dh * 2) * U
    gbs_lin = lin_bytes / (ms_lin * 1e-3) / 1e9
    gbs_cold = lin_bytes / (ms_lin_cold * 1e-3) / 1e9
    return {
        "workload": "decode_1p3b: B128 H16 d'16 d_v128 fp32 state + window-64 ring d_h128, bf16 tokens",
        "steps": steps,
        "fused_ms_per_step": round(ms_fused, 4),
        "fused_tokens_per_s": round(B / (ms_fused * 1e-3), 1),
        "fused_gbs": round((lin_bytes + swa_bytes) / (ms_fused * 1e-3) / 1e9, 1),
        "state_update_ms_per_step": round(ms_lin, 4),
        "state_update_tokens_per_s": round(B / (ms_lin * 1e-3), 1),
        "roofline": {"kernel": "based_decode_step (decode_step_kernel)", "bound": "hbm", "achieved": round(gbs_lin, 1),
                     "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": round(gbs_lin / PEAK_HBM_GBS, 4),
                     "algorithmic_bytes_per_launch": lin_bytes,
                     "traffic": measured_traffic("based_decode_step", wl.name)},
        "roofline_cold": {"kernel": "based_decode_step (decode_step_kernel), four rotating state buffers", "bound": "hbm",
                          "achieved": round(gbs_cold, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                          "frac": round(gbs_cold / PEAK_HBM_GBS, 4), "avg_ms": round(ms_lin_cold, 4),
                          "algorithmic_bytes_per_launch": lin_bytes, "traffic": None},
        # the decode loop captured once as a HIP graph ([fused step, advance positions] x 64) and replayed
        "graph_replay": graph,
        # variant: packed state (153 rows instead of 273), credited with its own, smaller byte count
        "packed_state": {
            "fused_ms_per_step": round(ms_fused_p, 4),
            "fused_tokens_per_s": round(B / (ms_fused_p * 1e-3), 1),
            "state_update_ms_per_step": round(ms_lin_p, 4),
            "state_update_tokens_per_s": round(B / (ms_lin_p * 1e-3), 1),
            "roofline": {"kernel": "based_decode_step_packed (decode_step_kernel, packed rows)", "bound": "hbm",
                         "achieved": round(lin_bytes_p / (ms_lin_p * 1e-3) / 1e9, 1), "peak": PEAK_HBM_GBS,
                         "unit": "GB/s", "frac": round(lin_bytes_p / (ms_lin_p * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                         "algorithmic_bytes_per_launch": lin_bytes_p,
                         "traffic": measured_traffic("based_decode_step_packed", wl.name)},
        },
    }


def projection_leg(torch, based, dev, B: int, N: int, d_model: int, H: int, dp: int, dv: int):
    """The layer's projections in the mixers' own layout: based_project_qkv (d_model -> H (2 d' + d_v), q, k, v
    written head-major from one pass over x) and based_project_out (head-major H d_v -> d_model): time per call
    and fraction of the bf16 MFMA peak (2 M K N flop)."""
    bf = torch.bfloat16
    res = {}
    M = B * N
    g = torch.Generator(device="cpu").manual_seed(11)
    xs = [(torch.randn((B, N, d_model), generator=g)).to(bf).to(dev) for _ in range(3)]
    Wqkv = (torch.randn((H * (2 * dp + dv), d_model), generator=g) / math.sqrt(d_model)).to(bf).to(dev)
    ys = [(torch.randn((B, H, N, dv), generator=g)).to(bf).to(dev) for _ in range(3)]
    Wo = (torch.randn((d_model, H * dv), generator=g) / math.sqrt(H * dv)).to(bf).to(dev)
    calls = (("qkv", d_model, H * (2 * dp + dv), "based_project_qkv", lambda i: based.project_qkv(xs[i % 3], Wqkv, H, dp, dv)),
             ("out", H * dv, d_model, "based_project_out", lambda i: based.project_out(ys[i % 3], Wo)))
    for name, K, Nf, entry, fn in calls:
        for i in range(3):
            fn(i)
        a = torch.cuda.Event(enable_timing=True); b = torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        R = 20
        for i in range(R):
            fn(i)
        b.record()
        torch.cuda.synchronize()
        ms = a.elapsed_time(b) / R   # (includes the allocation of the outputs by the binding's caching allocator)
        tf = 2.0 * M * K * Nf / (ms * 1e-3) / 1e12
        res[name] = {"M": M, "K": K, "N": Nf, "ms": round(ms, 4),
                     "roofline": {"kernel": f"{entry} (lin::linear_wide_kernel, 256 x 256 tiles)", "bound": "mfma", "achieved": round(tf, 1),
                                  "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(tf / PEAK_BF16_TFLOPS, 4)}}
    return res


def graph_replay_leg(torch, based, synth, dev, steps: int):
    """Fused decode for the next `steps` tokens, stream-ordered launches against one captured graph of
    64 [fused step, positions_advance] pairs replayed steps / 64 times.  Two shapes: the 360M-shaped batch
    of 8 (launch-bound: the step's kernel is a few microseconds) and the 1.3B-shaped batch of 128."""
    bf = torch.bfloat16
    T = 64
    reps = max(1, steps // T)
    out = {"tokens_per_graph": T, "replays": reps}
    for name in ("prefill_360m", "decode_1p3b"):
        wl = synth.WORKLOADS[name]
        B, H, dp, dv, dh, w = wl.B, wl.H, wl.d_feat, wl.d_v, wl.d_h, wl.w
        scale = 1.0 / math.sqrt(dh)
        state = based.alloc_state(B, H, dp, dv, dev)
        ring = based.alloc_swa_ring(B, H, w, dh, bf, dev)
        g = torch.Generator(device="cpu").manual_seed(7)
        mk = lambda d: (torch.randn((T, B, H, d), generator=g) * 0.5).to(bf).to(dev)
        tq, tk, tv, tsq, tsk, tsv = mk(dp), mk(dp), mk(dv), mk(dh), mk(dh), mk(dh)
        yl = torch.empty((T, B, H, dv), dtype=bf, device=dev)
        ys = torch.empty((T, B, H, dh), dtype=bf, device=dev)
        pos = torch.zeros((B,), dtype=torch.int32, device=dev)

        def loop():
            for t in range(T):
                based.decode_fused(tq[t], tk[t], tv[t], state, tsq[t], tsk[t], tsv[t], ring, pos, w, scale,
                                   y_lin=yl[t], y_swa=ys[t])
                based.positions_advance(pos)

        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            loop()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            loop()
        a = torch.cuda.Event(enable_timing=True); b = torch.cuda.Event(enable_timing=True)

        def timed(fn):
            pos.fill_(1)
            fn()
            torch.cuda.synchronize()
            a.record()
            for _ in range(reps):
                fn()
            b.record()
            torch.cuda.synchronize()
            return a.elapsed_time(b) / (reps * T)

        ms_eager = timed(loop)
        ms_graph = timed(graph.replay)
        out[name] = {
            "batch": B,
            "eager_ms_per_step": round(ms_eager, 5), "graph_ms_per_step": round(ms_graph, 5),
            "eager_tokens_per_s": round(B / (ms_eager * 1e-3), 1), "graph_tokens_per_s": round(B / (ms_graph * 1e-3), 1),
        }
        del graph
    return out


def cpu_baseline(wl, q, k, v, sq, sk, sv, scale):
    """The fp64 oracle as it stands, timed on this machine's host cores on a sample of units."""
    import oracle
    threads = oracle.threads()
    U = q.shape[0]
    units = min(U, max(2, threads // 2))
    while True:
        t0 = time.perf_counter()
        oracle.linattn_quadratic(q[:units], k[:units], v[:units])
        oracle.swa(sq[:units], sk[:units], sv[:units], wl.w, scale)
        dt = time.perf_counter() - t0
        if dt >= 8.0 or units >= U:
            break
        units = min(U, max(units + 1, int(units * min(4.0, 12.0 / max(dt, 1e-3)))))
    tokens = units * wl.N / wl.H   # a token of a sequence spans H units
    return {"value": round(tokens / dt, 1), "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": f"{units} of {U} (batch, head) units of the same workload, both prefill mixers "
                      f"(quadratic-form linear attention + windowed softmax), fp64, {dt:.1f} s; "
                      f"scaled as units / H sequences"}


if __name__ == "__main__":
    sys.exit(main())
