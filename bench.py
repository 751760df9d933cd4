#!/usr/bin/env python3
"""Benchmark of the chunk-wise attention hot path on one MI355X.

A step is one pass of the whole hot path over one synthetic layer of the named workload:
kvgrad_zero, then for every chunk in reverse order (Alg. 1, second loop) the forward of the
chunk against the cache and its backward (delta, dQ, dK/dV accumulated into gK/gV), one call
per chunk, in the method's order, on one stream.  Inputs are resident in HBM before timing.

Prints ONE JSON line: whole-job TFLOP/s (algorithmic FLOPs: 4*D per visible (row, col) pair
forward, 10*D backward), the roofline of the dominant kernel measured with HIP events around
its launches in every fifth step of the timed region, and the CPU oracle timed on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 matrix-core peak (published)
TOL = {"f32": {"o": 1e-4, "lse": 1e-4, "dq": 1e-4, "gk": 1e-4, "gv": 1e-4},
       "bf16": {"o": 1e-2, "lse": 1e-2, "dq": 2e-2, "gk": 2e-2, "gv": 2e-2}}


def hbm_traffic_per_launch(workload, kernel):
    """HBM bytes per launch of `kernel` in `workload`, from the committed table of rocprofv3 FETCH_SIZE / WRITE_SIZE
    measurements (profiles/hbm_traffic_per_launch.txt: one `workload kernel bytes` line per measured pair, with the
    commands and the calibration beside it).  None for a pair that has not been measured."""
    try:
        with open(os.path.join(ROOT, "profiles", "hbm_traffic_per_launch.txt")) as f:
            for line in f:
                parts = line.split("#")[0].split()
                if len(parts) == 3 and parts[0] == workload and parts[1] == kernel:
                    return float(parts[2])
    except OSError:
        pass
    return None


def pairs(j, C):
    """visible (row, col) pairs per head in the call for chunk j"""
    return C * j * C + C * (C + 1) // 2


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="cfg3",
                    help="workload of the headline figure (default: the 32K-token layer the metric is quoted on)")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the extra objects (cfg2, cfg4 and the Alg. 2 steps) of the default run")
    ap.add_argument("--device-inputs", action="store_true",
                    help="draw the inputs on the device (torch generator) instead of uploading the seeded host arrays "
                         "of `workloads`; no parity object then")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-layer32k", action="store_true")
    ap.add_argument("--no-profile", action="store_true", help="do not bracket kernels with events in the timed region")
    ap.add_argument("--calls", default="",
                    help="comma-separated chunk indices: instead of whole steps, time the forward + backward call pair "
                         "of just these chunks (per-kernel event times; used for counter collection)")
    ap.add_argument("--hbm-kernels", action="store_true",
                    help="also time the HBM-bound helpers (kvgrad_zero / accumulate, kv_append, kvgrad_readout) and "
                         "report their GB/s against the 8 TB/s HBM peak")
    ap.add_argument("--schedules", action="store_true",
                    help="also time a whole layer of --config under Alg. 1 and Alg. 2 (needs a config with spaco_t)")
    ap.add_argument("--transposed-order", action="store_true",
                    help="also time the step with the backward calls in the transposed order "
                         "(seco_chunk_attn_bwd_gather) and report it as transposed_backward_order")
    ap.add_argument("--context-scaling", action="store_true",
                    help="also time the backward loop of Alg. 2 (t = 8 selected chunks of 2048 tokens, evenly spaced) at "
                         "16K, 32K and 64K tokens, split into its dQ and dK/dV kernels: the paper's claim that the "
                         "backward cost is decoupled from the context length (Sec. 5), and what is left of it")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step into a HIP graph and time replays of it (removes the dispatch gaps between "
                         "the short kernels of small chunks); no per-kernel events in this mode")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch kvgrad_accumulate on a 1 GiB pair of buffers (a plain streaming kernel of known "
                         "size: reads 2 GiB, writes 1 GiB) so that rocprofv3 FETCH_SIZE / WRITE_SIZE can be scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build is single-GPU by design (one process, one MI355X, no collectives); "
                 "run with --gpus 1")

    import torch
    import paper_2505_16710_amd as seco
    from workloads import CONFIGS, f32_to_bf16_bits, head_slice

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    seco.load_library()
    dev = "cuda:0"
    cfg = CONFIGS[args.config]
    B, Hq, Hkv, D, N, C = cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.seq_len, cfg.chunk_len
    k_chunks = cfg.n_chunks
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    scale = cfg.scale
    G = Hq // Hkv
    # (batch, KV head) units whose host arrays are kept for the oracle: it is timed on them (cpu_baseline) and the
    # GPU results of the very same arrays are compared with what it returns (parity)
    oracle_units = [] if (args.no_cpu_baseline or args.device_inputs) else [(0, Hkv // 2), (B - 1, Hkv - 1)]
    host_units = {}

    def device_inputs(cx):
        gen = torch.Generator(device=dev).manual_seed(cx.seed)
        mk = lambda h: torch.randn(cx.batch, h, cx.seq_len, cx.head_dim, generator=gen, device=dev,
                                   dtype=torch.float32).to(tdt)
        return mk(cx.n_q_heads), mk(cx.n_kv_heads), mk(cx.n_kv_heads), mk(cx.n_q_heads)

    def uploaded_inputs(cx, keep):
        """The seeded host arrays of `workloads` (already rounded to the storage type), uploaded head by head; the
        fp32 host copies of the units in `keep` stay in host_units for the oracle."""
        out = {}
        for name, H in (("q", cx.n_q_heads), ("k", cx.n_kv_heads), ("v", cx.n_kv_heads), ("do", cx.n_q_heads)):
            t = torch.empty(cx.batch, H, cx.seq_len, cx.head_dim, dtype=tdt, device=dev)
            for b in range(cx.batch):
                for h in range(H):
                    x = head_slice(cx, name, b, h)
                    if cx.dtype == "bf16":
                        t[b, h] = torch.from_numpy(f32_to_bf16_bits(x).view(np.int16)).to(dev).view(torch.bfloat16)
                    else:
                        t[b, h] = torch.from_numpy(x).to(dev)
                    u = (b, h // (cx.n_q_heads // cx.n_kv_heads) if H == cx.n_q_heads else h)
                    if u in keep:
                        host_units.setdefault(u, {}).setdefault(name, []).append(x)
            out[name] = t
        return out["q"], out["k"], out["v"], out["do"]

    class Layer:
        """Device buffers of one layer of configuration cx; O is kept whole so that O and dO chunk views share
        strides."""

        def __init__(self, cx, inputs=None, seq_len=None):
            if seq_len is not None:                 # same shape, another context length (device-generated inputs)
                from dataclasses import replace
                cx = replace(cx, seq_len=seq_len)
            self.cx, self.N, self.C, self.k = cx, cx.seq_len, cx.chunk_len, cx.n_chunks
            self.q, self.kc, self.vc, self.do = inputs if inputs is not None else device_inputs(cx)
            Bx, Hqx, Hkvx, Dx = cx.batch, cx.n_q_heads, cx.n_kv_heads, cx.head_dim
            self.o = torch.empty_like(self.q)
            self.lse = torch.empty(self.k, Bx, Hqx, self.C, device=dev, dtype=torch.float32)   # kept per chunk
            self.dq = torch.empty_like(self.q)
            self.gk = torch.empty(Bx, Hkvx, self.N, Dx, device=dev, dtype=torch.float32)
            self.gv = torch.empty_like(self.gk)
            # workspaces sized by the library for this shape (delta; partial results of the short-chunk path)
            d = seco.binding.make_desc(self.rows(self.q, 0), self.kc, 0, scale, o=self.rows(self.o, 0), g=self.gk)
            nf = seco.seco_workspace_bytes(d, seco.binding.SECO_OP_FWD)
            nb = seco.seco_workspace_bytes(d, seco.binding.SECO_OP_BWD)
            self.ws_fwd = torch.empty(nf, device=dev, dtype=torch.uint8) if nf else False
            self.ws = torch.empty(max(nb, 256), device=dev, dtype=torch.uint8)

        def rows(self, t, j):
            return t[:, :, j * self.C:(j + 1) * self.C]

        def fwd(self, j):
            seco.seco_chunk_attn_fwd(self.rows(self.q, j), self.kc, self.vc, j * self.C, scale,
                                     o=self.rows(self.o, j), lse=self.lse[j], ws=self.ws_fwd)

        def bwd(self, j, weights=None, dq_weights=None):
            args = (self.rows(self.q, j), self.kc, self.vc, self.rows(self.o, j), self.lse[j], self.rows(self.do, j),
                    self.gk, self.gv, j * self.C, scale)
            if weights is None:
                seco.seco_chunk_attn_bwd(*args, d_q=self.rows(self.dq, j), ws=self.ws)
            else:
                seco.spaco_chunk_attn_bwd(*args, weights, self.C, d_q=self.rows(self.dq, j), ws=self.ws,
                                          dq_weight=dq_weights)

    t_in = time.perf_counter()
    L = Layer(cfg, None if args.device_inputs else uploaded_inputs(cfg, set(oracle_units)))
    torch.cuda.synchronize()
    input_seconds = time.perf_counter() - t_in

    def step():
        seco.kvgrad_zero(L.gk, L.gv)
        for j in range(k_chunks - 1, -1, -1):
            L.fwd(j)
            L.bwd(j)

    per_pair = D * Hq * B
    flops_fwd = sum(4 * pairs(j, C) for j in range(k_chunks)) * per_pair
    flops_dq = sum(6 * pairs(j, C) for j in range(k_chunks)) * per_pair
    flops_dkdv = sum(4 * pairs(j, C) for j in range(k_chunks)) * per_pair
    flops_step = flops_fwd + flops_dq + flops_dkdv

    if args.calls:
        per_call = {}
        for j in [int(x) for x in args.calls.split(",")]:
            for _ in range(max(args.warmup, 1)):
                L.fwd(j)
                L.bwd(j)
            torch.cuda.synchronize()
            seco.seco_profile_enable(True)
            for _ in range(args.steps):
                L.fwd(j)
                L.bwd(j)
            torch.cuda.synchronize()
            prof = seco.seco_profile_read()
            seco.seco_profile_enable(False)
            alg = {"fwd": 4, "dq": 6, "dkdv": 4}
            per_call[str(j)] = {k: {"avg_ms": round(prof[k][0] / args.steps, 5),
                                    "tflops": round(f * pairs(j, C) * per_pair * args.steps / (prof[k][0] * 1e-3) / 1e12, 1)}
                                for k, f in alg.items()}
        print(json.dumps({"metric": "per_call_kernel_times", "config": {"workload": cfg.name, "chunk_len": C,
                                                                       "seq_len": N}, "per_call": per_call}))
        return

    run_step = step
    if args.graph:
        # the library allocates nothing, never synchronises and clears gK/gV with a kernel, so a step can be captured
        args.no_profile = True
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        run_step = graph.replay

    bf16 = cfg.dtype == "bf16"
    peak = PEAK_BF16_TFLOPS if bf16 else 157.3

    def roofline_of(name, kind, alg_flops, ms, n, n_steps, where):
        """Roofline object of one kernel kind: algorithmic FLOPs of its launches / their summed event durations.
        bf16 kernels are dense MFMA contractions (2500 TFLOP/s); the fp32 parity kernels use the vector ALU only
        (256 CUs x 128 lanes x 2 FLOP x 2.4 GHz = 157.3 TFLOP/s)."""
        achieved = alg_flops * n_steps / (ms * 1e-3) / 1e12
        twice = 2.0 if (bf16 and kind == "dkdv") else 1.0       # dK/dV computes S and dP a second time
        return {"bound": "mfma" if bf16 else "alu", "kernel": kind + ("_bf16_kernel" if bf16 else "_f32_kernel"),
                "achieved": round(achieved, 2), "peak": peak, "unit": "TFLOP/s", "frac": round(achieved / peak, 4),
                "traffic": hbm_traffic_per_launch(name, kind),
                "avg_launch_ms": round(ms / n, 5), "launches": int(n),
                "executed_over_algorithmic": twice, "executed_frac": round(achieved * twice / peak, 4),
                "measured_in": where}

    def kernel_table(kprof, alg, n_steps):
        kern = {}
        for kind, (ms, n) in kprof.items():
            if n:
                kern[kind] = {"launches": int(n), "avg_ms": round(ms / n, 5), "total_ms_per_step": round(ms / n_steps, 4)}
                if kind in alg:
                    kern[kind]["tflops"] = round(alg[kind] * n_steps / (ms * 1e-3) / 1e12, 2)
                    if bf16:      # fraction of the dense bf16 matrix-core peak (algorithmic work)
                        kern[kind]["frac_of_mfma_peak"] = round(kern[kind]["tflops"] / PEAK_BF16_TFLOPS, 4)
        return kern

    # Per-kernel event times come from the warm-up steps (every launch bracketed).  In the timed steps only the
    # launches of the dominant kernel are bracketed, and only in every PROF_EVERY-th step: an event costs a gap of
    # about 5.6 us before the next kernel (rocprofv3 kernel trace), i.e. 11 us per bracketed launch; around every
    # launch that would slow the very region that gives `value` by 3 %, around the dominant kernel in every step
    # by 1.8 %, this way by 0.4 %.
    warm_prof = None
    for i in range(args.warmup):
        if not args.no_profile and i == args.warmup - 1:      # the last warm-up step is the profiled one
            torch.cuda.synchronize()
            seco.seco_profile_enable(True)
        run_step()
    torch.cuda.synchronize()
    if not args.no_profile and args.warmup > 0:
        warm_prof = seco.seco_profile_read()
        seco.seco_profile_enable(False)
    dom = None
    prof_kinds = None
    if not args.no_profile and warm_prof is not None:
        dom = max(("fwd", "dq", "dkdv"), key=lambda kd: warm_prof[kd][0])
        prof_kinds = [dom]
    PROF_EVERY = 5
    n_prof_steps = 0
    if not args.no_profile:
        seco.seco_profile_enable(False)             # also drops any earlier records
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(args.steps):
        bracket = not args.no_profile and i % PROF_EVERY == 0
        if bracket:
            seco.seco_profile_set(prof_kinds)       # host flag only: the records collected so far are kept
            n_prof_steps += 1
        run_step()
        if bracket:
            seco.seco_profile_set([])
        marks[i + 1].record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
    prof = None
    if not args.no_profile:
        prof = seco.seco_profile_read()
        seco.seco_profile_enable(False)
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    tflops = flops_step / (ms_per_step * 1e-3) / 1e12

    out = {
        "metric": "chunk_attn_fwd_bwd_tflops", "value": round(tflops, 2), "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: SeCO fwd+bwd (Alg. 1 second loop), one call pair per chunk, full gK/gV "
                               f"accumulation, {N}-token layer",
                   "batch": B, "n_q_heads": Hq, "n_kv_heads": Hkv, "head_dim": D, "seq_len": N, "chunk_len": C,
                   "n_chunks": k_chunks, "flops_per_step": flops_step,
                   "inputs": "device-generated (torch generator)" if args.device_inputs else
                             f"seeded host arrays of workloads.head_slice, uploaded ({input_seconds:.1f} s, untimed)"},
        "pct_of_bf16_mfma_peak": round(100 * tflops / PEAK_BF16_TFLOPS, 2),
        "launch_mode": "hip_graph_replay" if args.graph else "eager",
        "step_ms_min": round(per_step[0], 4), "step_ms_median": round(per_step[len(per_step) // 2], 4),
    }

    # what the device reports: compute units x 4096 bf16 FLOP per clock and CU x its maximum clock (the published
    # 2.5 PFLOP/s is 256 CUs at 2.4 GHz; the clock under load is lower and not readable from here)
    cus, clock_khz = seco.binding.seco_device_info()
    out["device"] = {"name": torch.cuda.get_device_properties(0).name, "compute_units": cus,
                     "max_clock_mhz": round(clock_khz / 1e3),
                     "bf16_peak_from_device_tflops": round(cus * 4096 * clock_khz * 1e3 / 1e12, 1)}

    if prof is not None:
        alg = {"fwd": flops_fwd, "dq": flops_dq, "dkdv": flops_dkdv}
        kprof, ksteps = (warm_prof, 1) if warm_prof is not None else (prof, n_prof_steps)
        kern = kernel_table(kprof, alg, ksteps)
        kern["measured_in"] = "last warm-up step (every launch bracketed by events)" if warm_prof is not None else "timed steps"
        if dom is None:
            dom = max(alg, key=lambda kd: prof[kd][0])
        ms, n = prof[dom]
        out["roofline"] = roofline_of(cfg.name, dom, alg[dom], ms, n, n_prof_steps,
                                      f"timed steps (HIP events around every launch of this kernel in {n_prof_steps} "
                                      f"of the {args.steps} timed steps)")
        out["kernels"] = kern

    # The outputs of the last timed step, brought to the host for the units the oracle is going to evaluate (the
    # comparison itself follows the oracle's timed run below).
    gpu_units = {}
    for (b, kvh) in oracle_units:
        hs = slice(kvh * G, (kvh + 1) * G)
        lse_full = torch.cat([L.lse[j][b:b + 1, hs] for j in range(k_chunks)], dim=2)
        gpu_units[(b, kvh)] = {"o": L.o[b:b + 1, hs].double().cpu().numpy(), "lse": lse_full.double().cpu().numpy(),
                               "dq": L.dq[b:b + 1, hs].double().cpu().numpy(),
                               "gk": L.gk[b:b + 1, kvh:kvh + 1].double().cpu().numpy(),
                               "gv": L.gv[b:b + 1, kvh:kvh + 1].double().cpu().numpy()}

    def other_workload(cx, selected=None, steps=5, warmup=2):
        """value + per-kernel table + roofline of the dominant kernel for another workload (device-generated inputs of
        the same distribution): the SeCO step, or with `selected` the Alg. 2 step (forward + backward calls of the
        selected chunks only, dK/dV restricted to selected chunks and weighted with the factor k/t)."""
        Lx = Layer(cx)
        kx, Cx = cx.n_chunks, cx.chunk_len
        pp = cx.head_dim * cx.n_q_heads * cx.batch
        calls = list(range(kx - 1, -1, -1)) if selected is None else list(selected)
        lam = 1.0 if selected is None else kx / len(selected)

        def sel_pairs(j):      # (row, col) pairs of call j whose columns lie in selected chunks
            if selected is None:
                return pairs(j, Cx)
            return sum(Cx * Cx for i in selected if i < j) + Cx * (Cx + 1) // 2

        alg = {"fwd": sum(4 * pairs(j, Cx) for j in calls) * pp, "dq": sum(6 * pairs(j, Cx) for j in calls) * pp,
               "dkdv": sum(4 * sel_pairs(j) for j in calls) * pp}
        total = sum(alg.values())

        def stepx():
            seco.kvgrad_zero(Lx.gk, Lx.gv)
            for j in calls:
                Lx.fwd(j)
                Lx.bwd(j, None if selected is None else seco.spaco_chunk_weights(selected, j, lam))

        for _ in range(warmup):
            stepx()
        torch.cuda.synchronize()
        a = time.perf_counter()
        for _ in range(steps):
            stepx()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - a) * 1e3 / steps
        seco.seco_profile_enable(True)
        stepx()
        torch.cuda.synchronize()
        kp = seco.seco_profile_read()
        seco.seco_profile_enable(False)
        domx = max(alg, key=lambda kd: kp[kd][0])
        tag = cx.name if selected is None else f"{cx.name}_spaco_t{len(selected)}"
        res = {"workload": f"{cx.name}: " + ("SeCO fwd+bwd, all chunks" if selected is None else
                                             f"Alg. 2 step, {len(selected)} of {kx} chunks selected {list(selected)}, factor {lam:g}"),
               "seq_len": cx.seq_len, "chunk_len": Cx, "value": round(total / (ms * 1e-3) / 1e12, 2), "unit": "TFLOP/s",
               "ms_per_step": round(ms, 4), "steps": steps, "warmup": warmup, "flops_per_step": total,
               "pct_of_bf16_mfma_peak": round(100 * total / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 2),
               "kernels": kernel_table(kp, alg, 1),
               "roofline": roofline_of(tag, domx, alg[domx], kp[domx][0], kp[domx][1], 1,
                                       "one extra step with HIP events around every launch")}
        del Lx
        torch.cuda.empty_cache()
        return res

    def layer_seconds(cx):
        """Seconds per layer of configuration cx under the two schedules (Alg. 1: k forwards, then forward +
        backward per chunk in reverse order; Alg. 2: k forwards, then forward + backward for the t selected
        chunks with factor k/t), best of 3."""
        Lx = Layer(cx)
        kx, tx = cx.n_chunks, cx.spaco_t
        sel = seco.spaco_select_chunks(cx.seed, 0, kx, tx)
        lam = kx / tx

        def seco_layer():
            for j in range(kx):
                Lx.fwd(j)
            seco.kvgrad_zero(Lx.gk, Lx.gv)
            for j in range(kx - 1, -1, -1):
                Lx.fwd(j)
                Lx.bwd(j)

        def spaco_layer():
            for j in range(kx):
                Lx.fwd(j)
            seco.kvgrad_zero(Lx.gk, Lx.gv)
            for j in sel:
                Lx.fwd(j)
                Lx.bwd(j, seco.spaco_chunk_weights(sel, j, lam))

        lse_full = torch.empty(cx.batch, cx.n_q_heads, cx.seq_len, device=dev, dtype=torch.float32)
        d_full = seco.binding.make_desc(Lx.q, Lx.kc, 0, scale, o=Lx.o)
        n_full = seco.seco_workspace_bytes(d_full, seco.binding.SECO_OP_FWD)
        ws_full = torch.empty(n_full, device=dev, dtype=torch.uint8) if n_full else False

        def prefill_stage1():           # stage 1 as ONE forward call over the whole sequence; LSE handed out per chunk
            seco.seco_chunk_attn_fwd(Lx.q, Lx.kc, Lx.vc, 0, scale, o=Lx.o, lse=lse_full, ws=ws_full)
            for j in range(kx):
                Lx.lse[j].copy_(lse_full[:, :, j * Lx.C:(j + 1) * Lx.C])

        def seco_layer_prefill_kept():  # whole-sequence stage 1 + kept outputs: stage 2 is backward calls only
            prefill_stage1()
            seco.kvgrad_zero(Lx.gk, Lx.gv)
            for j in range(kx - 1, -1, -1):
                Lx.bwd(j)

        def spaco_layer_prefill_kept():
            prefill_stage1()
            seco.kvgrad_zero(Lx.gk, Lx.gv)
            for j in sel:
                Lx.bwd(j, seco.spaco_chunk_weights(sel, j, lam))

        def seco_layer_kept():          # stage 2 takes O and LSE from stage 1 (kept per chunk) instead of recomputing
            for j in range(kx):
                Lx.fwd(j)
            seco.kvgrad_zero(Lx.gk, Lx.gv)
            for j in range(kx - 1, -1, -1):
                Lx.bwd(j)

        def spaco_layer_kept():
            for j in range(kx):
                Lx.fwd(j)
            seco.kvgrad_zero(Lx.gk, Lx.gv)
            for j in sel:
                Lx.bwd(j, seco.spaco_chunk_weights(sel, j, lam))

        # dQ visits the selected chunks only as well (given chunk j is drawn, an earlier chunk is drawn with probability
        # (t-1)/(k-1): weight (k-1)/(t-1) keeps the estimate of dQ unbiased); whole-sequence stage 1, kept outputs
        lam_q = (kx - 1) / (tx - 1) if tx > 1 else 0.0

        def spaco_layer_sparse_dq():
            prefill_stage1()
            seco.kvgrad_zero(Lx.gk, Lx.gv)
            for j in sel:
                Lx.bwd(j, seco.spaco_chunk_weights(sel, j, lam), seco.spaco_chunk_weights(sel, j, lam_q))

        stats_t = torch.empty(2, cx.batch, cx.n_q_heads, (cx.seq_len + 3) // 4 * 4, device=dev, dtype=torch.float32)

        def gather_bwd(j, row_weight=None):
            seco.seco_chunk_attn_bwd_gather(Lx.q[:, :, j * Lx.C:], Lx.kc, Lx.vc, Lx.rows(Lx.o, j), Lx.lse[j],
                                            Lx.do[:, :, j * Lx.C:], Lx.gk, Lx.gv, j * Lx.C, scale, Lx.C, stats_t,
                                            d_q=Lx.rows(Lx.dq, j), ws=Lx.ws, row_weight=row_weight,
                                            weight_chunk_len=Lx.C)

        def seco_layer_transposed():    # whole-sequence stage 1, kept outputs, backward calls in the transposed order
            prefill_stage1()
            seco.kvgrad_zero(Lx.gk, Lx.gv)
            for j in range(kx - 1, -1, -1):
                gather_bwd(j)

        def spaco_layer_transposed():
            prefill_stage1()
            seco.kvgrad_zero(Lx.gk, Lx.gv)
            for j in sel:
                gather_bwd(j, [1.0 if i == j else (lam if i in sel else 0.0) for i in range(j, kx)])

        def spaco_percall_layer():      # every chunk back-propagated, each call with its own draw of t earlier chunks
            for j in range(kx):
                Lx.fwd(j)
            seco.kvgrad_zero(Lx.gk, Lx.gv)
            for j in range(kx - 1, -1, -1):
                Lx.fwd(j)
                Lx.bwd(j, seco.spaco_percall_weights(cx.seed, 0, j, tx))

        def spaco_last_call():          # the single call of the last chunk with t sampled earlier chunks + itself
            j = kx - 1
            Lx.fwd(j)
            Lx.bwd(j, seco.spaco_percall_weights(cx.seed, 0, j, tx))

        res = {}
        for name, fn in (("seco", seco_layer), (f"spaco_t{tx}", spaco_layer), ("seco_kept_outputs", seco_layer_kept),
                         (f"spaco_t{tx}_kept_outputs", spaco_layer_kept),
                         ("seco_prefill_kept_outputs", seco_layer_prefill_kept),
                         (f"spaco_t{tx}_prefill_kept_outputs", spaco_layer_prefill_kept),
                         (f"spaco_t{tx}_prefill_kept_outputs_sparse_dq", spaco_layer_sparse_dq),
                         ("seco_prefill_kept_outputs_transposed", seco_layer_transposed),
                         (f"spaco_t{tx}_prefill_kept_outputs_transposed", spaco_layer_transposed),
                         (f"spaco_percall_t{tx}", spaco_percall_layer),
                         (f"spaco_last_call_t{tx}", spaco_last_call)):
            fn()
            torch.cuda.synchronize()
            best = 1e9
            for _ in range(3):
                a = time.perf_counter()
                fn()
                torch.cuda.synchronize()
                best = min(best, time.perf_counter() - a)
            res[name] = round(best, 5)
        res["selected_chunks"] = sel
        return res

    def transposed_order():
        """The same step with the backward calls in the transposed order (seco_chunk_attn_bwd_gather: the call of
        chunk j forms the finished gK/gV rows of chunk j from the query rows of chunks j..k-1, instead of adding
        to the rows of chunks 0..j): same forward calls, same dQ, same final gK/gV up to the order of summation."""
        stats = torch.empty(2, B, Hq, (N + 3) // 4 * 4, device=dev, dtype=torch.float32)

        def step_t():
            seco.kvgrad_zero(L.gk, L.gv)
            for j in range(k_chunks - 1, -1, -1):
                L.fwd(j)
                seco.seco_chunk_attn_bwd_gather(L.q[:, :, j * C:], L.kc, L.vc, L.rows(L.o, j), L.lse[j],
                                                L.do[:, :, j * C:], L.gk, L.gv, j * C, scale, C, stats,
                                                d_q=L.rows(L.dq, j), ws=L.ws)

        for _ in range(max(args.warmup, 1)):
            step_t()
        torch.cuda.synchronize()
        a = time.perf_counter()
        for _ in range(args.steps):
            step_t()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - a) * 1e3 / args.steps
        seco.seco_profile_enable(True)
        step_t()
        prof_t = seco.seco_profile_read()
        seco.seco_profile_enable(False)
        return {"ms_per_step": round(ms, 4), "tflops": round(flops_step / (ms * 1e-3) / 1e12, 2),
                "dkdv_ms_per_step": round(prof_t["dkdv"][0], 4), "dq_ms_per_step": round(prof_t["dq"][0], 4),
                "fwd_ms_per_step": round(prof_t["fwd"][0], 4)}

    if args.transposed_order and cfg.dtype == "bf16" and N % C == 0 and not args.graph:
        out["transposed_backward_order"] = transposed_order()

    def context_scaling():
        """Backward loop of Alg. 2 with C = 2048 and t = 8 fixed while the context grows (k = 8, 16, 32 chunks; the
        selected chunks evenly spaced, the last one included; factor k/t; stage-1 outputs kept, so the loop is the
        t backward calls only).  Per context length: milliseconds of the loop (host clock, best of 3) and, from the
        library's per-kernel events in one extra pass, of its dQ and dK/dV kernels; the same with the dQ of a call
        visiting the selected chunks only (spaco_chunk_attn_bwd_sparse_dq, weight (k-1)/(t-1))."""
        Cx, tx, res = 2048, 8, {}
        for Nx in (16384, 32768, 65536):
            Lx = Layer(CONFIGS["cfg3"], seq_len=Nx)          # cfg3's shape: chunks of 2048
            kx = Nx // Cx
            sel = [kx - 1 - i * (kx // tx) for i in range(tx)]
            lam, lam_q = kx / tx, (kx - 1) / (tx - 1)
            for j in range(kx):
                Lx.fwd(j)

            def loop(sparse_dq):
                seco.kvgrad_zero(Lx.gk, Lx.gv)
                for j in sel:
                    Lx.bwd(j, seco.spaco_chunk_weights(sel, j, lam),
                           seco.spaco_chunk_weights(sel, j, lam_q) if sparse_dq else None)

            row = {"n_chunks": kx, "selected_chunks": sel}
            for tag, sparse_dq in (("exact_dq", False), ("sparse_dq", True)):
                loop(sparse_dq)
                torch.cuda.synchronize()
                best = 1e9
                for _ in range(3):
                    a = time.perf_counter()
                    loop(sparse_dq)
                    torch.cuda.synchronize()
                    best = min(best, time.perf_counter() - a)
                seco.seco_profile_enable(True)
                loop(sparse_dq)
                prof = seco.seco_profile_read()
                seco.seco_profile_enable(False)
                row[tag] = {"loop_ms": round(best * 1e3, 3), "dq_ms": round(prof["dq"][0], 3),
                            "dkdv_ms": round(prof["dkdv"][0], 3)}
            res[str(Nx)] = row
            del Lx
            torch.cuda.empty_cache()
        return res

    if args.context_scaling and cfg.dtype == "bf16":
        out["context_scaling_c2048_t8"] = context_scaling()

    if args.schedules and cfg.dtype == "bf16" and cfg.spaco_t > 0:
        # the two schedules on the benchmarked configuration itself
        out["sec_per_layer"] = dict(layer_seconds(cfg), seq_len=N, chunk_len=C)

    if not args.no_other_workloads and cfg.dtype == "bf16" and not args.graph:
        # the other workloads the target spans (16K and 64K tokens) and the Alg. 2 steps (t = 4 at 32K, t = 8 at 64K,
        # seeded selections), each with its own whole-step TFLOP/s and the roofline of its dominant kernel
        L = None
        torch.cuda.empty_cache()
        others = {}
        for name in ("cfg2", "cfg3", "cfg4"):
            if name != cfg.name:
                others[name] = other_workload(CONFIGS[name])
        for name in ("cfg3", "cfg4"):
            cx = CONFIGS[name]
            sel = seco.spaco_select_chunks(cx.seed, 0, cx.n_chunks, cx.spaco_t)
            others[f"{name}_spaco_t{cx.spaco_t}"] = other_workload(cx, selected=sel)
        out["other_workloads"] = others

    if not args.no_layer32k and cfg.dtype == "bf16":
        # seconds per 32K-token layer: 16 chunks of 2048, t = 4
        L = None
        torch.cuda.empty_cache()
        out["sec_per_32k_layer"] = layer_seconds(CONFIGS["cfg3"])

    if oracle_units:
        # The oracle, as it stands, on whole (batch, KV head) units of the same workload and the same arrays the GPU
        # was given: the complete Alg. 1 loop of the unit (every forward and backward call), timed on the host cores;
        # its results are then compared element by element with what the last timed GPU step left for that unit.
        from oracle import attention as A
        try:
            from threadpoolctl import threadpool_info
            cores = max((p.get("num_threads", 1) for p in threadpool_info()), default=1)
        except Exception:
            cores = len(os.sched_getaffinity(0))
        unit_flops = 14 * sum(pairs(j, C) for j in range(k_chunks)) * D * G
        el, done = 0.0, []
        errs = {n: 0.0 for n in TOL[cfg.dtype]}
        errs_floor = dict(errs)
        for u in oracle_units:
            if u in done:
                continue
            h = host_units[u]
            xq, xdo = np.stack(h["q"])[None], np.stack(h["do"])[None]
            xk, xv = h["k"][0][None, None], h["v"][0][None, None]
            t_unit = time.perf_counter()
            ref = A.seco_layer(xq, xk, xv, xdo, C, scale)
            el += time.perf_counter() - t_unit
            done.append(u)
            for n, r in zip(("o", "lse", "dq", "gk", "gv"), ref):
                x = gpu_units[u][n]
                top = max(np.abs(r).max(), 1e-30)
                errs[n] = max(errs[n], float(np.abs(x - r).max() / top))
                errs_floor[n] = max(errs_floor[n], float((np.abs(x - r) / np.maximum(np.abs(r), 1e-3 * top)).max()))
            if el >= 10:          # bounded: about 10 - 30 s of oracle time
                break
        out["cpu_baseline"] = {"value": round(unit_flops * len(done) / el / 1e12, 5), "unit": "TFLOP/s",
                               "cores": int(cores), "kind": "oracle",
                               "sample": f"fp64 NumPy oracle, the whole Alg. 1 loop (forward + backward of all {k_chunks} "
                                         f"chunks) of {len(done)} of the {B * Hkv} (batch, KV head) units of {cfg.name} "
                                         f"{done}, {G} query heads each, {el:.1f} s",
                               "host_cores_available": len(os.sched_getaffinity(0))}
        tol = TOL[cfg.dtype]
        out["parity"] = {"against": "the oracle's results for the units above, same host arrays on both sides, GPU "
                                    "outputs of the last timed step, every element of the units",
                         "units": [list(u) for u in done],
                         "max_rel_err": {n: float(f"{e:.3e}") for n, e in errs.items()},
                         "max_elementwise_rel_err_floor_1e-3": {n: float(f"{e:.3e}") for n, e in errs_floor.items()},
                         "tolerance": tol, "pass": all(errs[n] <= tol[n] for n in tol)}

    if args.hbm_kernels:
        # the HBM-bound helpers on this configuration's buffers: bytes moved / time against the 8 TB/s of HBM3E
        Lh = Layer(cfg)
        j = k_chunks - 1
        knew = torch.randn(B, C, Hkv, D, device=dev).to(tdt).transpose(1, 2)
        dk = torch.empty(B, C, Hkv, D, device=dev, dtype=tdt).transpose(1, 2)
        dv = torch.empty_strided(dk.size(), dk.stride(), device=dev, dtype=tdt)
        g2 = torch.zeros_like(Lh.gk)
        eb = 2 if cfg.dtype == "bf16" else 4
        gbytes = Lh.gk.numel() * 4
        cases = {
            "kvgrad_zero": (lambda: seco.kvgrad_zero(Lh.gk, Lh.gv), 2 * gbytes),
            "kvgrad_accumulate": (lambda: seco.kvgrad_accumulate(Lh.gk, Lh.gv, g2, g2, 2.0), 2 * 3 * gbytes),
            "kv_append": (lambda: seco.kv_append(knew, knew, Lh.kc, Lh.vc, j * C), 2 * 2 * knew.numel() * eb),
            "kvgrad_readout": (lambda: seco.kvgrad_readout(Lh.gk, Lh.gv, j * C, C, tdt, d_k=dk, d_v=dv),
                               2 * knew.numel() * (4 + eb)),
        }
        n_rows = (1 << 30) // (Hkv * D * 4)
        big_dst = torch.zeros(1, Hkv, n_rows, D, device=dev, dtype=torch.float32)
        big_src = torch.ones_like(big_dst)
        cases["kvgrad_accumulate_1GiB"] = (lambda: seco.kvgrad_accumulate(big_dst, None, big_src, None, 0.5), 3 << 30)
        res = {"note": "only the 1 GiB case exceeds the 256 MB memory-side cache, i.e. streams from HBM; the others run "
                       "on this configuration's buffers and are partly cache-resident or launch-bound"}
        for name, (fn, nbytes) in cases.items():
            for _ in range(3):
                fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(20):
                fn()
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / 20
            res[name] = {"bytes": nbytes, "avg_us": round(us, 2), "GB_per_s": round(nbytes / us / 1e3, 1),
                         "frac_of_8TBps": round(nbytes / us / 1e3 / 8000.0, 3)}
        out["hbm_kernels"] = res
        del Lh

    if args.calibrate_copy:
        n_rows = (1 << 30) // (Hkv * D * 4)
        dst = torch.zeros(1, Hkv, n_rows, D, device=dev, dtype=torch.float32)
        src = torch.ones_like(dst)
        for _ in range(3):
            seco.kvgrad_accumulate(dst, None, src, None, 0.5)
        torch.cuda.synchronize()
        out["calibration"] = {"kernel": "kvgrad_kernel<true>", "launches": 3, "read_bytes_per_launch": 2 * dst.numel() * 4,
                              "write_bytes_per_launch": dst.numel() * 4}

    print(json.dumps(out))


if __name__ == "__main__":
    main()
