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
# HBM bytes per launch (mean over the 16 calls of cfg2) from rocprofv3 FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0; the
# factors come from a streaming kernel of known size in the same runs (profiles/cfg2_hbm_traffic_pmc.txt).
HBM_TRAFFIC_PER_LAUNCH = {("cfg2", "dkdv"): 254.7e6}


def pairs(j, C):
    """visible (row, col) pairs per head in the call for chunk j"""
    return C * j * C + C * (C + 1) // 2


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="cfg2")
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
        sys.exit("bench.py: this build is single-GPU by design (one process, one MI355X); run with --gpus 1")

    import torch
    import paper_2505_16710_amd as seco
    from workloads import CONFIGS

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    seco.load_library()
    dev = "cuda:0"
    cfg = CONFIGS[args.config]
    B, Hq, Hkv, D, N, C = cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.seq_len, cfg.chunk_len
    k_chunks = cfg.n_chunks
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    scale = cfg.scale

    def make_inputs(N):
        gen = torch.Generator(device=dev).manual_seed(cfg.seed)
        mk = lambda h: torch.randn(B, h, N, D, generator=gen, device=dev, dtype=torch.float32).to(tdt)
        return mk(Hq), mk(Hkv), mk(Hkv), mk(Hq)

    class Layer:
        """Device buffers of one layer; O is kept whole so that O and dO chunk views share strides."""

        def __init__(self, N, C):
            self.N, self.C, self.k = N, C, N // C
            self.q, self.kc, self.vc, self.do = make_inputs(N)
            self.o = torch.empty_like(self.q)
            self.lse = torch.empty(self.k, B, Hq, C, device=dev, dtype=torch.float32)   # kept per chunk
            self.dq = torch.empty_like(self.q)
            self.gk = torch.empty(B, Hkv, N, D, device=dev, dtype=torch.float32)
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

    L = Layer(N, C)

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
        "config": {"workload": f"{cfg.name}: SeCO fwd+bwd, one call pair per chunk, full gK/gV accumulation",
                   "batch": B, "n_q_heads": Hq, "n_kv_heads": Hkv, "head_dim": D, "seq_len": N, "chunk_len": C,
                   "n_chunks": k_chunks, "flops_per_step": flops_step},
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
        kern = {}
        kprof, ksteps = (warm_prof, 1) if warm_prof is not None else (prof, n_prof_steps)
        for kind, (ms, n) in kprof.items():
            if n:
                kern[kind] = {"launches": int(n), "avg_ms": round(ms / n, 5), "total_ms_per_step": round(ms / ksteps, 4)}
                if kind in alg:
                    kern[kind]["tflops"] = round(alg[kind] * ksteps / (ms * 1e-3) / 1e12, 2)
                    if cfg.dtype == "bf16":      # fraction of the dense bf16 matrix-core peak (algorithmic work)
                        kern[kind]["frac_of_mfma_peak"] = round(kern[kind]["tflops"] / PEAK_BF16_TFLOPS, 4)
        kern["measured_in"] = "last warm-up step (every launch bracketed by events)" if warm_prof is not None else "timed steps"
        if dom is None:
            dom = max(alg, key=lambda kd: prof[kd][0])
        ms, n = prof[dom]
        achieved = alg[dom] * n_prof_steps / (ms * 1e-3) / 1e12
        # bf16 kernels are dense MFMA contractions (2500 TFLOP/s); the fp32 parity kernels use the vector ALU only
        # (256 CUs x 128 lanes x 2 FLOP x 2.4 GHz = 157.3 TFLOP/s)
        bf16 = cfg.dtype == "bf16"
        peak = PEAK_BF16_TFLOPS if bf16 else 157.3
        out["roofline"] = {"bound": "mfma" if bf16 else "alu", "kernel": dom + ("_bf16_kernel" if bf16 else "_f32_kernel"),
                           "achieved": round(achieved, 2), "peak": peak, "unit": "TFLOP/s",
                           "frac": round(achieved / peak, 4),
                           "traffic": HBM_TRAFFIC_PER_LAUNCH.get((cfg.name, dom)),
                           "avg_launch_ms": round(ms / n, 5), "launches": int(n),
                           # matrix work the kernel executes per algorithmic FLOP (dK/dV computes S and dP again)
                           "executed_over_algorithmic": 2.0 if (bf16 and dom == "dkdv") else 1.0,
                           "executed_frac": round(achieved * (2.0 if (bf16 and dom == "dkdv") else 1.0) / peak, 4),
                           "measured_in": f"timed steps (HIP events around every launch of this kernel in {n_prof_steps} "
                                          f"of the {args.steps} timed steps)"}
        out["kernels"] = kern

    def layer_seconds(cx):
        """Seconds per layer of configuration cx under the two schedules (Alg. 1: k forwards, then forward +
        backward per chunk in reverse order; Alg. 2: k forwards, then forward + backward for the t selected
        chunks with factor k/t), best of 3."""
        Lx = Layer(cx.seq_len, cx.chunk_len)
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

        lse_full = torch.empty(B, Hq, cx.seq_len, device=dev, dtype=torch.float32)
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

        stats_t = torch.empty(2, B, Hq, (cx.seq_len + 3) // 4 * 4, device=dev, dtype=torch.float32)

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
            Lx = Layer(Nx, Cx)
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

    if not args.no_layer32k and cfg.dtype == "bf16":
        # seconds per 32K-token layer: 16 chunks of 2048, t = 4
        del L
        torch.cuda.empty_cache()
        out["sec_per_32k_layer"] = layer_seconds(CONFIGS["cfg3"])

    if not args.no_cpu_baseline:
        # the oracle, as it stands, on one independent (batch, KV head) unit of the same workload
        from oracle import attention as A
        from workloads import kv_group
        try:
            from threadpoolctl import threadpool_info
            cores = max((p.get("num_threads", 1) for p in threadpool_info()), default=1)
        except Exception:
            cores = len(os.sched_getaffinity(0))
        n_time = min(k_chunks, 16)
        chunks = list(range(k_chunks - 1, k_chunks - 1 - n_time, -1))
        done = units = 0
        fl = 0
        el = 0.0
        # whole (batch, KV head) units, one after the other, until about 10 s of oracle time have been spent
        for kvh in range(Hkv):
            grp = kv_group(cfg, 0, kvh)
            q = grp["q"][None].astype(np.float64)
            do = grp["do"][None].astype(np.float64)
            kk = grp["k"][None, None].astype(np.float64)
            vv = grp["v"][None, None].astype(np.float64)
            t_unit = time.perf_counter()
            for j in chunks:
                qs = q[:, :, j * C:(j + 1) * C]
                o_j, lse_j = A.chunk_attn_fwd(qs, kk, vv, j * C, scale)
                A.chunk_attn_bwd(qs, kk, vv, o_j, lse_j, do[:, :, j * C:(j + 1) * C], j * C, scale)
                done += 1
                fl += 14 * pairs(j, C) * D * (Hq // Hkv)
                if el + time.perf_counter() - t_unit > 25:
                    break
            unit_s = time.perf_counter() - t_unit
            el += unit_s
            units += 1
            if el >= 10 or el + unit_s > 25:
                break
        out["cpu_baseline"] = {"value": round(fl / el / 1e12, 5), "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
                               "sample": f"fp64 NumPy oracle, fwd+bwd of {done} chunk calls (the last {n_time} chunks of "
                                         f"{units} (batch, KV head) unit(s) of {cfg.name}, {Hq // Hkv} query heads each), "
                                         f"{el:.1f} s",
                               "host_cores_available": len(os.sched_getaffinity(0))}

    if args.hbm_kernels:
        # the HBM-bound helpers on this configuration's buffers: bytes moved / time against the 8 TB/s of HBM3E
        Lh = Layer(N, C)
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
