#!/usr/bin/env python3
"""Benchmark of the Swimba token-mixer hot path on one MI355X.

A step = one swimba_mixer_fwd call (router + mixing, cumsum + chunk state, state
scan, output: four launches) over one batch of the Mamba-2-130M-shaped workload, inputs resident in
HBM.  Prints ONE JSON line: whole-path tokens/s, the roofline of the dominant
kernel (timed alone with HIP events on the launch stream), per-kernel figures,
the decode step time, and the CPU oracle timed on the host cores.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 1|2|3] [--no-cpu]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# MI355X published peaks
PEAK_HBM_GBS = 8000.0
PEAK_BF16_TFLOPS = 2500.0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", type=int, default=1, choices=(1, 2, 3))
    ap.add_argument("--decode-steps", type=int, default=256)
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--no-decode", action="store_true")
    ap.add_argument("--proj", type=int, default=0, metavar="D_MODEL",
                    help="also time the routed expert in-projection from token features of this width")
    ap.add_argument("--xe", action="store_true",
                    help="also time the forward with one input stream per expert (rank-k injection)")
    ap.add_argument("--contrast", action="store_true",
                    help="also time the separated-SSM contrast (E state trajectories) on the same inputs")
    ap.add_argument("--stage", default=None,
                    help="run only this stage in the timed loop (for profilers): "
                         "mix|chunk_state|state_scan|output|step|copy")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "run with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2603_06938_amd import binding as sw
    from paper_2603_06938_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    w = synth.workload(args.workload)
    io = torch.bfloat16
    K, W = args.steps, args.warmup

    # ---- inputs: several identical-shape sets, rotated, so that a step does not find its
    # ---- inputs in the 256 MB last-level cache left by the previous step
    p = synth.make_inputs(w)

    def to_dev(a, is_io):
        t = torch.from_numpy(np.ascontiguousarray(a))
        return (t.to(io) if is_io else t).to(dev)

    base = {k: to_dev(v, k in ("x", "dt", "B_experts", "C_experts", "router_logits")) for k, v in p.items()}
    dims = sw.dims_of(base["x"], base["B_experts"], w.top_k, w.chunk)
    ws_bytes = sw.swimba_mixer_workspace_bytes(dims)
    set_bytes = sum(t.numel() * t.element_size() for t in base.values()) * 1 + ws_bytes \
        + base["x"].numel() * 2
    nsets = max(2, min(6, int(768e6 // set_bytes) + 1))
    sets = []
    for i in range(nsets):
        d = base if i == 0 else {k: v.clone() for k, v in base.items()}
        d["ws"] = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
        d["y"] = torch.empty_like(d["x"])
        d["h_final"] = torch.empty((w.batch, w.nheads, w.headdim, w.dstate), dtype=torch.float32, device=dev)
        sets.append(d)

    def step(i):
        d = sets[i % nsets]
        sw.swimba_mixer_fwd(d["x"], d["dt"], d["A"], d["D"], d["B_experts"], d["C_experts"],
                            d["router_logits"], w.top_k, w.chunk, None, y=d["y"], h_final=d["h_final"],
                            workspace=d["ws"])

    stages = {
        "mix": lambda d: sw.swimba_stage_mix(dims, d["B_experts"], d["C_experts"], d["router_logits"], d["ws"]),
        "chunk_state": lambda d: sw.swimba_stage_chunk_state(dims, d["x"], d["dt"], d["A"], d["B_experts"], d["ws"]),
        "state_scan": lambda d: sw.swimba_stage_state_scan(dims, None, d["h_final"], d["ws"]),
        "output": lambda d: sw.swimba_stage_output(dims, d["x"], d["dt"], d["D"], d["B_experts"],
                                                   d["C_experts"], d["y"], d["ws"]),
    }

    def time_loop(fn, n):
        """average ms per call of fn(i), measured with HIP events on the launch stream"""
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(n):
            fn(i)
        e1.record()
        e1.synchronize()
        return e0.elapsed_time(e1) / n

    # ---- profiler mode: one stage only --------------------------------------------------
    if args.stage:
        for i in range(nsets):
            step(i)   # every workspace holds valid router/cumsum/state data
        torch.cuda.synchronize()
        if args.stage == "copy":
            src = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
            dst = torch.empty_like(src)
            ms = time_loop(lambda i: sw.swimba_probe_copy(dst, src), K)
            print(json.dumps({"stage": "copy", "bytes_per_launch": src.numel(), "ms": ms,
                              "GBps_read_plus_write": 2 * src.numel() / ms / 1e6}))
        elif args.stage == "step":
            pass  # handled by the decode section below
        else:
            ms = time_loop(lambda i: stages[args.stage](sets[i % nsets]), K)
            print(json.dumps({"stage": args.stage, "ms": ms}))
            return 0
        if args.stage == "copy":
            return 0

    # ---- whole path ------------------------------------------------------------------------
    if not args.stage:
        for i in range(W):
            step(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(K):
            step(W + i)
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        ms_per_step = elapsed * 1e3 / K
        tokens_per_s = w.tokens * K / elapsed
        ev_ms = time_loop(lambda i: step(i), K)

    # ---- context: the same step on ONE input set (inputs and workspace found in the last-level
    # ---- cache), and what a plain copy and a register-resident MFMA loop reach on this GPU
    warm_ms = None
    achievable = None
    graph_ms = None
    if not args.stage:
        warm_ms = time_loop(lambda i: step(0), K)
        # the same K steps (input sets rotated as above) replayed from one HIP graph: no host
        # launch path between the kernels
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                for i in range(K):
                    step(i)
        torch.cuda.current_stream().wait_stream(side)
        graph.replay()
        torch.cuda.synchronize()
        graph_ms = time_loop(lambda i: graph.replay(), 3) / K
        del graph
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        time_loop(lambda i: sw.swimba_probe_copy(dst, src), 2)
        cms = time_loop(lambda i: sw.swimba_probe_copy(dst, src), 10)
        del src, dst
        sink = torch.zeros(1024 * 256, device=dev)
        time_loop(lambda i: sw.swimba_probe_mfma(sink, 1024, 2048), 2)
        mms = time_loop(lambda i: sw.swimba_probe_mfma(sink, 1024, 2048), 5)
        achievable = {"copy_GBps_read_plus_write": round(2 * (256 << 20) / cms / 1e6, 1),
                      "mfma_bf16_TFLOPs": round(1024 * 4 * 2048 * 32768.0 / mms / 1e9, 1)}

    # ---- per-kernel timing, each stage alone (workspaces already hold valid data) ----------
    T, H, P, N, G, E, k, Q = w.tokens, w.nheads, w.headdim, w.dstate, w.ngroups, w.nexperts, w.top_k, w.chunk
    nchunks = w.batch * ((w.seqlen + Q - 1) // Q)
    state_elems = nchunks * H * P * N
    # algorithmic work per launch: (HBM bytes, MFMA flops)
    NT = Q // 32
    cb_bytes = nchunks * G * (NT * (NT + 1) // 2) * 2048
    work = {
        # router + mixing: reads logits and the k active B and C rows; writes top-k, the mixed C
        # rows and the mixed B rows in two layouts (bf16)
        "mix": (T * (E * 2 + k * 8 + 2 * k * G * N * 2 + 3 * G * N * 2), 0.0),
        # cumsum + chunk state: reads x, dt, mixed B; writes cs and the bf16 chunk states
        "chunk_state": (T * (H * P * 2 + H * 2 + G * N * 2 + H * 4) + state_elems * 2, 2.0 * T * N * P * H),
        # reads the bf16 chunk states, writes the bf16 carried states in place, and h_final; the
        # same launch reads the mixed rows and writes the causal C.B^T tiles (dense count 2 T Q N G)
        "state_scan": (state_elems * (2 + 2) + w.batch * H * P * N * 4 + T * 2 * G * N * 2 + cb_bytes,
                       2.0 * T * Q * N * G),
        # reads x, dt, cs, carried states, mixed C, C.B^T tiles; writes y; masked (C B^T) X and
        # C.H per head on MFMA (dense counts; causally skipped tiles are counted)
        "output": (T * (2 * H * P * 2 + H * 2 + H * 4 + G * N * 2) + state_elems * 2 + cb_bytes,
                   2.0 * T * Q * P * H + 2.0 * T * N * P * H),
    }
    kernels = {}
    if not args.stage:
        for name, fn in stages.items():
            time_loop(lambda i: fn(sets[i % nsets]), 3)
            # K launches of the stage replayed from one HIP graph between two events: the launches
            # follow each other on the device without the host's launch path in between
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            sgraph = torch.cuda.CUDAGraph()
            with torch.cuda.stream(side):
                with torch.cuda.graph(sgraph, stream=side):
                    for i in range(K):
                        fn(sets[i % nsets])
            torch.cuda.current_stream().wait_stream(side)
            sgraph.replay()
            torch.cuda.synchronize()
            ms = time_loop(lambda i: sgraph.replay(), 3) / K
            del sgraph
            nbytes, flops = work[name]
            gbs, tfs = nbytes / ms / 1e6, flops / ms / 1e9
            # the roofline that bounds the kernel is the one with the larger time floor
            bound = "hbm" if nbytes / PEAK_HBM_GBS / 1e6 >= flops / PEAK_BF16_TFLOPS / 1e9 else "mfma"
            ach, peak, unit = (gbs, PEAK_HBM_GBS, "GB/s") if bound == "hbm" else (tfs, PEAK_BF16_TFLOPS, "TFLOP/s")
            kernels[name] = {"ms": round(ms, 5), "bound": bound, "achieved": round(ach, 2), "peak": peak,
                             "unit": unit, "frac": round(ach / peak, 4),
                             "hbm_GBps": round(gbs, 1), "mfma_TFLOPs": round(tfs, 1),
                             "mfma_frac": round(tfs / PEAK_BF16_TFLOPS, 4)}

    # ---- decode step (workload 4) ------------------------------------------------------------
    decode = None
    if not args.no_decode and (not args.stage or args.stage == "step"):
        wd = synth.workload(4)
        S = args.decode_steps
        pd = synth.make_decode_inputs(wd, steps=8)
        dd = {kk: to_dev(v, kk in ("x", "dt", "B_experts", "C_experts", "router_logits")) for kk, v in pd.items()}
        xs = dd["x"].transpose(0, 1).contiguous()
        dts = dd["dt"].transpose(0, 1).contiguous()
        Bs = dd["B_experts"].transpose(0, 1).contiguous()
        Cs = dd["C_experts"].transpose(0, 1).contiguous()
        gs = dd["router_logits"].transpose(0, 1).contiguous()
        # four independent state buffers, round-robin: 4 x 134 MB > last-level cache
        states = [dd["state"].clone() for _ in range(4)]
        yd = torch.empty_like(xs[0])
        dws = torch.empty(sw.swimba_step_workspace_bytes(
            sw.make_dims(wd.batch, 1, wd.nheads, wd.headdim, wd.dstate, wd.ngroups, wd.nexperts, wd.top_k, 0, io)),
            dtype=torch.uint8, device=dev)

        def dstep(i):
            t = i % 8
            sw.swimba_step(states[i % 4], xs[t], dts[t], dd["A"], dd["D"], Bs[t], Cs[t], gs[t], wd.top_k, y=yd, workspace=dws)

        time_loop(dstep, 8)
        ms = time_loop(dstep, S)
        dbytes = 2 * wd.batch * wd.nheads * wd.headdim * wd.dstate * 4 \
            + wd.batch * (2 * wd.nheads * wd.headdim * 2 + wd.nheads * 2 + wd.nexperts * 2
                          + 2 * wd.top_k * wd.ngroups * wd.dstate * 2)
        decode = {"workload": "decode_step: B64 H64 P64 N128 G1 E8 top2, fp32 state, bf16 io",
                  "us_per_step": round(ms * 1e3, 2), "steps": S, "tokens_per_s": round(wd.batch / ms * 1e3, 1),
                  "bound": "hbm", "achieved": round(dbytes / ms / 1e6, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                  "frac": round(dbytes / ms / 1e6 / PEAK_HBM_GBS, 4), "state_buffers_rotated": 4}
        # the same step with other router / group settings: G = 8 B/C groups (the long-sequence
        # layer's grouping), and 4 experts with top-1 routing (the paper's large model); random
        # device-side inputs of the same distributions, same state buffers
        variants = {}
        for vname, (vG, vE, vk) in {"G8_E8_top2": (8, 8, 2), "G1_E4_top1": (1, 4, 1)}.items():
            gen = torch.Generator(device=dev)
            gen.manual_seed(69384 + vG * 100 + vE)
            vB = (torch.randn((wd.batch, vE, vG, wd.dstate), generator=gen, device=dev) / wd.dstate ** 0.5).to(io)
            vC = (torch.randn((wd.batch, vE, vG, wd.dstate), generator=gen, device=dev) / wd.dstate ** 0.5).to(io)
            vg = torch.randn((wd.batch, vE), generator=gen, device=dev).to(io)
            vws = torch.empty(sw.swimba_step_workspace_bytes(
                sw.make_dims(wd.batch, 1, wd.nheads, wd.headdim, wd.dstate, vG, vE, vk, 0, io)),
                dtype=torch.uint8, device=dev)

            def vstep(i):
                sw.swimba_step(states[i % 4], xs[i % 8], dts[i % 8], dd["A"], dd["D"], vB, vC, vg, vk, y=yd, workspace=vws)

            time_loop(vstep, 8)
            vms = time_loop(vstep, S)
            variants[vname] = {"us_per_step": round(vms * 1e3, 2), "frac": round(dbytes / vms / 1e6 / PEAK_HBM_GBS, 4)}
        decode["variants"] = variants
        # several tokens per call (speculative / short-chunk decoding): same state bytes per call
        multi = {}
        for Lm in (4, 8):
            xm = dd["x"][:, :Lm].contiguous()
            dtm = dd["dt"][:, :Lm].contiguous()
            Bm = dd["B_experts"][:, :Lm].contiguous()
            Cm = dd["C_experts"][:, :Lm].contiguous()
            gm = dd["router_logits"][:, :Lm].contiguous()
            ym = torch.empty_like(xm)
            mws = torch.empty(sw.swimba_step_multi_workspace_bytes(
                sw.make_dims(wd.batch, Lm, wd.nheads, wd.headdim, wd.dstate, wd.ngroups, wd.nexperts, wd.top_k, 0, io)),
                dtype=torch.uint8, device=dev)

            def mstep(i):
                sw.swimba_step_multi(states[i % 4], xm, dtm, dd["A"], dd["D"], Bm, Cm, gm, wd.top_k, y=ym, workspace=mws)

            time_loop(mstep, 8)
            mms = time_loop(mstep, max(32, S // 4))
            multi["L%d" % Lm] = {"us_per_call": round(mms * 1e3, 2), "tokens_per_s": round(wd.batch * Lm / mms * 1e3, 1),
                                  "frac": round(dbytes / mms / 1e6 / PEAK_HBM_GBS, 4)}
        decode["multi_token"] = multi
        if args.stage == "step":
            print(json.dumps(decode))
            return 0

    # ---- separated-SSM contrast: E plain SSM passes through the same kernels --------------------
    contrast = None
    if args.contrast and not args.stage:
        d0 = sets[0]
        sws = torch.empty(sw.swimba_separated_workspace_bytes(dims), dtype=torch.uint8, device=dev)

        def sep(i):
            d = sets[i % nsets]
            sw.swimba_separated_fwd(d["x"], d["dt"], d["A"], d["D"], d["B_experts"], d["C_experts"],
                                    d["router_logits"], w.top_k, w.chunk, y=d["y"], workspace=sws)

        time_loop(sep, 2)
        ms = time_loop(sep, max(3, K // 5))
        contrast = {"what": "MoE of separated SSMs, %d state trajectories" % w.nexperts, "ms_per_step": round(ms, 4),
                    "tokens_per_s": round(w.tokens / ms * 1e3, 1), "slowdown_vs_mixed": round(ms / ev_ms, 2)}
        del sws, d0

    # ---- routed expert in-projection (upstream of the mixer): grouped GEMM on MFMA --------------
    proj_res = None
    if args.proj and not args.stage:
        Dm = args.proj
        gen = torch.Generator(device=dev)
        gen.manual_seed(69380 + 200 + args.workload)
        us = [torch.randn((w.batch, w.seqlen, Dm), generator=gen, device=dev).to(io) for _ in range(3)]
        WBs = (torch.randn((E, G, N, Dm), generator=gen, device=dev) / Dm ** 0.5).to(io)
        WCs = (torch.randn((E, G, N, Dm), generator=gen, device=dev) / Dm ** 0.5).to(io)
        pws = torch.empty(sw.swimba_expert_proj_workspace_bytes(dims, Dm), dtype=torch.uint8, device=dev)

        def proj_step(i):
            d = sets[i % nsets]
            sw.swimba_expert_proj(us[i % 3], WBs, WCs, d["router_logits"], w.top_k, B_experts=d["B_experts"],
                                  C_experts=d["C_experts"], workspace=pws)

        time_loop(proj_step, 3)
        ms = time_loop(proj_step, K)
        pflops = 2.0 * T * k * Dm * 2 * G * N
        pbytes = T * (Dm * 2 + E * 2 + k * 2 * G * N * 2) + 2 * E * G * N * Dm * 2
        proj_res = {"what": "routed expert in-projection, d_model %d -> B, C rows of the top-%d experts" % (Dm, k),
                    "ms": round(ms, 5), "mfma_TFLOPs": round(pflops / ms / 1e9, 1),
                    "mfma_frac": round(pflops / ms / 1e9 / PEAK_BF16_TFLOPS, 4),
                    "hbm_GBps": round(pbytes / ms / 1e6, 1), "hbm_frac": round(pbytes / ms / 1e6 / PEAK_HBM_GBS, 4)}
        # the router's linear map on the same features
        Wg = (torch.randn((E, Dm), generator=gen, device=dev) / Dm ** 0.5).to(io)
        lg = torch.empty((w.batch, w.seqlen, E), dtype=io, device=dev)
        time_loop(lambda i: sw.swimba_router_linear(us[i % 3], Wg, lg), 3)
        rl_ms = time_loop(lambda i: sw.swimba_router_linear(us[i % 3], Wg, lg), K)
        proj_res["router_linear"] = {"ms": round(rl_ms, 5),
                                     "hbm_GBps": round(T * (Dm * 2 + E * 2) / rl_ms / 1e6, 1)}
        # token features -> y in one call, selected streams only (no tensor with an expert axis),
        # against projection into the dense layout followed by the mixer forward
        fws = torch.empty(sw.swimba_mixer_proj_workspace_bytes(dims, Dm), dtype=torch.uint8, device=dev)

        def fused_step(i):
            d = sets[i % nsets]
            sw.swimba_mixer_fwd_proj(us[i % 3], WBs, WCs, d["x"], d["dt"], d["A"], d["D"], d["router_logits"],
                                     w.top_k, w.chunk, y=d["y"], h_final=d["h_final"], workspace=fws)

        def dense_step(i):
            proj_step(i)
            step(i)

        time_loop(fused_step, 3)
        fms = time_loop(fused_step, K)
        time_loop(dense_step, 3)
        dms = time_loop(dense_step, K)
        proj_res["features_to_y"] = {"selected_streams_ms": round(fms, 5), "dense_streams_ms": round(dms, 5),
                                     "tokens_per_s": round(T / fms * 1e3, 1)}
        # the projection overwrote the synthetic expert rows of every set with its own values
        del us, WBs, WCs, pws, fws

    # ---- one input stream per expert: k rank-1 passes through the same kernels ------------------
    xe_res = None
    if args.xe and not args.stage:
        gen = torch.Generator(device=dev)
        gen.manual_seed(69380 + 100 + args.workload)
        xes = [torch.randn((w.batch, w.seqlen, E, H, P), generator=gen, device=dev, dtype=torch.float32).to(io)
               for _ in range(2)]
        xws = torch.empty(sw.swimba_mixer_xe_workspace_bytes(dims), dtype=torch.uint8, device=dev)

        def xe_step(i):
            d = sets[i % nsets]
            sw.swimba_mixer_fwd_xe(xes[i % 2], d["dt"], d["A"], d["D"], d["B_experts"], d["C_experts"],
                                   d["router_logits"], w.top_k, w.chunk, None, y=d["y"], h_final=d["h_final"],
                                   workspace=xws)

        time_loop(xe_step, 3)
        ms = time_loop(xe_step, max(5, K // 2))
        xe_res = {"what": "mixed forward with one x stream per expert (rank-%d injection), %d passes" % (k, k),
                  "ms_per_step": round(ms, 4), "tokens_per_s": round(w.tokens / ms * 1e3, 1),
                  "slowdown_vs_shared_x": round(ms / ev_ms, 2)}
        del xes, xws

    # ---- CPU oracle on the host cores (reported baseline only) -------------------------------
    cpu = None
    if not args.no_cpu:
        from oracle import swimba_oracle as orc
        runs, t_cpu = 0, 0.0
        while t_cpu < 10.0 and runs < 400:      # about 10 s of host work, whatever the workload
            t0 = time.perf_counter()
            orc.mixer_fwd(p["x"], p["dt"], p["A"], p["D"], p["B_experts"], p["C_experts"],
                          p["router_logits"], w.top_k)
            t_cpu += time.perf_counter() - t0
            runs += 1
        cpu = {"value": round(w.tokens * runs / t_cpu, 1), "unit": "tokens/s", "cores": orc.num_threads(),
               "kind": "oracle",
               "sample": "the whole %s batch (%d tokens), %d passes, fp64 sequential recurrence, "
                         "OpenMP over (batch, head)" % (w.name, w.tokens, runs)}

    dom = max(kernels, key=lambda n: kernels[n]["ms"])
    roof = {kk: kernels[dom][kk] for kk in ("bound", "achieved", "peak", "unit", "frac")}
    roof["kernel"] = dom
    roof["mfma_frac"] = kernels[dom]["mfma_frac"]
    # HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (scaled by a
    # copy kernel of known size); recorded in profiles/ by hand after a counter run
    roof["traffic"] = None
    tf = os.path.join(ROOT, "profiles", "hbm_traffic_%s_%s.txt" % (dom, w.name))
    if os.path.exists(tf):
        for line in open(tf):
            if line.startswith("traffic_bytes_per_launch:"):
                roof["traffic"] = float(line.split(":")[1])
    out = {
        "metric": "Swimba mixer fwd tokens/s + % peak MFMA/HBM at 1 MI355X; decode step us",
        "value": round(tokens_per_s, 1),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": W,
        "ms_per_step": round(ms_per_step, 5),
        "ms_per_step_hip_events": round(ev_ms, 5),
        "ms_per_step_warm_cache": round(warm_ms, 5),
        "ms_per_step_hip_graph": round(graph_ms, 5),
        "peaks": {"hbm_GBps": PEAK_HBM_GBS, "mfma_bf16_TFLOPs": PEAK_BF16_TFLOPS},
        "achievable": achievable,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "%s: B%d L%d H%d P%d N%d G%d E%d top%d chunk%d, bf16 io / fp32 accumulate"
                               % (w.name, w.batch, w.seqlen, H, P, N, G, E, k, Q),
                   "input_sets_rotated": nsets},
        "roofline": roof,
        "kernels": kernels,
        "decode": decode,
        "cpu_baseline": cpu,
    }
    if contrast:
        out["separated_contrast"] = contrast
    if xe_res:
        out["expert_x"] = xe_res
    if proj_res:
        out["expert_proj"] = proj_res
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
