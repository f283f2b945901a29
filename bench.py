#!/usr/bin/env python3
"""Benchmark of the decomposed-layer hot path on one MI355X.

A "step" is one pass of the whole hot path of one decoder block over one batch of T
tokens: deinfer_lowrank_qkv -> deinfer_lowrank_linear (o) -> deinfer_lowrank_gateup_silu
-> deinfer_lowrank_down, enqueued back to back on one stream (attention core, norms,
RoPE and residual adds are not part of the path and are not run).  Inputs are seeded
synthetic tensors of the named shape, resident in HBM before the timed region.  To keep
the 256 MB last-level cache from serving the weights, consecutive steps rotate through
several independent copies of the packed weights (>= 1.5 GB in total).  The K steps are
timed twice, replayed from a captured HIP graph and with every call launched directly, and
the faster of the two is reported (config.launch names it, config.launch_ms holds both).

Prints ONE JSON line: metric, value (tokens/s of the step), ms_per_step, per-call timings,
"roofline" (the dominant launch of the call with the most work, timed with HIP events that the library
records around that launch on the launch stream, against the HBM or bf16 MFMA peak; "step_frac" inside
it is the whole step against the same peak; "measured_ceiling" is what a plain read of the same
bytes, or a loop of nothing but matrix products, reaches on the same device) and "cpu_baseline" (the
fp64 oracle on the host's cores, on a bounded sample of the same workload).

The default workload is the largest single-GPU configuration, the Llama-70B-shaped layer with GQA at
60 % parameter reduction, at its decode size (T = 128).  The default run adds, from child processes,
"prefill" (the same layer at T = 4096, with its own ms_per_step and MFMA roofline) and
"llama7b_keep80_decode_T64" (the 7B-shaped block at 64 tokens, its sweep over 1 / 8 / 32 tokens and
"second_row_r2357": the same block with the ranks the configuration prints instead of the ones its
rule gives).

--workload llama7b_keep80_kv_rebuild times a different step: keys and values of 8192 cached
tokens rebuilt from the paged low-rank cache (compacting copy, upward projections at the
buffer's capacity, rotary embedding of the keys), one captured graph.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

WORKLOADS = {
    # name: (block shape, default T, bound)
    "llama7b_keep80_decode": ("llama7b_keep80", 64, "hbm"),
    "llama7b_keep60_prefill": ("llama7b_keep60", 8192, "mfma"),
    "llama7b_keep40_prefill": ("llama7b_keep40", 8192, "mfma"),
    "llama13b_keep60_mixed": ("llama13b_keep60", 8256, "mfma"),
    # a chunk of a chunked prefill: between the decode sizes and the large prefill (first stages split over k)
    "llama7b_keep60_chunked_prefill": ("llama7b_keep60", 512, "mfma"),
    "llama70b_keep40_decode": ("llama70b_keep40", 128, "hbm"),
    "llama70b_keep40_prefill": ("llama70b_keep40", 4096, "mfma"),
    # keys and values of cached tokens rebuilt from the paged low-rank cache (a different step, see kv_rebuild)
    "llama7b_keep80_kv_rebuild": ("llama7b_keep80", 8192, "mfma"),
    # non-GLU block: the MLP is act(x U1 V1 + b1) then a second pair with bias (deinfer_lowrank_linear_act)
    # what ONE rank of an 8-way tensor-parallel group runs on its shard (no exchange is timed)
    "llama70b_keep40_tp8_rank_decode": ("llama70b_keep40", 128, "hbm"),
    "llama70b_keep40_tp8_rank_prefill": ("llama70b_keep40", 4096, "mfma"),
    "opt30b_keep60_decode": ("opt30b_keep60", 64, "hbm"),
    "opt30b_keep60_prefill": ("opt30b_keep60", 4096, "mfma"),
}
# The default run: the largest single-GPU configuration (70B-shaped layer with GQA, 60 % parameter
# reduction) at its decode size; its prefill size and the 7B-shaped block at 64 tokens are timed in child
# processes and reported as secondary objects of the same JSON line.
DEFAULT_WORKLOAD = "llama70b_keep40_decode"
HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 MFMA, published


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD, choices=sorted(WORKLOADS))
    ap.add_argument("--T", type=int, default=0, help="tokens per step (0 = the workload's default)")
    ap.add_argument("--launch", default="auto", choices=["auto", "graph", "direct"],
                    help="replay the step from a captured HIP graph, launch each call directly, or (auto) time the "
                         "K steps both ways and report the faster one (both times are kept in config.launch_ms)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--sweep", action="store_true", help="also time the other decode batch sizes")
    ap.add_argument("--seed", type=int, default=1)
    ap.add_argument("--dtype", default="bf16", choices=["bf16", "f16"], help="storage type of weights, activations and outputs")
    ap.add_argument("--rank-override", default="", help="e.g. gate=2357,up=2357,down=2357: ranks not taken from the rule")
    ap.add_argument("--traffic-calibration", type=int, default=0, metavar="MIB",
                    help="do nothing but five plain device-to-device copies of MIB MiB (a kernel of known traffic, for "
                         "scaling the FETCH_SIZE / WRITE_SIZE counters of rocprofv3 --pmc) and exit")
    ap.add_argument("--no-extra-rows", action="store_true",
                    help="default workload only: skip the secondary rows (the same layer at its prefill size, the 7B-shaped "
                         "block at 64 tokens with its sweep over smaller batches)")
    ap.add_argument("--no-second-row", action="store_true",
                    help="skip the second row of the default workload (the ranks that the configuration prints, 2357)")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); --gpus %d is not "
              "supported, run with --gpus 1" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import synth_inputs as si
    import paper_2604_17709_amd as dn

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    if args.traffic_calibration > 0:
        n = args.traffic_calibration << 20
        src = torch.empty(n, dtype=torch.uint8, device="cuda").fill_(3)
        dst = torch.empty(n, dtype=torch.uint8, device="cuda")
        torch.cuda.synchronize()
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"traffic_calibration": "5 copies", "bytes_read_per_copy": n, "bytes_written_per_copy": n}))
        return
    L = dn.lib()            # raises if the HIP library is missing: no fallback

    block_name, T_default, bound = WORKLOADS[args.workload]
    T = args.T or T_default
    if (args.workload.endswith("kv_rebuild") or "_tp8_rank_" in args.workload) and args.dtype != "bf16":
        print("bench.py: --dtype f16 is for the block workloads", file=sys.stderr)
        sys.exit(2)
    if args.workload.endswith("kv_rebuild"):
        return kv_rebuild(args, L, si.BLOCKS[block_name], T)
    if "_tp8_rank_" in args.workload:
        return tp_rank(args, L, si.BLOCKS[block_name], T, 8, bound if T > 128 else "hbm")
    if T <= 128:
        bound = "hbm"
    import dataclasses
    shape = dataclasses.replace(si.BLOCKS[block_name], dtype=args.dtype)
    tdt = torch.float16 if args.dtype == "f16" else torch.bfloat16
    proj = shape.projections()
    rho = 1.0 - shape.keep_num / shape.keep_den
    ranks = {p: dn.deinfer_rank_for_ratio(m, n, rho) for p, (m, n) in proj.items()}
    for item in filter(None, args.rank_override.split(",")):
        name, val = item.split("=")
        ranks[name] = int(val)

    # ---------------------------------------------------------------- inputs (host, seeded)
    t0 = time.time()
    host = si.block_tensors(shape, ranks, max(T, 1), args.seed)

    def dev(t):
        return torch.from_numpy(t.bits.view(np.int16)).cuda().view(tdt)

    params = sum(ranks[p] * (m + n) for p, (m, n) in proj.items())
    weight_bytes = 2 * params
    n_copies = max(2, int(np.ceil(1.5e9 / weight_bytes)))
    packed0 = {}
    for p in proj:
        raw = dn.raw_pair(dev(host["U_" + p]), dev(host["V_" + p]), rho)
        packed0[p] = dn.deinfer_pack_factors(raw)
        torch.cuda.synchronize()
        del raw
    copies = [packed0]
    for _ in range(1, n_copies):
        c = {}
        for p, pk in packed0.items():
            buf = pk._keep[0].clone()
            d = dn.Factors.from_buffer_copy(pk.desc)
            d.U = buf.data_ptr() + (pk.desc.U - pk._keep[0].data_ptr())
            d.V = buf.data_ptr() + (pk.desc.V - pk._keep[0].data_ptr())
            c[p] = dn.Pair(d, [buf])
        copies.append(c)
    x = dev(host["x"]); a = dev(host["a"]); h_in = dev(host["h_in"])
    if not shape.glu:
        b_gate = dev(host["b_gate"]).reshape(-1); b_down = dev(host["b_down"]).reshape(-1)
    bf = tdt
    q = torch.empty((T, proj["q"][1]), dtype=bf, device="cuda")
    k = torch.empty((T, proj["k"][1]), dtype=bf, device="cuda")
    v = torch.empty((T, proj["v"][1]), dtype=bf, device="cuda")
    o = torch.empty((T, proj["o"][1]), dtype=bf, device="cuda")
    h = torch.empty((T, proj["gate"][1]), dtype=bf, device="cuda")
    y = torch.empty((T, proj["down"][1]), dtype=bf, device="cuda")
    ws_bytes = max(dn.deinfer_workspace_bytes(T, [packed0["q"], packed0["k"], packed0["v"]]),
                   dn.deinfer_workspace_bytes(T, [packed0["o"]]),
                   dn.deinfer_workspace_bytes(T, [packed0["gate"], packed0["up"]] if shape.glu else [packed0["gate"]]),
                   dn.deinfer_workspace_bytes(T, [packed0["down"]]))
    ws = dn.Workspace(ws_bytes)
    torch.cuda.synchronize()
    setup_s = time.time() - t0

    # ---------------------------------------------------------------- the step (pre-marshalled C calls)
    def ld(t):
        return int(t.stride(0))

    def make_calls(c, stream_handle):
        B = ctypes.byref
        wsp, wsn = ws.buf.data_ptr(), ws.nbytes
        return {
            "qkv": (L.deinfer_lowrank_qkv, (x.data_ptr(), T, ld(x), B(c["q"].desc), B(c["k"].desc), B(c["v"].desc),
                                            q.data_ptr(), ld(q), k.data_ptr(), ld(k), v.data_ptr(), ld(v),
                                            None, 0, None, 0, wsp, wsn, stream_handle)),
            "o": (L.deinfer_lowrank_linear, (a.data_ptr(), T, ld(a), B(c["o"].desc), o.data_ptr(), ld(o), wsp, wsn, stream_handle)),
            "gateup": ((L.deinfer_lowrank_gateup_silu, (x.data_ptr(), T, ld(x), B(c["gate"].desc), B(c["up"].desc),
                                                        h.data_ptr(), ld(h), wsp, wsn, stream_handle)) if shape.glu else
                       (L.deinfer_lowrank_linear_act, (x.data_ptr(), T, ld(x), B(c["gate"].desc), b_gate.data_ptr(), dn.ACT_RELU,
                                                       h.data_ptr(), ld(h), wsp, wsn, stream_handle))),
            "down": ((L.deinfer_lowrank_down, (h_in.data_ptr(), T, ld(h_in), B(c["down"].desc), y.data_ptr(), ld(y), wsp, wsn, stream_handle))
                     if shape.glu else
                     (L.deinfer_lowrank_linear_act, (h_in.data_ptr(), T, ld(h_in), B(c["down"].desc), b_down.data_ptr(), dn.ACT_NONE,
                                                     y.data_ptr(), ld(y), wsp, wsn, stream_handle))),
        }

    def run_calls(calls, names=("qkv", "o", "gateup", "down")):
        for n in names:
            fn, a_ = calls[n]
            rc = fn(*a_)
            if rc != 0:
                raise RuntimeError("%s failed: %s" % (n, dn.last_error()))

    stream = torch.cuda.Stream()          # default priority
    sh = int(stream.cuda_stream)
    calls = [make_calls(c, sh) for c in copies]

    graphs = None
    launch_mode = "graph" if args.launch == "auto" else args.launch
    with torch.cuda.stream(stream):
        run_calls(calls[0])
    stream.synchronize()
    ws.check(stream)
    if launch_mode == "graph":
        try:
            graphs = []
            for i in range(n_copies):
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=stream):
                    run_calls(calls[i])
                graphs.append(g)
        except Exception as e:  # noqa: BLE001 - report and fall back to direct launches
            print("graph capture failed (%s); using direct launches" % e, file=sys.stderr)
            graphs = None
            launch_mode = "direct"

    def step(i):
        if graphs is not None:
            graphs[i % n_copies].replay()
        else:
            run_calls(calls[i % n_copies])

    ev_ms = {}                     # the same region between two events on the launch stream (device time only)

    def timed(fn, n, tag=None):
        ea = torch.cuda.Event(enable_timing=True); eb = torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t_a = time.perf_counter()
        with torch.cuda.stream(stream):
            ea.record(stream)
            for i in range(n):
                fn(i)
            eb.record(stream)
        stream.synchronize()
        torch.cuda.synchronize()
        t_b = time.perf_counter()
        if tag is not None:
            ev_ms[tag] = round(ea.elapsed_time(eb) / n, 5)
        return (t_b - t_a) / n

    with torch.cuda.stream(stream):
        for i in range(args.warmup):
            step(i)
    stream.synchronize()
    sec_per_step = timed(step, args.steps, launch_mode)
    launch_ms = {launch_mode: round(sec_per_step * 1e3, 5)}
    if args.launch == "auto" and graphs is not None:
        # the same K steps with every call launched directly (on this ROCm a replayed graph node costs a
        # little more than a launch the host has queued ahead); the faster way is the one reported
        direct = lambda i: run_calls(calls[i % n_copies])
        with torch.cuda.stream(stream):
            for i in range(args.warmup):
                direct(i)
        stream.synchronize()
        sec_direct = timed(direct, args.steps, "direct")
        launch_ms["direct"] = round(sec_direct * 1e3, 5)
        if sec_direct < sec_per_step:
            sec_per_step, launch_mode, step = sec_direct, "direct", direct
    ws.check(stream)
    # spread of the step time: the same steps once more in ten chunks, each timed on its own (the value
    # reported above is the mean over the K steps of the timed run; this says how far chunks scatter)
    n_chunk = max(1, args.steps // 10)
    chunk_ms = sorted(timed(step, n_chunk) * 1e3 for _ in range(10))
    spread = {"steps_per_chunk": n_chunk, "min": round(chunk_ms[0], 5), "median": round(0.5 * (chunk_ms[4] + chunk_ms[5]), 5),
              "max": round(chunk_ms[-1], 5)}

    # ---------------------------------------------------------------- per-call timing (HIP events on the launch stream)
    def time_call(name, n):
        e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
        with torch.cuda.stream(stream):
            for i in range(min(10, n)):
                run_calls(calls[i % n_copies], (name,))
            e0.record(stream)
            for i in range(n):
                run_calls(calls[i % n_copies], (name,))
            e1.record(stream)
        stream.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / n

    s = 2
    def call_bytes(names, outs):
        wb = s * sum(ranks[p] * (proj[p][0] + proj[p][1]) for p in names)
        return wb + s * T * proj[names[0]][0] + s * T * sum(outs)
    def call_flops(names):
        return 2.0 * T * sum(ranks[p] * (proj[p][0] + proj[p][1]) for p in names)
    call_defs = {
        "qkv": (("q", "k", "v"), [proj["q"][1], proj["k"][1], proj["v"][1]]),
        "o": (("o",), [proj["o"][1]]),
        "gateup": (("gate", "up") if shape.glu else ("gate",), [proj["gate"][1]]),
        "down": (("down",), [proj["down"][1]]),
    }
    n_call = max(20, min(args.steps, 200))
    per_call = {}
    for name, (ps, outs) in call_defs.items():
        sec = time_call(name, n_call)
        per_call[name] = {"us": round(sec * 1e6, 2), "bytes": call_bytes(ps, outs), "flops": call_flops(ps),
                          "GBs": round(call_bytes(ps, outs) / sec / 1e9, 1),
                          "TFLOPs": round(call_flops(ps) / sec / 1e12, 2)}
    # ---- the dominant kernel: the internal launches of the slowest call, each timed with HIP
    # events that the library records around that one launch on the launch stream
    # (the call with the most algorithmic work of the bounding kind, the slower one of equals: it is
    # also the slowest call in an undisturbed run, and the choice does not flip under a profiler)
    dom = max(per_call, key=lambda n: (per_call[n]["bytes" if bound == "hbm" else "flops"], per_call[n]["us"]))
    ps, outs = call_defs[dom]
    decode = T <= 128
    kinds = ({"down": dn.PROF_DECODE_DOWN, "reduce": dn.PROF_DECODE_REDUCE, "up": dn.PROF_DECODE_UP} if decode
             else {"down": dn.PROF_PREFILL_DOWN, "up": dn.PROF_PREFILL_UP})
    e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
    with torch.cuda.stream(stream):
        e0.record(stream); e1.record(stream)
    stream.synchronize()

    def time_kernel(kind, n):
        L.deinfer_set_profile_events(kind, e0.cuda_event, e1.cuda_event)
        tot, cnt = 0.0, 0
        with torch.cuda.stream(stream):
            for i in range(n + 3):
                # twice in a row on different weight copies: the events keep the brackets of the second
                # call, whose launches were queued while the first ran (a launch that finds the device
                # idle after a synchronisation takes 10 - 15 us longer between its events)
                run_calls(calls[i % n_copies], (dom,))
                run_calls(calls[(i + 1) % n_copies], (dom,))
                stream.synchronize()
                if i >= 3:
                    tot += e0.elapsed_time(e1); cnt += 1
        L.deinfer_set_profile_events(0, None, None)
        return tot * 1e-3 / cnt

    n_k = max(10, min(args.steps, 50))
    ktimes = {k: time_kernel(v, n_k) for k, v in kinds.items()}
    w_in = s * sum(ranks[p] * proj[p][0] for p in ps)       # U factors of the call
    w_out = s * sum(ranks[p] * proj[p][1] for p in ps)      # V factors of the call
    kbytes = {"down": w_in + s * T * proj[ps[0]][0], "up": w_out + s * T * sum(outs),
              "reduce": 6 * T * sum(ranks[p] for p in ps)}
    kflops = {"down": 2.0 * T * sum(ranks[p] * proj[p][0] for p in ps),
              "up": 2.0 * T * sum(ranks[p] * proj[p][1] for p in ps), "reduce": 0.0}
    if not decode:
        # the upward projections of all pairs of the call are one launch (the GLU call: both products
        # of a tile in one workgroup, h stored once)
        kbytes["up"] = w_out + s * T * sum(ranks[p] for p in ps) + s * T * sum(outs)
    # the dominant launch: the one with the most algorithmic work of the bounding kind (the slower of equals)
    kwork = kbytes if bound == "hbm" else kflops
    kdom = max(ktimes, key=lambda k: (kwork[k], ktimes[k]))
    ksec = ktimes[kdom]
    entry = {"qkv": "qkv", "o": "linear", "gateup": "gateup_silu" if shape.glu else "linear_act",
             "down": "down" if shape.glu else "linear_act"}[dom]
    # HBM bytes per launch of the dominant kernel from the rocprofv3 counter runs of the same command
    # (FETCH_SIZE, WRITE_SIZE, scaled by a copy of known size): a committed summary, not measured in this run
    traffic, traffic_source = None, None
    tfile = os.path.join(ROOT, "profiles", "hbm_traffic_%s_T%d.txt" % (args.workload, T))
    if os.path.exists(tfile):
        for line in open(tfile):
            if line.startswith("traffic_bytes_per_launch"):
                traffic = float(line.split("=")[1])
                traffic_source = "profiles/" + os.path.basename(tfile)
    if bound == "hbm":
        ach = kbytes[kdom] / ksec / 1e9
        roofline = {"bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": round(ach / HBM_PEAK_GBS, 4), "traffic": traffic}
    else:
        ach = kflops[kdom] / ksec / 1e12
        roofline = {"bound": "mfma", "achieved": round(ach, 1), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(ach / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": traffic}
    # (which kernel a launch is: the tile kernels up to 8 tokens, the streaming kernels up to 128 - for the
    # GLU call's second stage skinny_glu_kernel where its workgroups fill most of the device, else
    # skinny_kernel / stream_kernel -, prefill_kernel beyond; the rocprofv3 summaries under profiles/ name it)
    tiles16 = lambda n: (n + 15) // 16
    small = (T <= 8 and sum(tiles16(ranks[p]) for p in ps) <= 256 and sum(tiles16(proj[p][1]) for p in ps) <= 1024)
    kname = ("decode_kernel" if small else "skinny_glu_kernel / skinny_kernel" if (dom == "gateup" and shape.glu and kdom == "up" and T > 16)
             else "skinny_kernel / stream_kernel") if decode else "prefill_kernel"
    roofline["kernel"] = "%s (%s-projection launch of deinfer_lowrank_%s)" % (kname, kdom, entry)
    roofline["traffic_source"] = traffic_source
    roofline["avg_launch_us"] = round(ksec * 1e6, 2)
    roofline["algorithmic_bytes_per_launch"] = kbytes[kdom]
    roofline["algorithmic_flops_per_launch"] = kflops[kdom]
    roofline["launches_of_this_call_us"] = {k: round(v * 1e6, 2) for k, v in ktimes.items()}

    # ---- measured ceilings of this device beside the published ones (plain kernels of the library
    # that do nothing but read, or nothing but multiply; timed with events on the launch stream)
    def events_us(fn, n, warm=3):
        a0 = torch.cuda.Event(enable_timing=True); a1 = torch.cuda.Event(enable_timing=True)
        with torch.cuda.stream(stream):
            for i in range(warm):
                fn(i)
            a0.record(stream)
            for i in range(n):
                fn(warm + i)
            a1.record(stream)
        stream.synchronize()
        return a0.elapsed_time(a1) * 1e3 / n

    sink = torch.empty(dn.PROBE_SINK_BYTES, dtype=torch.uint8, device="cuda")
    if bound == "hbm":
        pool = torch.empty(2 << 30, dtype=torch.uint8, device="cuda").random_(0, 256)
        nb = (int(kbytes[kdom]) + 1023) // 1024 * 1024
        slots = max(1, pool.numel() // nb)
        torch.cuda.synchronize()           # the fill ran on another stream
        p0, sk, skn = pool.data_ptr(), sink.data_ptr(), sink.numel()      # plain integers: no per-launch host work
        def rd(off, n):
            if L.deinfer_probe_stream_read(p0 + off, n, sk, skn, sh) != 0:
                raise RuntimeError(dn.last_error())
        same_us = events_us(lambda i: rd((i % slots) * nb, nb), 60)
        long_us = events_us(lambda i: rd(0, pool.numel()), 5, warm=1)
        roofline["measured_ceiling"] = {
            "what": "deinfer_probe_stream_read: a plain coalesced read, rotating through a 2 GiB pool",
            "read_of_the_same_bytes_us": round(same_us, 2), "read_of_the_same_bytes_GBs": round(nb / same_us / 1e3, 1),
            "long_stream_GBs": round(pool.numel() / long_us / 1e3, 1),
            "launch_time_over_plain_read_time": round(ksec * 1e6 / same_us, 3)}
        del pool
    else:
        fl = [0.0]
        def mf(i):
            fl[0] = dn.deinfer_probe_mfma_bf16(x, 4000, sink, stream)
        torch.cuda.synchronize()
        mf_us = events_us(mf, 5, warm=1)
        Kd, Nd = ((ranks[ps[-1]], proj[ps[-1]][1]) if kdom == "up" else (proj[ps[0]][0], sum(ranks[p] for p in ps)))
        ga = torch.randn((T, Kd), device="cuda").to(bf); gb = (torch.randn((Kd, Nd), device="cuda") * 0.02).to(bf)
        gc = torch.empty((T, Nd), dtype=bf, device="cuda")
        torch.cuda.synchronize()
        gemm_us = events_us(lambda i: torch.matmul(ga, gb, out=gc), 20)
        Kp = (Kd + 31) // 32 * 32          # the k extent of the packed format (zero padded)
        gap = torch.zeros((T, Kp), dtype=bf, device="cuda"); gap[:, :Kd] = ga
        gbp = torch.zeros((Kp, Nd), dtype=bf, device="cuda"); gbp[:Kd] = gb
        torch.cuda.synchronize()
        gemm_pad_us = events_us(lambda i: torch.matmul(gap, gbp, out=gc), 20)
        roofline["measured_ceiling"] = {
            "what": "deinfer_probe_mfma_bf16: back-to-back 32x32x16 bf16 products on register operands (activation values), "
                    "one wavefront per SIMD, no memory traffic",
            "products_only_TFLOPs": round(fl[0] / mf_us / 1e6, 1),
            "frac_of_products_only": round(ach / (fl[0] / mf_us / 1e6), 4),
            "context_vendor_gemm": {"what": "torch.matmul (bf16, random operands) of the same T x K x N as this launch, "
                                            "without its epilogue work; not part of the path",
                                    "K": int(Kd), "N": int(Nd), "us": round(gemm_us, 2),
                                    "TFLOPs": round(2.0 * T * Kd * Nd / gemm_us / 1e6, 1),
                                    "us_with_K_zero_padded_to_%d" % Kp: round(gemm_pad_us, 2)}}
        del ga, gb, gc, gap, gbp

    step_bytes = sum(c["bytes"] for c in per_call.values())
    step_flops = sum(c["flops"] for c in per_call.values())
    out = {
        "metric": "decomposed-layer tokens/sec; % HBM roofline (decode) / % MFMA peak (prefill)",
        "value": round(T / sec_per_step, 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(sec_per_step * 1e3, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": args.dtype, "data": "synthetic",
        "config": {"workload": "%s T=%d (%s of one block)" % (args.workload, T, "qkv+o+gateup_silu+down" if shape.glu else
                                                              "qkv+o+linear_act(bias, ReLU)+linear_act(bias)"),
                   "ranks": ranks, "weight_MB": round(weight_bytes / 1e6, 1), "weight_copies": n_copies,
                   "launch": launch_mode, "launch_ms": launch_ms},
        "ms_per_step_chunks": spread,
        # the timed K steps between two events on the launch stream: without the host's share of the
        # bracket (first launch, wake-up after the synchronisation), which counts for a small K
        "ms_per_step_device": ev_ms.get(launch_mode),
        "step_GBs": round(step_bytes / sec_per_step / 1e9, 1),
        "step_TFLOPs": round(step_flops / sec_per_step / 1e12, 2),
        "step_frac_of_roofline": round((step_bytes / sec_per_step / 1e9 / HBM_PEAK_GBS) if bound == "hbm"
                                       else (step_flops / sec_per_step / 1e12 / MFMA_BF16_PEAK_TFLOPS), 4),
        "calls": per_call,
        "roofline": roofline,
        "setup_s": round(setup_s, 1),
    }
    roofline["step_frac"] = out["step_frac_of_roofline"]     # the whole step against the same peak, beside the dominant launch

    # ---------------------------------------------------------------- other decode sizes
    if args.sweep and T <= 128:
        sweep = {}
        for Ts in (1, 8, 32, 64, 128):
            if Ts == T or Ts > host["x"].shape[0]:
                continue
            sub = [{n: (fn, tuple(Ts if (i == 1) else v_ for i, v_ in enumerate(a_))) for n, (fn, a_) in c.items()} for c in calls]
            with torch.cuda.stream(stream):
                for i in range(10):
                    run_calls(sub[i % n_copies])
            stream.synchronize()
            sub_step, mode = (lambda i: run_calls(sub[i % n_copies])), "direct"
            if launch_mode == "graph":       # as the main measurement: the step replayed from a graph per weight copy, if that won there
                try:
                    sub_graphs = []
                    for i in range(n_copies):
                        g = torch.cuda.CUDAGraph()
                        with torch.cuda.graph(g, stream=stream):
                            run_calls(sub[i])
                        sub_graphs.append(g)
                    sub_step, mode = (lambda i: sub_graphs[i % n_copies].replay()), "graph"
                except Exception as e:  # noqa: BLE001 - report and keep the direct launches
                    print("graph capture failed in the sweep (%s); using direct launches" % e, file=sys.stderr)
            with torch.cuda.stream(stream):
                for i in range(args.warmup):
                    sub_step(i)
            sec = timed(sub_step, args.steps)
            sweep["T=%d" % Ts] = {"tokens_per_s": round(Ts / sec, 1), "us_per_step": round(sec * 1e6, 2), "launch": mode}
        out["sweep"] = sweep

    # ---------------------------------------------------------------- second row: the ranks the configuration prints
    # (its rule gives 2388 for gate / up / down, its text 2357; the rule is what is benchmarked
    # above, the printed value here, in a child process with the same settings)
    if args.workload == "llama7b_keep80_decode" and not args.rank_override and not args.no_second_row and args.dtype == "bf16":
        import subprocess
        cmd = [sys.executable, os.path.abspath(__file__), "--workload", args.workload, "--T", str(T), "--steps", str(args.steps),
               "--warmup", str(args.warmup), "--launch", args.launch, "--seed", str(args.seed), "--no-cpu-baseline",
               "--rank-override", "gate=2357,up=2357,down=2357"]
        res = subprocess.run(cmd, capture_output=True, text=True)
        try:
            row = json.loads(res.stdout.strip().splitlines()[-1])
            out["second_row_r2357"] = {"ranks": row["config"]["ranks"], "weight_MB": row["config"]["weight_MB"],
                                       "ms_per_step": row["ms_per_step"], "value": row["value"],
                                       "step_frac_of_roofline": row["step_frac_of_roofline"]}
        except Exception as e:  # noqa: BLE001 - the main row stands on its own
            out["second_row_r2357"] = {"error": "%s: %s" % (type(e).__name__, res.stderr[-300:])}

    # ---------------------------------------------------------------- secondary rows of the default run (child processes)
    if args.workload == DEFAULT_WORKLOAD and not args.no_extra_rows and not args.rank_override and args.dtype == "bf16" and not args.T:
        import subprocess

        def child(extra):
            cmd = [sys.executable, os.path.abspath(__file__), "--steps", str(args.steps), "--warmup", str(args.warmup),
                   "--launch", args.launch, "--seed", str(args.seed), "--no-cpu-baseline", "--no-extra-rows"] + extra
            res = subprocess.run(cmd, capture_output=True, text=True)
            try:
                return json.loads(res.stdout.strip().splitlines()[-1])
            except Exception as e:  # noqa: BLE001 - the main row stands on its own
                return {"error": "%s: %s" % (type(e).__name__, res.stderr[-300:])}

        keep = ("value", "unit", "ms_per_step", "ms_per_step_chunks", "ms_per_step_device", "step_frac_of_roofline", "step_GBs", "step_TFLOPs", "calls", "roofline", "config")
        # free this process's copies of the weights first: the children need the memory bandwidth, not the space
        row = child(["--workload", "llama70b_keep40_prefill"])
        out["prefill"] = row if "error" in row else {k_: row[k_] for k_ in keep if k_ in row}
        row = child(["--workload", "llama7b_keep80_decode", "--sweep"])
        out["llama7b_keep80_decode_T64"] = row if "error" in row else {k_: row[k_] for k_ in keep + ("sweep", "second_row_r2357") if k_ in row}

    # ---------------------------------------------------------------- CPU baseline: the oracle, as it stands
    if not args.no_cpu_baseline:
        import oracle
        rows = min(T, 64)
        f64 = lambda t: t.values.astype(np.float64)
        xs, as_, hs = f64(host["x"])[:rows], f64(host["a"])[:rows], f64(host["h_in"])[:rows]
        W = {n: f64(host[n]) for n in host if n[:2] in ("U_", "V_")}
        passes, cpu_s = 0, 0.0
        while cpu_s < 10.0 and passes < 50:
            t_a = time.perf_counter()
            oracle.lowrank_qkv(xs, W["U_q"], W["V_q"], W["U_k"], W["V_k"], W["U_v"], W["V_v"])
            oracle.lowrank_linear(as_, W["U_o"], W["V_o"])
            if shape.glu:
                oracle.lowrank_gateup_silu(xs, W["U_gate"], W["V_gate"], W["U_up"], W["V_up"])
                oracle.lowrank_down(hs, W["U_down"], W["V_down"])
            else:
                oracle.lowrank_linear_act(xs, W["U_gate"], W["V_gate"], f64(host["b_gate"]).reshape(-1), oracle.ACT_RELU)
                oracle.lowrank_linear_act(hs, W["U_down"], W["V_down"], f64(host["b_down"]).reshape(-1), oracle.ACT_NONE)
            cpu_s += time.perf_counter() - t_a
            passes += 1
        out["cpu_baseline"] = {"value": round(rows * passes / cpu_s, 2), "unit": "tokens/s", "cores": oracle.num_threads(),
                               "kind": "oracle",
                               "sample": "%d of %d token rows of the same block, %d passes, fp64 loops, %.1f s in total"
                                         % (rows, T, passes, cpu_s)}
    print(json.dumps(out))


def tp_rank(args, L, shape, T, P, bound):
    """Step = the calls of ONE rank of a P-way tensor-parallel group for one block (Sec. 4.1): first
    sub-layers: downward projections with the rank's column slice of U, [all-gather, not run],
    upward projections with its column shard of V; second sub-layers: downward projection with
    its row slice of U, [reduce-sum, not run], the replicated upward projection.  The gathered /
    summed rank-space rows are stand-in tensors of the right shape."""
    import numpy as np
    import torch
    import synth_inputs as si
    import paper_2604_17709_amd as dn
    bf = torch.bfloat16
    proj = shape.projections()
    rho = 1.0 - shape.keep_num / shape.keep_den
    ranks = {p: dn.deinfer_rank_for_ratio(m, n, rho) for p, (m, n) in proj.items()}
    cdiv = lambda a, b: (a + b - 1) // b
    g = torch.Generator(device="cuda"); g.manual_seed(args.seed)
    rnd = lambda *sh, std=0.02: (torch.randn(sh, generator=g, device="cuda") * std).to(bf)
    t0 = time.time()

    def pair_u(d_in, r):          # a pair used for its downward matrix only
        return dn.deinfer_pack_factors(dn.raw_pair(rnd(d_in, r), rnd(r, 16), rho))

    def pair_v(r, d_out):         # a pair used for its upward matrix only
        return dn.deinfer_pack_factors(dn.raw_pair(rnd(16, r), rnd(r, d_out), rho))

    H, Fd = shape.hidden, shape.ffn
    n_copies = 8                  # rotate the weights so that the 256 MB cache does not serve them
    sets = []
    for _ in range(n_copies):
        sets.append({
            "qkv_d": [pair_u(H, cdiv(ranks[n], P)) for n in ("q", "k", "v")],
            "qkv_u": [pair_v(ranks[n], proj[n][1] // P) for n in ("q", "k", "v")],
            "o_d": pair_u(H // P, ranks["o"]), "o_u": pair_v(ranks["o"], H),
            "gu_d": [pair_u(H, cdiv(ranks[n], P)) for n in ("gate", "up")],
            "gu_u": [pair_v(ranks[n], Fd // P) for n in ("gate", "up")],
            "dn_d": pair_u(Fd // P, ranks["down"]), "dn_u": pair_v(ranks["down"], H)})
    w_bytes = 0
    s0 = sets[0]
    for k, v in s0.items():
        for p_ in (v if isinstance(v, list) else [v]):
            w_bytes += 2 * (p_.r * p_.d_in if k.endswith("_d") else p_.r * p_.d_out)
    pad8 = lambda r: (r + 7) // 8 * 8
    x = rnd(T, H, std=1.0); a_sh = rnd(T, H // P, std=1.0); h_sh = rnd(T, Fd // P, std=1.0)
    tg = {n: torch.zeros((T, pad8(ranks[n])), dtype=bf, device="cuda") for n in ranks}     # gathered / summed rank-space rows
    for n in tg:
        tg[n][:, :ranks[n]] = rnd(T, ranks[n], std=0.3)
    ts = {n: torch.zeros((T, pad8(cdiv(ranks[n], P))), dtype=bf, device="cuda") for n in ("q", "k", "v", "gate", "up")}
    tpart = {n: torch.zeros((T, pad8(ranks[n])), dtype=bf, device="cuda") for n in ("o", "down")}
    outs = {n: torch.empty((T, proj[n][1] // P), dtype=bf, device="cuda") for n in ("q", "k", "v")}
    outs["o"] = torch.empty((T, H), dtype=bf, device="cuda"); outs["down"] = torch.empty((T, H), dtype=bf, device="cuda")
    outs["h"] = torch.empty((T, Fd // P), dtype=bf, device="cuda")
    need = 0
    for v in s0.values():
        need = max(need, dn.deinfer_workspace_bytes(T, v if isinstance(v, list) else [v]))
    ws = dn.Workspace(need)
    torch.cuda.synchronize()
    setup_s = time.time() - t0
    stream = torch.cuda.Stream(); sh = int(stream.cuda_stream)
    B = ctypes.byref
    wsp, wsn = ws.buf.data_ptr(), ws.nbytes
    FP = ctypes.POINTER(dn.Factors)

    def down_proj(xin, pairs, touts):
        n = len(pairs)
        fa = (FP * n)(*[ctypes.pointer(p_.desc) for p_ in pairs])
        ta = (ctypes.c_void_p * n)(*[t.data_ptr() for t in touts])
        la = (ctypes.c_int64 * n)(*[t.stride(0) for t in touts])
        return (L.deinfer_lowrank_down_proj, (xin.data_ptr(), T, xin.stride(0), fa, n, ta, la, wsp, wsn, sh))

    def up(tin, p_, out):
        return (L.deinfer_lowrank_up, (tin.data_ptr(), T, tin.stride(0), B(p_.desc), out.data_ptr(), out.stride(0), wsp, wsn, sh))

    def calls_of(c):
        return {
            "qkv_down": [down_proj(x, c["qkv_d"], [ts["q"], ts["k"], ts["v"]])],
            "qkv_up": [up(tg[n], c["qkv_u"][i], outs[n]) for i, n in enumerate(("q", "k", "v"))],
            "o_down": [down_proj(a_sh, [c["o_d"]], [tpart["o"]])],
            "o_up": [up(tg["o"], c["o_u"], outs["o"])],
            "gateup_down": [down_proj(x, c["gu_d"], [ts["gate"], ts["up"]])],
            "gateup_up": [(L.deinfer_lowrank_up_glu_silu, (tg["gate"].data_ptr(), tg["gate"].stride(0), tg["up"].data_ptr(),
                                                           tg["up"].stride(0), T, B(c["gu_u"][0].desc), B(c["gu_u"][1].desc),
                                                           outs["h"].data_ptr(), outs["h"].stride(0), wsp, wsn, sh))],
            "down_down": [down_proj(h_sh, [c["dn_d"]], [tpart["down"]])],
            "down_up": [up(tg["down"], c["dn_u"], outs["down"])],
        }
    calls = [calls_of(c) for c in sets]
    order = list(calls[0].keys())

    def run(i, names=None):
        for n in (names or order):
            for fn, a_ in calls[i % n_copies][n]:
                if fn(*a_) != 0:
                    raise RuntimeError("%s failed: %s" % (n, dn.last_error()))

    with torch.cuda.stream(stream):
        run(0)
    stream.synchronize(); ws.check(stream)
    graphs = []
    for i in range(n_copies):
        gph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gph, stream=stream):
            run(i)
        graphs.append(gph)
    with torch.cuda.stream(stream):
        for i in range(args.warmup):
            graphs[i % n_copies].replay()
    stream.synchronize(); torch.cuda.synchronize()
    t_a = time.perf_counter()
    with torch.cuda.stream(stream):
        for i in range(args.steps):
            graphs[i % n_copies].replay()
    stream.synchronize(); torch.cuda.synchronize()
    sec = (time.perf_counter() - t_a) / args.steps

    def ev(names, n):
        a0 = torch.cuda.Event(enable_timing=True); a1 = torch.cuda.Event(enable_timing=True)
        with torch.cuda.stream(stream):
            for i in range(5): run(i, names)
            a0.record(stream)
            for i in range(n): run(i, names)
            a1.record(stream)
        stream.synchronize()
        return a0.elapsed_time(a1) * 1e-3 / n
    per_call = {n: round(ev((n,), 50) * 1e6, 2) for n in order}
    # dominant launch: the replicated upward projection of the MLP's second layer
    decode = T <= 128
    kind = dn.PROF_DECODE_UP if decode else dn.PROF_PREFILL_UP
    e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
    with torch.cuda.stream(stream):
        e0.record(stream); e1.record(stream)
    stream.synchronize()
    L.deinfer_set_profile_events(kind, e0.cuda_event, e1.cuda_event)
    tot = 0.0
    for i in range(23):
        with torch.cuda.stream(stream):
            run(i, ("down_up",))
        stream.synchronize()
        if i >= 3: tot += e0.elapsed_time(e1)
    L.deinfer_set_profile_events(0, None, None)
    ksec = tot * 1e-3 / 20
    kb = 2 * (ranks["down"] * H + T * ranks["down"] + T * H)
    kf = 2.0 * T * ranks["down"] * H
    step_bytes = w_bytes + 2 * T * (2 * H + H // P + Fd // P) + 2 * T * (sum(proj[n][1] // P for n in ("q", "k", "v")) + 2 * H + Fd // P)
    step_flops = 2.0 * T * w_bytes / 2
    if bound == "hbm":
        ach = kb / ksec / 1e9
        roof = {"bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBS, 4)}
    else:
        ach = kf / ksec / 1e12
        roof = {"bound": "mfma", "achieved": round(ach, 1), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": round(ach / MFMA_BF16_PEAK_TFLOPS, 4)}
    roof.update({"traffic": None, "kernel": "%s kernel (deinfer_lowrank_up of the replicated V_down)" % ("skinny_kernel" if decode else "prefill_kernel"),
                 "avg_launch_us": round(ksec * 1e6, 2), "algorithmic_bytes_per_launch": kb, "algorithmic_flops_per_launch": kf})
    out = {
        "metric": "decomposed-layer tokens/sec; % HBM roofline (decode) / % MFMA peak (prefill)",
        "value": round(T / sec, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(sec * 1e3, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s T=%d (one rank of %d: its shard of qkv, o, gate/up, down as downward-projection and "
                               "upward-projection calls; the exchanges between them are not run)" % (args.workload, T, P),
                   "ranks_full": ranks, "weight_MB_per_rank": round(w_bytes / 1e6, 1), "weight_copies": n_copies, "launch": "graph"},
        "step_GBs": round(step_bytes / sec / 1e9, 1), "step_TFLOPs": round(step_flops / sec / 1e12, 2),
        "step_frac_of_roofline": round((step_bytes / sec / 1e9 / HBM_PEAK_GBS) if bound == "hbm"
                                       else (step_flops / sec / 1e12 / MFMA_BF16_PEAK_TFLOPS), 4),
        "calls_us": per_call, "roofline": roof, "setup_s": round(setup_s, 1),
    }
    if not args.no_cpu_baseline:
        import oracle
        rows = min(T, 64)
        f64 = lambda t: t[:rows].to(torch.float32).cpu().numpy().astype(np.float64)
        Vd = np.random.default_rng(args.seed).standard_normal((ranks["down"], H)) * 0.02
        Ud = np.random.default_rng(args.seed + 1).standard_normal((Fd // P, ranks["down"])) * 0.02
        hs, td = f64(h_sh), f64(tg["down"])[:, :ranks["down"]]
        passes, cpu_s = 0, 0.0
        while cpu_s < 10.0 and passes < 50:
            t_a = time.perf_counter()
            oracle.down_projection(hs, Ud); oracle.up_projection(td, Vd)
            cpu_s += time.perf_counter() - t_a
            passes += 1
        out["cpu_baseline"] = {"value": round(rows * passes / cpu_s, 2), "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
                               "sample": "%d of %d token rows, the two calls of the MLP's second layer only (%.0f %% of the rank's weights), "
                                         "%d passes, %.1f s in total" % (rows, T, 100.0 * 2 * ranks["down"] * (Fd // P + H) / w_bytes, passes, cpu_s)}
    print(json.dumps(out))


def kv_rebuild(args, L, shape, T):
    """Step = keys and values of T cached tokens rebuilt from the paged low-rank cache: compacting
    copy of k_low_rank and v_low_rank, two upward projections at the buffer's capacity, rotary
    embedding of the keys; one captured graph, block tables of a 16-sequence batch."""
    import numpy as np
    import torch
    import synth_inputs as si
    import paper_2604_17709_amd as dn
    bf = torch.bfloat16
    proj = shape.projections()
    rho = 1.0 - shape.keep_num / shape.keep_den
    d_in, d_kv = proj["k"]
    r = dn.deinfer_rank_for_ratio(d_in, d_kv, rho)
    head_dim = 128
    n_heads = d_kv // head_dim
    bt, pitch = 16, (r + 7) // 8 * 8
    n_seqs = 16
    blocks_per_seq = T // bt // n_seqs
    cap_blocks = n_seqs * blocks_per_seq
    T = cap_blocks * bt
    n_pool = 2 * cap_blocks
    # cache state: prompts of 3/4 of the length allocated in one go, the rest block by block while decoding
    prompt = [blocks_per_seq * 3 // 4] * n_seqs
    decode = [blocks_per_seq - prompt[0]] * n_seqs
    table, n_blocks = si.paged_block_tables(args.seed, prompt, decode, n_pool, recycled=n_pool // 8)
    plan, remap, pos = dn.deinfer_kv_compact_plan(table, n_blocks, n_pool, cap_blocks, bt)
    t0 = time.time()
    host = {n: si.make(args.seed, i + 1, sh, 0.02, "bf16") for i, (n, sh) in
            enumerate({"V_k": (r, d_kv), "V_v": (r, d_kv), "U": (d_in, r)}.items())}
    dev = lambda t: torch.from_numpy(t.bits.view(np.int16)).cuda().view(bf)
    pairs = {n: dn.deinfer_pack_factors(dn.raw_pair(dev(host["U"]), dev(host["V_" + n]), rho)) for n in ("k", "v")}
    pools = {n: torch.zeros((n_pool, bt, pitch), dtype=bf, device="cuda") for n in ("k", "v")}
    for n in pools:
        pools[n][:, :, :r] = torch.randn((n_pool, bt, r), device="cuda").to(bf)
    bufs = {n: torch.zeros((T, pitch), dtype=bf, device="cuda") for n in ("k", "v")}
    outs = {n: torch.empty((T, d_kv), dtype=bf, device="cuda") for n in ("k", "v")}
    plan_d = torch.from_numpy(plan).cuda(); pos_d = torch.from_numpy(pos).cuda()
    ws = dn.Workspace(dn.deinfer_workspace_bytes(T, [pairs["k"]]))
    torch.cuda.synchronize()
    setup_s = time.time() - t0
    stream = torch.cuda.Stream(); sh = int(stream.cuda_stream)
    block_bytes = bt * pitch * 2
    cap_runs = (plan.size - dn.KV_PLAN_HEADER) // 3
    B = ctypes.byref

    table_d = torch.empty((T, head_dim), dtype=torch.float32, device="cuda")

    def run(names=("copy", "table", "up")):
        # "up": keys through the projection whose epilogue rotates them, values through the plain one;
        # "up_plain" + "rope": the keys the other way (projection, then rotation in place), timed for comparison
        if "table" in names:
            rc = L.deinfer_rope_table(pos_d.data_ptr(), T, head_dim, 10000.0, table_d.data_ptr(), sh)
            if rc: raise RuntimeError(dn.last_error())
        for n in ("k", "v"):
            if "copy" in names:
                rc = L.deinfer_kv_compact_copy(pools[n].data_ptr(), n_pool, block_bytes, plan_d.data_ptr(), cap_runs,
                                               bufs[n].data_ptr(), cap_blocks, sh)
                if rc: raise RuntimeError(dn.last_error())
            if "up" in names and n == "k":
                rc = L.deinfer_lowrank_up_rope(bufs[n].data_ptr(), T, pitch, B(pairs[n].desc), table_d.data_ptr(), head_dim,
                                               outs[n].data_ptr(), d_kv, ws.buf.data_ptr(), ws.nbytes, sh)
                if rc: raise RuntimeError(dn.last_error())
            elif "up" in names or "up_plain" in names:
                rc = L.deinfer_lowrank_up(bufs[n].data_ptr(), T, pitch, B(pairs[n].desc), outs[n].data_ptr(), d_kv,
                                          ws.buf.data_ptr(), ws.nbytes, sh)
                if rc: raise RuntimeError(dn.last_error())
        if "rope" in names:
            rc = L.deinfer_rope_inplace(outs["k"].data_ptr(), T, d_kv, n_heads, head_dim, pos_d.data_ptr(), 10000.0, dn.BF16, sh)
            if rc: raise RuntimeError(dn.last_error())

    with torch.cuda.stream(stream):
        run()
    stream.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=stream):
        run()

    def timed(fn, n):
        torch.cuda.synchronize()
        t_a = time.perf_counter()
        with torch.cuda.stream(stream):
            for i in range(n):
                fn()
        stream.synchronize(); torch.cuda.synchronize()
        return (time.perf_counter() - t_a) / n

    with torch.cuda.stream(stream):
        for i in range(args.warmup):
            graph.replay()
    stream.synchronize()
    sec = timed(graph.replay, args.steps)

    def ev(fn, n):
        a0 = torch.cuda.Event(enable_timing=True); a1 = torch.cuda.Event(enable_timing=True)
        with torch.cuda.stream(stream):
            for i in range(3): fn()
            a0.record(stream)
            for i in range(n): fn()
            a1.record(stream)
        stream.synchronize()
        return a0.elapsed_time(a1) * 1e-3 / n
    parts = {n: ev(lambda n=n: run((n,)), 50) for n in ("copy", "table", "up", "up_plain", "rope")}
    # the dominant kernel: one upward projection (the GEMM "of large size", bf16 MFMA)
    e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
    with torch.cuda.stream(stream):
        e0.record(stream); e1.record(stream)
    stream.synchronize()
    L.deinfer_set_profile_events(dn.PROF_PREFILL_UP, e0.cuda_event, e1.cuda_event)
    tot = 0.0
    for i in range(23):
        with torch.cuda.stream(stream):
            rc = L.deinfer_lowrank_up_rope(bufs["k"].data_ptr(), T, pitch, B(pairs["k"].desc), table_d.data_ptr(), head_dim,
                                           outs["k"].data_ptr(), d_kv, ws.buf.data_ptr(), ws.nbytes, sh)
            if rc: raise RuntimeError(dn.last_error())
        stream.synchronize()
        if i >= 3: tot += e0.elapsed_time(e1)
    L.deinfer_set_profile_events(0, None, None)
    ksec = tot * 1e-3 / 20
    kflops = 2.0 * T * r * d_kv
    ach = kflops / ksec / 1e12
    n_run_blocks = int(plan[1])
    traffic = None
    tfile = os.path.join(ROOT, "profiles", "hbm_traffic_%s_T%d.txt" % (args.workload, T))
    if os.path.exists(tfile):
        for line in open(tfile):
            if line.startswith("traffic_bytes_per_launch"):
                traffic = float(line.split("=")[1])
    copy_bytes = 2 * 2 * n_run_blocks * block_bytes                  # k and v, read + write
    rope_bytes = 2 * T * d_kv * 2
    out = {
        "metric": "decomposed-layer tokens/sec; % HBM roofline (decode) / % MFMA peak (prefill)",
        "value": round(T / sec, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(sec * 1e3, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s T=%d (keys and values of T cached tokens rebuilt from the paged low-rank cache: "
                               "compacting copy k, v + table of rotary angles + upward projection k with the rotary "
                               "embedding in its epilogue + upward projection v)" % (args.workload, T),
                   "ranks": {"k": r, "v": r}, "block_tokens": bt, "sequences": n_seqs, "runs": int(plan[0]),
                   "blocks": n_run_blocks, "launch": "graph"},
        "calls": {"copy_k_v": {"us": round(parts["copy"] * 1e6, 2), "bytes": copy_bytes, "GBs": round(copy_bytes / parts["copy"] / 1e9, 1)},
                  "up_k_v": {"us": round(parts["up"] * 1e6, 2), "flops": 2 * kflops, "TFLOPs": round(2 * kflops / parts["up"] / 1e12, 2)},
                  "rope_table": {"us": round(parts["table"] * 1e6, 2)},
                  "not_in_the_step": {"up_k_v_plain_us": round(parts["up_plain"] * 1e6, 2),
                                      "rope_k_in_place": {"us": round(parts["rope"] * 1e6, 2), "bytes": rope_bytes,
                                                          "GBs": round(rope_bytes / parts["rope"] / 1e9, 1)}}},
        "roofline": {"bound": "mfma", "achieved": round(ach, 1), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(ach / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": traffic,
                     "kernel": "prefill_kernel kernel (upward projection of k with the rotary epilogue: deinfer_lowrank_up_rope)",
                     "avg_launch_us": round(ksec * 1e6, 2), "algorithmic_flops_per_launch": kflops,
                     "algorithmic_bytes_per_launch": 2 * (r * d_kv + T * r + T * d_kv)},
        "setup_s": round(setup_s, 1),
    }
    if not args.no_cpu_baseline:
        import oracle
        from oracle import paged_cache as pc
        rows = 64
        Vk = host["V_k"].values.astype(np.float64); Vv = host["V_v"].values.astype(np.float64)
        pk = pools["k"].to(torch.float32).cpu().numpy().astype(np.float64)
        small_nb = np.minimum(n_blocks, 1).astype(np.int32)             # one block per sequence: 16 x 16 = 256 token slots
        passes, cpu_s = 0, 0.0
        while cpu_s < 10.0 and passes < 50:
            t_a = time.perf_counter()
            runs_o, _ = pc.contiguous_runs(table, n_blocks)
            g = pc.copy_runs(pk[:, :, :r], pc.contiguous_runs(table, small_nb)[0], n_seqs)
            tk = g.reshape(-1, r)[:rows]
            kk = oracle.up_projection(tk, Vk); oracle.up_projection(tk, Vv)
            pc.rope(kk, pos[:rows], n_heads, head_dim)
            cpu_s += time.perf_counter() - t_a
            passes += 1
        out["cpu_baseline"] = {"value": round(rows * passes / cpu_s, 2), "unit": "tokens/s", "cores": oracle.num_threads(),
                               "kind": "oracle",
                               "sample": "%d of %d token rows (full scan of the block tables, copy of one block per sequence, "
                                         "both upward projections, rotary embedding), %d passes, %.1f s in total"
                                         % (rows, T, passes, cpu_s)}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
