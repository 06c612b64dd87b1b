#!/usr/bin/env python3
"""Benchmark of the MoQAE hot path on one MI355X.

A step is one pass of the whole path over one layer of the workload: route every chunk
(Eq. (1)-(2)), quantise-and-pack K and V at the routed bit-widths, and one decode-attention
call over the packed cache.  Inputs (fp16 K, V, q, router weights) are resident in HBM before
the timed region.  The decode call of step i reads the arena packed in step i-1 (two arenas
alternate), so the 256 MB last-level cache cannot hold what it reads.

Prints ONE JSON line: metric = decode-attention HBM GB/s (algorithmic packed bytes / time of
the whole decode call, made on the plan that was left in its workspace when the cache was packed),
`roofline` for its main kernel timed alone (HIP events the library records around it), the same
call without a plan (`decode_call_unplanned` = moqae_decode_attn), `stream_ceiling` = what a plain
read-only streaming kernel reaches on the same GPU, route+pack chunks/s with a roofline object
each, and the CPU oracle timed on the same workload.  The timed steps rotate over three kinds (whole
planned call / main kernel alone / whole unplanned call), so the default 150 steps give 50 samples
of each; averages, medians and minima are reported.
"""
from __future__ import annotations

import argparse
import dataclasses
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0        # MI355X HBM3E, vendor figure

# What the decode contraction computes in (the `dtype` of the JSON line): one query head per KV head: code bytes
# times base-128 digits of a 21-bit fixed-point copy of q / of the softmax weights on v_mfma_i32_16x16x64_i8, exact
# integer sums; grouped queries: fp16 code fields times fp16 weights on v_mfma_f32_16x16x32_f16; softmax and all
# accumulation in binary32 (no narrower than the FP16 de-quantisation of the paper's "Limitations" section).
DTYPE = {1: "i8-mfma fixed-point 21b / f32 accumulate", 0: "f16-mfma / f32 accumulate"}


def measured_traffic(workload):
    """HBM bytes per decode call (fetched + written) from the rocprofv3 FETCH_SIZE / WRITE_SIZE runs summarised in
    profiles/hbm_traffic_<workload>.md (its line `traffic_bytes_per_decode_call: N`); counters cannot be read from
    inside this process, so a workload without such a summary reports null."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}.md")
    if os.path.exists(path):
        for line in open(path):
            if line.startswith("traffic_bytes_per_decode_call:"):
                return int(line.split(":")[1].split()[0])
    return None


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class HipEvents:
    """Raw HIP events (ctypes on the HIP runtime torch has loaded): the library records a pair around
    its main decode kernel, on the stream that kernel is launched on."""

    def __init__(self, n):
        import ctypes as C
        self.C = C
        self.hip = C.CDLL("libamdhip64.so")
        self.ev = []
        for _ in range(2 * n):
            e = C.c_void_p()
            assert self.hip.hipEventCreate(C.byref(e)) == 0
            self.ev.append(e)

    def pair(self, i):
        return self.ev[2 * i], self.ev[2 * i + 1]

    def elapsed_ms(self, i):
        C = self.C
        ms = C.c_float()
        assert self.hip.hipEventSynchronize(self.ev[2 * i + 1]) == 0
        assert self.hip.hipEventElapsedTime(C.byref(ms), self.ev[2 * i], self.ev[2 * i + 1]) == 0
        return float(ms.value)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="timed steps (default: 150 for one layer, 10 for the stack)")
    ap.add_argument("--warmup", type=int, default=None,
                    help="untimed steps (default 60 for one layer: after the seconds of host-side input generation the GPU needs "
                         "some 40 steps, about 40 ms, before its kernel times settle; 2 for the stack)")
    ap.add_argument("--workload", default="llama13b_128k")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--decode-only", action="store_true",
                    help="profiling aid: after set-up run only decode calls in the timed loop")
    ap.add_argument("--force-bits", type=int, default=0,
                    help="sweep aid (implies --decode-only): every chunk takes the expert of this bit-width")
    ap.add_argument("--sweep", choices=["chunk", "share"], default=None,
                    help="trend sweeps on synthetic data (the paper's ablations, Table 3 and Table 5): 'chunk' runs the "
                         "chosen single-layer workload at chunk sizes 8, 16, 32, 64, 128 and 256; 'share' runs an 8-layer cut of the "
                         "stack workload with routing-sharing groups of 1, 2, 4 and 8 layers")
    ap.add_argument("--ragged", action="store_true",
                    help="decode attention over a batch of 16 sequences of 2k ... 32k tokens (one layer of the stack "
                         "workload's shape) through moqae_decode_attn_ragged, beside the uniform call at full length")
    ap.add_argument("--per-channel", action="store_true",
                    help="quantise the keys per channel (cfg.k_per_channel = 1: groups of G tokens of one dim) instead of per token")
    ap.add_argument("--kquant-error", action="store_true",
                    help="attention error against unquantised fp64 attention of caches quantised uniformly at 2, 4 and 8 bits, keys per "
                         "token vs per channel, on the first 16k tokens of four heads of the chosen workload's synthetic K, V")
    ap.add_argument("--copy-probe", action="store_true",
                    help="counter calibration: run a plain elementwise kernel that reads 1 GiB and writes 1 GiB, "
                         "five times, and exit (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE are scaled by what they read for it)")
    args = ap.parse_args()
    if args.copy_probe:
        import torch
        src = torch.zeros(1 << 28, dtype=torch.int32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(5):
            torch.add(src, 1, out=dst)
        torch.cuda.synchronize()
        print(json.dumps({"copy_probe": "torch add(int32, 1)", "read_bytes": 1 << 30, "write_bytes": 1 << 30, "launches": 5}))
        return 0
    if args.force_bits:
        args.decode_only = True
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        return 2

    from paper_2506_07533_amd import synth

    w = synth.WORKLOADS[args.workload]
    stack_like = w.n_layers > 1 or args.sweep == "share"
    if args.steps is None:
        args.steps = 10 if stack_like else 150
    if args.warmup is None:
        args.warmup = 2 if stack_like else 60
    if args.sweep == "chunk":
        if w.n_layers > 1:
            print("bench.py: --sweep chunk takes a single-layer workload", file=sys.stderr)
            return 2
        args.no_cpu_baseline = True
        rows = []
        for N in (8, 16, 32, 64, 128, 256):
            r = bench_layer(args, dataclasses.replace(w, chunk=N, name=f"{w.name}/chunk{N}"))
            rows.append({"chunk": N, "chunks": r["config"]["chunks"], "packed_bytes": r["config"]["packed_bytes"],
                         "realised_mix": r["config"]["realised_mix"],
                         "route_us": round(r["roofline_route"]["avg_ms"] * 1e3, 1),
                         "pack_us": round(r["roofline_pack"]["avg_ms"] * 1e3, 1),
                         "decode_call_us": round(r["decode_call"]["avg_ms"] * 1e3, 1),
                         "decode_kernel_us": round(r["roofline"]["avg_ms"] * 1e3, 1),
                         "decode_GBps": r["value"], "route_pack_chunks_per_s": r["route_pack_chunks_per_s"]})
            log(f"[sweep] {rows[-1]}")
        print(json.dumps({"sweep": "chunk", "workload": w.name, "data": "synthetic", "rows": rows}), flush=True)
        return 0
    if args.sweep == "share":
        base = synth.WORKLOADS["stack32_32k"]
        rows = []
        for g in (1, 2, 4, 8):
            r = bench_stack(args, dataclasses.replace(base, n_layers=8, share_group=g, name=f"{base.name}/8layers/share{g}"))
            rows.append({"share_group": g, "layers": 8, "routed_layers": r["routed_layers"],
                         "prefill_route_ms": r["prefill_route_ms"], "prefill_pack_ms": r["prefill_pack_ms"],
                         "route_pack_chunks_per_s": r["route_pack_chunks_per_s"],
                         "decode_step_ms": round(r["roofline"]["avg_ms"] * 8, 4)})
            log(f"[sweep] {rows[-1]}")
        print(json.dumps({"sweep": "share", "workload": base.name + " (8 layers)", "data": "synthetic", "rows": rows}), flush=True)
        return 0
    if args.ragged:
        print(json.dumps(bench_ragged(args)), flush=True)
        return 0
    if args.kquant_error:
        print(json.dumps(kquant_error(args, w)), flush=True)
        return 0
    res = bench_stack(args, w) if w.n_layers > 1 else bench_layer(args, w)
    print(json.dumps(res), flush=True)
    return 0


def bench_layer(args, w):
    """One layer: a step = route + pack + one decode call (see the module docstring)."""
    import torch
    from paper_2506_07533_amd import binding as mq, synth
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    BH, C, T, M = w.batch * w.n_kv_heads, w.n_chunks, w.n_tail, len(w.expert_bits)
    cfg = mq.Cfg(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.chunk, w.group, w.expert_bits, w.freeze_chunks,
                 1 if args.per_channel else 0)

    t0 = time.time()
    d = synth.make_workload(w)
    log(f"[bench] synthetic {w.name}: K,V {d['K'].shape} generated in {time.time() - t0:.1f}s")
    K = torch.from_numpy(d["K"]).to(dev); V = torch.from_numpy(d["V"]).to(dev)
    W1, W2, W3 = (torch.from_numpy(d[k]).to(dev) for k in ("W1", "W2", "W3"))
    q = torch.from_numpy(d["q"]).to(dev)
    Kt = torch.zeros((w.batch, w.n_kv_heads, w.chunk, w.head_dim), dtype=torch.float16, device=dev)
    Vt = torch.zeros_like(Kt)
    if T:
        Kt[:, :, :T] = K[:, :, C * w.chunk:]; Vt[:, :, :T] = V[:, :, C * w.chunk:]

    expert = torch.zeros((BH, C), dtype=torch.uint8, device=dev)
    votes = torch.zeros((BH, C, M), dtype=torch.int32, device=dev)
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    # first pass sizes the arenas (realised mix), then two arenas alternate
    mq.route_chunks(cfg, K, 0, C, W1, W2, W3, None, expert, votes)
    if args.force_bits:
        expert.fill_(list(w.expert_bits).index(args.force_bits))
    torch.cuda.synchronize()
    e_host = expert.cpu().numpy()
    bits_of = np.array(w.expert_bits)[e_host]
    blk = {b: mq.chunk_block_bytes(cfg, b) for b in w.expert_bits}
    packed_bytes = int(sum(blk[b] * int((bits_of == b).sum()) for b in w.expert_bits))
    mix = {str(b): round(float((bits_of == b).mean()), 4) for b in w.expert_bits}
    cap = int(sum(-(-blk[b] // 256) * 256 * int((bits_of == b).sum()) for b in w.expert_bits)) + 4096   # every block starts on a multiple of 256
    arenas = [torch.zeros(cap, dtype=torch.uint8, device=dev) for _ in range(2)]
    useds = [torch.zeros(1, dtype=torch.int64, device=dev) for _ in range(2)]
    offs = [torch.zeros((BH, C), dtype=torch.int64, device=dev) for _ in range(2)]
    out = torch.zeros((w.batch, w.n_q_heads, w.head_dim), dtype=torch.float32, device=dev)
    # one decode workspace per arena: the plan of a cache (moqae_decode_plan) is made when it is packed and serves the
    # decode calls on it, as in serving, where hundreds of decode steps follow on unchanged tables
    wss = [torch.zeros(mq.decode_workspace_bytes(cfg, C), dtype=torch.uint8, device=dev) for _ in range(2)]
    scale = 1.0 / float(np.sqrt(w.head_dim))

    hev = HipEvents(args.steps)
    L = mq.lib()
    ws_unplanned = torch.zeros(mq.decode_workspace_bytes(cfg, C), dtype=torch.uint8, device=dev)

    def step(i, ev=None, k=None):
        a = i & 1
        kind = None if k is None else k % 3              # 0: planned call, 1: its main kernel alone, 2: unplanned call
        useds[a].zero_()
        if ev: ev[0].record()
        if not args.decode_only:
            mq.route_chunks(cfg, K, 0, C, W1, W2, W3, None, expert, votes)
        if ev: ev[1].record()
        if not args.decode_only:
            mq.quantize_pack(cfg, K, V, 0, C, expert, arenas[a], useds[a], offs[a], status)
            mq.decode_plan(cfg, expert, C, wss[a])       # counted with the pack call
        if ev: ev[2].record()
        if kind == 1: L.moqae_bench_time_decode_kernel(*hev.pair(k))
        if kind == 2:
            mq.decode_attn(cfg, q, arenas[a ^ 1], offs[a ^ 1], expert, C, Kt if T else None, Vt if T else None, T,
                           scale, out, ws_unplanned)
        else:
            mq.decode_attn(cfg, q, arenas[a ^ 1], offs[a ^ 1], expert, C, Kt if T else None, Vt if T else None, T,
                           scale, out, wss[a ^ 1], planned=True)
        if kind == 1: L.moqae_bench_time_decode_kernel(None, None)
        if ev: ev[3].record()

    for a in range(2):                                   # both arenas packed before anything is timed
        useds[a].zero_()
        mq.quantize_pack(cfg, K, V, 0, C, expert, arenas[a], useds[a], offs[a], status)
        mq.decode_plan(cfg, expert, C, wss[a])
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    assert int(status.item()) == 0, "arena overflow"

    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i, evs[i], i)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t_start) * 1e3
    assert int(status.item()) == 0, "arena overflow"
    t_route = np.array([e[0].elapsed_time(e[1]) for e in evs])
    t_pack = np.array([e[1].elapsed_time(e[2]) for e in evs])
    # the whole planned call (two kernels) on steps 0, 3, ..., where nothing else is recorded inside it; its main
    # kernel alone on steps 1, 4, ...; the whole unplanned call (three kernels) on steps 2, 5, ...
    t_attn = np.array([e[2].elapsed_time(e[3]) for i, e in enumerate(evs) if i % 3 == 0])
    t_split = np.array([hev.elapsed_ms(i) for i in range(args.steps) if i % 3 == 1]) if args.steps > 1 else t_attn
    t_unpl = np.array([e[2].elapsed_time(e[3]) for i, e in enumerate(evs) if i % 3 == 2]) if args.steps > 2 else t_attn
    ms_per_step = wall_ms / args.steps

    n_units = BH * C
    kv_bytes = n_units * w.chunk * w.head_dim * 2
    attn_bytes = packed_bytes + n_units * 9 + 2 * BH * T * w.head_dim * 2 + q.numel() * 2 + out.numel() * 4
    route_bytes = kv_bytes + n_units * (1 + 4 * M)
    pack_bytes = 2 * kv_bytes + packed_bytes + n_units * 9

    def roof(bytes_, t_ms):
        g = bytes_ / (t_ms.mean() * 1e-3) / 1e9
        return {"bound": "hbm", "achieved": round(g, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": round(g / HBM_PEAK_GBPS, 4), "traffic": None,
                "bytes_per_launch": int(bytes_), "avg_ms": round(float(t_ms.mean()), 4),
                "min_ms": round(float(t_ms.min()), 4), "median_ms": round(float(np.median(t_ms)), 4)}

    res = {
        "metric": "decode_attn_hbm_GBps", "value": None, "unit": "GB/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": DTYPE[1 if w.n_q_heads == w.n_kv_heads else 0], "data": "synthetic",
        "config": {"workload": w.name, "batch": w.batch, "q_heads": w.n_q_heads, "kv_heads": w.n_kv_heads,
                   "head_dim": w.head_dim, "cached_tokens": w.seq, "chunk": w.chunk, "group": w.group,
                   "expert_bits": list(w.expert_bits), "k_per_channel": int(args.per_channel), "realised_mix": mix, "chunks": n_units,
                   "packed_bytes": packed_bytes, "fp16_equiv_bytes": 2 * kv_bytes},
        # the dominant kernel, timed alone by a pair of HIP events the library records around it
        "roofline": dict(roof(attn_bytes, t_split), kernel="attn_split_kernel"),
        # the decode call as a whole (moqae_decode_attn_planned): attn_split_kernel + attn_merge_kernel and the gap; the
        # plan of the tables is made once per packed cache (with the pack call above), not per decode step
        "decode_call": dict(roof(attn_bytes, t_attn), entry_point="moqae_decode_attn_planned", samples=int(t_attn.size)),
        # the same call with the plan made inside it (moqae_decode_attn: attn_prep_kernel + the two kernels above)
        "decode_call_unplanned": dict(roof(attn_bytes, t_unpl), entry_point="moqae_decode_attn", samples=int(t_unpl.size)),
        "pct_of_hbm_peak": None,
    }
    res["roofline"]["samples"] = int(t_split.size)
    res["stream_ceiling"] = stream_ceiling(mq, dev)
    if not args.force_bits:
        res["roofline"]["traffic"] = measured_traffic(w.name)
    res["value"] = res["decode_call"]["achieved"]
    res["pct_of_hbm_peak"] = round(100 * res["decode_call"]["frac"], 2)
    if not args.decode_only:
        res["roofline_route"] = dict(roof(route_bytes, t_route), kernel="route_kernel")
        res["roofline_pack"] = dict(roof(pack_bytes, t_pack), kernel="plan_rows_kernel + pack_kernel + arena_end_kernel (+ attn_prep_kernel: the decode plan)")
        res["route_pack_chunks_per_s"] = round(n_units / ((t_route.mean() + t_pack.mean()) * 1e-3), 1)
        res["route_chunks_per_s"] = round(n_units / (t_route.mean() * 1e-3), 1)
        res["pack_chunks_per_s"] = round(n_units / (t_pack.mean() * 1e-3), 1)

    if not args.decode_only:
        # the same compression in ONE kernel on the paged store (moqae_route_pack_paged: router, page, quantiser per chunk;
        # K is read from HBM once), timed beside the two-call path above
        pages = tuple(int((bits_of == b).sum()) + 8 for b in w.expert_bits)
        p_arena = torch.zeros(mq.pool_arena_bytes(cfg, pages), dtype=torch.uint8, device=dev)
        p_state = torch.zeros(mq.pool_state_bytes(cfg, pages) // 4, dtype=torch.int32, device=dev)
        p_off = torch.zeros((BH, C), dtype=torch.int64, device=dev)
        p_expert = torch.zeros((BH, C), dtype=torch.uint8, device=dev)
        n_f = max(10, args.steps // 3)
        fev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_f)]
        for i in range(3 + n_f):
            mq.pool_init(cfg, pages, p_state)
            if i >= 3: fev[i - 3][0].record()
            mq.route_pack_paged(cfg, pages, K, V, 0, C, (W1, W2, W3, None), p_expert, votes, p_arena, p_state, p_off, status)
            if i >= 3: fev[i - 3][1].record()
        torch.cuda.synchronize()
        assert int(status.item()) == 0 and torch.equal(p_expert, expert), "paged path"
        t_f = np.array([a.elapsed_time(b) for a, b in fev])
        fused_bytes = 2 * kv_bytes + packed_bytes + n_units * (9 + 1 + 4 * M)
        res["roofline_route_pack_paged"] = dict(roof(fused_bytes, t_f), kernel="route_pack_kernel (router + page + quantiser, one pass)",
                                                samples=n_f)
        res["route_pack_paged_chunks_per_s"] = round(n_units / (t_f.mean() * 1e-3), 1)
        # the second half of the headline metric, both ways of doing the same work
        res["quantize_route_chunks_per_s"] = {"two_calls (moqae_route_chunks + moqae_quantize_pack)": res["route_pack_chunks_per_s"],
                                              "one_call (moqae_route_pack_paged)": res["route_pack_paged_chunks_per_s"],
                                              "best": max(res["route_pack_chunks_per_s"], res["route_pack_paged_chunks_per_s"])}
        del p_arena

    if not args.decode_only and not args.per_channel and w.n_q_heads // w.n_kv_heads <= 2:
        # four new tokens per sequence in one call (moqae_decode_attn_multi): the same bytes serve four queries
        Qn = 4
        qm = torch.randn((w.batch, Qn, w.n_q_heads, w.head_dim), dtype=torch.float16, device=dev)
        om = torch.zeros((w.batch, Qn, w.n_q_heads, w.head_dim), dtype=torch.float32, device=dev)
        wsm = torch.zeros(mq.decode_workspace_bytes_multi(cfg, C, Qn), dtype=torch.uint8, device=dev)
        Ktm = torch.randn((w.batch, w.n_kv_heads, w.chunk, w.head_dim), dtype=torch.float16, device=dev); Vtm = torch.randn_like(Ktm)
        mev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(20)]
        for i in range(23):
            a = i & 1
            if i >= 3: mev[i - 3][0].record()
            mq.decode_attn_multi(cfg, qm, arenas[a], offs[a], expert, C, Ktm, Vtm, Qn, scale, om, wsm)
            if i >= 3: mev[i - 3][1].record()
        torch.cuda.synchronize()
        t_m = np.array([a.elapsed_time(b) for a, b in mev])
        res["decode_call_4_queries"] = dict(roof(attn_bytes, t_m), entry_point="moqae_decode_attn_multi", queries=Qn, samples=20)

    if not args.decode_only:
        # router fine-tuning (Sec. 3.3): loss and gradient over every cached key row of the layer, synthetic L_nll
        nll = torch.full((w.batch,), 2.0, dtype=torch.float32, device=dev)
        loss = torch.zeros(3, dtype=torch.float32, device=dev)
        g1 = torch.zeros((w.head_dim, M), dtype=torch.float32, device=dev); g2 = torch.zeros_like(g1)
        g3 = torch.zeros((M, M), dtype=torch.float32, device=dev); gb = torch.zeros(M, dtype=torch.float32, device=dev)
        tev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(10)]
        for i in range(12):
            if i >= 2: tev[i - 2][0].record()
            mq.router_loss_grad(cfg, K, 0, C * w.chunk, W1, W2, W3, None, nll, None, None, 0.5, loss, g1, g2, g3, gb)
            if i >= 2: tev[i - 2][1].record()
        torch.cuda.synchronize()
        t_t = np.array([a.elapsed_time(b) for a, b in tev])
        rows = BH * C * w.chunk
        flop = rows * (8 * M * w.head_dim)               # 2*M*D multiply-adds forward and as many for dW1, dW2
        tf = flop / (t_t.mean() * 1e-3) / 1e12
        res["router_train"] = {"bound": "alu", "achieved": round(tf, 2), "peak": 157.3, "unit": "TFLOP/s", "frac": round(tf / 157.3, 4),
                               "rows": rows, "flop_per_row": 8 * M * w.head_dim, "avg_ms": round(float(t_t.mean()), 4),
                               "min_ms": round(float(t_t.min()), 4), "rows_per_s": round(rows / (t_t.mean() * 1e-3), 1),
                               "kernel": "router_train_kernel (Eq. (3)-(5): loss + gradient, binary32)", "loss": [round(float(v), 6) for v in loss.cpu()]}

    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(w, d, scale)
    return res


def kquant_error(args, w):
    """How much the quantiser of the keys costs in attention accuracy on keys with outlier channels (the structure Sec. 2.2
    quotes): uniform 2 / 4 / 8-bit caches, keys per token vs per channel, against fp64 attention over the raw fp16 K, V."""
    import torch
    from paper_2506_07533_amd import binding as mq, synth
    dev = torch.device("cuda:0")
    H, S = 4, 16384
    ws_ = dataclasses.replace(w, batch=1, n_q_heads=H, n_kv_heads=H, seq=S, name=w.name + "/4heads16k")
    d = synth.make_workload(ws_)
    K, V, q = d["K"], d["V"], d["q"]
    scale = 1.0 / float(np.sqrt(w.head_dim))
    Kf, Vf, qf = K.astype(np.float64), V.astype(np.float64), q.astype(np.float64)
    sc = scale * np.einsum("bhsd,bhd->bhs", Kf, qf); sc -= sc.max(-1, keepdims=True)
    p = np.exp(sc); p /= p.sum(-1, keepdims=True)
    o_ref = np.einsum("bhs,bhsd->bhd", p, Vf)
    C = S // w.chunk
    Kd, Vd, qd = (torch.from_numpy(x).to(dev) for x in (K, V, q))
    rows = []
    for bits in (2, 4, 8):
        row = {"bits": bits}
        for kpc in (0, 1):
            cfg = mq.Cfg(1, H, H, w.head_dim, w.chunk, w.group, (bits, 16), 0, kpc)
            expert = torch.zeros((H, C), dtype=torch.uint8, device=dev)
            arena = torch.zeros(mq.arena_upper_bound(cfg, H * C), dtype=torch.uint8, device=dev)
            used = torch.zeros(1, dtype=torch.int64, device=dev); status = torch.zeros(1, dtype=torch.int32, device=dev)
            off = torch.zeros((H, C), dtype=torch.int64, device=dev)
            mq.quantize_pack(cfg, Kd, Vd, 0, C, expert, arena, used, off, status)
            out = torch.zeros((1, H, w.head_dim), dtype=torch.float32, device=dev)
            wsb = torch.zeros(mq.decode_workspace_bytes(cfg, C), dtype=torch.uint8, device=dev)
            mq.decode_attn(cfg, qd, arena, off, expert, C, None, None, 0, scale, out, wsb)
            torch.cuda.synchronize()
            assert int(status.item()) == 0
            o = out.cpu().numpy().astype(np.float64)
            err = np.abs(o - o_ref).max(-1) / np.abs(o_ref).max(-1)
            row["per_channel" if kpc else "per_token"] = round(float(err.max()), 5)
        rows.append(row)
        log(f"[kquant] {row}")
    return {"kquant_error": "max-norm relative error of the attention output against fp64 attention over the raw fp16 cache",
            "workload": ws_.name, "chunk": w.chunk, "group": w.group, "data": "synthetic (four outlier channels per head, x10)", "rows": rows}


def stream_ceiling(mq, dev):
    """What a plain read-only streaming kernel (csrc/stream_probe.hip: 16-byte loads, 2 GiB read once per launch,
    eight times the 256 MB last-level cache) reaches on this GPU: the practical ceiling of any read-bound kernel."""
    import ctypes as C
    import torch
    L = mq.lib()
    L.moqae_bench_stream_sink_words.restype = C.c_uint32
    L.moqae_bench_stream_read.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p, C.c_void_p]
    nbytes = 2 << 30
    buf = torch.zeros(nbytes // 4, dtype=torch.int32, device=dev)
    sink = torch.zeros(int(L.moqae_bench_stream_sink_words()), dtype=torch.int32, device=dev)
    st = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    n = 20
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
    for i in range(3 + n):
        if i >= 3: ev[i - 3][0].record()
        assert L.moqae_bench_stream_read(C.c_void_p(buf.data_ptr()), nbytes, C.c_void_p(sink.data_ptr()), st) == 0
        if i >= 3: ev[i - 3][1].record()
    torch.cuda.synchronize()
    t = np.array([a.elapsed_time(b) for a, b in ev])
    g = nbytes / (np.median(t) * 1e-3) / 1e9
    return {"achieved": round(float(g), 1), "unit": "GB/s", "frac_of_peak": round(float(g / HBM_PEAK_GBPS), 4),
            "bytes_per_launch": nbytes, "median_ms": round(float(np.median(t)), 4), "min_ms": round(float(t.min()), 4),
            "kernel": "stream_read_kernel (read-only, 16-byte loads)", "samples": n}


def bench_stack(args, w):
    """The multi-layer workload: prefill compression of every layer with routing sharing (one routed
    layer per group), then decode steps that append one token to every layer and attend over it.
    A step here = one decode step over all layers (append + decode call per layer)."""
    import math
    import torch
    from paper_2506_07533_amd import binding as mq, cache, synth
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    N, D, B, H = w.chunk, w.head_dim, w.batch, w.n_kv_heads
    C0 = w.seq // N
    cfg = mq.Cfg(B, w.n_q_heads, H, D, N, w.group, w.expert_bits, w.freeze_chunks)
    blk = [mq.chunk_block_bytes(cfg, b) for b in w.expert_bits]
    mean_blk = sum(sz * p for sz, p in zip(blk, w.mix))
    arena_bytes = int(B * H * (C0 + 2) * mean_blk * 1.08)
    stack = cache.KVStack(cfg, w.n_layers, w.share_group, C0 + 1, arena_bytes=[arena_bytes] * w.n_layers)
    routers = {}
    t_route = t_pack = 0.0
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    for l in range(w.n_layers):
        d = synth.make_layer_device(w, l, dev)
        routers[l] = (d["W1"], d["W2"], d["W3"], None)
        lc = stack.layers[l]
        # one untimed pass first (the first kernel to touch freshly written tensors of this size pays several
        # milliseconds of address-translation warm-up that has nothing to do with the method)
        if stack.is_leader(l):
            lc.route(d["K"], 0, C0, routers[l])
        else:
            lc.share_decisions_from(stack.layers[stack.leader_of(l)], 0, C0)
        lc.pack(d["K"], d["V"], 0, C0)
        lc.arena_used.zero_()
        torch.cuda.synchronize()
        ev[0].record()
        if stack.is_leader(l):
            lc.route(d["K"], 0, C0, routers[l])
        else:
            lc.share_decisions_from(stack.layers[stack.leader_of(l)], 0, C0)
        ev[1].record()
        lc.pack(d["K"], d["V"], 0, C0)
        ev[2].record()
        torch.cuda.synchronize()
        lc.n_chunks, lc.n_tail = C0, 0
        t_route += ev[0].elapsed_time(ev[1]); t_pack += ev[1].elapsed_time(ev[2])
        lc.check_status()
        del d
        log(f"[bench] layer {l} compressed: {'route' if stack.is_leader(l) else 'share'} {ev[0].elapsed_time(ev[1]):.3f} ms, "
            f"pack {ev[1].elapsed_time(ev[2]):.3f} ms")
    packed = sum(int(lc.arena_used.item()) for lc in stack.layers)
    n_units = B * H * C0 * w.n_layers

    scale = 1.0 / math.sqrt(D)
    g = torch.Generator(device=dev); g.manual_seed(99)
    kn = torch.randn((B, H, D), generator=g, device=dev, dtype=torch.float16)
    vn = torch.randn((B, H, D), generator=g, device=dev, dtype=torch.float16)
    q = torch.randn((B, w.n_q_heads, D), generator=g, device=dev, dtype=torch.float16)
    out = torch.zeros((B, w.n_q_heads, D), dtype=torch.float32, device=dev)

    def step():
        for l in range(w.n_layers):
            stack.append(l, kn, vn, routers)
            stack.layers[l].decode(q, out, scale)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    gpu_ms = e0.elapsed_time(e1)
    n_tail = stack.layers[0].n_tail
    step_bytes = packed + w.n_layers * (B * H * C0 * 9 + 2 * B * H * n_tail * D * 2 + q.numel() * 2 + out.numel() * 4)
    gbps = step_bytes / (gpu_ms / args.steps * 1e-3) / 1e9
    res = {
        "metric": "decode_attn_hbm_GBps", "value": round(gbps, 1), "unit": "GB/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(wall_ms / args.steps, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": DTYPE[1 if w.n_q_heads == H else 0], "data": "synthetic",
        "config": {"workload": w.name, "batch": B, "q_heads": w.n_q_heads, "kv_heads": H, "head_dim": D,
                   "cached_tokens": w.seq, "chunk": N, "group": w.group, "layers": w.n_layers,
                   "routing_sharing_group": w.share_group, "chunks": n_units, "packed_bytes": packed,
                   "step": "one decode step over all layers: append one token and one decode call per layer"},
        "roofline": {"bound": "hbm", "achieved": round(gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(gbps / HBM_PEAK_GBPS, 4), "traffic": None, "bytes_per_launch": int(step_bytes // w.n_layers),
                     "avg_ms": round(gpu_ms / args.steps / w.n_layers, 4),
                     "kernel": "decode calls of a step, appends included (GPU time of the step / layers)"},
        "pct_of_hbm_peak": round(100 * gbps / HBM_PEAK_GBPS, 2),
        "prefill_route_ms": round(t_route, 3), "prefill_pack_ms": round(t_pack, 3),
        "route_pack_chunks_per_s": round(n_units / ((t_route + t_pack) * 1e-3), 1),
        "routed_layers": sum(1 for l in range(w.n_layers) if stack.is_leader(l)),
    }
    return res


def bench_ragged(args):
    """One layer of the stack workload's shape (16 sequences x 32 KV heads, chunk 128, planted mix) packed to 32k
    tokens; the sequences then attend to 2k, 4k, ... 32k tokens of it (plus residuals of different lengths)."""
    import math
    import torch
    from paper_2506_07533_amd import binding as mq, cache, synth
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    w = dataclasses.replace(synth.WORKLOADS["stack32_32k"], n_layers=1, share_group=1, name="ragged16_2k-32k")
    N, D, B, H = w.chunk, w.head_dim, w.batch, w.n_kv_heads
    C0 = w.seq // N
    cfg = mq.Cfg(B, w.n_q_heads, H, D, N, w.group, w.expert_bits, w.freeze_chunks)
    d = synth.make_layer_device(w, 0, dev)
    lc = cache.LayerCache(cfg, C0)
    lc.route(d["K"], 0, C0, (d["W1"], d["W2"], d["W3"], None))
    lc.pack(d["K"], d["V"], 0, C0)
    torch.cuda.synchronize()
    lc.check_status()
    lens_c = [(b + 1) * C0 // B for b in range(B)]                 # 16, 32, ... 256 chunks
    lens_t = [(37 * b) % N for b in range(B)]
    lc.K_tail.copy_(d["K"][:, :, :N]); lc.V_tail.copy_(d["V"][:, :, :N])
    nc = torch.tensor(lens_c, dtype=torch.int32, device=dev); nt = torch.tensor(lens_t, dtype=torch.int32, device=dev)
    q = d["q"]
    out = torch.zeros((B, w.n_q_heads, D), dtype=torch.float32, device=dev)
    ws = torch.zeros(mq.decode_workspace_bytes_ragged(cfg, C0), dtype=torch.uint8, device=dev)
    scale = 1.0 / math.sqrt(D)
    e_host = lc.expert[:, :C0].cpu().numpy()
    blk = np.array([mq.chunk_block_bytes(cfg, b) for b in w.expert_bits], np.int64)
    sizes = blk[e_host]                                             # [B*H, C0]
    bytes_r = sum(int(sizes[b * H:(b + 1) * H, :lens_c[b]].sum()) + lens_c[b] * H * 9 + 2 * H * lens_t[b] * D * 2 for b in range(B))
    bytes_u = int(sizes.sum()) + B * H * C0 * 9
    bytes_r += q.numel() * 2 + out.numel() * 4; bytes_u += q.numel() * 2 + out.numel() * 4
    # a second cache of the same contents, so that consecutive calls do not read what the last-level cache holds
    lc2 = cache.LayerCache(cfg, C0)
    lc2.expert.copy_(lc.expert); lc2.pack(d["K"], d["V"], 0, C0); lc2.K_tail.copy_(lc.K_tail); lc2.V_tail.copy_(lc.V_tail)
    torch.cuda.synchronize()
    caches = [lc, lc2]

    def run(ragged, i):
        c = caches[i & 1]
        if ragged:
            mq.decode_attn_ragged(cfg, q, c.arena, c.chunk_off, c.expert, nc, C0, c.K_tail, c.V_tail, nt, scale, out, ws)
        else:
            mq.decode_attn(cfg, q, c.arena, c.chunk_off, c.expert, C0, None, None, 0, scale, out, ws)

    def timed(ragged):
        for i in range(args.warmup):
            run(ragged, i)
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
        torch.cuda.synchronize()
        for i, (e0, e1) in enumerate(ev):
            e0.record(); run(ragged, i); e1.record()
        torch.cuda.synchronize()
        return np.array([e0.elapsed_time(e1) for e0, e1 in ev])

    t_r, t_u = timed(True), timed(False)
    g_r = bytes_r / (t_r.mean() * 1e-3) / 1e9; g_u = bytes_u / (t_u.mean() * 1e-3) / 1e9
    return {"metric": "decode_attn_hbm_GBps", "value": round(g_r, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
            "warmup": args.warmup, "ms_per_step": round(float(t_r.mean()), 4), "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": DTYPE[1], "data": "synthetic",
            "config": {"workload": w.name, "batch": B, "q_heads": w.n_q_heads, "kv_heads": H, "head_dim": D, "chunk": N,
                       "group": w.group, "chunks_per_sequence": lens_c, "residual_rows": lens_t, "packed_bytes_read": bytes_r},
            "roofline": {"bound": "hbm", "achieved": round(g_r, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                         "frac": round(g_r / HBM_PEAK_GBPS, 4), "traffic": None, "bytes_per_launch": bytes_r,
                         "avg_ms": round(float(t_r.mean()), 4), "min_ms": round(float(t_r.min()), 4),
                         "kernel": "whole moqae_decode_attn_ragged call"},
            "uniform_call_full_length": {"achieved": round(g_u, 1), "frac": round(g_u / HBM_PEAK_GBPS, 4),
                                         "bytes_per_launch": bytes_u, "avg_ms": round(float(t_u.mean()), 4)}}


def cpu_baseline(w, d, scale):
    """The CPU oracle as it stands, timed on the first KV heads of the same workload."""
    from oracle import moqae_ref as R
    threads = R.num_threads()
    # every (sequence 0, KV head) row when that is at most four per thread (about 10 s of CPU work at 128k tokens), else two per thread
    rows0 = w.batch * w.n_kv_heads if w.batch == 1 else w.n_kv_heads
    Hs = rows0 if rows0 <= 4 * threads else max(1, 2 * threads)
    rep = w.n_q_heads // w.n_kv_heads
    C, T = w.n_chunks, w.n_tail
    rcfg = R.RefCfg(1, Hs * rep, Hs, w.head_dim, w.chunk, w.group, w.expert_bits, w.freeze_chunks)
    K = d["K"][:1, :Hs]; V = d["V"][:1, :Hs]; q = np.ascontiguousarray(d["q"][:1, :Hs * rep])
    t0 = time.perf_counter()
    e, _ = R.route_chunks(rcfg, K, 0, C, d["W1"], d["W2"], d["W3"])
    t1 = time.perf_counter()
    sizes = np.array([R.chunk_block_bytes(rcfg, b) for b in w.expert_bits], np.uint64)[e]
    arena = np.zeros(int(sizes.sum()) + 4096, np.uint8); used = np.zeros(1, np.uint64); off = np.zeros(e.shape, np.uint64)
    t2 = time.perf_counter()
    assert R.quantize_pack(rcfg, K, V, 0, C, e, arena, used, off) == 0
    t3 = time.perf_counter()
    Kt = np.zeros((1, Hs, w.chunk, w.head_dim), np.float16); Vt = np.zeros_like(Kt)
    if T:
        Kt[:, :, :T] = K[:, :, C * w.chunk:]; Vt[:, :, :T] = V[:, :, C * w.chunk:]
    R.decode_attn(rcfg, q, arena, off, e, C, Kt, Vt, T, scale)
    t4 = time.perf_counter()
    n = Hs * C
    return {"value": round(float(sizes.sum()) / (t4 - t3) / 1e9, 4), "unit": "GB/s", "cores": threads, "kind": "oracle",
            "sample": f"first {Hs} of {w.batch * w.n_kv_heads} (sequence, KV head) rows of the same workload, all "
                      f"{C} chunks each: route, pack and one decode-attention call",
            "route_pack_chunks_per_s": round(n / ((t1 - t0) + (t3 - t2)), 1),
            "route_s": round(t1 - t0, 3), "pack_s": round(t3 - t2, 3), "attn_s": round(t4 - t3, 3)}


if __name__ == "__main__":
    sys.exit(main())
