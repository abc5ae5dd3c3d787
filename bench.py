#!/usr/bin/env python3
"""Benchmark of the capped-memory training step on one MI355X.

Default workload: the largest of the five that one GPU holds with its slow-tier pool, the Llama-7B-shaped decoder
(32 layers, d=4096, 32 heads, SwiGLU 11008, vocabulary 32000, seq 2048, batch 4: 8192 tokens per step), bf16 with
fp32 AdamW state, memory cap 96 GB, synthetic seeded weights and tokens.  One step = forward, backward, AdamW
under the plan, with the slow tier paced to --bw bytes/s per direction (25 GB/s).  Its 118 GB pool is more than
these boxes can pin in host memory, so it is a device buffer outside the capped arena (said in config.slow_tier);
--workload gpt2_small_bf16 runs the GPT-2-small-shaped workload (40 % cap) with the pool in pinned host memory.
--slow-tier file puts the slow tier into a file instead (direct I/O at whatever the file system delivers; probed first).

Prints one JSON line: tokens/s under the cap (value), the uncapped ideal and the migration bound
beside it, the MFMA roofline of the GEMM kernel measured with HIP events in the timed region, and
the CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

GEMM_OPS = (2, 9, 10)          # forward, dX, dW contractions (one kernel template)
ATTN_OPS = (4, 17)
# memory-bound operators by trace op code
HBM_CLASSES = {"norm": (1, 14, 15), "activation": (5, 6, 12, 13), "rope": (3, 18), "cross_entropy": (7,),
               "embedding": (0, 19, 20), "adamw": (21,)}
PEAK_BF16_TFLOPS = 2500.0
PEAK_FP32_VECTOR_TFLOPS = 157.3


def gemm_traffic(workload):
    """Bytes per GEMM launch that cross between the L2s and the fabric, measured offline with rocprofv3 --pmc
    FETCH_SIZE / WRITE_SIZE runs of this command and kept with their provenance in profiles/gemm_traffic.json
    (workload -> bytes_per_launch, profile file, commit of the kernels measured).  None where no such run exists."""
    try:
        with open(os.path.join(ROOT, "profiles", "gemm_traffic.json")) as f:
            return json.load(f).get(workload)
    except OSError:
        return None


def probe_file_bw(path, total=2 << 30, block=8 << 20, threads=4):
    """Sequential write then read of `total` bytes in `block` pieces from `threads` threads, direct I/O if the file
    system has it: the bandwidth the file tier can expect.  Returns bytes/s per direction."""
    import mmap
    import threading
    flags = os.O_RDWR | os.O_CREAT
    try:
        fd = os.open(path, flags | os.O_DIRECT, 0o600)
        direct = True
    except OSError:
        fd = os.open(path, flags, 0o600)
        direct = False
    try:
        os.ftruncate(fd, total)
        try:
            os.posix_fallocate(fd, 0, total)
        except OSError:
            pass
        bufs = [mmap.mmap(-1, block) for _ in range(threads)]      # page aligned
        for b in bufs:
            b.write(os.urandom(4096) * (block // 4096))
        nblk = total // block

        def run(fn):
            def body(i):
                for j in range(i, nblk, threads):
                    fn(bufs[i], j * block)
            th = [threading.Thread(target=body, args=(i,)) for i in range(threads)]
            t0 = time.perf_counter()
            for t in th:
                t.start()
            for t in th:
                t.join()
            return total / (time.perf_counter() - t0)
        w = run(lambda b, off: os.pwrite(fd, b, off))
        if not direct:
            os.fsync(fd)
        r = run(lambda b, off: os.preadv(fd, [b], off))
        # both directions at once, as in a training step: even blocks are written while odd blocks are read
        bufs2 = [mmap.mmap(-1, block) for _ in range(threads)]
        res = {}

        def both(kind):
            def body(i):
                for j in range(2 * i + (kind == "r"), nblk, 2 * threads):
                    (os.pwrite(fd, bufs[i], j * block) if kind == "w" else os.preadv(fd, [bufs2[i]], j * block))
            th = [threading.Thread(target=body, args=(i,)) for i in range(threads)]
            t0 = time.perf_counter()
            for t in th:
                t.start()
            for t in th:
                t.join()
            res[kind] = (total / 2) / (time.perf_counter() - t0)
        tw, tr = threading.Thread(target=both, args=("w",)), threading.Thread(target=both, args=("r",))
        tw.start(); tr.start(); tw.join(); tr.join()
    finally:
        os.close(fd)
        if os.path.exists(path):
            os.remove(path)
    return {"write_Bps": w, "read_Bps": r, "duplex_write_Bps": res["w"], "duplex_read_Bps": res["r"], "direct": direct}


def _union(iv):
    out = []
    for a, b in sorted(iv):
        if b <= a:
            continue
        if out and a <= out[-1][1]:
            out[-1][1] = max(out[-1][1], b)
        else:
            out.append([a, b])
    return out


def interval_overlap(kernels, copies):
    """Both arguments: lists of (begin, end).  Returns the length of (union of copies) that lies inside (union of
    kernels), the length of the union of copies, and their ratio."""
    K, Cp = _union(kernels), _union(copies)
    both, i = 0, 0
    for a, b in Cp:
        while i < len(K) and K[i][1] <= a:
            i += 1
        j = i
        while j < len(K) and K[j][0] < b:
            both += max(0, min(b, K[j][1]) - max(a, K[j][0]))
            j += 1
    busy = sum(b - a for a, b in Cp)
    return {"copy_busy_ms": busy / 1e6, "copy_busy_under_kernels_ms": both / 1e6,
            "frac_of_copy_time_with_a_kernel_running": (both / busy) if busy else None,
            "kernel_busy_ms": sum(b - a for a, b in K) / 1e6}


def planner_times(names=("tiny_gpt_fp32", "gpt2_small_bf16", "llama_7b_bf16", "llama_13b_bf16", "llama_30b_bf16")):
    """CPU only: wall time of lifetime analysis + Algorithm 1 in the library and in the oracle, on the canonical
    traces of the five workloads with modelled kernel times, each at its stated capacity and bandwidth.  The
    library's planner also assigns addresses and lowers the planning capacity until the layout fits the arena
    (library_search_s: everything); the oracle runs Algorithm 1 once at the capacity the library settled on
    (oracle_single_s), and the library is timed on that single pass as well (library_single_s: unlimited arena).
    The single passes must give the same entries.  One JSON line."""
    import paper_2506_06472_amd as tio
    from oracle import plan as op, trace as ot
    from synth import CONFIGS
    rows = []
    for name in names:
        cfg = CONFIGS[name]
        bw = cfg.get("slow_tier_bw", 25 * 10**9)
        lt = tio.tio_trace_build(cfg)
        t0 = time.perf_counter()
        ll = tio.tio_analyze_lifetimes(lt)
        cap = cfg.get("cap_bytes") or int(int(ll.export()["M"].max()) * cfg["cap_frac"])
        pe = tio.tio_build_plan(lt, ll, cap, bw, min_bytes=1 << 20).export()
        t1 = time.perf_counter()
        single = tio.tio_build_plan(lt, ll, pe["planning_cap"], bw, min_bytes=1 << 20, arena_bytes=2**62).export()
        t2 = time.perf_counter()
        tr = ot.build_trace(cfg)
        t3 = time.perf_counter()
        ref = op.build_plan(tr, op.analyze_lifetimes(tr), pe["planning_cap"], bw, min_bytes=1 << 20)
        t4 = time.perf_counter()
        same = single["entries"] == ref["entries"] and pe["entries"] == ref["entries"]
        rows.append({"workload": name, "kernels": int(lt.export()["n_kernels"]), "entries": len(pe["entries"]),
                     "cap_bytes": int(cap), "planning_cap_bytes": int(pe["planning_cap"]),
                     "library_search_s": t1 - t0, "library_single_s": t2 - t1, "oracle_single_s": t4 - t3,
                     "same_plan": bool(same)})
        print(f"{name}: library {t1 - t0:.3f} s (search) / {t2 - t1:.3f} s (one pass), oracle {t4 - t3:.2f} s (one pass), "
              f"same plan {same}", file=sys.stderr, flush=True)
    out = {"planner_wall_time": rows, "cores": 1, "kernel_times": "modelled"}
    print(json.dumps(out))
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--retime", type=int, default=16,
                    help="re-timing passes of the planner (0: the paper's plan alone); with passes, the paper's plan is timed as well")
    ap.add_argument("--workload", default="llama_7b_bf16")
    ap.add_argument("--bw", type=float, default=-1, help="slow-tier bytes/s per direction; 0 = unthrottled; default: the workload's (25e9)")
    ap.add_argument("--min-bytes", type=int, default=1 << 20)
    ap.add_argument("--file", default="/tmp/teraio_slow_tier.bin", help="--slow-tier file: path of the file (created, removed at the end)")
    ap.add_argument("--staging-mb", type=int, default=256, help="--slow-tier file: pinned staging buffer, MiB")
    ap.add_argument("--chunk-mb", type=int, default=8, help="--slow-tier file: transfer chunk, MiB")
    ap.add_argument("--slow-tier", choices=["auto", "host", "device", "file"], default="auto",
                    help="where the slow-tier pool lives: pinned host memory, or a device buffer outside the arena "
                         "(auto: host unless the pool exceeds what this kind of box can pin, about 28 GB)")
    ap.add_argument("--shared-channel", choices=["auto", "yes", "no"], default="auto",
                    help="plan with one channel shared by offloads and prefetches instead of one per direction "
                         "(auto: yes for the file tier, whose two directions share the device's bandwidth)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--modelled-tau", action="store_true", help="plan from modelled instead of measured kernel times")
    ap.add_argument("--dump-tau", default="", help="write the measured kernel times (ns, one per line: the format sweep --tau reads) to this file")
    ap.add_argument("--host-tier-bw", type=float, default=0,
                    help="bytes/s per direction of a second, host-memory destination beside the slow tier (the paper's "
                         "mixed mode); 0 = none; not the headline configuration")
    ap.add_argument("--host-budget", type=float, default=0, help="bytes of host memory the second destination may hold")
    ap.add_argument("--split-batch", action="store_true",
                    help="with --micro-batches n: split the workload's own batch into n groups instead of running n "
                         "batches per step (same tokens per step as the headline, smaller activations)")
    ap.add_argument("--micro-batches", type=int, default=1,
                    help="n > 1: a step is n micro-batches of the workload's batch with gradient accumulation and one "
                         "AdamW update (n times the tokens per step, same memory cap); not the headline configuration")
    ap.add_argument("--layers", type=int, default=0,
                    help="run the workload at reduced depth: this many decoder layers at the workload's widths, sequence "
                         "length and batch, with the memory cap scaled by (uncapped peak at this depth) / (uncapped peak at "
                         "full depth); for workloads whose arena plus slow-tier pool exceed one GPU's memory")
    ap.add_argument("--planner-times", action="store_true",
                    help="no GPU: time the library's and the oracle's planner on the five workloads' traces and exit")
    args = ap.parse_args()
    if args.planner_times:
        planner_times()
        return
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2506_06472_amd as tio
    from synth import CONFIGS, gen_params, gen_tokens, iter_params_pooled, to_bf16_round

    cfg = dict(CONFIGS[args.workload])
    full_layers, cap_scale = cfg["L"], 1.0
    if args.layers and args.layers != cfg["L"]:
        peak_of = lambda c: int(tio.tio_analyze_lifetimes(tio.tio_trace_build(c)).export()["M"].max())
        full_peak = peak_of(cfg)
        cfg["L"] = args.layers
        cap_scale = peak_of(cfg) / full_peak
    base_peak = None
    if args.micro_batches > 1:
        # the cap stays that of the workload itself (a fraction of the single-batch peak, or its byte figure)
        if "cap_frac" in cfg:
            base_peak = int(tio.tio_analyze_lifetimes(tio.tio_trace_build(cfg)).export()["M"].max())
        if not args.split_batch:
            cfg["B"] *= args.micro_batches
        elif cfg["B"] % args.micro_batches:
            raise SystemExit("--split-batch: the batch is not a multiple of --micro-batches")
        cfg["micro_batches"] = args.micro_batches
    t_start = time.perf_counter()
    log = lambda *a: print(f"[{time.perf_counter() - t_start:7.1f}s]", *a, file=sys.stderr, flush=True)
    bw = int(args.bw if args.bw >= 0 else cfg.get("slow_tier_bw", 25e9))
    file_probe = None
    shared = args.shared_channel == "yes" or (args.shared_channel == "auto" and args.slow_tier == "file")
    if args.slow_tier == "file":
        # the file system sets the pace: plan with what it delivers to four concurrent direct-I/O streams
        file_probe = probe_file_bw(args.file + ".probe")
        if args.bw <= 0:
            both = file_probe["duplex_write_Bps"] + file_probe["duplex_read_Bps"]
            bw = int(min(both, file_probe["write_Bps"], file_probe["read_Bps"])) if shared else \
                int(min(file_probe["duplex_write_Bps"], file_probe["duplex_read_Bps"]))
        log(f"file tier probe: write {file_probe['write_Bps'] / 1e9:.2f} GB/s, read {file_probe['read_Bps'] / 1e9:.2f} GB/s alone; "
            f"{file_probe['duplex_write_Bps'] / 1e9:.2f} + {file_probe['duplex_read_Bps'] / 1e9:.2f} GB/s together; "
            f"direct I/O {file_probe['direct']}; planning with {bw / 1e9:.2f} GB/s {'shared by both directions' if shared else 'per direction'}")
    S = cfg["B"] * cfg["T"]
    plist = tio.tio_param_list(cfg)
    n_params = sum(r * c for _, r, c in plist)
    specs = [(n, (r, c) if r > 1 else (c,), "normal" if (r > 1) else ("ones" if n.endswith("_g") else "zeros"))
             for n, r, c in plist]
    tok, lab = gen_tokens(cfg["B"], cfg["T"], cfg["V"], 0)
    small = n_params <= 10**9
    params = None
    if small:
        params = gen_params(specs, 0)
        if cfg["precision"] == "bf16":
            params = {k: to_bf16_round(v) for k, v in params.items()}

    def load_params(ctx):
        if small:
            ctx.tio_params_load(params)
        else:                       # one tensor at a time from a seeded pool (the library rounds to bf16 itself)
            for name, arr in iter_params_pooled(specs, 0):
                ctx.tio_params_load({name: arr})

    # ---- sizes: uncapped layout, and a preliminary capped plan (modelled kernel times) for the pool size
    lt = tio.tio_trace_build(cfg)
    ll = tio.tio_analyze_lifetimes(lt)
    M = ll.export()["M"]
    peak = int(M.max())
    cap = (int(cfg["cap_bytes"] * cap_scale) if "cap_bytes" in cfg else int((base_peak or peak) * cfg["cap_frac"])) // 256 * 256
    up = tio.tio_build_plan(lt, ll, 2**62, 0)
    upe = up.export()
    prelim = tio.tio_build_plan(lt, ll, cap, bw, duplex=not shared, min_bytes=args.min_bytes).export()
    host_bytes = int(max(upe["host_needed"], prelim["host_needed"] * 1.15)) + (1 << 20)
    arena_bytes = max(upe["arena_needed"], cap)
    log(f"{args.workload}: {n_params / 1e9:.3f} B parameters, uncapped peak {peak / 1e9:.2f} GB, cap {cap / 1e9:.2f} GB, "
        f"slow-tier pool {host_bytes / 1e9:.2f} GB at {bw / 1e9:.1f} GB/s")
    tier = args.slow_tier if args.slow_tier != "auto" else ("host" if host_bytes <= 28 * 10**9 else "device")
    arena = torch.empty(arena_bytes + 8192, dtype=torch.uint8, device="cuda:0")
    file_kw = {}
    if tier == "file":
        host = None
        host_bytes = int(host_bytes * 1.05) + (64 << 20)          # every range of the file is padded to 4 KiB
        file_kw = dict(slow_tier_file=args.file, staging_bytes=args.staging_mb << 20, file_chunk_bytes=args.chunk_mb << 20)
    elif tier == "host":
        host = torch.empty(host_bytes, dtype=torch.uint8, pin_memory=True)
    else:
        log("slow tier placed in device memory outside the arena (the box cannot pin a pool of this size)")
        host = torch.empty(host_bytes, dtype=torch.uint8, device="cuda:0")
    log("buffers allocated")

    # ---- profile on the uncapped layout, measure the ideal
    ctx = tio.tio_ctx_create(cfg, upe["arena_needed"], host_bytes, 0, arena=arena, host=host, **file_kw)
    load_params(ctx)
    log("parameters loaded; profiling on the uncapped layout")
    measured = ctx.tio_profile_iteration(tok, lab, tio.PROFILE_MEASURED)
    tau = measured.export()["tau"]
    log("sum of kernel times ms", tau.sum() / 1e6)
    if args.dump_tau:
        np.savetxt(args.dump_tau, tau, fmt="%d")
    for _ in range(args.warmup):
        ctx.tio_train_step(tok, lab, None)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):                      # timed like the capped loop below (events around every launch)
        ctx.tio_train_step(tok, lab, None, time_kernels=True)
    torch.cuda.synchronize()
    ideal_s = (time.perf_counter() - t0) / args.steps
    ctx.close()
    del ctx

    # ---- plan under the cap
    if not args.modelled_tau:
        lt.set_tau(tau)
    tp0 = time.perf_counter()
    plan_kw = dict(duplex=not shared, min_bytes=args.min_bytes, host_bw=int(args.host_tier_bw), host_budget=int(args.host_budget))
    plan = tio.tio_build_plan(lt, ll, cap, bw, retime_passes=args.retime, **plan_kw)
    plan_s = time.perf_counter() - tp0
    pe = plan.export()
    # the paper's plan (Algorithm 1 run once on the kernel times) beside the re-timed one, when they differ
    paper_plan = tio.tio_build_plan(lt, ll, cap, bw, **plan_kw) if pe["retime_pass"] > 0 else None
    ppe = paper_plan.export() if paper_plan is not None else None
    log('ideal ms', ideal_s * 1e3, 'plan: entries', len(pe['entries']), 'moved GB', pe['bytes_per_direction'] / 1e9, 'planner s', plan_s)
    host_needed = max(pe["host_needed"], ppe["host_needed"] if ppe else 0)
    if tier == "file":
        host_bytes = max(host_bytes, int(host_needed * 1.05) + (64 << 20))
    elif host_needed + (1 << 20) > host_bytes:
        host = None
        host_bytes = host_needed + (1 << 20)
        host = torch.empty(host_bytes, dtype=torch.uint8, pin_memory=True) if tier == "host" else \
            torch.empty(host_bytes, dtype=torch.uint8, device="cuda:0")

    # ---- capped run: the context sees only `cap` bytes of the arena
    ctx = tio.tio_ctx_create(cfg, cap, host_bytes, bw, arena=arena, host=host,
                             host_tier_bytes=max(pe["host_tier_needed"], ppe["host_tier_needed"] if ppe else 0) + 4096
                             if pe["host_tier_needed"] else 0,
                             host_tier_bw=int(args.host_tier_bw), **file_kw)
    load_params(ctx)
    first = ctx.tio_train_step(tok, lab, plan)
    # at initialisation the normalised hidden state has unit entries and the head weights are N(0, 0.02^2):
    # the logits are N(0, 0.0004 d) and the expected loss is ln V + 0.0002 d
    expect0 = np.log(cfg["V"]) + 0.0002 * cfg["d"]
    if abs(first["loss"] - expect0) > 0.05:
        raise RuntimeError(f"loss at initialisation {first['loss']} is not ln(V) + 0.0002 d = {expect0}")
    for _ in range(max(0, args.warmup - 1)):
        ctx.tio_train_step(tok, lab, plan)
    torch.cuda.synchronize()
    N = len(M)
    ops = lt.export()["op"]
    flops = lt.export()["flops"].astype(np.float64)
    ktimes = np.zeros(N, dtype=np.float64)
    d2h = h2d = 0
    loss = None
    t0 = time.perf_counter()
    for _ in range(args.steps):
        st = ctx.tio_train_step(tok, lab, plan, time_kernels=True)
        ktimes += ctx.tio_kernel_times(N)
        d2h += st["d2h_bytes"]
        h2d += st["h2d_bytes"]
        loss = st["loss"]
    torch.cuda.synchronize()
    step_s = (time.perf_counter() - t0) / args.steps
    # one more step, outside the timed region, with every kernel and every copy stamped on its own stream: the
    # compute/copy overlap is the share of the time a copy is in flight during which a kernel is running too
    ctx.tio_train_step(tok, lab, plan, timeline=True)
    k0, k1, c0, c1 = ctx.tio_step_timeline(N, len(pe["entries"]))
    overlap = interval_overlap(list(zip(k0.tolist(), k1.tolist())), [(a, b) for a, b in zip(c0.tolist(), c1.tolist()) if a >= 0])
    file_info = ctx.tio_file_tier_info() if tier == "file" else None
    paper = None
    if paper_plan is not None:
        # the same context goes on training under the paper's plan: one untimed step to settle, then the timed ones
        ctx.tio_train_step(tok, lab, paper_plan)
        torch.cuda.synchronize()
        tq = time.perf_counter()
        for _ in range(args.steps):
            ctx.tio_train_step(tok, lab, paper_plan, time_kernels=True)
        torch.cuda.synchronize()
        paper_s = (time.perf_counter() - tq) / args.steps
        paper = {"what": "Algorithm 1 and the urgent pass run once, on the measured kernel times (Section 3.2 as printed)",
                 "tokens_per_s": S / paper_s, "ms_per_step": paper_s * 1e3,
                 "model_predicted_ms_per_step": tio.tio_plan_simulate_engine(lt, paper_plan, bw, duplex=not shared)[0] / 1e6
                 if (bw and tier != "file") else tio.tio_plan_simulate(lt, paper_plan, bw, duplex=not shared)[0] / 1e6,
                 "bytes_per_direction": ppe["bytes_per_direction"], "greedy_pairs": ppe["n_greedy"], "urgent_pairs": ppe["n_forced"],
                 "planning_cap_bytes": ppe["planning_cap"]}
    ctx.close()
    if tier == "file" and os.path.exists(args.file):
        os.remove(args.file)
    ktimes /= args.steps

    gemm = np.isin(ops, GEMM_OPS)
    attn = np.isin(ops, ATTN_OPS)
    gemm_ns, gemm_flops, n_gemm = ktimes[gemm].sum(), flops[gemm].sum(), int(gemm.sum())
    tv = lt.export()
    gemm_bytes = sum(int(tv["tensor_bytes"][tv["operand_tensor"][tv["operand_off"][k]:tv["operand_off"][k + 1]]].sum())
                     for k in np.nonzero(gemm)[0])
    # memory-bound kernels: algorithmic bytes = operand tensor sizes, once per read and once per write
    kb = np.array([sum(int(tv["tensor_bytes"][t]) * ((int(f) & 1) + ((int(f) >> 1) & 1))
                       for t, f in zip(tv["operand_tensor"][tv["operand_off"][k]:tv["operand_off"][k + 1]],
                                       tv["operand_flags"][tv["operand_off"][k]:tv["operand_off"][k + 1]]))
                   for k in range(N)], dtype=np.float64)
    hbm = {}
    for label, codes in HBM_CLASSES.items():
        sel = np.isin(ops, codes)
        if sel.any():
            hbm[label] = {"GBps": kb[sel].sum() / ktimes[sel].sum(), "GBps_without_migration": kb[sel].sum() / float(tau[sel].sum()),
                          "ms_per_step": ktimes[sel].sum() / 1e6, "launches": int(sel.sum())}
    gemm_tflops = gemm_flops / gemm_ns / 1e3
    traffic = gemm_traffic(args.workload) if args.micro_batches == 1 else None
    bf16 = cfg["precision"] == "bf16"
    gemm_peak = PEAK_BF16_TFLOPS if bf16 else PEAK_FP32_VECTOR_TFLOPS
    attn_tflops = flops[attn].sum() / ktimes[attn].sum() / 1e3
    comp_s = ktimes.sum() / 1e9
    mig_bound_s = (pe["bytes_per_direction"] * (2 if shared else 1) / bw) if bw else 0.0
    bound_s = max(ideal_s, mig_bound_s)

    out = {
        "metric": "train tokens/s on 1 MI355X under GPU-mem cap", "value": S / step_s, "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": step_s * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": cfg["precision"],
        "data": "synthetic",
        "config": {"workload": args.workload, "layers_run": cfg["L"], "layers_of_the_workload": full_layers,
                   "cap_scaled_by": cap_scale, "micro_batches": args.micro_batches, "batch_split": bool(args.split_batch), "tokens_per_step": S, "mem_cap_bytes": cap, "uncapped_peak_bytes": peak,
                   "cap_frac_of_peak": cap / peak, "slow_tier_bw_bytes_per_s": bw, "channels": "one shared" if shared else "one per direction", 
                   "slow_tier": {"host": "pinned host memory", "device": "device memory outside the arena (stand-in)",
                                 "file": "file, direct I/O through a pinned staging ring"}[tier], "min_bytes": args.min_bytes,
                   "kernel_times": "modelled" if args.modelled_tau else "measured"},
        "ideal_tokens_per_s": S / ideal_s, "ideal_ms_per_step": ideal_s * 1e3,
        # the engine of a paced tier serves a ready queue in 16 MiB chunks, urgent requests first; unthrottled tiers and the
        # file tier serve in the order submitted
        "model_predicted_ms_per_step": (tio.tio_plan_simulate_engine(lt, plan, bw, duplex=not shared)[0] if (bw and tier != "file")
                                        else tio.tio_plan_simulate(lt, plan, bw, duplex=not shared)[0]) / 1e6,
        "model_first_come_first_served_ms_per_step": tio.tio_plan_simulate(lt, plan, bw, duplex=not shared)[0] / 1e6,
        "frac_of_ideal": ideal_s / step_s,
        "migration_bound_ms": mig_bound_s * 1e3, "frac_of_min_ideal_migration_bound": bound_s / step_s,
        "plan": {"how": ("Algorithm 1 re-run on the stalled timeline: pass %d kept (0 = the paper's plan, 1-%d fully stretched, %d-%d stretched from the memory peak on)"
                         % (pe["retime_pass"], args.retime, args.retime + 1, 2 * args.retime))
                        if args.retime else "Algorithm 1 run once",
                 "entries": len(pe["entries"]), "greedy_pairs": pe["n_greedy"], "urgent_pairs": pe["n_forced"],
                 "host_tier_pairs": sum(pe["tier"]), "host_tier_peak_bytes": pe["host_peak"],
                 "host_tier_bw_bytes_per_s": int(args.host_tier_bw), "host_tier_budget_bytes": int(args.host_budget),
                 "bytes_per_direction": pe["bytes_per_direction"], "planning_cap_bytes": pe["planning_cap"],
                 "arena_bytes_needed": pe["arena_needed"], "planner_seconds": plan_s},
        "copy": {"d2h_GBps": d2h / args.steps / step_s / 1e9, "h2d_GBps": h2d / args.steps / step_s / 1e9,
                 "cap_GBps": bw / 1e9},
        "kernel_ms_per_step": comp_s * 1e3, "kernel_share_of_step": comp_s / step_s,
        "overlap": overlap,
        "attention_tflops": attn_tflops, "loss": loss,
        "hbm_kernels": {"peak_GBps": 8000.0, "bytes": "operand tensor sizes, counted once per read and once per write",
                        "classes": hbm},
        # fp32 workloads (the tiny parity configurations) run the contractions on the fp32 vector ALU
        "roofline": {"bound": "mfma" if bf16 else "alu",
                     "kernel": ("gemm_bf16_dl_k" if bf16 else "gemm_f32_k") + " (forward, dX and dW contractions)",
                     "achieved": gemm_tflops, "peak": gemm_peak, "unit": "TFLOP/s",
                     "frac": gemm_tflops / gemm_peak, "traffic": (traffic or {}).get("bytes_per_launch"),
                     "traffic_unit": "bytes per launch missing the L2 (rocprofv3 FETCH_SIZE + WRITE_SIZE, calibrated); "
                                     "measured offline, not in this run",
                     "traffic_provenance": ({k: traffic[k] for k in ("profile", "kernels_as_of_commit")} if traffic else None),
                     "algorithmic_bytes_per_launch": gemm_bytes / n_gemm,
                     "launches_per_step": n_gemm, "avg_launch_us": gemm_ns / n_gemm / 1e3,
                     "achieved_without_migration": gemm_flops / float(tau[gemm].sum()) / 1e3,
                     "flops_per_step": gemm_flops},
    }

    if tier == "file":
        out["file_tier"] = {"path": args.file, "direct_io": bool(file_info["direct_io"]), "file_bytes": file_info["file_bytes"],
                            "probe_write_GBps": file_probe["write_Bps"] / 1e9, "probe_read_GBps": file_probe["read_Bps"] / 1e9,
                            "probe_duplex_write_GBps": file_probe["duplex_write_Bps"] / 1e9,
                            "probe_duplex_read_GBps": file_probe["duplex_read_Bps"] / 1e9,
                            "staging_bytes": args.staging_mb << 20, "chunk_bytes": args.chunk_mb << 20}
    if paper is not None:
        out["paper_plan"] = paper
    log('capped ms/step', step_s * 1e3, 'loss', loss, 'paper plan ms/step', paper and paper["ms_per_step"])
    if not args.no_cpu_baseline:
        # the oracle as it stands, fp32, on all host cores (numpy's BLAS threads), on the step's whole batch
        from oracle import model as om
        if small:
            cpu_tokens = S
            tr = om.Trainer(cfg, params, dtype=np.float32)
            tc = time.perf_counter()
            tr.step(tok, lab)
            cpu_s = time.perf_counter() - tc
            what = (f"one full step (forward, backward, AdamW; numpy fp32) of the same model on the same batch "
                    f"({S} tokens), {cpu_s:.1f} s")
        else:
            # one decoder layer at the workload's widths (small vocabulary, so that embedding and head are negligible) on
            # the whole batch; the step of the whole model is taken as n_layers times that: an extrapolation
            sample = dict(cfg, L=1, V=1024, B=CONFIGS[args.workload]["B"])
            sample.pop("micro_batches", None)
            sspecs = [(n, (r, c) if r > 1 else (c,), "normal" if (r > 1) else ("ones" if n.endswith("_g") else "zeros"))
                      for n, r, c in tio.tio_param_list(sample)]
            sparams = gen_params(sspecs, 0)
            stok, slab = gen_tokens(sample["B"], cfg["T"], 1024, 0)
            cpu_tokens = sample["B"] * cfg["T"]
            tr = om.Trainer(sample, sparams, dtype=np.float32)
            tc = time.perf_counter()
            tr.step(stok, slab)
            cpu_s = (time.perf_counter() - tc) * cfg["L"]
            what = (f"EXTRAPOLATED: one decoder layer of the workload's widths (forward, backward, AdamW; numpy fp32, "
                    f"vocabulary 1024) on the whole batch of {sample['B'] * cfg['T']} tokens took {cpu_s / cfg['L']:.1f} s; times "
                    f"{cfg['L']} layers, embedding and head left out")
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info() if p.get("user_api") == "blas"] or [1])
        except Exception:
            cores = len(os.sched_getaffinity(0))
        out["cpu_baseline"] = {"value": cpu_tokens / cpu_s,
                               "unit": "tokens/s", "cores": cores, "kind": "oracle", "dtype": "f32",
                               "sample": what}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
