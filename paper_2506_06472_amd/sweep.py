"""Performance-model sweeps from the library's own trace, lifetimes, planner and model (CPU only).

  python -m paper_2506_06472_amd.sweep --workload llama_7b_bf16 --bw 8 16 25 32 48 64

For every slow-tier bandwidth: build the plan under the workload's memory cap, run tio_plan_simulate, and
print the predicted step time, tokens/s and fraction of the uncapped ideal (the study of Section 2.2 and
Figure 3 of the paper: training throughput against migration bandwidth).  --characterize adds what Figures
1 and 2 of the paper show for their models: the share of the allocated bytes that a kernel actually
touches, and the distribution of the tensors' inactive periods.  Kernel times are the library's modelled
ones unless --tau FILE gives measured times (one integer of nanoseconds per kernel, e.g. written from
tio_profile_iteration).  --measure-layer (needs the GPU) measures them on a one-layer model of the same widths
and gives every launch of the full model the time of the launch with the same operator, flops and operand sizes:
kernel times for configurations whose slow-tier pool no single box can hold.
"""
from __future__ import annotations

import argparse
import sys

import numpy as np

from . import binding as tio


def _cfg(name, micro_batches):
    from synth import CONFIGS
    cfg = dict(CONFIGS[name])
    base_peak = None
    if micro_batches > 1:
        if "cap_frac" in cfg:
            base_peak = int(tio.tio_analyze_lifetimes(tio.tio_trace_build(cfg)).export()["M"].max())
        cfg["B"] *= micro_batches
        cfg["micro_batches"] = micro_batches
    return cfg, base_peak


def sweep(name, bws, micro_batches=1, tau=None, min_bytes=1 << 20, out=sys.stdout, host_bw=0, host_budgets=(0,),
          shared_channel=False, benefits=(False,), retime_passes=0):
    """benefits: which benefit definitions to plan with, one row each: False = the formula of Algorithm 1, True = the
    prose form in which a kernel counts only with the bytes it is over capacity (tio_plan_opts.clamp_benefit)."""
    cfg, base_peak = _cfg(name, micro_batches)
    lt = tio.tio_trace_build(cfg)
    if tau is not None:
        lt.set_tau(tau)
    ll = tio.tio_analyze_lifetimes(lt)
    M = ll.export()["M"]
    peak = int(M.max())
    cap = int(cfg["cap_bytes"]) if "cap_bytes" in cfg else int((base_peak or peak) * cfg["cap_frac"]) // 256 * 256
    tokens = cfg["B"] * cfg["T"]
    print(f"{name}: {len(M)} kernels, uncapped peak {peak / 1e9:.2f} GB, cap {cap / 1e9:.2f} GB, {tokens} tokens/step, "
          f"micro-batches {micro_batches}, kernel times {'measured' if tau is not None else 'modelled'}"
          f"{', one channel shared by both directions' if shared_channel else ''}"
          f"{f', host-memory tier at {host_bw / 1e9:.0f} GB/s' if host_bw else ''}"
          f"{f', planner re-timed ({retime_passes} passes)' if retime_passes else ''}", file=out)
    print(f"{'GB/s':>7} {'host GB':>8} {'benefit':>8} {'step ms':>10} {'tokens/s':>10} {'of ideal':>9} {'GB/direction':>13} {'pairs':>6} {'urgent':>7} {'to host':>8}", file=out)
    rows = []
    for bw in bws:
        for hb in host_budgets:
            entries = []
            for clamp in benefits:
                plan = tio.tio_build_plan(lt, ll, cap, int(bw), duplex=not shared_channel, min_bytes=min_bytes,
                                          host_bw=int(host_bw) if hb else 0, host_budget=int(hb), clamp_benefit=clamp,
                                          retime_passes=retime_passes)
                pe = plan.export()
                step, comp = tio.tio_plan_simulate(lt, plan, int(bw), duplex=not shared_channel)
                gb = pe["bytes_per_direction"] / 1e9
                rows.append((bw, hb, step, comp, pe))
                entries.append(pe["entries"])
                print(f"{bw / 1e9:7.1f} {hb / 1e9:8.1f} {'prose' if clamp else 'formula':>8} {step / 1e6:10.1f} {tokens / (step / 1e9):10.0f} {comp / step:9.3f} {gb:13.2f} "
                      f"{pe['n_greedy'] + pe['n_forced']:6d} {pe['n_forced']:7d} {sum(pe['tier']):8d}", file=out)
            if len(entries) == 2:
                print(f"        the two benefit definitions give {'the same plan' if entries[0] == entries[1] else 'different plans'}", file=out)
    return rows


def _signatures(tv):
    off, ten, size = tv["operand_off"], tv["operand_tensor"], tv["tensor_bytes"]
    return [(int(tv["op"][k]), int(tv["flops"][k]), tuple(sorted(int(size[t]) for t in ten[off[k]:off[k + 1]])))
            for k in range(tv["n_kernels"])]


def measure_layer_tau(name, micro_batches=1, out=sys.stdout):
    """Kernel times of workload `name` from a measured iteration of the same model with one layer (GPU): the
    median-of-three time of each launch, averaged over the launches with the same signature (operator, flops,
    operand sizes), is given to every launch of the full trace with that signature."""
    from synth import gen_tokens, iter_params_pooled
    cfg, _ = _cfg(name, micro_batches)
    one = dict(cfg, L=1)
    lt1 = tio.tio_trace_build(one)
    up = tio.tio_build_plan(lt1, tio.tio_analyze_lifetimes(lt1), 2**62, 0).export()
    plist = tio.tio_param_list(one)
    specs = [(n, (r, c) if r > 1 else (c,), "normal" if r > 1 else ("ones" if n.endswith("_g") else "zeros")) for n, r, c in plist]
    tok, lab = gen_tokens(one["B"], one["T"], one["V"], 0)
    ctx = tio.tio_ctx_create(one, up["arena_needed"], up["host_needed"] + (1 << 20), 0)
    try:
        for pname, arr in iter_params_pooled(specs, 0):
            ctx.tio_params_load({pname: arr})
        tau1 = ctx.tio_profile_iteration(tok, lab, tio.PROFILE_MEASURED).export()["tau"]
    finally:
        ctx.close()
    acc = {}
    for sig, t in zip(_signatures(lt1.export()), tau1):
        acc.setdefault(sig, []).append(int(t))
    mean = {sig: int(round(sum(v) / len(v))) for sig, v in acc.items()}
    full = _signatures(tio.tio_trace_build(cfg).export())
    missing = sorted({sig[:2] for sig in full if sig not in mean})
    if missing:
        raise RuntimeError(f"launches of the full model without a counterpart in the one-layer model: {missing[:5]}")
    tau = np.array([mean[sig] for sig in full], dtype=np.int64)
    print(f"{name}: kernel times measured on one layer ({len(tau1)} launches, {len(mean)} distinct), sum over the full model "
          f"{tau.sum() / 1e6:.1f} ms", file=out)
    return tau


def characterize(name, micro_batches=1, out=sys.stdout):
    cfg, _ = _cfg(name, micro_batches)
    lt = tio.tio_trace_build(cfg)
    tv = lt.export()
    ll = tio.tio_analyze_lifetimes(lt).export()
    M = ll["M"].astype(np.float64)
    size = tv["tensor_bytes"].astype(np.float64)
    off = tv["operand_off"]
    act = np.array([size[tv["operand_tensor"][off[k]:off[k + 1]]].sum() for k in range(tv["n_kernels"])])
    share = act / M
    tau = tv["tau"].astype(np.float64)
    w = tau / tau.sum()
    print(f"{name}: share of the allocated bytes a kernel touches (time-weighted mean {np.sum(share * w):.4f}, "
          f"median {np.median(share):.4f}, 90th percentile {np.quantile(share, 0.9):.4f}, max {share.max():.4f})", file=out)
    # inactive periods in time: from the end of the bounding kernel `start` to the start of kernel `end`
    t_end = np.cumsum(tau)
    t_beg = t_end - tau
    total = tau.sum()
    N = tv["n_kernels"]
    s, e, b = ll["start"], ll["end"], ll["bytes"].astype(np.float64)
    length = np.where(e < N, t_beg[e % N] - t_end[s], total - t_end[s] + t_beg[e % N])
    edges = [0, 1e4, 1e5, 1e6, 1e7, 1e8, 1e9, 1e10, np.inf]
    labels = ["<10us", "10-100us", "0.1-1ms", "1-10ms", "10-100ms", "0.1-1s", "1-10s", ">10s"]
    print(f"  {len(length)} inactive periods; by length (modelled kernel times): count, share of the period bytes", file=out)
    for lo, hi, lab in zip(edges[:-1], edges[1:], labels):
        m = (length >= lo) & (length < hi)
        if m.any():
            print(f"    {lab:>9}: {int(m.sum()):6d}  {b[m].sum() / b.sum():6.3f}", file=out)
    big = b >= 10e6
    print(f"  periods of tensors of at least 10 MB: {int(big.sum())} of {len(b)}, {b[big].sum() / b.sum():.3f} of the bytes", file=out)


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--workload", nargs="+", default=["gpt2_small_bf16"])
    ap.add_argument("--bw", nargs="+", type=float, default=[8, 16, 25, 32, 48, 64], help="GB/s per direction")
    ap.add_argument("--micro-batches", type=int, default=1)
    ap.add_argument("--min-bytes", type=int, default=1 << 20)
    ap.add_argument("--tau", help="file with measured kernel times in ns, one per line")
    ap.add_argument("--characterize", action="store_true")
    ap.add_argument("--measure-layer", action="store_true", help="kernel times measured on a one-layer model (needs the GPU)")
    ap.add_argument("--host-bw", type=float, default=0, help="GB/s per direction of a host-memory tier beside the slow tier")
    ap.add_argument("--host-budget", nargs="+", type=float, default=[0], help="GB of host memory that tier may hold (one row each)")
    ap.add_argument("--shared-channel", action="store_true", help="offloads and prefetches share one channel (a single storage device)")
    ap.add_argument("--benefit", choices=["formula", "prose", "both"], default="formula",
                    help="benefit of a candidate: Algorithm 1's formula, the prose form (only the bytes over capacity count), or a row for each")
    ap.add_argument("--retime", type=int, default=0,
                    help="re-timing passes of the planner (Algorithm 1 run again on the stalled timeline); 0 = the paper's plan")
    a = ap.parse_args(argv)
    tau = np.loadtxt(a.tau, dtype=np.int64) if a.tau else None
    for name in a.workload:
        if a.measure_layer:
            tau = measure_layer_tau(name, a.micro_batches)
        sweep(name, [int(b * 1e9) for b in a.bw], a.micro_batches, tau, a.min_bytes, host_bw=a.host_bw * 1e9,
              host_budgets=[h * 1e9 for h in a.host_budget], shared_channel=a.shared_channel,
              benefits={"formula": (False,), "prose": (True,), "both": (False, True)}[a.benefit], retime_passes=a.retime)
        if a.characterize:
            characterize(name, a.micro_batches)
        print()


if __name__ == "__main__":
    main()
