"""CPU oracle: plan checker and performance model.

TEST INFRASTRUCTURE ONLY; shares no code with the HIP library.

check_plan verifies, from nothing but the trace and the plan entries, the
properties any correct plan must have (Section 3.2: memory is reduced only
between t_offloaded and t_prefetch; the loop ends when max(M') <= M_GPU):
every operand is resident when its kernel runs, the resident bytes never exceed
the capacity, entries pair up around exactly one inactive period, and the bytes
moved per direction are at least peak minus capacity.

simulate is the performance model of Section 2.2: kernel times are fixed at
their profiled values, migrations run at the designated bandwidth one at a time
per direction, and a kernel waits while a tensor it needs (or memory it is to
reuse) is still being migrated; the waiting time is added to the iteration.

check_layout verifies an address assignment produced by the library: tensors
whose residencies overlap in (cyclic) kernel time never overlap in address, and
everything lies inside the arena.
"""
from __future__ import annotations

from .plan import OFFLOAD, PREFETCH


def absent_windows(entries, N):
    """{pair: (tensor, k_off, k_pre, start, end)} from the entry list."""
    off, pre = {}, {}
    for (t, kind, trig, dl, urgent, pair) in entries:
        (off if kind == OFFLOAD else pre)[pair] = (t, trig, dl)
    assert off.keys() == pre.keys(), "every offload needs exactly one prefetch"
    out = {}
    for pair in off:
        t, trig_o, dl_o = off[pair]
        t2, trig_p, dl_p = pre[pair]
        assert t == t2
        out[pair] = (t, dl_o, trig_p - 1, trig_o - 1, dl_p)
    return out


def check_plan(trace, life, plan, cap, host_budget=None):
    """With host_budget: also recounts the bytes held by the host tier at every kernel (a host-tier pair
    occupies it for its whole inactive period) and checks them against the budget."""
    N = len(trace["kernels"])
    entries = plan["entries"]
    win = absent_windows(entries, N)
    periods = set(life["periods"])
    seen = set()
    M2 = list(life["M"])
    moved = 0
    for pair, (t, k_off, k_pre, start, end) in win.items():
        s = trace["tensors"][t][0]
        assert (t, s, start, end) in periods, f"pair {pair}: not an inactive period of tensor {t}"
        assert (t, start) not in seen, "period selected twice"
        seen.add((t, start))
        assert start < k_off <= k_pre + 1 <= end, (pair, start, k_off, k_pre, end)
        for k in range(k_off, k_pre + 1):
            M2[k % N] -= s
            assert (k % N) not in life["active"][t], f"tensor {t} absent at its own kernel {k % N}"
        moved += s
    assert M2 == list(plan["Mp"]), "planner's memory estimate differs from a recount"
    assert max(M2) <= cap, "resident bytes exceed the capacity"
    tier = plan.get("tier") or [0] * len(win)
    assert len(tier) == len(win) and all(x in (0, 1) for x in tier)
    Mh = [0] * N
    for pair, (t, k_off, k_pre, start, end) in win.items():
        if tier[pair]:
            for k in range(start + 1, end):
                Mh[k % N] += trace["tensors"][t][0]
    if host_budget is not None:
        assert max(Mh) <= host_budget, "host tier holds more than its budget"
        assert max(Mh) == plan.get("host_peak", 0)
    else:
        assert not any(tier), "host-tier pairs in a single-tier plan"
    if entries:
        assert moved >= max(life["M"]) - cap, "moved fewer bytes than peak - capacity"
    # sorted in issue order
    key = lambda e: (e[2] % N, e[1], -e[4], e[0], e[5])
    assert list(entries) == sorted(entries, key=key)
    return dict(bytes_per_direction=moved, pairs=len(win), host_pairs=sum(tier), host_peak=max(Mh),
                host_bytes_per_direction=sum(trace["tensors"][win[p][0]][0] for p in win if tier[p]))


def simulate(trace, plan, bw, duplex=True, iterations=3, host_bw=0):
    """Predicted duration (ns) of the last simulated iteration, and the compute-only time.  Pairs of the
    host tier move on that tier's own two channels at host_bw."""
    tau = trace["tau"]
    N = len(tau)
    entries = plan["entries"]
    by_trigger = [[] for _ in range(N)]
    for e in entries:
        by_trigger[e[2] % N].append(e)
    pre_deadline = [[] for _ in range(N)]
    off_deadline = [[] for _ in range(N)]
    for (t, kind, trig, dl, urgent, pair) in entries:
        (off_deadline if kind == OFFLOAD else pre_deadline)[dl % N].append(pair)
    size = {e[5]: trace["tensors"][e[0]][0] for e in entries}
    tier = plan.get("tier") or [0] * (len(entries) // 2)
    rate = (bw, host_bw)

    def dur(pair):
        r = rate[tier[pair]]
        return -(-size[pair] * 10**9 // r) if r else 0

    off_done, pre_done = {}, {}
    d2h_free, h2d_free = [0, 0], [0, 0]      # per tier
    done_prev = 0            # completion of the previous kernel
    mem_ready = 0            # completion of every offload whose deadline has been passed
    t_iter = []
    for it in range(iterations):
        t0 = done_prev
        for k in range(N):
            for p in off_deadline[k]:
                mem_ready = max(mem_ready, off_done.get(p, 0))
            for (t, kind, trig, dl, urgent, pair) in by_trigger[k]:
                d = dur(pair)
                w = tier[pair]
                if kind == OFFLOAD:
                    st = max(d2h_free[w], done_prev)
                    off_done[pair] = d2h_free[w] = st + d
                    if not duplex:
                        h2d_free[w] = d2h_free[w]
                else:
                    st = max(h2d_free[w], done_prev, off_done.get(pair, 0), mem_ready)
                    pre_done[pair] = h2d_free[w] = st + d
                    if not duplex:
                        d2h_free[w] = h2d_free[w]
            st = max(done_prev, mem_ready)
            for p in pre_deadline[k]:
                st = max(st, pre_done.get(p, 0))
            for p in off_deadline[k]:           # offloads issued at this very trigger point
                st = max(st, off_done.get(p, 0))
            done_prev = st + tau[k]
        t_iter.append(done_prev - t0)
    return dict(step_ns=t_iter[-1], compute_ns=sum(tau), per_iteration=t_iter)


def check_layout(trace, life, plan, allocs, arena_bytes):
    """allocs: list of (tensor, first_kernel, last_kernel, address) with kernel indices unrolled
    (last may be >= N for a residency that crosses the iteration boundary)."""
    N = len(trace["kernels"])
    per_kernel = [[] for _ in range(N)]
    for (t, k0, k1, addr) in allocs:
        s = trace["tensors"][t][0]
        assert addr % 256 == 0 and 0 <= addr and addr + s <= arena_bytes, (t, addr, s)
        assert k1 - k0 < N
        for k in range(k0, k1 + 1):
            per_kernel[k % N].append((addr, addr + s, t))
    for k in range(N):
        iv = sorted(per_kernel[k])
        for (a0, a1, t0), (b0, b1, t1) in zip(iv, iv[1:]):
            assert a1 <= b0, f"kernel {k}: tensors {t0} and {t1} overlap in the arena"
    # every operand has an address at its kernel
    covered = [set() for _ in range(N)]
    for (t, k0, k1, addr) in allocs:
        for k in range(k0, k1 + 1):
            covered[k % N].add(t)
    for k, (_, operands, _) in enumerate(trace["kernels"]):
        for t, _ in operands:
            assert t in covered[k], f"operand {t} of kernel {k} has no address"
    return True
