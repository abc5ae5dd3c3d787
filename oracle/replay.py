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
    stretched = [0] * N      # last iteration: a kernel's own time plus the stall in front of it
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
            stretched[k] = st + tau[k] - done_prev
            done_prev = st + tau[k]
        t_iter.append(done_prev - t0)
    return dict(step_ns=t_iter[-1], compute_ns=sum(tau), per_iteration=t_iter, stretched=stretched)


def simulate_engine(trace, plan, bw, duplex=True, iterations=3, host_bw=0, chunk_bytes=16 << 20, urgent_first=True):
    """Performance model of the migration engine with a ready queue per channel (Section 3.2, "Minimize kernel
    stalls": urgent migrations go ahead of the other pending ones; Section 3.3).  Reading:

      * kernel times are fixed (Section 2.2); the entries triggered at kernel k are issued when kernel k-1 completes;
      * a channel (one per direction and tier; one per tier when duplex is off) moves one chunk of at most chunk_bytes
        at a time, ceil(bytes * 1e9 / bandwidth) ns per chunk;
      * a request is ready once it has been issued and, for a prefetch, once its own offload and every offload whose
        deadline had been reached when the prefetch was issued are complete (the memory it lands in is free);
      * whenever a channel is free it takes the next chunk of the first ready urgent request in issue order, else of
        the first ready request in issue order: an urgent request overtakes pending ones at a chunk boundary,
        and a request that is not ready never holds up one that is (urgent_first=False: no priority, ready
        requests in issue order);
      * kernel k starts when kernel k-1, the prefetches due at k and every offload whose deadline is k or earlier
        are complete.

    Returns the duration of every simulated iteration and the compute-only time, like simulate."""
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
    tier = plan.get("tier") or [0] * (len(entries) // 2)
    rate = (bw, host_bw)

    class Req:
        pass

    n_chan = 4
    chan_of = lambda kind, w: 2 * w + (kind if duplex else 0)
    queue = [[] for _ in range(n_chan)]            # issued, unfinished requests in issue order
    busy_until = [None] * n_chan                   # end of the chunk in flight
    in_flight = [None] * n_chan
    last_off, last_pre = {}, {}                    # pair -> latest request
    due = []                                       # offload requests whose deadline has been reached, not yet known complete

    def done(r, now):
        return r.done_at is not None and r.done_at <= now

    def issue(k, now):
        for p in off_deadline[k]:
            if p in last_off:
                due.append(last_off[p])
        for (t, kind, trig, dl, urgent, pair) in by_trigger[k]:
            r = Req()
            r.kind, r.pair, r.urgent, r.left, r.done_at = kind, pair, urgent, trace["tensors"][t][0], None
            r.rate = rate[tier[pair]]
            r.deps = []
            if kind == PREFETCH:
                if pair in last_off:
                    r.deps.append(last_off[pair])
                r.deps += [q for q in due if not done(q, now)]
                last_pre[pair] = r
            else:
                last_off[pair] = r
            queue[chan_of(kind, tier[pair])].append(r)
        for p in off_deadline[k]:                  # offloads issued at this very trigger point
            if p in last_off and last_off[p] not in due:
                due.append(last_off[p])

    def pick(c, now):
        ready = [r for r in queue[c] if all(done(q, now) for q in r.deps)]
        if urgent_first:
            for r in ready:
                if r.urgent:
                    return r
        return ready[0] if ready else None

    def kernel_may_start(k, now):
        due[:] = [q for q in due if not done(q, now)]
        if due:
            return False
        return all(done(last_pre[p], now) for p in pre_deadline[k] if p in last_pre)

    now, k_glob, running_until = 0, 0, None
    total = iterations * N
    t_iter, t_iter_start = [], 0
    issue(0, 0)
    while k_glob < total:
        changed = True
        while changed and k_glob < total:           # everything that happens at `now`
            changed = False
            for c in range(n_chan):                  # chunks that end now
                if in_flight[c] is not None and busy_until[c] <= now:
                    r = in_flight[c]
                    if r.left == 0:
                        r.done_at = busy_until[c]
                        queue[c].remove(r)
                    in_flight[c] = None
                    changed = True
            if running_until is not None and running_until <= now:      # the kernel that ends now
                running_until = None
                k_glob += 1
                if k_glob % N == 0:
                    t_iter.append(now - t_iter_start)
                    t_iter_start = now
                if k_glob < total:
                    issue(k_glob % N, now)
                changed = True
                continue
            for c in range(n_chan):                  # free channels take their next chunk
                if in_flight[c] is None:
                    r = pick(c, now)
                    if r is not None:
                        n = min(r.left, chunk_bytes) if chunk_bytes else r.left
                        r.left -= n
                        busy_until[c] = now + (-(-n * 10**9 // r.rate) if r.rate else 0)
                        in_flight[c] = r
                        changed = True
            if running_until is None and kernel_may_start(k_glob % N, now):
                running_until = now + tau[k_glob % N]
                changed = True
        if k_glob >= total:
            break
        pending = [busy_until[c] for c in range(n_chan) if in_flight[c] is not None]
        if running_until is not None:
            pending.append(running_until)
        assert pending and min(pending) > now, "nothing in flight and nothing can start"
        now = min(pending)
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
