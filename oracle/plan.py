"""CPU oracle for the lifetime analysis and the migration planner.

TEST INFRASTRUCTURE ONLY; shares no code with the HIP library.

analyze_lifetimes follows Section 3.1 ("Analyzing tensor activity patterns"):
a tensor is active at the kernels that read or write it; the gap between two
consecutive active kernels is an inactive period; intermediate tensors live
from first to last use, global tensors (weights, optimizer state) always, and
their last period wraps into the next iteration.

build_plan follows Algorithm 1 of Section 3.2 in the paper's order and
notation (I, M, M', tau, t_offloaded, t_prefetch, C, B), on an integer
nanosecond timeline, with the readings listed in this repository's design
notes (cyclic timeline, one transfer at a time per direction, kernel-index
conversion of the two times, tie-breaks).  When the loop ends with memory
still above capacity, the forced pass realises the "kernel stalls / urgent
migrations" paragraph of Section 3.2: at each over-capacity kernel the
inactive tensor whose next use is furthest away is evicted and marked urgent.

Two destinations ("Decide offloading destination", Section 3.2): with host_bw > 0 there is, besides the
slow tier (the paper's SSDs: preferred, unlimited), a host-memory tier with its own pair of channels, its
own bandwidth and a byte budget.  Reading: the slow tier is saturated for a candidate when the transfers
already planned on its channels displace the candidate (its offload cannot begin when the tensor becomes
inactive, or its prefetch cannot end when it becomes active again, or it does not fit at all); only then
is the candidate also evaluated on the host tier, provided the budget still has room for it during its
whole inactive period, and it goes to the host when that gives the larger benefit.  Forced (urgent)
evictions of periods not selected before go to the host when the budget has room, because a stalled
kernel waits for exactly these transfers.

Pins (tests/test_oracle_plan.py): hand-worked cases under tests/golden/,
capacity >= peak gives the empty plan, traffic lower bound, invariance under
permutation of the period list, exhaustive search on tiny traces, and the
residency invariants checked by oracle/replay.py.  The paper prints no worked
example of Algorithm 1: numeric parity with the paper's planner is unpinned.
"""
from __future__ import annotations

import bisect

from .trace import K_INPUT

OFFLOAD, PREFETCH = 0, 1


# ----------------------------------------------------------------------------
# Section 3.1: lifetimes
# ----------------------------------------------------------------------------
def analyze_lifetimes(trace):
    """Returns dict(periods=[(t, s, start, end)], M=[bytes per kernel], active=[[k,...] per tensor]).

    start/end are the active kernels that bound the period; end may exceed N-1
    for the wrap-around period of a persistent tensor (end - N is its first
    active kernel of the next iteration).
    """
    N = len(trace["kernels"])
    nt = len(trace["tensors"])
    npers = trace["n_persistent"]
    active = [[] for _ in range(nt)]
    for k, (_, operands, _) in enumerate(trace["kernels"]):
        for t, _ in operands:
            active[t].append(k)
    M = [0] * N
    periods = []
    for t in range(nt):
        s, kind, _ = trace["tensors"][t]
        a = active[t]
        if t < npers:
            for k in range(N):
                M[k] += s
        elif a:
            for k in range(a[0], a[-1] + 1):
                M[k] += s
        if not a or kind == K_INPUT:      # input buffers are rewritten by the host every iteration
            continue
        for i in range(len(a) - 1):
            if a[i + 1] - a[i] >= 2:
                periods.append((t, s, a[i], a[i + 1]))
        if t < npers and a[0] + N - a[-1] >= 2:
            periods.append((t, s, a[-1], a[0] + N))
    return dict(periods=periods, M=M, active=active)


# ----------------------------------------------------------------------------
# I/O bandwidth usage state: one channel = busy intervals on the cyclic timeline
# ----------------------------------------------------------------------------
class Channel:
    def __init__(self, period_ns):
        self.P = period_ns
        self.b, self.e = [], []             # sorted, disjoint, non-touching [b, e), 0 <= b < e <= P

    def _forward(self, lo, hi):
        """Busy intervals intersecting [lo, hi) in unrolled time, ascending."""
        for j in range(lo // self.P, (hi - 1) // self.P + 1):
            off = j * self.P
            i = bisect.bisect_right(self.e, lo - off)          # first interval ending after lo
            while i < len(self.b) and self.b[i] + off < hi:
                yield self.b[i] + off, self.e[i] + off
                i += 1

    def _backward(self, lo, hi):
        """The same intervals, descending."""
        for j in range((hi - 1) // self.P, lo // self.P - 1, -1):
            off = j * self.P
            i = bisect.bisect_left(self.b, hi - off) - 1       # last interval beginning before hi
            while i >= 0 and self.e[i] + off > lo:
                yield self.b[i] + off, self.e[i] + off
                i -= 1

    def earliest_gap(self, lo, hi, dur):
        """Smallest t >= lo with [t, t+dur) free and t+dur <= hi, or None."""
        if hi - lo < dur:
            return None
        t = lo
        for b, e in self._forward(lo, hi):
            if t + dur <= b:
                break
            t = max(t, e)
            if t + dur > hi:
                return None
        return t if t + dur <= hi else None

    def latest_gap(self, lo, hi, dur):
        """Largest t with [t, t+dur) free, t >= lo and t+dur <= hi, or None."""
        if hi - lo < dur:
            return None
        t = hi - dur
        for b, e in self._backward(lo, hi):
            if e <= t:
                break
            t = min(t, b - dur)
            if t < lo:
                return None
        return t if t >= lo else None

    def insert(self, t0, t1):
        """Marks [t0, t1) (unrolled time, length <= P) busy; touching intervals are merged."""
        if t1 <= t0:
            return
        a, z = t0 % self.P, t0 % self.P + (t1 - t0)
        for (x, y) in ([(a, z)] if z <= self.P else [(a, self.P), (0, z - self.P)]):
            i = bisect.bisect_left(self.b, x)
            assert (i == 0 or self.e[i - 1] <= x) and (i == len(self.b) or y <= self.b[i]), "overlap"
            if i > 0 and self.e[i - 1] == x and i < len(self.b) and self.b[i] == y:
                self.e[i - 1] = self.e[i]
                del self.b[i], self.e[i]
            elif i > 0 and self.e[i - 1] == x:
                self.e[i - 1] = y
            elif i < len(self.b) and self.b[i] == y:
                self.b[i] = x
            else:
                self.b.insert(i, x)
                self.e.insert(i, y)

    def busy_ns(self):
        return sum(e - b for b, e in zip(self.b, self.e))


# ----------------------------------------------------------------------------
# Section 3.2: Algorithm 1 and the forced (urgent) pass
# ----------------------------------------------------------------------------
def build_plan(trace, life, cap, bw, duplex=True, min_bytes=0, host_bw=0, host_budget=0, clamp_benefit=False):
    """Returns dict(entries=[(tensor, kind, trigger, deadline, urgent, pair)], Mp=[...], n_greedy, n_forced,
    tier=[0 slow tier | 1 host tier, per pair], host_peak=bytes).

    trigger/deadline are unrolled kernel indices in [0, 2N]: an entry is issued
    just before kernel (trigger mod N) is launched, after kernel trigger-1 has
    completed; an offload must have completed before kernel deadline may reuse the
    memory, a prefetch before kernel deadline (its next use) runs.  `pair` numbers
    the selected periods in selection order; the tensor is counted out of GPU
    memory at kernels [offload deadline, prefetch trigger - 1].

    clamp_benefit: the benefit of the prose ("Quantify the benefit and cost": the integral of the reduction in
    critical memory pressure), B = sum over C of min(s, M'[k] - capacity) * tau[k], instead of the listing's
    B = s * sum over C of tau[k]; candidates are compared by the exact fraction B / s.
    """
    from fractions import Fraction
    tau = trace["tau"]
    N = len(tau)
    T = [0] * (2 * N + 1)                                  # T[k] = start of kernel k, unrolled
    for k in range(2 * N):
        T[k + 1] = T[k] + tau[k % N]
    Ttot = T[N]
    Mp = list(life["M"])
    I = sorted(p for p in life["periods"] if p[1] >= min_bytes)
    small = sorted(p for p in life["periods"] if p[1] < min_bytes)
    ch_off = Channel(Ttot)
    ch_pre = ch_off if not duplex else Channel(Ttot)
    two_tier = host_bw > 0 and host_budget > 0
    hch_off = Channel(Ttot)                                # the host tier's own channels
    hch_pre = hch_off if not duplex else Channel(Ttot)
    Mh = [0] * N                                           # bytes held in host memory while kernel k runs
    sel = []                     # [t, s, start, end, k_off, k_pre, urgent_off, urgent_pre] in selection order
    tier = []                    # destination of each selected period

    def dur(s):                                            # bw == 0 stands for unlimited bandwidth
        return -(-s * 10**9 // bw) if bw else 0

    def hdur(s):
        return -(-s * 10**9 // host_bw)

    def host_fits(s, start, end):
        """room in the host budget while the tensor is away: kernels start+1 .. end-1"""
        return all(Mh[k % N] + s <= host_budget for k in range(start + 1, end))

    def host_take(s, start, end):
        for k in range(start + 1, end):
            Mh[k % N] += s

    clamp_size = [0]                                       # size of the candidate being evaluated

    def evaluate(c_off, c_pre, lo, hi, d, over):
        """(score, g, t_offloaded, t_prefetch, k_off, k_pre) of a candidate on one tier's channels, or None"""
        g = c_off.earliest_gap(lo, hi, d)
        if g is None:
            return None
        t_offloaded = g + d
        g2 = c_pre.latest_gap(lo, hi, d)
        if g2 is None:
            return None
        t_prefetch = g2
        if not t_offloaded < t_prefetch:
            return None
        k_off = bisect.bisect_left(T, t_offloaded)               # first kernel starting at or after
        k_pre = bisect.bisect_right(T, t_prefetch) - 2           # last kernel ending at or before
        if k_off > k_pre:
            return None
        score = over[k_pre + 1] - over[k_off]                    # B / s = sum of tau over C
        if score <= 0:
            return None
        if clamp_benefit:
            s = clamp_size[0]
            B = sum(min(s, Mp[k % N] - cap) * tau[k % N] for k in range(k_off, k_pre + 1) if Mp[k % N] > cap)
            score = Fraction(B, s)
        return score, g, t_offloaded, t_prefetch, k_off, k_pre

    # ---- Algorithm 1
    while max(Mp) > cap:
        over = [0] * (2 * N + 1)                           # prefix sums of tau over kernels above capacity
        for k in range(2 * N):
            over[k + 1] = over[k] + (tau[k % N] if Mp[k % N] > cap else 0)
        best = None
        for (t, s, start, end) in I:
            d = dur(s)
            lo, hi = T[start + 1], T[end]
            clamp_size[0] = s
            ev, where = evaluate(ch_off, ch_pre, lo, hi, d, over), 0
            if two_tier:
                # slow tier saturated for this candidate: planned transfers displace it (or leave it no room)
                displaced = ev is None or ev[1] > lo or ev[3] + d < hi
                if displaced and host_fits(s, start, end):
                    hev = evaluate(hch_off, hch_pre, lo, hi, hdur(s), over)
                    if hev is not None and (ev is None or hev[0] > ev[0]):
                        ev, where, d = hev, 1, hdur(s)
            if ev is None:
                continue
            score, g, t_offloaded, t_prefetch, k_off, k_pre = ev
            key = (score, s, -start, -t, -end)
            if best is None or key > best[0]:
                best = (key, (t, s, start, end), g, t_offloaded, t_prefetch, k_off, k_pre, d, where)
        if best is None:
            break
        _, per, g, t_offloaded, t_prefetch, k_off, k_pre, d, where = best
        t, s, start, end = per
        sel.append([t, s, start, end, k_off, k_pre, 0, 0])
        tier.append(where)
        for k in range(k_off, k_pre + 1):
            Mp[k % N] -= s
        if where == 0:
            ch_off.insert(g, t_offloaded)
            ch_pre.insert(t_prefetch, t_prefetch + d)
        else:
            hch_off.insert(g, t_offloaded)
            hch_pre.insert(t_prefetch, t_prefetch + d)
            host_take(s, start, end)
        I.remove(per)
    n_greedy = len(sel)

    # ---- forced pass: stalls and urgent migrations
    def frame(start, end, k):
        """k or k+N, whichever lies strictly inside (start, end); else None."""
        if start < k < end:
            return k
        if start < k + N < end:
            return k + N
        return None

    for k in range(N):
        while Mp[k] > cap:
            best = None
            # (a) periods already selected whose window does not cover k, (b) unselected periods
            for idx, (t, s, start, end, k_off, k_pre, _, _) in enumerate(sel):
                kk = frame(start, end, k)
                if kk is None or k_off <= kk <= k_pre or (min_bytes and s < min_bytes):
                    continue
                key = (end - kk, s, -start, -t)
                if best is None or key > best[0]:
                    best = (key, ("sel", idx), kk)
            for (t, s, start, end) in I:
                kk = frame(start, end, k)
                if kk is None:
                    continue
                key = (end - kk, s, -start, -t)
                if best is None or key > best[0]:
                    best = (key, ("new", (t, s, start, end)), kk)
            if best is None:                                # last resort: tensors below min_bytes
                for idx, (t, s, start, end, k_off, k_pre, _, _) in enumerate(sel):
                    kk = frame(start, end, k)
                    if kk is None or k_off <= kk <= k_pre:
                        continue
                    key = (end - kk, s, -start, -t)
                    if best is None or key > best[0]:
                        best = (key, ("sel", idx), kk)
                for (t, s, start, end) in small:
                    kk = frame(start, end, k)
                    if kk is None:
                        continue
                    key = (end - kk, s, -start, -t)
                    if best is None or key > best[0]:
                        best = (key, ("new", (t, s, start, end)), kk)
            if best is None:
                raise ValueError(f"operands of kernel {k} alone exceed the capacity")
            _, (what, ref), kk = best
            if what == "new":
                t, s, start, end = ref
                (I if ref in I else small).remove(ref)
                rec = [t, s, start, end, kk, kk - 1, 1, 1]          # empty window, grown below
                sel.append(rec)
                if two_tier and host_fits(s, start, end):           # a stalled kernel waits for these transfers
                    tier.append(1)
                    host_take(s, start, end)
                else:
                    tier.append(0)
            else:
                rec = sel[ref]
            t, s, start, end, k_off, k_pre = rec[:6]
            if kk < k_off:                                          # pull the offload deadline forward
                for j in range(kk, k_off):
                    Mp[j % N] -= s
                rec[4], rec[6] = kk, 1
            else:                                                   # push the prefetch back
                last = kk
                for j in range(kk, end):
                    if Mp[j % N] > cap:
                        last = j
                for j in range(k_pre + 1, last + 1):
                    Mp[j % N] -= s
                rec[5], rec[7] = last, 1

    entries = []
    for pair, (t, s, start, end, k_off, k_pre, u_off, u_pre) in enumerate(sel):
        entries.append((t, OFFLOAD, start + 1, k_off, u_off, pair))
        entries.append((t, PREFETCH, k_pre + 1, end, u_pre, pair))
    entries.sort(key=lambda e: (e[2] % N, e[1], -e[4], e[0], e[5]))
    return dict(entries=entries, Mp=Mp, n_greedy=n_greedy, n_forced=len(sel) - n_greedy, tier=tier, host_peak=max(Mh))
