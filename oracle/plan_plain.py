"""CPU oracle, plain form of the migration planner (Algorithm 1 of Section 3.2 plus the urgent pass).

TEST INFRASTRUCTURE ONLY; shares no code with the HIP library and none with oracle/plan.py.

This file exists to pin oracle/plan.py (which is organised for speed: sorted interval arrays, binary
searches, prefix sums, a folded cyclic timeline) against the same reading of the paper written out as
directly as possible:

  * time is an integer-nanosecond line on which iteration j occupies [j*P, (j+1)*P), P = sum of tau; the
    kernel with unrolled index k (k = j*N + k') starts at start_of(k), a table made by adding up tau;
  * the "I/O bandwidth usage state" of a direction is a plain list of the transfers placed so far, each
    one interval [b, e); because every iteration repeats the same plan, a transfer is busy at [b + j*P,
    e + j*P) for every integer j, and the list is scanned in full for every question asked of it;
  * t_offloaded and t_prefetch come from the definition: the earliest (latest) start of a free slot of
    the transfer's length inside the period's idle window;
  * C, the benefit B and the update of M' are loops over kernel indices.

Nothing here is sorted, merged, folded or cached.  It is meant for traces of at most a few hundred
kernels; tests/test_oracle_plan_plain.py asserts that oracle/plan.py gives the same plan on the
hand-worked examples, on the small model traces and on random traces at finite bandwidth.

Readings (the paper leaves these open; they are the ones listed in this repository's design notes):
a candidate's offload may start once kernel `start` has ended and its prefetch must end before kernel
`end` starts; the tensor counts as absent at the kernels that lie entirely between t_offloaded and
t_prefetch; score = B / s with B = s * sum of tau over the absent kernels whose M' exceeds the capacity
(clamp_benefit: B = sum of min(s, M'[k] - capacity) * tau[k], the prose form of "Quantify the benefit and
cost", compared as the exact fraction B / s); ties go to the larger tensor, then the earlier start, the smaller
tensor id, the earlier end.  After the loop, kernels still above capacity evict, one at a time, the tensor
that is counted present, is not an operand, and whose next use is furthest away ("Minimize kernel stalls"):
an unselected period becomes absent from that kernel up to the last over-capacity kernel before its next use;
a selected period's absence is stretched to reach the kernel (backwards: down to the kernel; forwards: up
to the last over-capacity kernel before its next use); the entries touched are urgent.
"""
from __future__ import annotations

from fractions import Fraction

OFFLOAD, PREFETCH = 0, 1
K_INPUT = 4          # tensor kind of the token / label buffers (the host rewrites them every iteration)


def inactive_periods(trace):
    """Section 3.1: (tensor, bytes, start, end) for every gap of at least one kernel between two uses; a
    persistent tensor's last use pairs with its first use of the next iteration.  Also M[k]."""
    N = len(trace["kernels"])
    periods, M = [], [0] * N
    for t, (s, kind, _name) in enumerate(trace["tensors"]):
        uses = [k for k in range(N) if any(op_t == t for op_t, _ in trace["kernels"][k][1])]
        persistent = t < trace["n_persistent"]
        for k in range(N):
            if persistent or (uses and uses[0] <= k <= uses[-1]):
                M[k] += s
        if not uses or kind == K_INPUT:
            continue
        nxt = uses[1:] + ([uses[0] + N] if persistent else [])
        for a, b in zip(uses, nxt):
            if b - a >= 2:
                periods.append((t, s, a, b))
    return periods, M


class Timeline:
    """Start times of the kernels of three consecutive iterations, by adding up tau (a table of the definition
    start_of(k+1) = start_of(k) + tau[k mod N]); the two look-ups scan it from the beginning."""

    def __init__(self, tau):
        self.tau = list(tau)
        self.N = len(tau)
        self.P = sum(tau)
        self.starts = [0]
        for k in range(3 * self.N):
            self.starts.append(self.starts[-1] + self.tau[k % self.N])

    def start_of(self, k):
        return self.starts[k]

    def first_kernel_starting_at_or_after(self, time):
        for k, t in enumerate(self.starts):
            if t >= time:
                return k
        raise AssertionError("time beyond the table")

    def last_kernel_ending_at_or_before(self, time):
        """-1 if not even kernel 0 has ended by then (kernel k ends where kernel k+1 starts)."""
        last = -1
        for k in range(len(self.starts) - 1):
            if self.starts[k + 1] <= time:
                last = k
            else:
                break
        return last


def _copies(transfers, P, lo, hi):
    """Every repetition [b + j*P, e + j*P) of the placed transfers that could touch [lo, hi)."""
    out = []
    for (b, e) in transfers:
        j = (lo - e) // P - 1
        while b + j * P < hi:
            if e + j * P > lo:
                out.append((b + j * P, e + j * P))
            j += 1
    return out


def _free(busy, t, d):
    return all(not (b < t + d and t < e) for (b, e) in busy)


def earliest_slot(transfers, P, lo, hi, d):
    """Smallest t >= lo with t + d <= hi and [t, t + d) clear of every placed transfer; None if there is none.
    Such a t is lo itself or the end of a transfer."""
    busy = _copies(transfers, P, lo, hi)
    for t in sorted([lo] + [e for (_, e) in busy if e > lo]):
        if t + d > hi:
            return None
        if _free(busy, t, d):
            return t
    return None


def latest_slot(transfers, P, lo, hi, d):
    """Largest t with t >= lo, t + d <= hi and [t, t + d) clear; it ends at hi or at the beginning of a transfer."""
    busy = _copies(transfers, P, lo, hi)
    for t in sorted([hi - d] + [b - d for (b, _) in busy if b < hi], reverse=True):
        if t < lo:
            return None
        if _free(busy, t, d):
            return t
    return None


def build_plan(trace, cap, bw, duplex=True, min_bytes=0, clamp_benefit=False):
    """Same result format as oracle/plan.py build_plan (single destination)."""
    tl = Timeline(trace["tau"])
    N, P, tau = tl.N, tl.P, tl.tau
    periods, M = inactive_periods(trace)
    Mp = list(M)
    offloads = []                                   # placed transfers of the offloading direction
    prefetches = offloads if not duplex else []     # one shared list when both directions share the channel
    chosen = []                                     # dicts in selection order

    def dur(s):
        return 0 if bw == 0 else (s * 10**9 + bw - 1) // bw

    remaining = [p for p in periods if p[1] >= min_bytes]
    small = [p for p in periods if p[1] < min_bytes]

    # ---- Algorithm 1
    while max(Mp) > cap:
        best = None
        for (t, s, start, end) in remaining:
            d = dur(s)
            lo, hi = tl.start_of(start + 1), tl.start_of(end)
            g = earliest_slot(offloads, P, lo, hi, d)
            if g is None:
                continue
            t_offloaded = g + d
            t_prefetch = latest_slot(prefetches, P, lo, hi, d)
            if t_prefetch is None or not t_offloaded < t_prefetch:
                continue
            k_off = tl.first_kernel_starting_at_or_after(t_offloaded)
            k_pre = tl.last_kernel_ending_at_or_before(t_prefetch)
            C = [k for k in range(k_off, k_pre + 1) if Mp[k % N] > cap]
            if not C:
                continue
            if clamp_benefit:
                score = Fraction(sum(min(s, Mp[k % N] - cap) * tau[k % N] for k in C), s)
            else:
                score = sum(tau[k % N] for k in C)
            key = (score, s, -start, -t, -end)
            if best is None or key > best[0]:
                best = (key, (t, s, start, end), g, t_prefetch, k_off, k_pre, d)
        if best is None:
            break
        _, per, g, t_prefetch, k_off, k_pre, d = best
        t, s, start, end = per
        chosen.append(dict(t=t, s=s, start=start, end=end, k_off=k_off, k_pre=k_pre, u_off=0, u_pre=0))
        for k in range(k_off, k_pre + 1):
            Mp[k % N] -= s
        if d > 0:
            offloads.append((g, g + d))
            prefetches.append((t_prefetch, t_prefetch + d))
        remaining.remove(per)
    n_greedy = len(chosen)

    # ---- urgent pass
    def inside(start, end, k):
        """The unrolled index of kernel k that lies strictly inside (start, end), if any."""
        for kk in (k, k + N):
            if start < kk < end:
                return kk
        return None

    for k in range(N):
        while Mp[k] > cap:
            def candidates(pool_new, allow_small_selected):
                out = []
                for c in chosen:
                    kk = inside(c["start"], c["end"], k)
                    if kk is None or c["k_off"] <= kk <= c["k_pre"]:
                        continue                                        # not its period, or already absent there
                    if c["s"] < min_bytes and not allow_small_selected:
                        continue
                    out.append(((c["end"] - kk, c["s"], -c["start"], -c["t"]), c, None, kk))
                for per in pool_new:
                    kk = inside(per[2], per[3], k)
                    if kk is not None:
                        out.append(((per[3] - kk, per[1], -per[2], -per[0]), None, per, kk))
                return out
            cands = candidates(remaining, False) or candidates(small, True)
            if not cands:
                raise ValueError(f"operands of kernel {k} alone exceed the capacity")
            # keys are distinct: two periods differ in tensor id or in start
            _, c, per, kk = max(cands, key=lambda x: x[0])
            if c is None:
                t, s, start, end = per
                (remaining if per in remaining else small).remove(per)
                c = dict(t=t, s=s, start=start, end=end, k_off=kk, k_pre=kk - 1, u_off=1, u_pre=1)
                chosen.append(c)
            if kk < c["k_off"]:
                for j in range(kk, c["k_off"]):
                    Mp[j % N] -= c["s"]
                c["k_off"], c["u_off"] = kk, 1
            else:
                last = kk
                for j in range(kk, c["end"]):
                    if Mp[j % N] > cap:
                        last = j
                for j in range(c["k_pre"] + 1, last + 1):
                    Mp[j % N] -= c["s"]
                c["k_pre"], c["u_pre"] = last, 1

    entries = []
    for pair, c in enumerate(chosen):
        entries.append((c["t"], OFFLOAD, c["start"] + 1, c["k_off"], c["u_off"], pair))
        entries.append((c["t"], PREFETCH, c["k_pre"] + 1, c["end"], c["u_pre"], pair))
    # issue order: by trigger point; there offloads before prefetches, urgent first within a direction
    entries.sort(key=lambda e: (e[2] % N, e[1], -e[4], e[0], e[5]))
    return dict(entries=entries, Mp=Mp, n_greedy=n_greedy, n_forced=len(chosen) - n_greedy)
