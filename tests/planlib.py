"""Helpers shared by the planner tests: tiny synthetic traces and golden-file parsing.
Holds no planner arithmetic."""
import os

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def mini_trace(tau, tensors):
    """tensors: list of (name, bytes, persistent, [active kernels]); persistent ones must come first."""
    N = len(tau)
    ops = [[] for _ in range(N)]
    tl = []
    npers = 0
    for tid, (name, nbytes, pers, act) in enumerate(tensors):
        if pers:
            assert npers == tid, "persistent tensors first"
            npers += 1
        tl.append((nbytes, 0 if pers else 5, name))
        for k in act:
            ops[k].append((tid, 3))
    kernels = [(0, sorted(o), 0) for o in ops]
    return dict(tensors=tl, kernels=kernels, tau=list(tau), n_persistent=npers,
                ids={t[0]: i for i, t in enumerate(tensors)})


def load_golden(name):
    tau = cap = bw = None
    tensors, entries, Mp, err = [], [], None, False
    for line in open(os.path.join(GOLDEN, name)):
        w = line.split("#")[0].split()
        if not w:
            continue
        if w[0] == "tau":
            tau = [int(x) for x in w[1:]]
        elif w[0] == "cap":
            cap = int(w[1])
        elif w[0] == "bw":
            bw = int(w[1])
        elif w[0] == "tensor":
            tensors.append((w[1], int(w[2]), w[3] == "persistent", [int(x) for x in w[4:]]))
        elif w[0] == "entry":
            entries.append((w[1],) + tuple(int(x) for x in w[2:]))
        elif w[0] == "Mp":
            Mp = [int(x) for x in w[1:]]
        elif w[0] == "expect":
            err = True
    tr = mini_trace(tau, tensors)
    entries = [(tr["ids"][e[0]],) + e[1:] for e in entries]
    return tr, cap, bw, entries, Mp, err


def golden_options(name):
    """Planner options a golden file states beside the fields of load_golden (currently: min_bytes)."""
    out = {}
    for line in open(os.path.join(GOLDEN, name)):
        w = line.split("#")[0].split()
        if w and w[0] == "min_bytes":
            out["min_bytes"] = int(w[1])
    return out


def load_golden_two_tier(name):
    """Golden file with a host tier: the fields of load_golden plus host_bw, host_budget and the tier of each pair."""
    tr, cap, bw, entries, Mp, err = load_golden(name)
    extra = {}
    for line in open(os.path.join(GOLDEN, name)):
        w = line.split("#")[0].split()
        if w and w[0] in ("host_bw", "host_budget"):
            extra[w[0]] = int(w[1])
        elif w and w[0] == "tier":
            extra["tier"] = [int(x) for x in w[1:]]
    return dict(trace=tr, cap=cap, bw=bw, entries=entries, Mp=Mp, **extra)


def random_trace(rng, N, n_pers, n_trans, max_bytes=1000):
    """Random small trace: every kernel has at least one operand, sizes multiples of 8."""
    tensors = []
    for i in range(n_pers):
        act = sorted(set(rng.choice(N, size=rng.integers(1, 3), replace=False).tolist()))
        tensors.append((f"p{i}", int(rng.integers(1, max_bytes // 8)) * 8, True, act))
    for i in range(n_trans):
        a = int(rng.integers(0, N - 1))
        b = int(rng.integers(a + 1, N))
        mid = [int(k) for k in range(a + 1, b) if rng.random() < 0.2]
        tensors.append((f"t{i}", int(rng.integers(1, max_bytes // 8)) * 8, False, sorted({a, b, *mid})))
    tau = [int(x) for x in rng.integers(50, 500, size=N)]
    # transient ids must follow first-write order only for the model traces; not needed here
    return mini_trace(tau, tensors)
