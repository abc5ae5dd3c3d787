// Lifetime analysis (Section 3.1), Algorithm 1 with the urgent pass (Section 3.2) and the arena
// address assignment.  Integer arithmetic only; every tie is broken deterministically.
#include "analysis.h"

#include <algorithm>
#include <map>
#include <numeric>
#include <tuple>

namespace tio {

typedef unsigned __int128 u128;

// ------------------------------------------------------------------------------------------------
// trace
// ------------------------------------------------------------------------------------------------
static uint64_t mix(uint64_t h, uint64_t v) {
    h ^= v + 0x9E3779B97F4A7C15ull + (h << 6) + (h >> 2);
    return h * 0xBF58476D1CE4E5B9ull;
}

void Trace::rehash() {
    uint64_t h = 0x1234567ull;
    h = mix(h, (uint64_t)n_kernels); h = mix(h, (uint64_t)n_tensors); h = mix(h, (uint64_t)n_persistent);
    for (auto v : op) h = mix(h, (uint64_t)v);
    for (auto v : operand_off) h = mix(h, (uint64_t)v);
    for (auto v : operand_tensor) h = mix(h, (uint64_t)v);
    for (auto v : operand_flags) h = mix(h, (uint64_t)v);
    for (auto v : tensor_bytes) h = mix(h, v);
    structure_hash = h;
}

Trace trace_from_program(const Program &P) {
    Trace t;
    t.n_kernels = (int32_t)P.kernels.size();
    t.n_tensors = (int32_t)P.tensors.size();
    t.n_persistent = P.n_persistent;
    t.operand_off.push_back(0);
    for (const KernelRec &k : P.kernels) {
        std::map<int32_t, int32_t> fl;            // sorted by tensor id, flags merged
        for (int r = 0; r < kMaxRoles; ++r)
            if (k.t[r] >= 0) fl[k.t[r]] |= k.fl[r];
        for (auto &kv : fl) { t.operand_tensor.push_back(kv.first); t.operand_flags.push_back(kv.second); }
        t.operand_off.push_back((int32_t)t.operand_tensor.size());
        t.op.push_back(k.op);
        t.flops.push_back(k.flops);
    }
    for (const TensorInfo &ti : P.tensors) { t.tensor_bytes.push_back(ti.bytes); t.tensor_kind.push_back(ti.kind); }
    t.tau.assign(t.n_kernels, 0);
    model_tau(t);
    t.rehash();
    return t;
}

void model_tau(Trace &t) {
    // half of the dense bf16 MFMA peak, half of the HBM peak, a fixed launch cost
    const u128 F = 1250000000000000ull, Wb = 4000000000000ull;
    const int64_t launch = 4000;
    for (int k = 0; k < t.n_kernels; ++k) {
        u128 bytes = 0;
        for (int i = t.operand_off[k]; i < t.operand_off[k + 1]; ++i) bytes += t.tensor_bytes[t.operand_tensor[i]];
        u128 tf = ((u128)t.flops[k] * 1000000000ull + F - 1) / F;
        u128 tb = (bytes * 1000000000ull + Wb - 1) / Wb;
        t.tau[k] = (int64_t)std::max(tf, tb) + launch;
    }
}

// ------------------------------------------------------------------------------------------------
// Section 3.1: active kernels -> inactive periods and memory demand
// ------------------------------------------------------------------------------------------------
Lifetimes analyze(const Trace &t) {
    Lifetimes L;
    const int N = t.n_kernels;
    L.n_kernels = N;
    L.structure_hash = t.structure_hash;
    L.active.assign(t.n_tensors, {});
    for (int k = 0; k < N; ++k)
        for (int i = t.operand_off[k]; i < t.operand_off[k + 1]; ++i) L.active[t.operand_tensor[i]].push_back(k);
    // difference array for the transient lifetimes
    std::vector<int64_t> diff(N + 1, 0);
    uint64_t always = 0;
    for (int id = 0; id < t.n_tensors; ++id) {
        const auto &a = L.active[id];
        const uint64_t s = t.tensor_bytes[id];
        const bool persistent = id < t.n_persistent;
        if (persistent) always += s;
        else if (!a.empty()) { diff[a.front()] += (int64_t)s; diff[a.back() + 1] -= (int64_t)s; }
        if (a.empty() || t.tensor_kind[id] == KIND_INPUT) continue;   // host rewrites inputs every iteration
        for (size_t i = 0; i + 1 < a.size(); ++i)
            if (a[i + 1] - a[i] >= 2) L.periods.push_back({id, s, a[i], a[i + 1]});
        if (persistent && a.front() + N - a.back() >= 2) L.periods.push_back({id, s, a.back(), a.front() + N});
    }
    L.M.assign(N, 0);
    int64_t run = 0;
    for (int k = 0; k < N; ++k) { run += diff[k]; L.M[k] = always + (uint64_t)run; }
    for (const Period &p : L.periods) {
        L.v_tensor.push_back(p.tensor); L.v_bytes.push_back(p.bytes);
        L.v_start.push_back(p.start); L.v_end.push_back(p.end);
    }
    return L;
}

// ------------------------------------------------------------------------------------------------
// I/O bandwidth usage state of one migration direction: busy intervals on the cyclic timeline
// ------------------------------------------------------------------------------------------------
namespace {

struct Channel {
    int64_t P;
    std::vector<int64_t> b, e;       // sorted, disjoint, merged when touching; 0 <= b < e <= P

    // smallest t >= lo with [t,t+dur) free and t+dur <= hi; -1 if none
    int64_t earliest(int64_t lo, int64_t hi, int64_t dur) const {
        if (hi - lo < dur) return -1;
        int64_t t = lo;
        for (int64_t j = lo / P; j <= (hi - 1) / P; ++j) {
            const int64_t off = j * P;
            size_t i = std::upper_bound(e.begin(), e.end(), lo - off) - e.begin();
            for (; i < b.size() && b[i] + off < hi; ++i) {
                if (t + dur <= b[i] + off) return t;
                t = std::max(t, e[i] + off);
                if (t + dur > hi) return -1;
            }
        }
        return t + dur <= hi ? t : -1;
    }
    // largest t >= lo with [t,t+dur) free and t+dur <= hi; -1 if none
    int64_t latest(int64_t lo, int64_t hi, int64_t dur) const {
        if (hi - lo < dur) return -1;
        int64_t t = hi - dur;
        for (int64_t j = (hi - 1) / P; j >= lo / P; --j) {
            const int64_t off = j * P;
            int64_t i = (int64_t)(std::lower_bound(b.begin(), b.end(), hi - off) - b.begin()) - 1;
            for (; i >= 0 && e[i] + off > lo; --i) {
                if (e[i] + off <= t) return t;
                t = std::min(t, b[i] + off - dur);
                if (t < lo) return -1;
            }
        }
        return t >= lo ? t : -1;
    }
    void put(int64_t x, int64_t y) {
        size_t i = std::lower_bound(b.begin(), b.end(), x) - b.begin();
        const bool left = i > 0 && e[i - 1] == x, right = i < b.size() && b[i] == y;
        if (left && right) { e[i - 1] = e[i]; b.erase(b.begin() + i); e.erase(e.begin() + i); }
        else if (left) e[i - 1] = y;
        else if (right) b[i] = x;
        else { b.insert(b.begin() + i, x); e.insert(e.begin() + i, y); }
    }
    void insert(int64_t t0, int64_t t1) {
        if (t1 <= t0) return;
        const int64_t a = t0 % P, z = a + (t1 - t0);
        if (z <= P) put(a, z);
        else { put(a, P); put(0, z - P); }
    }
};

struct Cand { int32_t tensor; uint64_t bytes; int32_t start, end; bool alive; };

// lexicographic "better" for the forced pass: furthest next use, larger tensor, earlier start, smaller id
struct ForcedKey {
    int64_t dist; uint64_t bytes; int32_t start, tensor;
    bool better_than(const ForcedKey &o) const {
        return std::make_tuple(dist, bytes, -start, -tensor) > std::make_tuple(o.dist, o.bytes, -o.start, -o.tensor);
    }
};

}  // namespace

void select_periods(const Trace &t, const Lifetimes &life, uint64_t cap, uint64_t bw, bool duplex,
                    uint64_t min_bytes, uint64_t host_bw, uint64_t host_budget, bool clamp_benefit, Plan &out) {
    const int N = t.n_kernels;
    const std::vector<int64_t> &tau = t.tau;
    std::vector<int64_t> T(2 * N + 1, 0);
    for (int k = 0; k < 2 * N; ++k) T[k + 1] = T[k] + tau[k % N];
    const int64_t Ttot = T[N];
    std::vector<uint64_t> Mp = life.M;
    std::vector<Cand> I, small;
    for (const Period &p : life.periods)
        (p.bytes >= min_bytes ? I : small).push_back({p.tensor, p.bytes, p.start, p.end, true});
    Channel ch_off{Ttot, {}, {}}, ch_pre_own{Ttot, {}, {}};
    Channel &ch_pre = duplex ? ch_pre_own : ch_off;
    // Destination choice (Section 3.2): besides the slow tier a host-memory tier with its own channels, its own
    // bandwidth and a byte budget.  The slow tier is saturated for a candidate when the transfers already planned
    // on its channels displace it (or leave it no room); only then is the candidate also evaluated on the host
    // tier, provided the budget has room for it during its whole inactive period, and it goes there when that
    // gives the larger benefit.
    const bool two_tier = host_bw > 0 && host_budget > 0;
    Channel hch_off{Ttot, {}, {}}, hch_pre_own{Ttot, {}, {}};
    Channel &hch_pre = duplex ? hch_pre_own : hch_off;
    std::vector<uint64_t> Mh(N, 0);                     // bytes held in host memory while kernel k runs
    auto host_fits = [&](uint64_t s, int32_t start, int32_t end) {
        for (int k = start + 1; k < end; ++k) if (Mh[k % N] + s > host_budget) return false;
        return true;
    };
    auto host_take = [&](uint64_t s, int32_t start, int32_t end) {
        for (int k = start + 1; k < end; ++k) Mh[k % N] += s;
    };
    std::vector<Pair> sel;
    auto dur = [&](uint64_t s) -> int64_t { return bw ? (int64_t)(((u128)s * 1000000000ull + bw - 1) / bw) : 0; };
    auto hdur = [&](uint64_t s) -> int64_t { return (int64_t)(((u128)s * 1000000000ull + host_bw - 1) / host_bw); };
    // score: sum of tau over the region C (= B / s of Algorithm 1).  With clamp_benefit the benefit is the prose form of
    // "Quantify the benefit and cost", B = sum over C of min(s, M'[k] - capacity) * tau[k]: only the bytes a kernel is
    // actually over capacity count.  Candidates are then ranked by the exact fraction B / s (cross-multiplied in 128 bits).
    struct Eval { bool ok; int64_t score, g, t_offloaded, t_prefetch; int32_t k_off, k_pre; u128 B; };
    auto compare_scores = [&](const Eval &a, uint64_t sa, const Eval &b, uint64_t sb) -> int {
        if (!clamp_benefit) return a.score < b.score ? -1 : (a.score > b.score ? 1 : 0);
        const u128 l = a.B * (u128)sb, r = b.B * (u128)sa;
        return l < r ? -1 : (l > r ? 1 : 0);
    };

    // ---- Algorithm 1
    std::vector<int64_t> over(2 * N + 1);
    while (*std::max_element(Mp.begin(), Mp.end()) > cap) {
        over[0] = 0;
        for (int k = 0; k < 2 * N; ++k) over[k + 1] = over[k] + (Mp[k % N] > cap ? tau[k % N] : 0);
        int best = -1;
        int64_t bd = 0;
        Eval best_ev{false, 0, 0, 0, 0, 0, 0, 0};
        // benefit of a candidate on one tier's channels
        auto evaluate = [&](Channel &c_off, Channel &c_pre, int64_t lo, int64_t hi, int64_t d, uint64_t bytes) -> Eval {
            Eval e{false, 0, 0, 0, 0, 0, 0, 0};
            e.g = c_off.earliest(lo, hi, d);
            if (e.g < 0) return e;
            e.t_offloaded = e.g + d;
            e.t_prefetch = c_pre.latest(lo, hi, d);
            if (e.t_prefetch < 0 || !(e.t_offloaded < e.t_prefetch)) return e;
            e.k_off = (int32_t)(std::lower_bound(T.begin(), T.end(), e.t_offloaded) - T.begin());
            e.k_pre = (int32_t)(std::upper_bound(T.begin(), T.end(), e.t_prefetch) - T.begin()) - 2;
            if (e.k_off > e.k_pre) return e;
            e.score = over[e.k_pre + 1] - over[e.k_off];             // B / s = sum of tau over the region C
            e.ok = e.score > 0;
            if (e.ok && clamp_benefit)
                for (int k = e.k_off; k <= e.k_pre; ++k) {
                    const uint64_t m = Mp[k % N];
                    if (m > cap) e.B += (u128)std::min<uint64_t>(bytes, m - cap) * (u128)tau[k % N];
                }
            return e;
        };
        int best_tier = 0;
        for (int i = 0; i < (int)I.size(); ++i) {
            const Cand &c = I[i];
            if (!c.alive) continue;
            int64_t d = dur(c.bytes);
            const int64_t lo = T[c.start + 1], hi = T[c.end];
            Eval ev = evaluate(ch_off, ch_pre, lo, hi, d, c.bytes);
            int where = 0;
            if (two_tier) {
                const bool displaced = !ev.ok || ev.g > lo || ev.t_prefetch + d < hi;
                if (displaced && host_fits(c.bytes, c.start, c.end)) {
                    const Eval hev = evaluate(hch_off, hch_pre, lo, hi, hdur(c.bytes), c.bytes);
                    if (hev.ok && (!ev.ok || compare_scores(hev, c.bytes, ev, c.bytes) > 0)) { ev = hev; where = 1; d = hdur(c.bytes); }
                }
            }
            if (!ev.ok) continue;
            bool take = best < 0;
            if (!take) {
                const Cand &o = I[best];
                const int by_score = compare_scores(ev, c.bytes, best_ev, o.bytes);
                take = by_score > 0 || (by_score == 0 && std::make_tuple(c.bytes, -c.start, -c.tensor, -c.end) >
                                                             std::make_tuple(o.bytes, -o.start, -o.tensor, -o.end));
            }
            if (take) { best = i; best_ev = ev; bd = d; best_tier = where; }
        }
        if (best < 0) break;
        Cand &c = I[best];
        const int64_t bg = best_ev.g, bto = best_ev.t_offloaded, btp = best_ev.t_prefetch;
        const int32_t bko = best_ev.k_off, bkp = best_ev.k_pre;
        sel.push_back({c.tensor, c.bytes, c.start, c.end, bko, bkp, 0, 0});
        sel.back().tier = best_tier;
        for (int k = bko; k <= bkp; ++k) Mp[k % N] -= c.bytes;
        if (best_tier == 0) {
            ch_off.insert(bg, bto);
            ch_pre.insert(btp, btp + bd);
        } else {
            hch_off.insert(bg, bto);
            hch_pre.insert(btp, btp + bd);
            host_take(c.bytes, c.start, c.end);
        }
        c.alive = false;
    }
    out.n_greedy = (int32_t)sel.size();

    // ---- urgent pass: at every kernel still above capacity evict the inactive tensor whose next use
    //      is furthest away, either by widening an already selected window or by selecting a new period
    auto frame = [&](int32_t start, int32_t end, int k) -> int32_t {
        if (start < k && k < end) return k;
        if (start < k + N && k + N < end) return k + N;
        return -1;
    };
    for (int k = 0; k < N; ++k) {
        while (Mp[k] > cap) {
            int what = 0, ref = -1; int32_t bkk = 0;     // what: 1 selected pair, 2 period in I, 3 period in small
            ForcedKey bk{};
            auto consider = [&](int w, int r, int32_t kk, int32_t end, uint64_t bytes, int32_t start, int32_t tensor) {
                ForcedKey key{(int64_t)end - kk, bytes, start, tensor};
                if (!what || key.better_than(bk)) { what = w; ref = r; bkk = kk; bk = key; }
            };
            for (int pass = 0; pass < 2 && !what; ++pass) {
                for (int i = 0; i < (int)sel.size(); ++i) {
                    const Pair &p = sel[i];
                    const int32_t kk = frame(p.start, p.end, k);
                    if (kk < 0 || (p.k_off <= kk && kk <= p.k_pre)) continue;
                    if (pass == 0 && min_bytes && p.bytes < min_bytes) continue;
                    consider(1, i, kk, p.end, p.bytes, p.start, p.tensor);
                }
                std::vector<Cand> &pool = pass == 0 ? I : small;
                for (int i = 0; i < (int)pool.size(); ++i) {
                    const Cand &c = pool[i];
                    if (!c.alive) continue;
                    const int32_t kk = frame(c.start, c.end, k);
                    if (kk < 0) continue;
                    consider(pass == 0 ? 2 : 3, i, kk, c.end, c.bytes, c.start, c.tensor);
                }
            }
            if (!what)
                throw PlanError{TIO_ERR_ACTIVE_SET_EXCEEDS_CAP,
                                "operands of kernel " + std::to_string(k) + " alone exceed the capacity"};
            int idx = ref;
            if (what != 1) {
                Cand &c = (what == 2 ? I : small)[ref];
                c.alive = false;
                sel.push_back({c.tensor, c.bytes, c.start, c.end, bkk, bkk - 1, 1, 1});   // empty window, grown below
                idx = (int)sel.size() - 1;
                // a stalled kernel waits for exactly these transfers: the faster tier when its budget has room
                if (two_tier && host_fits(c.bytes, c.start, c.end)) {
                    sel.back().tier = 1;
                    host_take(c.bytes, c.start, c.end);
                }
            }
            Pair &p = sel[idx];
            if (bkk < p.k_off) {                       // pull the offload deadline forward
                for (int j = bkk; j < p.k_off; ++j) Mp[j % N] -= p.bytes;
                p.k_off = bkk; p.urgent_off = 1;
            } else {                                   // push the prefetch back
                int32_t last = bkk;
                for (int j = bkk; j < p.end; ++j) if (Mp[j % N] > cap) last = j;
                for (int j = p.k_pre + 1; j <= last; ++j) Mp[j % N] -= p.bytes;
                p.k_pre = last; p.urgent_pre = 1;
            }
        }
    }
    out.n_forced = (int32_t)sel.size() - out.n_greedy;
    out.host_peak = *std::max_element(Mh.begin(), Mh.end());
    out.host_bw = host_bw;
    out.n_kernels = N;
    out.Mp = Mp;
    out.pairs = sel;
    out.entries.clear();
    out.bytes_moved = 0;
    for (int i = 0; i < (int)sel.size(); ++i) {
        const Pair &p = sel[i];
        out.entries.push_back({p.tensor, TIO_OFFLOAD, p.start + 1, p.k_off, p.urgent_off, i});
        out.entries.push_back({p.tensor, TIO_PREFETCH, p.k_pre + 1, p.end, p.urgent_pre, i});
        out.bytes_moved += p.bytes;
    }
    std::sort(out.entries.begin(), out.entries.end(), [N](const tio_plan_entry &a, const tio_plan_entry &b) {
        // at one trigger point offloads are issued before prefetches (a prefetch may reuse the range an
        // offload of the same point empties), urgent ones first within each direction
        return std::make_tuple(a.trigger % N, a.kind, -a.urgent, a.tensor, a.pair) <
               std::make_tuple(b.trigger % N, b.kind, -b.urgent, b.tensor, b.pair);
    });
}

// ------------------------------------------------------------------------------------------------
// address assignment
// ------------------------------------------------------------------------------------------------
static bool time_conflict(const Alloc &x, const Alloc &y, int N) {
    if (x.whole_cycle || y.whole_cycle) return true;
    auto ov = [](int a0, int a1, int b0, int b1) { return a0 <= b1 && b0 <= a1; };
    return ov(x.first, x.last, y.first, y.last) || ov(x.first, x.last, y.first + N, y.last + N) ||
           ov(x.first + N, x.last + N, y.first, y.last);
}

bool assign_addresses(const Trace &t, const Lifetimes &life, uint64_t arena_bytes, Plan &plan) {
    const int N = t.n_kernels;
    plan.allocs.clear();
    plan.alloc_of.assign(t.n_tensors, {});
    std::vector<std::vector<int>> pairs_of(t.n_tensors);
    for (int i = 0; i < (int)plan.pairs.size(); ++i) pairs_of[plan.pairs[i].tensor].push_back(i);
    for (int id = 0; id < t.n_tensors; ++id) {
        const auto &a = life.active[id];
        auto &ps = pairs_of[id];
        std::sort(ps.begin(), ps.end(), [&](int x, int y) { return plan.pairs[x].start < plan.pairs[y].start; });
        auto add = [&](int first, int last, int born, int ended, bool whole) {
            Alloc al;
            al.tensor = id; al.born_by_pair = born; al.ended_by_pair = ended; al.whole_cycle = whole;
            if (first >= N) { first -= N; last -= N; }
            al.first = first; al.last = last;
            plan.allocs.push_back(al);
            const int idx = (int)plan.allocs.size() - 1;
            plan.alloc_of[id].push_back(idx);
            if (born >= 0) plan.pairs[born].alloc_after = idx;
            if (ended >= 0) plan.pairs[ended].alloc_before = idx;
        };
        if (id < t.n_persistent) {
            if (ps.empty()) { add(0, N - 1, -1, -1, true); continue; }
            for (size_t i = 0; i < ps.size(); ++i) {
                const Pair &cur = plan.pairs[ps[i]];
                const bool wrap = i + 1 == ps.size();
                const Pair &nxt = plan.pairs[ps[wrap ? 0 : i + 1]];
                add(cur.k_pre + 1, nxt.k_off - 1 + (wrap ? N : 0), ps[i], ps[wrap ? 0 : i + 1], false);
            }
        } else {
            if (a.empty()) continue;
            int cur = a.front(), born = -1;
            for (int pi : ps) {
                const Pair &p = plan.pairs[pi];
                add(cur, p.k_off - 1, born, pi, false);
                cur = p.k_pre + 1; born = pi;
            }
            add(cur, a.back(), born, -1, false);
        }
    }
    // first fit, largest first
    const int A = (int)plan.allocs.size();
    std::vector<int> order(A);
    std::iota(order.begin(), order.end(), 0);
    std::sort(order.begin(), order.end(), [&](int x, int y) {
        const Alloc &ax = plan.allocs[x], &ay = plan.allocs[y];
        const uint64_t sx = t.tensor_bytes[ax.tensor], sy = t.tensor_bytes[ay.tensor];
        return std::make_tuple(sy, ax.first, ax.tensor, ax.last) < std::make_tuple(sx, ay.first, ay.tensor, ay.last);
    });
    std::vector<int> placed;
    std::vector<std::pair<uint64_t, uint64_t>> busy;
    uint64_t top = 0;
    for (int idx : order) {
        Alloc &al = plan.allocs[idx];
        const uint64_t s = t.tensor_bytes[al.tensor];
        busy.clear();
        for (int j : placed) {
            const Alloc &o = plan.allocs[j];
            if (time_conflict(al, o, N)) busy.push_back({o.address, o.address + t.tensor_bytes[o.tensor]});
        }
        std::sort(busy.begin(), busy.end());
        uint64_t addr = 0;
        for (auto &iv : busy) {
            if (addr + s <= iv.first) break;
            addr = std::max(addr, iv.second);
        }
        al.address = addr;
        top = std::max(top, addr + s);
        placed.push_back(idx);
    }
    plan.arena_needed = top;

    // slow-tier slots: a home slot for every persistent tensor, one slot per migrated transient period
    uint64_t h = 0;
    plan.persistent_home.assign(t.n_persistent, 0);
    for (int id = 0; id < t.n_persistent; ++id) { plan.persistent_home[id] = h; h += t.tensor_bytes[id]; }
    for (Pair &p : plan.pairs) {
        if (p.tier != 0) continue;
        if (p.tensor < t.n_persistent) p.host_offset = plan.persistent_home[p.tensor];
        else { p.host_offset = h; h += p.bytes; }
    }
    plan.host_needed = h;
    // host-memory tier: a pair holds its slot during its whole inactive period; slots are reused over time
    // (first fit, selection order), so the pool stays close to the peak the budget allows
    {
        std::vector<int> placed;
        uint64_t top = 0;
        auto overlap = [&](const Pair &x, const Pair &y) {
            auto ov = [](int a0, int a1, int b0, int b1) { return a0 <= b1 && b0 <= a1; };
            const int x0 = x.start + 1, x1 = x.end - 1, y0 = y.start + 1, y1 = y.end - 1;
            return ov(x0, x1, y0, y1) || ov(x0, x1, y0 + N, y1 + N) || ov(x0 + N, x1 + N, y0, y1);
        };
        for (int i = 0; i < (int)plan.pairs.size(); ++i) {
            Pair &p = plan.pairs[i];
            if (p.tier != 1) continue;
            std::vector<std::pair<uint64_t, uint64_t>> busy;
            for (int j : placed) if (overlap(p, plan.pairs[j])) busy.push_back({plan.pairs[j].host_offset, plan.pairs[j].host_offset + plan.pairs[j].bytes});
            std::sort(busy.begin(), busy.end());
            uint64_t addr = 0;
            for (auto &iv : busy) {
                if (addr + p.bytes <= iv.first) break;
                addr = std::max(addr, iv.second);
            }
            p.host_offset = addr;
            top = std::max(top, addr + p.bytes);
            placed.push_back(i);
        }
        plan.host_tier_needed = top;
    }
    plan.pair_tier.clear();
    for (const Pair &p : plan.pairs) plan.pair_tier.push_back(p.tier);

    // address reuse: the first writer of an allocation waits for the offload that emptied the range.
    // Sweep two cycles of the issue order with a map "address range -> last occupant".
    std::vector<std::vector<int>> born_at(N);       // allocations that start at kernel k, prefetches first
    for (const tio_plan_entry &e : plan.entries)
        if (e.kind == TIO_PREFETCH) born_at[e.trigger % N].push_back(plan.pairs[e.pair].alloc_after);
    for (int i = 0; i < A; ++i) {
        const Alloc &al = plan.allocs[i];
        if (al.born_by_pair < 0 && !al.whole_cycle) born_at[al.first % N].push_back(i);
    }
    std::map<uint64_t, std::pair<uint64_t, int>> occ;   // start -> (end, alloc)
    for (int cycle = 0; cycle < 2; ++cycle)
        for (int k = 0; k < N; ++k)
            for (int ai : born_at[k]) {
                Alloc &al = plan.allocs[ai];
                const uint64_t a0 = al.address, a1 = a0 + t.tensor_bytes[al.tensor];
                if (cycle == 1) al.wait_pairs.clear();
                auto it = occ.lower_bound(a0);
                if (it != occ.begin()) { auto pv = std::prev(it); if (pv->second.first > a0) it = pv; }
                std::vector<std::pair<uint64_t, std::pair<uint64_t, int>>> keep;
                while (it != occ.end() && it->first < a1) {
                    const uint64_t b0 = it->first, b1 = it->second.first;
                    const int who = it->second.second;
                    const int ep = plan.allocs[who].ended_by_pair;
                    if (cycle == 1 && ep >= 0 && std::find(al.wait_pairs.begin(), al.wait_pairs.end(), ep) == al.wait_pairs.end())
                        al.wait_pairs.push_back(ep);
                    if (b0 < a0) keep.push_back({b0, {a0, who}});
                    if (b1 > a1) keep.push_back({a1, {b1, who}});
                    it = occ.erase(it);
                }
                for (auto &kv : keep) occ[kv.first] = kv.second;
                occ[a0] = {a1, ai};
            }

    // executor tables
    plan.entries_at.assign(N, {});
    plan.kernel_wait_pre.assign(N, {});
    plan.kernel_wait_off.assign(N, {});
    plan.kernel_needs_event.assign(N, 0);
    for (int i = 0; i < (int)plan.entries.size(); ++i) {
        const tio_plan_entry &e = plan.entries[i];
        plan.entries_at[e.trigger % N].push_back(i);
        plan.kernel_needs_event[(e.trigger - 1 + N) % N] = 1;
    }
    for (int i = 0; i < (int)plan.pairs.size(); ++i) plan.kernel_wait_pre[plan.pairs[i].end % N].push_back(i);
    for (int i = 0; i < A; ++i) {
        const Alloc &al = plan.allocs[i];
        if (al.born_by_pair < 0 && !al.whole_cycle)
            for (int p : al.wait_pairs) plan.kernel_wait_off[al.first % N].push_back(p);
    }
    plan.v_allocs.clear();
    for (const Alloc &al : plan.allocs) plan.v_allocs.push_back({al.tensor, al.first, al.last, al.address});
    return top <= arena_bytes;
}

SimResult simulate_plan(const Trace &t, const Plan &plan, uint64_t bw, bool duplex, int iterations,
                        std::vector<int64_t> *stretched) {
    const int N = t.n_kernels;
    const size_t np = plan.pairs.size();
    if (stretched) stretched->assign(N, 0);
    // entry indices by trigger point, in the plan's issue order (the executor tables may not have been built yet)
    std::vector<std::vector<int32_t>> entries_at(N);
    for (int i = 0; i < (int)plan.entries.size(); ++i) entries_at[plan.entries[i].trigger % N].push_back(i);
    std::vector<std::vector<int32_t>> pre_deadline(N), off_deadline(N);
    for (const tio_plan_entry &e : plan.entries)
        (e.kind == TIO_OFFLOAD ? off_deadline : pre_deadline)[e.deadline % N].push_back(e.pair);
    // pairs of the host-memory tier move on that tier's own two channels at the plan's host bandwidth
    auto dur = [&](const Pair &p) -> int64_t {
        const uint64_t r = p.tier ? plan.host_bw : bw;
        return r ? (int64_t)(((u128)p.bytes * 1000000000ull + r - 1) / r) : 0;
    };
    std::vector<int64_t> off_done(np, 0), pre_done(np, 0);
    int64_t d2h_free[2] = {0, 0}, h2d_free[2] = {0, 0};
    int64_t done_prev = 0;          // completion of the previous kernel
    int64_t mem_ready = 0;          // completion of every offload whose deadline has been passed
    int64_t last = 0, compute = 0;
    for (int k = 0; k < N; ++k) compute += t.tau[k];
    for (int it = 0; it < iterations; ++it) {
        const int64_t t0 = done_prev;
        for (int k = 0; k < N; ++k) {
            for (int32_t p : off_deadline[k]) mem_ready = std::max(mem_ready, off_done[p]);
            for (int32_t ei : entries_at[k]) {
                const tio_plan_entry &e = plan.entries[ei];
                const int64_t d = dur(plan.pairs[e.pair]);
                const int w = plan.pairs[e.pair].tier;
                if (e.kind == TIO_OFFLOAD) {
                    const int64_t st = std::max(d2h_free[w], done_prev);
                    off_done[e.pair] = d2h_free[w] = st + d;
                    if (!duplex) h2d_free[w] = d2h_free[w];
                } else {
                    const int64_t st = std::max(std::max(h2d_free[w], done_prev), std::max(off_done[e.pair], mem_ready));
                    pre_done[e.pair] = h2d_free[w] = st + d;
                    if (!duplex) d2h_free[w] = h2d_free[w];
                }
            }
            int64_t st = std::max(done_prev, mem_ready);
            for (int32_t p : pre_deadline[k]) st = std::max(st, pre_done[p]);
            for (int32_t p : off_deadline[k]) st = std::max(st, off_done[p]);     // offloads issued at this very trigger point
            if (stretched) (*stretched)[k] = st + t.tau[k] - done_prev;           // the kernel and the stall in front of it
            done_prev = st + t.tau[k];
        }
        last = done_prev - t0;
    }
    return SimResult{last, compute};
}

// Discrete-event model of the engine with ready queues.  Events are the end of a chunk on one of the four channels
// (direction x tier) and the end of the running kernel; at every event time the model first retires what ends,
// issues the entries whose trigger point was reached, then lets every free channel take a chunk and the compute
// stream start the next kernel if its migrations are complete.
SimResult simulate_engine(const Trace &t, const Plan &plan, uint64_t bw, bool duplex, int iterations, uint64_t chunk_bytes,
                          bool urgent_first) {
    const int N = t.n_kernels;
    const size_t np = plan.pairs.size();
    struct Request {
        int kind, pair, urgent;
        uint64_t left, rate;
        int64_t done_at;                       // -1 while unfinished
        std::vector<int> deps;                 // requests that must be complete before the first chunk
    };
    std::vector<Request> req;
    std::vector<std::vector<int32_t>> pre_deadline(N), off_deadline(N);
    for (const tio_plan_entry &e : plan.entries)
        (e.kind == TIO_OFFLOAD ? off_deadline : pre_deadline)[e.deadline % N].push_back(e.pair);
    constexpr int NC = 4;
    std::vector<int> queue[NC];                // issued and unfinished, in issue order
    int in_flight[NC] = {-1, -1, -1, -1};
    int64_t busy_until[NC] = {0, 0, 0, 0};
    std::vector<int> last_off(np, -1), last_pre(np, -1), due;
    auto done = [&](int r, int64_t now) { return req[r].done_at >= 0 && req[r].done_at <= now; };
    auto issue = [&](int k, int64_t now) {
        for (int32_t p : off_deadline[k]) if (last_off[p] >= 0) due.push_back(last_off[p]);
        for (int32_t ei : plan.entries_at[k]) {
            const tio_plan_entry &e = plan.entries[ei];
            const Pair &pr = plan.pairs[e.pair];
            Request r{e.kind, e.pair, e.urgent, pr.bytes, pr.tier ? plan.host_bw : bw, -1, {}};
            const int id = (int)req.size();
            if (e.kind == TIO_PREFETCH) {
                if (last_off[e.pair] >= 0) r.deps.push_back(last_off[e.pair]);
                for (int q : due) if (!done(q, now)) r.deps.push_back(q);
                last_pre[e.pair] = id;
            } else {
                last_off[e.pair] = id;
            }
            req.push_back(std::move(r));
            queue[2 * pr.tier + (duplex ? e.kind : 0)].push_back(id);
        }
        for (int32_t p : off_deadline[k])      // offloads issued at this very trigger point
            if (last_off[p] >= 0 && std::find(due.begin(), due.end(), last_off[p]) == due.end()) due.push_back(last_off[p]);
    };
    auto ready = [&](int r, int64_t now) {
        for (int q : req[r].deps) if (!done(q, now)) return false;
        return true;
    };
    auto pick = [&](int c, int64_t now) {
        int first = -1;
        for (int r : queue[c]) {
            if (!ready(r, now)) continue;
            if (urgent_first && req[r].urgent) return r;
            if (first < 0) first = r;
            if (!urgent_first) break;
        }
        return first;
    };
    auto kernel_may_start = [&](int k, int64_t now) {
        due.erase(std::remove_if(due.begin(), due.end(), [&](int q) { return done(q, now); }), due.end());
        if (!due.empty()) return false;
        for (int32_t p : pre_deadline[k]) if (last_pre[p] >= 0 && !done(last_pre[p], now)) return false;
        return true;
    };
    int64_t compute = 0;
    for (int k = 0; k < N; ++k) compute += t.tau[k];
    const int64_t total = (int64_t)iterations * N;
    int64_t now = 0, k_glob = 0, running_until = -1, iter_start = 0, last = 0;
    issue(0, 0);
    while (k_glob < total) {
        bool changed = true;
        while (changed && k_glob < total) {
            changed = false;
            for (int c = 0; c < NC; ++c)
                if (in_flight[c] >= 0 && busy_until[c] <= now) {
                    const int r = in_flight[c];
                    if (req[r].left == 0) {
                        req[r].done_at = busy_until[c];
                        queue[c].erase(std::find(queue[c].begin(), queue[c].end(), r));
                    }
                    in_flight[c] = -1;
                    changed = true;
                }
            if (running_until >= 0 && running_until <= now) {
                running_until = -1;
                ++k_glob;
                if (k_glob % N == 0) { last = now - iter_start; iter_start = now; }
                if (k_glob < total) issue((int)(k_glob % N), now);
                changed = true;
                continue;
            }
            for (int c = 0; c < NC; ++c)
                if (in_flight[c] < 0) {
                    const int r = pick(c, now);
                    if (r < 0) continue;
                    const uint64_t n = chunk_bytes ? std::min(req[r].left, chunk_bytes) : req[r].left;
                    req[r].left -= n;
                    busy_until[c] = now + (req[r].rate ? (int64_t)(((u128)n * 1000000000ull + req[r].rate - 1) / req[r].rate) : 0);
                    in_flight[c] = r;
                    changed = true;
                }
            if (running_until < 0 && kernel_may_start((int)(k_glob % N), now)) {
                running_until = now + t.tau[k_glob % N];
                changed = true;
            }
        }
        if (k_glob >= total) break;
        int64_t next = running_until >= 0 ? running_until : INT64_MAX;
        for (int c = 0; c < NC; ++c) if (in_flight[c] >= 0) next = std::min(next, busy_until[c]);
        if (next == INT64_MAX || next <= now) throw PlanError{TIO_ERR_PLAN_INVALID, "performance model: nothing in flight and nothing can start"};
        now = next;
    }
    return SimResult{last, compute};
}

uint64_t address_at(const Plan &plan, int32_t tensor, int32_t k) {
    const int N = plan.n_kernels;
    for (int ai : plan.alloc_of[tensor]) {
        const Alloc &al = plan.allocs[ai];
        if (al.whole_cycle || (al.first <= k && k <= al.last) || (al.first <= k + N && k + N <= al.last)) return al.address;
    }
    return UINT64_MAX;
}

// ------------------------------------------------------------------------------------------------
// Re-timing (an extension; the paper plans once, on the kernel times of an iteration that does not stall).  When the
// bytes that must move take longer than the compute, the iteration stalls, and the timeline Algorithm 1 plans on (the
// sum of the kernel times) is several times shorter than the iteration the engine will run: the channels look full
// after a fraction of the bytes, the rest is evicted by the urgent pass at the kernels where memory overflows (all
// offloads in the forward pass, all prefetches in the backward pass), and the two directions end up working one
// after the other.  Re-timing runs Algorithm 1 again on the timeline of the iteration as the performance model says
// it executes under the previous plan: kernel k takes its own time plus the stall in front of it.  On that timeline
// the channels have the time they really have, and the greedy loop spreads both directions over the whole iteration.
// Every pass is simulated on the true kernel times and the passes are ranked by predicted iteration, the earlier pass
// first among equals; the caller keeps the best one whose address layout fits the arena (pass 0 is the paper's plan,
// so with room in the arena the result is never predicted slower than it).  A plan's validity does not depend on kernel times
// (residency is counted per kernel index), so every pass yields a valid plan for the same trace.
// ------------------------------------------------------------------------------------------------
void select_periods_retimed(const Trace &t, const Lifetimes &life, uint64_t cap, uint64_t bw, bool duplex,
                            uint64_t min_bytes, uint64_t host_bw, uint64_t host_budget, bool clamp_benefit, int passes,
                            const Plan &proto, std::vector<Plan> &out) {
    out.clear();
    std::vector<int64_t> steps;
    auto fresh = [&]() {
        Plan p;
        p.cap = proto.cap; p.planning_cap = proto.planning_cap; p.bw = proto.bw; p.structure_hash = proto.structure_hash;
        return p;
    };
    out.push_back(fresh());
    select_periods(t, life, cap, bw, duplex, min_bytes, host_bw, host_budget, clamp_benefit, out.back());
    out.back().retime_pass = 0;
    if (passes <= 0 || bw == 0) return;
    std::vector<int64_t> first;
    steps.push_back(simulate_plan(t, out.back(), bw, duplex, 3, &first).step_ns);
    // Two chains of passes from the same start.  Chain A plans on the fully stretched timeline.  Chain B stretches
    // only the kernels from the first kernel of largest memory demand on: before that point memory grows and the
    // stalls wait for offloads, and a timeline stretched there invites the planner to offload exactly there again
    // (at the Llama-7B shape: the forward pass keeps stalling on activation offloads while the offload channel has
    // spare time in the backward pass); with the kernels before the peak at their own times, those offloads do not
    // fit, and the planner keeps more optimizer state out across the forward pass instead.
    const int N = t.n_kernels;
    const int kpeak = (int)(std::max_element(life.M.begin(), life.M.end()) - life.M.begin());
    Trace tt = t;
    for (int chain = 0; chain < 2; ++chain) {
        std::vector<int64_t> stretched = first;
        for (int pass = 1; pass <= passes; ++pass) {
            for (int k = 0; k < N; ++k) tt.tau[k] = (chain == 1 && k < kpeak) ? t.tau[k] : stretched[k];
            out.push_back(fresh());
            select_periods(tt, life, cap, bw, duplex, min_bytes, host_bw, host_budget, clamp_benefit, out.back());
            out.back().retime_pass = chain * passes + pass;
            steps.push_back(simulate_plan(t, out.back(), bw, duplex, 3, &stretched).step_ns);
        }
    }
    // shortest predicted iteration first, the earlier pass among equals
    std::vector<int> order(out.size());
    for (int i = 0; i < (int)order.size(); ++i) order[i] = i;
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return steps[a] < steps[b]; });
    std::vector<Plan> sorted;
    for (int i : order) { out[i].predicted_step_ns = steps[i]; sorted.push_back(std::move(out[i])); }
    out = std::move(sorted);
}

// ------------------------------------------------------------------------------------------------
// plan = selection + layout, with the planning capacity lowered until the layout fits the arena
// ------------------------------------------------------------------------------------------------
Plan build_plan(const Trace &t, const Lifetimes &life, uint64_t cap, uint64_t bw, const tio_plan_opts &o) {
    if (t.structure_hash != life.structure_hash) throw PlanError{TIO_ERR_PLAN_STALE, "lifetimes belong to another trace"};
    const uint64_t peak = *std::max_element(life.M.begin(), life.M.end());
    const uint64_t arena = o.arena_bytes ? o.arena_bytes : cap;
    const int retries = o.layout_retries > 0 ? o.layout_retries : 24;
    uint64_t pc = std::min(cap, peak);
    const uint64_t step = std::max<uint64_t>(256, std::min(cap, peak) / 50);
    // Selections at one planning capacity, best predicted first (one selection without re-timing); p = the first whose
    // layout fits the arena, top = the prediction of the best one whether it fits or not
    auto attempt = [&](uint64_t planning_cap, Plan &p, int64_t &top) {
        Plan proto;
        proto.cap = cap; proto.planning_cap = planning_cap; proto.bw = bw; proto.structure_hash = t.structure_hash;
        std::vector<Plan> cands;
        select_periods_retimed(t, life, planning_cap, bw, o.duplex != 0, o.min_bytes, o.host_bw, o.host_budget,
                               o.clamp_benefit != 0, o.retime_passes, proto, cands);
        top = cands.front().predicted_step_ns;
        for (Plan &c : cands)
            if (assign_addresses(t, life, arena, c)) { p = std::move(c); return true; }
        return false;
    };
    // The planning capacity goes down in steps of 2 % until a layout fits.  With re-timing, several selections compete at
    // every capacity and the first that fits may be predicted far slower than the best one, which may fit a step
    // further down at the price of 2 % more bytes: the search goes on while a lower capacity can still win (the best
    // found so far is predicted slower than the best selection of the current capacity, fitting or not), at most two
    // steps (one on long traces, where a step takes seconds) beyond the last improvement.
    Plan best;
    bool have = false;
    uint64_t best_pc = 0;
    int best_r = 0, since = 0;
    const int patience = t.n_kernels <= 4096 ? 2 : 1;
    for (int r = 0; r <= retries; ++r) {
        Plan p;
        int64_t top = 0;
        const bool ok = attempt(pc, p, top);
        if (ok && (!have || p.predicted_step_ns < best.predicted_step_ns)) {
            best = std::move(p); have = true; best_pc = pc; best_r = r; since = 0;
        } else if (have) {
            ++since;
        }
        if (have && (best.predicted_step_ns <= top || since >= patience)) break;
        if (pc <= step) break;
        pc -= step;
    }
    if (!have) throw PlanError{TIO_ERR_ARENA_TOO_SMALL, "no address assignment fits the arena"};
    // the step above the chosen capacity did not do as well: look between the two for a larger planning capacity that
    // does (every byte of it is a byte that need not move), halving the interval a few times; fewer times for long
    // traces, where one attempt takes seconds
    uint64_t lo = best_pc, hi = best_r > 0 ? best_pc + step : best_pc;
    const int halvings = t.n_kernels <= 4096 ? 4 : t.n_kernels <= 16384 ? 2 : 0;
    for (int i = 0; i < halvings && hi - lo >= 512; ++i) {
        const uint64_t mid = (lo + (hi - lo) / 2) / 256 * 256;
        Plan q;
        int64_t top = 0;
        if (attempt(mid, q, top) && q.predicted_step_ns <= best.predicted_step_ns) { lo = mid; best = std::move(q); } else hi = mid;
    }
    // With re-timing the result is never predicted slower than the plan built without it for the same arena: that plan
    // may sit at a planning capacity the search above did not reach.
    if (o.retime_passes > 0 && bw != 0 && best.retime_pass != 0) {
        tio_plan_opts once = o;
        once.retime_passes = 0;
        try {
            Plan paper = build_plan(t, life, cap, bw, once);
            paper.predicted_step_ns = simulate_plan(t, paper, bw, o.duplex != 0, 3, nullptr).step_ns;
            if (paper.predicted_step_ns < best.predicted_step_ns) return paper;
        } catch (const PlanError &) {
        }
    }
    return best;
}

void validate_plan(const Trace &t, const Lifetimes &life, const Plan &plan) {
    const int N = t.n_kernels;
    if (plan.structure_hash != t.structure_hash || plan.n_kernels != N) throw PlanError{TIO_ERR_PLAN_STALE, "plan belongs to another trace"};
    std::vector<uint64_t> M2 = life.M;
    for (const Pair &p : plan.pairs) {
        if (!(p.start < p.k_off && p.k_off <= p.k_pre + 1 && p.k_pre + 1 <= p.end))
            throw PlanError{TIO_ERR_PLAN_INVALID, "window outside its inactive period"};
        for (int k = p.k_off; k <= p.k_pre; ++k) M2[k % N] -= p.bytes;
    }
    for (int k = 0; k < N; ++k) {
        if (M2[k] != plan.Mp[k]) throw PlanError{TIO_ERR_PLAN_INVALID, "memory estimate differs from a recount"};
        if (M2[k] > plan.planning_cap) throw PlanError{TIO_ERR_PLAN_INVALID, "residency above capacity at kernel " + std::to_string(k)};
        for (int i = t.operand_off[k]; i < t.operand_off[k + 1]; ++i)
            if (address_at(plan, t.operand_tensor[i], k) == UINT64_MAX)
                throw PlanError{TIO_ERR_PLAN_INVALID, "operand not resident at kernel " + std::to_string(k)};
    }
    const int A = (int)plan.allocs.size();
    for (int i = 0; i < A; ++i)
        for (int j = i + 1; j < A; ++j) {
            const Alloc &x = plan.allocs[i], &y = plan.allocs[j];
            const uint64_t x1 = x.address + t.tensor_bytes[x.tensor], y1 = y.address + t.tensor_bytes[y.tensor];
            if (x.address < y1 && y.address < x1 && time_conflict(x, y, N))
                throw PlanError{TIO_ERR_PLAN_INVALID, "two resident tensors overlap in the arena"};
        }
}

}  // namespace tio
