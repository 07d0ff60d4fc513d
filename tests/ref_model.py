"""A second, independently written evaluation of the plan model, used only to cross-check
the C++ oracle on tiny inputs.  It is deliberately built differently: the pipeline time is
the longest path of an explicitly constructed dependency graph (Kahn order), partitions
and reroute vectors are enumerated with itertools and then sorted into index order, and
all arithmetic is Python's unbounded int.  It does not call the oracle.
"""
import itertools
from collections import defaultdict, deque

INF = (1 << 63) - 1


def one_f_one_b_order(S, M, s):
    w = min(S - 1 - s, M)
    seq = [("F", j) for j in range(w)]
    for j in range(M - w):
        seq += [("F", w + j), ("B", j)]
    seq += [("B", j) for j in range(M - w, M)]
    return seq


def dag_makespan(F, B, M):
    """longest path through the 1F1B dependency graph (Estimator, eq. (transition))"""
    S = len(F)
    cost, preds = {}, defaultdict(list)
    for s in range(S):
        seq = one_f_one_b_order(S, M, s)
        for n, (kind, j) in enumerate(seq):
            v = (s, kind, j)
            cost[v] = F[s] if kind == "F" else B[s]
            if n:
                preds[v].append((s,) + seq[n - 1])
            if kind == "F" and s > 0:
                preds[v].append((s - 1, "F", j))
            if kind == "B":
                preds[v].append((s + 1, "B", j) if s < S - 1 else (s, "F", j))
    succs, indeg = defaultdict(list), {v: 0 for v in cost}
    for v, ps in preds.items():
        for p in set(ps):
            succs[p].append(v)
            indeg[v] += 1
    end, q, seen = {}, deque(v for v in cost if indeg[v] == 0), 0
    start = defaultdict(int)
    while q:
        v = q.popleft()
        seen += 1
        end[v] = start[v] + cost[v]
        for u in succs[v]:
            start[u] = max(start[u], end[v])
            indeg[u] -= 1
            if indeg[u] == 0:
                q.append(u)
    assert seen == len(cost), "dependency graph has a cycle"
    return max(end.values())


def scale(x, q):
    return (x * q + 32768) // 65536


def colex_partitions(L, k):
    """all k-subsets of cut positions 1..L-1, in combinatorial-number-system order
    (compare the largest cut first)"""
    return sorted(itertools.combinations(range(1, L), k), key=lambda c: tuple(reversed(c)))


def reroute_vectors(parts, total, cap):
    """all vectors of `parts` non-negative entries summing to `total`, each <= cap if cap>0,
    in lexicographic order"""
    hi = total if cap <= 0 else min(total, cap)
    return sorted(v for v in itertools.product(range(hi + 1), repeat=parts) if sum(v) == total)


def layout_p0(L, S):
    sizes = [L // S + (1 if s >= S - L % S else 0) for s in range(S)]
    b = [0]
    for x in sizes:
        b.append(b[-1] + x)
    return b


def distribute(total, nodes):
    N = sum(nodes)
    out = [total * n // N if n else 0 for n in nodes]
    left, d = total - sum(out), 0
    while left:
        if nodes[d]:
            out[d] += 1
            left -= 1
        d = (d + 1) % len(nodes)
    while True:
        alive = [d for d in range(len(nodes)) if nodes[d]]
        empty = [d for d in alive if out[d] == 0]
        big = max(alive, key=lambda d: (out[d], -d))
        if not empty or out[big] < 2:
            return out
        out[big] -= 1
        out[empty[0]] += 1


def greedy_rounds(L, devices):
    """Restorer, "Asymmetric Communication": colour the layers in index order with the smallest colour not
    used by an earlier layer that shares a device; `devices` is a list of sets of layers"""
    colour = {}
    for l in range(L):
        seen = {colour[o] for dev in devices if l in dev for o in dev if o < l}
        c = 0
        while c in seen:
            c += 1
        colour[l] = c
    return max(colour.values()) + 1 if colour else 0


class Model:
    def __init__(self, sc):
        self.sc = sc
        self.L, self.S, self.D, self.M = sc["L"], sc["PP"], sc["DP"], sc["M"]
        self.f = [int(x) for x in sc["fwd_us"]]
        self.b = [int(x) for x in sc["bwd_us"]]
        self.m = [int(x) for x in sc["mem_mib"]]
        act = sc.get("act_mib")
        self.a = [int(x) for x in act] if act is not None else [0] * len(self.m)
        q = sc.get("speed_q16")
        self.q = [[int(q[d * self.S + s]) if q is not None else 65536 for s in range(self.S)] for d in range(self.D)]
        self.dead = [[(d * self.S + s) in sc["failed_nodes"] for s in range(self.S)] for d in range(self.D)]
        self.p0 = layout_p0(self.L, self.S)
        self.K = sc["horizon_steps"]
        self.cap_r = sc.get("reroute_cap", 0)
        S, D = self.S, self.D
        fail_rep = [sum(self.dead[d]) for d in range(D)]
        fail_stage = [sum(self.dead[d][s] for d in range(D)) for s in range(S)]
        self.fail_rep = fail_rep
        hasA = S >= 2 and not any(self.dead[d][s] and self.dead[d][(s - 1) % S] for d in range(D) for s in range(S))
        left = {S - n for n in fail_rep if n}
        hasB = len(sc["failed_nodes"]) > 0 and len(left) == 1 and min(left) >= 1
        self.SB = min(left) if hasB else 0
        self.mbB = distribute(D * self.M, [S - n for n in fail_rep]) if hasB else None
        self.affected = [s for s in range(S) if fail_stage[s]]
        self.peers = [[d for d in range(D) if not self.dead[d][s]] for s in self.affected]
        hasC = all(fail_stage[s] < D for s in range(S))
        self.vecs = []
        if hasC:
            for a, s in enumerate(self.affected):
                self.vecs.append(reroute_vectors(len(self.peers[a]), fail_stage[s] * self.M, self.cap_r))
                hasC = hasC and len(self.vecs[-1]) > 0
        self.has = [hasA, hasB, hasC]

    def seg(self, tab, lo, hi):
        return sum(tab[lo:hi])

    def missing(self, a, b, a0, b0):
        return sum(self.m[l] for l in range(a, b) if not (a0 <= l < b0))

    def cost(self, strategy, cuts, rr=()):
        terms = self.terms(strategy, cuts, rr)
        return INF if terms is None else self.K * terms[0] + terms[1]

    def terms(self, strategy, cuts, rr=()):
        """(step time, transition time) of a plan, None when it does not fit in memory"""
        sc, S, D, M = self.sc, self.S, self.D, self.M
        bounds = [0] + list(cuts) + [self.L]
        n = len(bounds) - 1
        fs = [self.seg(self.f, bounds[j], bounds[j + 1]) for j in range(n)]
        bs = [self.seg(self.b, bounds[j], bounds[j + 1]) for j in range(n)]
        ms = [self.seg(self.m, bounds[j], bounds[j + 1]) for j in range(n)]
        av = [self.seg(self.a, bounds[j], bounds[j + 1]) for j in range(n)]
        cap, comm = sc["mem_cap_mib"], sc["comm_us"]

        def peak(static, act, length, pos):      # Memory Estimator: static + (stages - position) x activations
            return static + (length - pos) * act

        if strategy == 0:
            for d in range(D):
                alive = [j for j in range(S) if not self.dead[d][j]]
                for pos, j in enumerate(alive):
                    nx = (j + 1) % S
                    if peak(ms[j] + ms[nx], av[j] + av[nx], len(alive), pos) > cap:
                        return None
            t = 0
            for d in range(D):
                alive = [j for j in range(S) if not self.dead[d][j]]
                F = [scale(fs[j] + fs[(j + 1) % S], self.q[d][j]) for j in alive]
                B = [scale(bs[j] + bs[(j + 1) % S], self.q[d][j]) for j in alive]
                t = max(t, dag_makespan(F, B, M) + (len(alive) - 1) * comm)
            miss = sum(self.missing(bounds[j], bounds[j + 1], self.p0[j], self.p0[j + 1]) for j in range(S))
        elif strategy == 1:
            if any(peak(ms[j], av[j], n, j) > cap for j in range(n)):
                return None
            t, miss = 0, 0
            for d in range(D):
                if self.fail_rep[d] == 0:
                    if any(peak(self.seg(self.m, self.p0[j], self.p0[j + 1]), self.seg(self.a, self.p0[j], self.p0[j + 1]), S, j) > cap
                           for j in range(S)):
                        return None
                    F = [scale(self.seg(self.f, self.p0[j], self.p0[j + 1]), self.q[d][j]) for j in range(S)]
                    B = [scale(self.seg(self.b, self.p0[j], self.p0[j + 1]), self.q[d][j]) for j in range(S)]
                    t = max(t, dag_makespan(F, B, self.mbB[d]) + (S - 1) * comm)
                else:
                    host = [j for j in range(S) if not self.dead[d][j]]
                    F = [scale(fs[j], self.q[d][host[j]]) for j in range(n)]
                    B = [scale(bs[j], self.q[d][host[j]]) for j in range(n)]
                    t = max(t, dag_makespan(F, B, self.mbB[d]) + (n - 1) * comm)
                    fetch = [[self.missing(bounds[j], bounds[j + 1], self.p0[host[i]], self.p0[host[i] + 1]) for j in range(n)]
                             for i in range(n)]                 # fetch[i][j]: survivor i becomes the node of new stage j
                    if sc.get("transfer_assign", 0):            # Restorer: the one-to-one assignment of least total transfer
                        miss_d = min(sum(fetch[perm[j]][j] for j in range(n)) for perm in itertools.permutations(range(n)))
                    else:
                        miss_d = sum(fetch[j][j] for j in range(n))
                    miss = max(miss, miss_d)
        else:
            if any(peak(ms[j], av[j], S, j) > cap for j in range(S)):
                return None
            t = 0
            for d in range(D):
                qq = [65536 if self.dead[d][j] else self.q[d][j] for j in range(S)]
                t = max(t, dag_makespan([scale(fs[j], qq[j]) for j in range(S)],
                                        [scale(bs[j], qq[j]) for j in range(S)], M))
            t += (S - 1) * comm
            for a, s in enumerate(self.affected):
                t += max(rr[a][i] * (scale(fs[s], self.q[d][s]) + scale(bs[s], self.q[d][s]))
                         for i, d in enumerate(self.peers[a]))
            miss = sum(self.missing(bounds[j], bounds[j + 1], self.p0[j], self.p0[j + 1]) for j in range(S))
        if sc.get("allreduce_us", 0):
            stage = [set(range(bounds[j], bounds[j + 1])) for j in range(n)]
            devices = []
            for d in range(D):
                alive = [j for j in range(S) if not self.dead[d][j]]
                if strategy == 0:
                    devices += [stage[j] | stage[(j + 1) % S] for j in alive]
                elif strategy == 1 and self.fail_rep[d]:
                    devices += stage
                elif strategy == 1:
                    devices += [set(range(self.p0[j], self.p0[j + 1])) for j in range(S)]
                else:
                    devices += [stage[j] for j in alive]
            t += sc["allreduce_us"] * greedy_rounds(self.L, devices)
        return t, sc["reconf_us"][strategy] + sc["xfer_us_per_mib"] * miss

    def all_costs(self):
        """cost of every plan in global index order"""
        out = []
        if self.has[0]:
            out += [self.cost(0, c) for c in colex_partitions(self.L, self.S - 1)]
        if self.has[1]:
            out += [self.cost(1, c) for c in colex_partitions(self.L, self.SB - 1)]
        if self.has[2]:
            joint = list(itertools.product(*self.vecs)) if self.vecs else [()]
            for c in colex_partitions(self.L, self.S - 1):
                out += [self.cost(2, c, rr) for rr in joint]
        return out


# ----------------------------------------------------------------------------- re-planning (Algorithm 1)
def replan(rp):
    """Independent evaluation of the search over DP/PP degrees: even integer partition of the node
    count, proportional micro-batches, per pipeline the best split by explicit-graph longest path,
    least-transfer matching by scipy, candidates ranked with exact fractions."""
    from fractions import Fraction
    from scipy.optimize import linear_sum_assignment
    import numpy as np
    L = rp["L"]
    f, b, m = ([int(x) for x in rp[k]] for k in ("fwd_us", "bwd_us", "mem_mib"))
    a = [int(x) for x in rp["act_mib"]] if rp.get("act_mib") is not None else [0] * L
    old_pp = rp["old_pp"]
    p0 = layout_p0(L, old_pp)
    held = [(p0[n % old_pp], p0[n % old_pp + 1]) for n in range(rp["old_dp"] * old_pp) if n not in rp["failed_nodes"]]
    N = len(held)
    best, n_cand = None, 0
    for dp in range(rp["dp_min"], rp["dp_max"] + 1):
        if dp > N:
            continue
        lens = sorted([N // dp] * (dp - N % dp) + [N // dp + 1] * (N % dp))
        if min(lens) < rp["pp_min"] or max(lens) > rp["pp_max"] or max(lens) > L or rp["micro_batches"] < dp:
            continue
        n_cand += 1
        mb = distribute(rp["micro_batches"], lens)
        plan, ok = [], True
        for n, M in zip(lens, mb):
            choice = None
            for cuts in colex_partitions(L, n - 1):
                bounds = [0] + list(cuts) + [L]
                if any(sum(m[bounds[j]:bounds[j + 1]]) + (n - j) * sum(a[bounds[j]:bounds[j + 1]]) > rp["mem_cap_mib"] for j in range(n)):
                    continue
                t = dag_makespan([sum(f[bounds[j]:bounds[j + 1]]) for j in range(n)],
                                 [sum(b[bounds[j]:bounds[j + 1]]) for j in range(n)], M)
                if choice is None or t < choice[0]:
                    choice = (t, list(cuts))
            if choice is None:
                ok = False
                break
            plan.append(choice)
        if not ok:
            continue
        pipeline_us = [t + (n - 1) * rp["comm_us"] for (t, _), n in zip(plan, lens)]
        t_step = max(pipeline_us)
        pos = []
        for (t, cuts), n in zip(plan, lens):
            bounds = [0] + cuts + [L]
            pos += [(bounds[j], bounds[j + 1]) for j in range(n)]
        rounds = 0
        if rp.get("allreduce_us", 0):
            rounds = greedy_rounds(L, [set(range(lo, hi)) for lo, hi in pos])
            t_step += rp["allreduce_us"] * rounds
        cost = np.array([[sum(m[l] for l in range(lo, hi) if not (hl <= l < hh)) for (lo, hi) in pos] for (hl, hh) in held])
        r, c = linear_sum_assignment(cost)
        fetch = int(cost[r, c].sum())
        t_trans = rp["restart_us"] + rp["xfer_us_per_mib"] * fetch
        score = Fraction(rp["horizon_us"] - t_trans, t_step)
        if best is None or score > best[0]:
            best = (score, {"found": True, "dp": dp, "length": lens, "micro_batches": mb, "cuts": [c for _, c in plan],
                            "pipeline_us": pipeline_us, "t_step_us": t_step, "fetch_mib": fetch, "t_trans_us": t_trans,
                            "comm_rounds": rounds})
    if best is None:
        return {"found": False, "n_candidates": n_cand}
    return dict(best[1], n_candidates=n_cand)
