"""A second, independent statement of the search in exact Python arithmetic.

Used only to pin the C oracle on tiny inputs: integers are Python ints,
accuracies are exact rationals (fractions.Fraction of the fp64 inputs), the
critical path and the accuracy are computed by a dynamic program over a
topological order (the C oracle enumerates paths instead), and the prune is
written with sorting and set operations (the C oracle uses flag arrays).
Follows Section 3.2 of the paper, Eq. 2, 3, 5-8, 11-13, with one
(variant, partition, batch) tuple per task.
"""
from __future__ import annotations

import itertools
from fractions import Fraction
from typing import Dict, List, Optional, Tuple


class PyRef:
    def __init__(self, pb):
        self.pb = pb
        self.T, self.V, self.P, self.B, self.C = pb.T, pb.V, pb.P, pb.B, pb.C
        self.lat = pb.latency_us.reshape(pb.T, pb.C).astype(object)
        self.thr = pb.thr_mrps.reshape(pb.T, pb.C).astype(object)
        self.m = [int(x) for x in pb.mult_milli]
        self.q = int(pb.queue_factor)
        self.preds: List[List[int]] = [[] for _ in range(pb.T)]
        self.succs: List[List[int]] = [[] for _ in range(pb.T)]
        for a, b in zip(pb.src.tolist(), pb.dst.tolist()):
            self.preds[b].append(a)
            self.succs[a].append(b)
        # topological order by repeated removal
        indeg = [len(p) for p in self.preds]
        order, ready = [], [t for t in range(pb.T) if indeg[t] == 0]
        while ready:
            t = ready.pop()
            order.append(t)
            for s in self.succs[t]:
                indeg[s] -= 1
                if indeg[s] == 0:
                    ready.append(s)
        assert len(order) == pb.T, "cycle"
        self.order = order
        self.sinks = [t for t in range(pb.T) if not self.succs[t]]
        self.sink_total = sum(self.m[s] for s in self.sinks)
        self.accF = [[Fraction(float(pb.accuracy[t, v])) for v in range(pb.V)] for t in range(pb.T)]
        self.amax = self._acc([max(range(pb.V), key=lambda v: (self.accF[t][v], -v))
                               for t in range(pb.T)])

    # -- search-space restrictions (Section 4.3, Appendix B) --------------------------
    space = (True, True, True)          # accuracy scaling, spatial partitioning, graph-informed

    def _reference(self):
        """Per task, for its most accurate variant over the allowed partitions and all
        batches: highest latency, and units / throughput of the highest-throughput tuple."""
        A, S, T = self.space
        wp = max(range(self.P), key=lambda p: (int(self.pb.units[p]), -p))
        out = []
        for t in range(self.T):
            v = max(range(self.V), key=lambda v: (self.accF[t][v], -v))
            tuples = [(p, b) for p in range(self.P) if S or p == wp for b in range(self.B)]
            lmax = max(int(self.lat[t][(v * self.P + p) * self.B + b]) for p, b in tuples)
            p, b = max(tuples, key=lambda pb_: (int(self.thr[t][(v * self.P + pb_[0]) * self.B + pb_[1]]),
                                                -pb_[0], -pb_[1]))
            out.append((v, wp, lmax, int(self.pb.units[p]), int(self.thr[t][(v * self.P + p) * self.B + b])))
        return out

    def resource_shares(self):
        """Exact per-task shares of S_avail when budgets are static (None if not)."""
        if self.space[2] or int(self.pb.capacity_units) == 0:
            return None
        ref = self._reference()
        e = [Fraction(self.m[t] * ref[t][3], ref[t][4]) for t in range(self.T)]
        return [int(self.pb.capacity_units) * x / sum(e) for x in e]

    def allowed(self, D: int, slo_l: int, t: int, c: int) -> bool:
        A, S, T = self.space
        ref = self._reference()
        if not A and self.variant(c) != ref[t][0]:
            return False
        if not S and self.part(c) != ref[t][1]:
            return False
        if not T:
            lmax = [r[2] for r in ref]
            up, down = {}, {}
            for u in self.order:
                up[u] = max([up[p] + lmax[p] for p in self.preds[u]], default=0)
            for u in reversed(self.order):
                down[u] = max([down[s] + lmax[s] for s in self.succs[u]], default=0)
            worst = up[t] + lmax[t] + down[t]          # heaviest path through t
            if self.q * int(self.lat[t][c]) * worst > slo_l * lmax[t]:
                return False
            shares = self.resource_shares()
            if shares is not None and self.rep_cost(D, t, c)[1] > shares[t].numerator // shares[t].denominator:
                return False
        return True

    def variant(self, c: int) -> int:
        return c // (self.P * self.B)

    def part(self, c: int) -> int:
        return (c // self.B) % self.P

    def _acc(self, variants) -> Fraction:
        """Sum over paths of (request fraction x product of accuracies), as a
        node recursion: G(t) = a_t * sum_pred share(pred->t) * G(pred)."""
        G: Dict[int, Fraction] = {}
        for t in self.order:
            a = self.accF[t][variants[t]]
            if not self.preds[t]:
                G[t] = a
            else:
                tot = sum(self.m[p] for p in self.preds[t])
                G[t] = a * sum(Fraction(self.m[p], tot) * G[p] for p in self.preds[t])
        return sum(Fraction(self.m[s], self.sink_total) * G[s] for s in self.sinks)

    def _acc_values(self, vals) -> Fraction:
        """The same recursion for given per-task accuracies (exact rationals)."""
        G: Dict[int, Fraction] = {}
        for t in self.order:
            if not self.preds[t]:
                G[t] = vals[t]
            else:
                tot = sum(self.m[p] for p in self.preds[t])
                G[t] = vals[t] * sum(Fraction(self.m[p], tot) * G[p] for p in self.preds[t])
        return sum(Fraction(self.m[s], self.sink_total) * G[s] for s in self.sinks)

    def latency(self, choice) -> int:
        fin: Dict[int, int] = {}
        for t in self.order:
            fin[t] = int(self.lat[t][choice[t]]) + max([fin[p] for p in self.preds[t]], default=0)
        return self.q * max(fin[s] for s in self.sinks)

    def rep_cost(self, D: int, t: int, c: int) -> Tuple[int, int]:
        need = D * self.m[t]                       # micro-requests per second
        per = 1000 * int(self.thr[t][c])
        rep = max(1, -(-need // per))
        return rep, rep * int(self.pb.units[self.part(c)])

    def lists(self, D: int, slo_l: int, cap: int) -> Tuple[List[List[int]], bool]:
        if cap == 0:
            return [[c for c in range(self.C) if self.allowed(D, slo_l, t, c)] for t in range(self.T)], False
        # longest path through t with other tasks at their fastest choice:
        # longest chain ending just before t plus longest chain starting just after it
        lo = [min(int(x) for x in self.lat[t]) for t in range(self.T)]
        up = {}
        for t in self.order:
            up[t] = max([up[p] + lo[p] for p in self.preds[t]], default=0)
        down = {}
        for t in reversed(self.order):
            down[t] = max([down[s] + lo[s] for s in self.succs[t]], default=0)
        out, truncated = [], False
        for t in range(self.T):
            through = up[t] + down[t]
            rows = []
            for c in range(self.C):
                if self.allowed(D, slo_l, t, c) and self.q * (int(self.lat[t][c]) + through) <= slo_l:
                    rows.append((int(self.lat[t][c]), self.accF[t][self.variant(c)],
                                 self.rep_cost(D, t, c)[1], c))
            front = []
            for r in rows:
                beaten = False
                for o in rows:
                    if o is r:
                        continue
                    if o[0] <= r[0] and o[1] >= r[1] and o[2] <= r[2]:
                        if (o[0], o[1], o[2]) != (r[0], r[1], r[2]) or o[3] < r[3]:
                            beaten = True
                            break
                if not beaten:
                    front.append(r)
            if len(front) > cap:
                truncated = True
                quota = cap // self.V
                kept = []
                for v in range(self.V):
                    mine = sorted((r for r in front if self.variant(r[3]) == v),
                                  key=lambda r: (r[0], r[3]))
                    n = len(mine)
                    if n <= quota:
                        kept += mine
                    else:
                        kept += [mine[(j * (n - 1)) // (quota - 1)] for j in range(quota)]
                front = kept
            out.append(sorted(r[3] for r in front))
        return out, truncated

    def search_objective(self, D: int, slo_l: int, slo_a: float, cap: int, alpha: float, beta: float):
        """Eq. 14 in exact rationals: the feasible candidate with the largest
        alpha*A_obj - beta*cost; ties -> lower cost -> lower index.  Returns
        (best (idx, cost, lat, acc, choice, obj) or None, gap to the best candidate
        with other variants or None)."""
        lists, _ = self.lists(D, slo_l, cap)
        K = [len(l) for l in lists]
        if not all(K):
            return None, None
        al, be, slo = Fraction(float(alpha)), Fraction(float(beta)), Fraction(float(slo_a))
        capu = int(self.pb.capacity_units)
        strides = [1] * self.T
        for t in range(1, self.T):
            strides[t] = strides[t - 1] * K[t - 1]
        feas = []
        for digits in itertools.product(*[range(k) for k in reversed(K)]):
            digits = digits[::-1]
            idx = sum(d * s for d, s in zip(digits, strides))
            choice = [lists[t][digits[t]] for t in range(self.T)]
            lat = self.latency(choice)
            cost = sum(self.rep_cost(D, t, choice[t])[1] for t in range(self.T))
            variants = tuple(self.variant(c) for c in choice)
            acc = self._acc(variants) / self.amax
            if lat <= slo_l and acc >= slo and (capu == 0 or cost <= capu):
                feas.append((-(al * acc - be * cost), cost, idx, lat, acc, choice, variants))
        if not feas:
            return None, None
        w = min(feas, key=lambda r: r[:3])
        others = [-r[0] for r in feas if r[6] != w[6]]
        gap = (-w[0] - max(others)) if others else None
        return (w[2], w[1], w[3], w[4], w[5], -w[0]), gap

    # -- per-variant multiplicative factors (Eq. 4, 5) ---------------------------------
    def demands(self, D: int, variants, factor_milli) -> List[int]:
        """Demand of every task in micro-requests/s for one choice of variants: D*m_t at a
        source, elsewhere the sum over incoming edges of floor(demand of the tail x factor of
        the tail's variant / 1000).  factor_milli[e][v] in the edge order of the problem."""
        edges = list(zip(self.pb.src.tolist(), self.pb.dst.tolist()))
        need: Dict[int, int] = {}
        for t in self.order:
            inc = [(a, e) for e, (a, b) in enumerate(edges) if b == t]
            if not inc:
                need[t] = D * self.m[t]
            else:
                need[t] = sum(need[a] * int(factor_milli[e][variants[a]]) // 1000 for a, e in inc)
        return [need[t] for t in range(self.T)]

    def search_factors(self, D: int, slo_l: int, slo_a: float, factor_milli, objective=None):
        """Brute force over the whole (allowed) space with per-variant factors; every
        candidate computes its own demands.  objective = None: cheapest feasible, ties to the
        lowest full index; (alpha, beta): largest alpha*A - beta*cost, then cheaper, then
        lowest full index.  Returns (full_index, cost, latency, accuracy, choice, replicas,
        objective or None) or None, and the number of candidates."""
        lists = [[c for c in range(self.C) if self.allowed(D, slo_l, t, c)] for t in range(self.T)]
        slo = Fraction(float(slo_a))
        capu = int(self.pb.capacity_units)
        best, count = None, 0
        for choice in itertools.product(*lists):
            count += 1
            variants = [self.variant(c) for c in choice]
            need = self.demands(D, variants, factor_milli)
            reps = []
            for t, c in enumerate(choice):
                per = 1000 * int(self.thr[t][c])
                reps.append(max(1, -(-need[t] // per)))
            cost = sum(r * int(self.pb.units[self.part(c)]) for r, c in zip(reps, choice))
            lat = self.latency(choice)
            acc = self._acc(variants) / self.amax
            if not (lat <= slo_l and acc >= slo and (capu == 0 or cost <= capu)):
                continue
            full = sum(c * self.C ** t for t, c in enumerate(choice))
            if objective is None:
                key, obj = (cost, full), None
            else:
                obj = Fraction(float(objective[0])) * acc - Fraction(float(objective[1])) * cost
                key = (-obj, cost, full)
            if best is None or key < best[0]:
                best = (key, (full, cost, lat, acc, list(choice), reps, obj))
        return (best[1] if best else None), count

    # -- mixtures of two tuples per task (Eq. 2, 6, 7, 9, 10) ---------------------------
    def mix_options(self, D: int, slo_l: int, t: int) -> List[dict]:
        """All options of task t, ascending id.  Mixtures are found from the side of the
        second tuple: for every count m2 of c2 the smallest count m1 of c1 that completes the
        demand, kept if one replica of c2 less would not do."""
        need = D * self.m[t]
        capu = int(self.pb.capacity_units)
        ok = [c for c in range(self.C) if self.allowed(D, slo_l, t, c)]
        out = []
        for c in ok:
            rep, cost = self.rep_cost(D, t, c)
            if capu and cost > capu:
                continue
            a = self.accF[t][self.variant(c)]
            out.append(dict(id=c, c1=c, c2=0xFFFF, m1=rep, m2=0, lat=int(self.lat[t][c]), cost=cost,
                            acc=float(self.pb.accuracy[t, self.variant(c)]), accF=a))
        for c1, c2 in itertools.combinations(ok, 2):
            h1, h2 = 1000 * int(self.thr[t][c1]), 1000 * int(self.thr[t][c2])
            u1, u2 = int(self.pb.units[self.part(c1)]), int(self.pb.units[self.part(c2)])
            m2 = 1
            while m2 * h2 < need:
                m1 = -(-(need - m2 * h2) // h1)
                if m1 * h1 + (m2 - 1) * h2 < need:
                    cost = m1 * u1 + m2 * u2
                    if capu == 0 or cost <= capu:
                        a1, a2 = self.accF[t][self.variant(c1)], self.accF[t][self.variant(c2)]
                        w1, w2 = float(m1 * h1), float(m2 * h2)
                        f1 = float(self.pb.accuracy[t, self.variant(c1)])
                        f2 = float(self.pb.accuracy[t, self.variant(c2)])
                        out.append(dict(id=self.C + (c1 * self.C + c2) * 65536 + m1, c1=c1, c2=c2, m1=m1, m2=m2,
                                        lat=max(int(self.lat[t][c1]), int(self.lat[t][c2])), cost=cost,
                                        acc=(w1 * f1 + w2 * f2) / (w1 + w2),
                                        accF=(m1 * h1 * a1 + m2 * h2 * a2) / (m1 * h1 + m2 * h2)))
                m2 += 1
        return sorted(out, key=lambda o: o["id"])

    def mix_lists(self, D: int, slo_l: int, cap: int):
        """Surviving options per task and whether anything was thinned.  Dominance compares the
        fp64 accuracies (both implementations must take that decision in the same precision)."""
        lo = [min(int(x) for x in self.lat[t]) for t in range(self.T)]
        up, down = {}, {}
        for t in self.order:
            up[t] = max([up[p] + lo[p] for p in self.preds[t]], default=0)
        for t in reversed(self.order):
            down[t] = max([down[s] + lo[s] for s in self.succs[t]], default=0)
        lists, truncated = [], False
        for t in range(self.T):
            opts = self.mix_options(D, slo_l, t)
            if cap:
                opts = [o for o in opts if self.q * (o["lat"] + up[t] + down[t]) <= slo_l]
                # skyline: walk by (cost, latency, -accuracy, id); an option survives if nothing
                # seen before it is at least as fast and at least as accurate
                opts.sort(key=lambda o: (o["cost"], o["lat"], -o["acc"], o["id"]))
                front = []
                for o in opts:
                    if not any(f["lat"] <= o["lat"] and f["acc"] >= o["acc"] for f in front):
                        front.append(o)
                if len(front) > cap:
                    truncated = True
                    # grid over latency and accuracy: isqrt(cap) latency bands of near-equal
                    # size, each thinned to cap // bands options evenly spaced by accuracy rank
                    import math
                    bands = math.isqrt(cap)
                    per = cap // bands
                    n = len(front)
                    front.sort(key=lambda o: (o["lat"], o["id"]))
                    groups = [[] for _ in range(bands)]
                    for r, o in enumerate(front):
                        groups[r * bands // n].append(o)
                    front = []
                    for grp in groups:
                        grp.sort(key=lambda o: (o["acc"], o["id"]))
                        if len(grp) <= per:
                            front += grp
                        else:
                            front += [grp[(j * (len(grp) - 1)) // (per - 1)] for j in range(per)]
                opts = sorted(front, key=lambda o: o["id"])
            lists.append(opts)
        return lists, truncated

    def search_mix(self, D: int, slo_l: int, slo_a: float, cap: int, max_space: int = 300000, objective=None):
        """Returns (best or None, K, truncated, margin); best = (idx, cost, lat, acc, options).
        objective = (alpha, beta): the largest alpha*A_obj - beta*cost wins instead of the lowest
        cost (then lower cost, then lower index), and a sixth field holds its exact value."""
        lists, truncated = self.mix_lists(D, slo_l, cap)
        K = [len(l) for l in lists]
        space = 1
        for k in K:
            space *= k
        if space > max_space:
            raise OverflowError(space)
        slo = Fraction(float(slo_a))
        capu = int(self.pb.capacity_units)
        best, margin = None, None
        if all(K):
            strides = [1] * self.T
            for t in range(1, self.T):
                strides[t] = strides[t - 1] * K[t - 1]
            for digits in itertools.product(*[range(k) for k in reversed(K)]):
                digits = digits[::-1]
                idx = sum(d * s for d, s in zip(digits, strides))
                opts = [lists[t][digits[t]] for t in range(self.T)]
                fin: Dict[int, int] = {}
                for t in self.order:
                    fin[t] = opts[t]["lat"] + max([fin[p] for p in self.preds[t]], default=0)
                lat = self.q * max(fin[s] for s in self.sinks)
                cost = sum(o["cost"] for o in opts)
                acc = self._acc_values([o["accF"] for o in opts]) / self.amax
                d = abs(acc - slo)
                margin = d if margin is None or d < margin else margin
                if lat <= slo_l and acc >= slo and (capu == 0 or cost <= capu):
                    if objective is None:
                        if best is None or (cost, idx) < (best[1], best[0]):
                            best = (idx, cost, lat, acc, opts)
                    else:
                        obj = Fraction(float(objective[0])) * acc - Fraction(float(objective[1])) * cost
                        if best is None or (-obj, cost, idx) < (-best[5], best[1], best[0]):
                            best = (idx, cost, lat, acc, opts, obj)
        return best, K, truncated, margin

    def search(self, D: int, slo_l: int, slo_a: float, cap: int):
        """Returns (best index or None, cost, latency, accuracy Fraction, K list,
        truncated, min |A - slo| seen)."""
        lists, truncated = self.lists(D, slo_l, cap)
        K = [len(l) for l in lists]
        best = None
        margin = None
        slo = Fraction(float(slo_a))
        capu = int(self.pb.capacity_units)
        if all(K):
            strides = [1] * self.T
            for t in range(1, self.T):
                strides[t] = strides[t - 1] * K[t - 1]
            for digits in itertools.product(*[range(k) for k in reversed(K)]):
                digits = digits[::-1]            # digits[t] for task t; task 0 fastest
                idx = sum(d * s for d, s in zip(digits, strides))
                choice = [lists[t][digits[t]] for t in range(self.T)]
                lat = self.latency(choice)
                cost = sum(self.rep_cost(D, t, choice[t])[1] for t in range(self.T))
                acc = self._acc([self.variant(c) for c in choice]) / self.amax
                d = abs(acc - slo)
                margin = d if margin is None or d < margin else margin
                ok = lat <= slo_l and acc >= slo and (capu == 0 or cost <= capu)
                if ok and (best is None or (cost, idx) < (best[1], best[0])):
                    best = (idx, cost, lat, acc, choice)
        return best, K, truncated, margin
