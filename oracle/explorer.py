"""Plain Python restatement of the paper's fusion exploration (Section 5), TEST INFRASTRUCTURE ONLY.

Only tests may import this module; the product never does.  It shares no code with the library: the
graph structure comes from the workload descriptor, and the two things the search cannot know by
itself -- the score of a pattern and whether a kernel can run it -- are passed in as a callback.

What the paper fixes, and how it is read here (each reading is listed in the design notes):
  * Section 5.2: vertices are visited from the last to the first; the candidate patterns of a vertex
    are built from the candidate patterns of its consumers (PatternReduction).  Consumers are taken in
    groups of at most two; inside a group every combination of "one candidate pattern of the consumer,
    the consumer alone, or nothing" is joined with the vertex; larger consumer lists are halved
    recursively and the halves' results are pooled (the paper's text) and, beyond the text, also
    joined pairwise, since a vertex with three consumers could otherwise never share a pattern with
    consumers from both halves.  Only the top-k patterns by score are kept (k = 3).
  * Section 5.2: patterns with a cyclic dependence, and patterns the code generator cannot process,
    are discarded.  A pattern that no kernel runs *yet* is kept as "tentative" (with the score it
    would have at streaming rate) so that it can grow into one a kernel family covers; tentative
    patterns never enter a plan and are not grown across a graph output.
  * Section 5.3: beam search of width 3 over the vertices from producers to consumers, appending a
    vertex's candidate patterns to every kept plan they do not overlap, ranking by accumulated score plus a
    look-ahead over the ops not visited yet (best score per op of any candidate holding the op); at the last
    vertex this is the paper's ranking by accumulated score.
  * Section 5.2, remote fusion: patterns of the plan that no edge joins are merged greedily when their union
    is runnable and gains over running them apart (`remote_fusion`).
  * Seeds: everything downstream of a vertex, the same stopped at graph outputs, and the connected component a
    vertex starts are offered as candidates too and escape the top-k cut (a kernel family can be runnable as a
    whole while parts of it are not, and the cut favours ever larger patterns).

Four of these go beyond the paper's text: the pairwise joining of the halves' candidates, the tentative patterns,
the look-ahead in the beam's ranking and the seeds.  `explore` takes a switch for each (tentative patterns arise
only when the score callback reports "unsupported"), and with all of them off it is the procedure of Section 5.2 /
5.3 alone.

Pins (tests/test_explorer_pins.py, fixtures tests/golden/explorer_*.txt: tiny graphs with hand-written score
tables, every expected value derived by hand in the fixture's comments):
  explore           candidate patterns per vertex and the beam's plans on a chain, a diamond, a vertex with three
                    consumers and the cyclic-dependence triangle of Section 5.2, additions off; the three-consumer
                    case also with the halves joined
  plan_is_acyclic   the cyclic pattern of the triangle / diamond; two patterns that wait for each other
  remote_fusion     two independent chains and a lone op (hand gains), and a merge that a cycle forbids
  brute_force_best  hand-enumerated optimum on each fixture
"""
from __future__ import annotations

from typing import Callable, Dict, List, Optional, Sequence, Tuple

Ops = Tuple[int, ...]
# score(ops) -> (status, f, f_optimistic): status 0 = runnable; "unsupported" = convex but no kernel;
# anything else = not a pattern (cyclic dependence, dtype boundary)
ScoreFn = Callable[[Ops], Tuple[object, Optional[float], float]]


class GraphView:
    """Op-level structure of a workload descriptor: who reads whose result."""

    def __init__(self, spec):
        self.n = len(spec.ops)
        producer = {op.out: i for i, op in enumerate(spec.ops)}
        outputs = {name for name, _ in spec.outputs}
        self.consumers: List[List[int]] = [[] for _ in range(self.n)]
        self.producers: List[List[int]] = [[] for _ in range(self.n)]
        readers: Dict[str, List[int]] = {}
        for i, op in enumerate(spec.ops):
            for name in op.inputs:
                readers.setdefault(name, []).append(i)
                if name in producer:
                    j = producer[name]
                    if i not in self.consumers[j]:
                        self.consumers[j].append(i)
                    if j not in self.producers[i]:
                        self.producers[i].append(j)
        for c in self.consumers:
            c.sort()
        # ops that share an operand (a graph input or an intermediate) are neighbours as well
        self.sharing: List[List[int]] = [[] for _ in range(self.n)]
        for i, op in enumerate(spec.ops):
            for name in op.inputs:
                self.sharing[i].extend(readers[name])
        self.is_output = [op.out in outputs for op in spec.ops]
        # ops that wait for an op's result through a computation outside the graph (Section 1: compute-intensive ops
        # are not fused): they run after it, and never in the same kernel
        self.waiting: List[List[int]] = [[] for _ in range(self.n)]
        for src, dst in getattr(spec, "external", ()):
            for i in readers.get(dst, []):
                if i not in self.waiting[producer[src]]:
                    self.waiting[producer[src]].append(i)
        # desc: everything that reads an op's result, directly or not (what a pattern grown from the op may hold)
        # after: the same plus what waits for it through external computations (what decides the order of execution)
        self.desc: List[set] = [set() for _ in range(self.n)]
        self.after: List[set] = [set() for _ in range(self.n)]
        for i in range(self.n - 1, -1, -1):
            for c in self.consumers[i]:
                self.desc[i].add(c)
                self.desc[i] |= self.desc[c]
                self.after[i].add(c)
                self.after[i] |= self.after[c]
            for c in self.waiting[i]:
                self.after[i].add(c)
                self.after[i] |= self.after[c]


def plan_is_acyclic(view: GraphView, groups: Sequence[Sequence[int]]) -> bool:
    """Section 5.2's "no cyclic dependence", for a whole plan: the graph whose vertices are the plan's patterns (and
    the ops outside them, one each) must have a topological order.  Patterns that are convex one by one can still wait
    for each other: {a, d} and {b, c} with edges a -> b and c -> d."""
    gid = {}
    for k, p in enumerate(groups):
        for o in p:
            gid[o] = k
    for o in range(view.n):
        gid.setdefault(o, len(groups) + o)
    succ: Dict[int, set] = {}
    waiting: Dict[int, int] = {k: 0 for k in set(gid.values())}
    for o in range(view.n):
        for c in list(view.consumers[o]) + list(view.waiting[o]):
            if gid[c] != gid[o] and gid[c] not in succ.setdefault(gid[o], set()):
                succ[gid[o]].add(gid[c])
                waiting[gid[c]] += 1
    ready = [k for k, w in waiting.items() if w == 0]
    done = 0
    while ready:
        k = ready.pop()
        done += 1
        for c in succ.get(k, ()):
            waiting[c] -= 1
            if waiting[c] == 0:
                ready.append(c)
    return done == len(waiting)


class Pat:
    __slots__ = ("ops", "f", "tentative")

    def __init__(self, ops: Ops, f: float, tentative: bool):
        self.ops, self.f, self.tentative = ops, f, tentative


def _key(p: Pat):
    return (-p.f, p.ops)


def explore(view: GraphView, score: ScoreFn, top_k: int = 3, beam_width: int = 3, max_tentative_ops: int = 24,
            join_halves: bool = True, seeds: bool = True, lookahead: bool = True):
    """Returns (candidate patterns per vertex, the beam's plans as [(patterns, accumulated score)]).
    join_halves / seeds / lookahead switch the additions to Section 5.2 / 5.3 described in the module header."""
    n = view.n

    def reads_own_output(ops: Ops) -> bool:
        s = set(ops)
        return any(view.is_output[o] and any(c in s for c in view.consumers[o]) for o in ops)

    def consider(ops: Ops, out: List[Pat]) -> None:
        if not plan_is_acyclic(view, [ops]):   # Section 5.2: fusing these ops creates a cyclic dependence
            return
        status, f, f_opt = score(ops)
        if status == 0:
            if f > 0:
                out.append(Pat(ops, f, False))
        elif status == "unsupported" and f_opt > 0 and len(ops) <= max_tentative_ops and not reads_own_output(ops):
            out.append(Pat(ops, f_opt, True))

    def keep_top(v: List[Pat]) -> List[Pat]:
        v = sorted(v, key=_key)
        uniq: List[Pat] = []
        for p in v:
            if not uniq or uniq[-1].ops != p.ops:
                uniq.append(p)
        kept, n_real, n_tent = [], 0, 0
        for p in uniq:
            if p.tentative and n_tent < top_k:
                kept.append(p)
                n_tent += 1
            elif not p.tentative and n_real < top_k:
                kept.append(p)
                n_real += 1
        return kept

    cand: List[List[Pat]] = [[] for _ in range(n)]

    def unite(a: Sequence[int], b: Sequence[int]) -> Ops:
        return tuple(sorted(set(a) | set(b)))

    def reduce_group(v: int, group: List[int]) -> List[Pat]:
        out: List[Pat] = []
        if len(group) <= 2:
            choices = [[(), (c,)] + [p.ops for p in cand[c]] for c in group]
            combos = [[]]
            for ch in choices:
                combos = [prev + [x] for prev in combos for x in ch]
            for combo in combos:
                if all(len(x) == 0 for x in combo):
                    continue
                u: Ops = (v,)
                for x in combo:
                    u = unite(u, x)
                consider(u, out)
            return keep_top(out)
        half = len(group) // 2
        a = reduce_group(v, group[:half])
        b = reduce_group(v, group[half:])
        out = a + b
        if join_halves:
            for x in a:
                for y in b:
                    consider(unite(x.ops, y.ops), out)
        return keep_top(out)

    for v in range(n - 1, -1, -1):
        if view.consumers[v]:
            cand[v] = reduce_group(v, view.consumers[v])

    # seeds: the downstream cone of every vertex, and the connected component a vertex starts
    comp = [-1] * n
    for v in range(n):
        if comp[v] >= 0:
            continue
        comp[v] = v
        stack = [v]
        while stack:
            o = stack.pop()
            for x in view.consumers[o] + view.producers[o] + view.sharing[o]:
                if comp[x] < 0:
                    comp[x] = v
                    stack.append(x)
    for v in range(n if seeds else 0):
        seed_pats: List[Pat] = []
        cone = tuple([v] + sorted(x for x in view.desc[v]))
        if len(cone) > 1:
            consider(cone, seed_pats)
        # the same cone, not continued past a graph output
        inside = {v}
        for x in range(v, n):
            if x in inside and not view.is_output[x]:
                inside.update(view.consumers[x])
        bounded = tuple(sorted(inside))
        if len(bounded) > 1 and bounded != cone:
            consider(bounded, seed_pats)
        if comp[v] == v:
            whole = tuple(x for x in range(n) if comp[x] == v)
            if len(whole) > 1 and whole != cone and whole != bounded:
                consider(whole, seed_pats)
        # seeds escape the top-k cut
        for sd in seed_pats:
            if all(p.ops != sd.ops for p in cand[v]):
                cand[v].append(sd)
        cand[v].sort(key=_key)

    # beam search from producers to consumers; plans are ranked by accumulated score plus a look-ahead: every op
    # not visited yet and still uncovered counts with the best score per op of any candidate that holds it
    per_op = [0.0] * n
    for v in range(n):
        for p in cand[v]:
            if not p.tentative:
                share = p.f / len(p.ops)
                for o in p.ops:
                    per_op[o] = max(per_op[o], share)

    def rank(covered, f, v):
        r = f
        for u in range(v + 1, n if lookahead else 0):
            if u not in covered:
                r += per_op[u]
        return r

    sets: List[Tuple[List[Ops], frozenset, float]] = [([], frozenset(), 0.0)]
    for v in range(n):
        nxt = list(sets)
        for patterns, covered, f in sets:
            for p in cand[v]:
                if p.tentative or any(o in covered for o in p.ops):
                    continue
                if not plan_is_acyclic(view, patterns + [p.ops]):
                    continue
                nxt.append((patterns + [p.ops], covered | frozenset(p.ops), f + p.f))
        nxt.sort(key=lambda s: (-rank(s[1], s[2], v), s[0]))
        sets = nxt[:beam_width]
    return cand, [(patterns, f) for patterns, _, f in sets]


def remote_fusion(patterns: List[Ops], n_ops: int, score: ScoreFn, view: Optional[GraphView] = None) -> Tuple[List[Ops], float]:
    """Section 5.2, remote fusion, read greedily: of all pairs of the plan's patterns (ops left alone count as
    patterns of one) whose union is runnable and leaves the plan free of cyclic dependences (checked when `view`
    is given), merge the pair that gains the most; repeat until none gains.
    Returns (all groups of the plan after merging, total gain)."""
    covered = {o for p in patterns for o in p}
    groups = sorted([tuple(p) for p in patterns] + [(o,) for o in range(n_ops) if o not in covered])
    if len(groups) > 64:
        return groups, 0.0

    def f_of(p: Ops) -> float:
        return score(p)[1] if len(p) > 1 else 0.0

    total = 0.0
    while True:
        best_gain, pair = 0.0, None
        for i in range(len(groups)):
            for j in range(i + 1, len(groups)):
                u = tuple(sorted(set(groups[i]) | set(groups[j])))
                status, f, _ = score(u)
                if status != 0:
                    continue
                gain = f - f_of(groups[i]) - f_of(groups[j])
                if gain > best_gain:
                    merged = [g for k, g in enumerate(groups) if k not in (i, j)] + [u]
                    if view is not None and not plan_is_acyclic(view, merged):
                        continue
                    best_gain, pair = gain, (i, j)
        if pair is None:
            break
        i, j = pair
        u = tuple(sorted(set(groups[i]) | set(groups[j])))
        del groups[j]
        groups[i] = u
        groups.sort()
        total += best_gain
    return groups, total


def brute_force_best(view: GraphView, score: ScoreFn, max_ops: int = 10) -> float:
    """Largest total score over ALL ways of cutting a tiny graph into runnable patterns (exhaustive)."""
    n = view.n
    assert n <= max_ops, "exhaustive search is for tiny graphs only"
    best = 0.0
    cache: Dict[Ops, Optional[float]] = {}

    def f_of(ops: Ops) -> Optional[float]:
        if ops not in cache:
            if len(ops) == 1:
                cache[ops] = 0.0
            else:
                status, f, _ = score(ops)
                cache[ops] = f if status == 0 else None
        return cache[ops]

    blocks: List[Ops] = []

    def rec(remaining: Tuple[int, ...], total: float) -> None:
        nonlocal best
        if not remaining:
            if plan_is_acyclic(view, blocks):
                best = max(best, total)
            return
        first, rest = remaining[0], remaining[1:]
        # the block that holds `first`: first plus any subset of the rest
        for mask in range(1 << len(rest)):
            block = (first,) + tuple(rest[i] for i in range(len(rest)) if (mask >> i) & 1)
            f = f_of(block)
            if f is None:
                continue
            blocks.append(block)
            rec(tuple(x for x in rest if x not in block), total + f)
            blocks.pop()

    rec(tuple(range(n)), 0.0)
    return best
