"""CPU checker for the replication planner.  TEST INFRASTRUCTURE ONLY.

Pure-Python integers (exact, unbounded), one function per step, in the order the
paper takes them.  Shares no code with the library's planner; the library never
imports it.

Steps and where they come from:
  aggregate_load        Alg. 1, first statement: W_s = W summed over batches.
  expert_copies         Alg. 1's Placement "number of replicas assigned for each
                        expert": the paper names it and gives no rule; the reading
                        here is largest-quotient first (copy to the expert with the
                        largest load per copy), which minimises the largest
                        per-copy load.
  placement             Sec. 4.2.2 step 5: most-loaded expert copy onto the
                        least-loaded device with free capacity.
  est_max_rank_load     Alg. 1 inner loops: a copy of e carries floor(W/c_e);
                        a rank's load is the sum over the copies it holds.
  greedy_allocation     unit greedy on that cost model: repeatedly add the replica
                        with the largest reduction of the estimated maximum rank
                        load per byte until the budget is spent.
  mckp_allocation       Alg. 2, the paper's exact multiple-choice knapsack DP (used
                        as a checker for the greedy, and for the paper's objective).
  capacity_assignment   Alg. 3, interleaved per-layer per-rank expert capacity.
  make_plan             Sec. 4.2 workflow, steps 3-5, then per-layer reporting
                        (balancedness = average / maximum rank load, Sec. 3.1).
  replication_benefit   Alg. 1 in full: every profiling batch replayed under the
                        placement for each candidate replica count; per-layer mean
                        balancedness gain over placement-only.
  choose_replication_factor  Sec. 4.2.1 step 2: the R with the highest balancedness
                        gain per replica (parity unpinned: the paper gives no rule,
                        the tests pin this reading only).
  make_plan_paper       the paper's own pipeline: Alg. 1 -> (R) -> Alg. 2 -> Alg. 3 ->
                        placement.
  plan_diff             Sec. 4.3 step 3: the weights a rank must fetch or may drop when
                        one plan replaces another.
  make_plan_uniform     the comparison plans of Sec. 5: placement only (n = 0) and the
                        same number of replicas in every layer (n = D is the uniform
                        replication baseline).
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence, Tuple


def aggregate_load(W: Sequence[Sequence[Sequence[int]]]) -> List[List[int]]:
    """W[b][l][e] -> W_s[l][e]."""
    B = len(W)
    L = len(W[0])
    E = len(W[0][0])
    return [[sum(int(W[b][l][e]) for b in range(B)) for e in range(E)] for l in range(L)]


def expert_copies(ws: Sequence[int], n: int, D: int) -> List[int]:
    """Copies per expert after handing out n replicas one at a time, each to the
    expert with the largest load per current copy (exact rational comparison,
    lowest expert id on ties); an expert never gets more copies than ranks."""
    E = len(ws)
    c = [1] * E
    for _ in range(n):
        best = -1
        for e in range(E):
            if c[e] >= D:
                continue
            if best < 0 or ws[e] * c[best] > ws[best] * c[e]:
                best = e
        if best < 0:
            raise ValueError("more replicas than E*(D-1)")
        c[best] += 1
    return c


def canonical_capacities(total: int, D: int) -> List[int]:
    """floor(total/D) everywhere, one more on the lowest-numbered total mod D ranks."""
    return [total // D + (1 if g < total % D else 0) for g in range(D)]


def placement(ws: Sequence[int], copies: Sequence[int], cap: Sequence[int]
              ) -> Tuple[List[List[Tuple[int, int]]], List[int]]:
    """Greedy placement of expert copies on ranks under per-rank capacities.

    Items are all copies; copy q of expert e weighs floor(ws[e] / copies[e]).
    Items are taken heaviest first (ties: lower expert, then lower copy).  Each goes
    to the rank that still has room and does not yet hold a copy of the same expert,
    with the smallest load so far (ties: more room left, then lower rank id).  If
    every rank with room already holds that expert, the distinct-rank wish is
    dropped for this item.  Returns (held[g] = list of (e, q), load[g]).
    """
    D = len(cap)
    E = len(ws)
    if sum(cap) != sum(copies):
        raise ValueError("capacities do not add up to the number of copies")
    items = [(ws[e] // copies[e], e, q) for e in range(E) for q in range(copies[e])]
    items.sort(key=lambda it: (-it[0], it[1], it[2]))
    room = list(cap)
    load = [0] * D
    held: List[List[Tuple[int, int]]] = [[] for _ in range(D)]
    has = [set() for _ in range(D)]
    for wgt, e, q in items:
        def pick(distinct: bool) -> int:
            best = -1
            for g in range(D):
                if room[g] <= 0 or (distinct and e in has[g]):
                    continue
                if best < 0 or (load[g], -room[g]) < (load[best], -room[best]):
                    best = g
            return best
        g = pick(True)
        if g < 0:
            g = pick(False)
        held[g].append((e, q))
        has[g].add(e)
        load[g] += wgt
        room[g] -= 1
    return held, load


def est_max_rank_load(ws: Sequence[int], n: int, D: int) -> int:
    """M(n): estimated maximum rank load of a layer given n replicas."""
    E = len(ws)
    c = expert_copies(ws, n, D)
    _, load = placement(ws, c, canonical_capacities(E + n, D))
    return max(load)


def greedy_allocation(Ws: Sequence[Sequence[int]], D: int,
                      bytes_per_replica: Optional[Sequence[int]], budget: int
                      ) -> Tuple[List[int], List[Tuple[int, int]]]:
    """Replicas per layer under a byte budget, one replica at a time.

    Each step looks at the layers whose next replica still fits the budget and
    whose experts are not all at D copies, and picks the one with the largest
    M(x) - M(x+1) per byte (compared exactly; ties: larger current M, then lower
    layer).  Steps with no gain are still taken, so the budget is always spent.
    Returns (x, order) where order lists (layer, spent_after) per step.
    """
    L = len(Ws)
    E = len(Ws[0])
    by = [1] * L if bytes_per_replica is None else [int(b) for b in bytes_per_replica]
    if any(b <= 0 for b in by):
        raise ValueError("bytes_per_replica must be positive")
    x = [0] * L
    cur = [est_max_rank_load(Ws[l], 0, D) for l in range(L)]
    nxt: List[Optional[int]] = [None] * L
    spent = 0
    order: List[Tuple[int, int]] = []
    while True:
        best = -1
        for l in range(L):
            if spent + by[l] > budget or x[l] >= E * (D - 1):
                continue
            if nxt[l] is None:
                nxt[l] = est_max_rank_load(Ws[l], x[l] + 1, D)
            if best < 0:
                best = l
                continue
            dl, db = cur[l] - nxt[l], cur[best] - nxt[best]
            lhs, rhs = dl * by[best], db * by[l]
            if lhs > rhs or (lhs == rhs and cur[l] > cur[best]):
                best = l
        if best < 0:
            break
        x[best] += 1
        spent += by[best]
        cur[best] = nxt[best]
        nxt[best] = None
        order.append((best, spent))
    return x, order


def mckp_allocation(Tmap: Dict[int, Sequence[float]], C: int) -> List[int]:
    """Alg. 2: every layer takes one replica count, 0 or one of the counts Alg. 1 scored, the
    counts add up to exactly C, and the summed gain is as large as possible.  Returns the count
    per layer, or raises when no selection adds up to C.

    One pass over the layers keeps, for every total c, the best summed gain the layers seen so
    far can reach with exactly c replicas (None: unreachable), and remembers per layer which
    count it took to get there.  A layer's options are tried as 0 first, then the scored counts
    from the smallest up, and an option only displaces the one before it when strictly better:
    equal gains keep fewer replicas.  The answer is read back from the last layer to the first.
    """
    counts = sorted(Tmap)
    L = len(Tmap[counts[0]])
    reach: List[Optional[float]] = [None] * (C + 1)      # reach[c]: best gain at total c so far
    reach[0] = 0.0
    took: List[List[int]] = []                           # took[l][c]: layer l's count in that best
    for l in range(L):
        after = list(reach)                              # this layer takes nothing
        mine = [0] * (C + 1)
        for r in counts:
            gain = Tmap[r][l]
            for c in range(r, C + 1):
                if reach[c - r] is None:
                    continue
                v = reach[c - r] + gain
                if after[c] is None or v > after[c]:
                    after[c], mine[c] = v, r
        took.append(mine)
        reach = after
    if reach[C] is None:
        raise ValueError("no selection of replica counts sums to C")
    x = [0] * L
    left = C
    for l in range(L - 1, -1, -1):
        x[l] = took[l][left]
        left -= x[l]
    return x


def interleave_select(idx: Sequence[int], k: int) -> List[int]:
    """k entries of idx, evenly spread: positions floor(i * len / k), i = 0..k-1.

    This is the spacing of the paper's worked example (Sec. 4.2.2: four tied
    devices, two extras -> devices 0 and 2), which the example fixes more firmly
    than the one-line description of the helper in Alg. 3."""
    n = len(idx)
    return [idx[(i * n) // k] for i in range(k)]


def capacity_assignment(D: int, R: Sequence[int]) -> List[List[int]]:
    """Alg. 3.  R[l] = physical experts (base + replicas) of layer l.
    Returns A[l][g] = experts held by rank g in layer l.

    Every rank holds floor(R[l] / D) experts of layer l; the R[l] mod D experts left over go
    one each to the ranks that have collected the fewest such extras in the layers before
    (the floors are the same for all ranks, so only the extras tell ranks apart).  Ranks are
    taken in order of extras so far; the last level that only partly fits is a tie, and there
    the takers are spread evenly over the tied ranks in rank order (interleave_select)."""
    extras = [0] * D
    A: List[List[int]] = []
    for total in R:
        row = [total // D] * D
        need = total % D
        if need:
            by_fill = sorted(range(D), key=lambda g: (extras[g], g))
            level = extras[by_fill[need - 1]]            # fill of the last rank that still gets one
            below = [g for g in by_fill if extras[g] < level]
            tied = [g for g in by_fill if extras[g] == level]
            for g in below + interleave_select(tied, need - len(below)):
                row[g] += 1
                extras[g] += 1
        A.append(row)
    return A


def layer_tables(held: Sequence[Sequence[Tuple[int, int]]]) -> Tuple[List[int], List[int]]:
    """Slot numbering of one layer: rank-major, within a rank by (expert, copy).
    Returns (slot_expert[S], rank_slot_off[D+1])."""
    slot_expert: List[int] = []
    off = [0]
    for g in range(len(held)):
        for e, _q in sorted(held[g]):
            slot_expert.append(e)
        off.append(len(slot_expert))
    return slot_expert, off


def make_plan(W, D: int, bytes_per_replica: Optional[Sequence[int]], budget: int) -> dict:
    """The whole planner.  W[b][l][e] integer loads."""
    Ws = aggregate_load(W)
    L, E = len(Ws), len(Ws[0])
    x, order = greedy_allocation(Ws, D, bytes_per_replica, budget)
    A = capacity_assignment(D, [E + x[l] for l in range(L)])
    layers = []
    for l in range(L):
        c = expert_copies(Ws[l], x[l], D)
        held, load = placement(Ws[l], c, A[l])
        slot_expert, off = layer_tables(held)
        mx = max(load)
        bal = 1.0 if mx == 0 else (sum(load) / D) / mx
        layers.append(dict(n_replicas=x[l], copies=c, slot_expert=slot_expert,
                           rank_slot_off=off, capacity=A[l], rank_load=load,
                           est_max_rank_load=mx, est_balancedness=bal))
    total = sum(x)
    return dict(L=L, E=E, D=D, x=x, order=order, layers=layers, total_replicas=total,
                replication_factor=total / D,
                memory_saving_vs_uniform=(L * D / total) if total else float("inf"))


def geometric_counts(D: int, E: int) -> List[int]:
    """Sec. 4.2.1 step 1: the candidate replica counts 1, 2, 4, ... up to D (and never
    more than a layer can take: every expert on every rank, E * (D - 1) replicas)."""
    out, r = [], 1
    while r <= D and r <= E * (D - 1):
        out.append(r)
        r *= 2
    return out


def replication_benefit(W, D: int, counts: Optional[Sequence[int]] = None
                        ) -> Tuple[List[int], List[float], Dict[int, List[float]]]:
    """Alg. 1.  W[b][l][e] integer loads.  Returns (counts, base[l], T[r][l]).

    For r = 0 and every candidate count r the layer is placed once on the loads
    summed over batches (r replicas by expert_copies, capacities floor/ceil of
    (E + r) / D with the extras on the lowest ranks, greedy placement).  Every batch
    is then replayed under that placement: each copy of expert e carries
    floor(W[b][l][e] / copies[e]) on the rank that holds it, and the batch scores
    (average rank load) / (maximum rank load); a batch that sends nothing to the
    layer scores 1.  base[l] is the mean score over batches at r = 0 and
    T[r][l] the mean score at r minus base[l].  (The listing's single `base` is read
    per layer: it is assigned from BAL[l].)  Arithmetic: integer loads; one double
    division of the load sum by D, one by the maximum, a running double sum over
    batches in order, one division by B, one subtraction.
    """
    Ws = aggregate_load(W)
    B, L, E = len(W), len(Ws), len(Ws[0])
    counts = geometric_counts(D, E) if counts is None else [int(r) for r in counts]
    base = [0.0] * L
    T: Dict[int, List[float]] = {}
    for r in [0] + list(counts):
        mean = [0.0] * L
        for l in range(L):
            c = expert_copies(Ws[l], r, D)
            held, _ = placement(Ws[l], c, canonical_capacities(E + r, D))
            bal = 0.0
            for b in range(B):
                G = [0] * D
                for g in range(D):
                    for e, _q in held[g]:
                        G[g] += int(W[b][l][e]) // c[e]
                mx = max(G)
                bal += 1.0 if mx == 0 else (sum(G) / D) / mx
            mean[l] = bal / B
        if r == 0:
            base = mean
        else:
            T[r] = [mean[l] - base[l] for l in range(L)]
    return list(counts), base, T


def mckp_table(Tmap: Dict[int, Sequence[float]], C: int):
    """The value table of Alg. 2 for every capacity 0..C at once: best[c] = the maximum
    total gain of a selection that sums to exactly c (None when no selection does)."""
    keys = sorted(Tmap.keys())
    L = len(Tmap[keys[0]])
    prev: List[Optional[float]] = [None] * (C + 1)
    prev[0] = 0.0
    for l in range(1, L + 1):
        cur: List[Optional[float]] = [None] * (C + 1)
        for c in range(C + 1):
            cur[c] = prev[c]
            for r in keys:
                if c >= r and prev[c - r] is not None:
                    cand = prev[c - r] + Tmap[r][l - 1]
                    if cur[c] is None or cand > cur[c]:
                        cur[c] = cand
        prev = cur
    return prev


def choose_replication_factor(Tmap: Dict[int, Sequence[float]], D: int, R_max: int) -> int:
    """Sec. 4.2.1 step 2, automatic mode: the replication factor R in 1..R_max whose best
    allocation of R * D replicas has the highest total gain per replica (exact-sum
    allocations as in Alg. 2; an R no selection sums to is skipped; ties keep the
    smaller R).  Returns 0 when no R in range is reachable.
    Parity unpinned against the paper, which does not give the rule: the tests pin this
    reading of the sentence by brute force over all allocations, not the paper's choice."""
    best_tab = mckp_table(Tmap, R_max * D)
    best_R, best_v = 0, 0.0
    for R in range(1, R_max + 1):
        v = best_tab[R * D]
        if v is None:
            continue
        per = v / (R * D)
        if best_R == 0 or per > best_v:
            best_R, best_v = R, per
    return best_R


def _finish_plan(Ws, D: int, x: Sequence[int], extra: dict) -> dict:
    L, E = len(Ws), len(Ws[0])
    A = capacity_assignment(D, [E + x[l] for l in range(L)])
    layers = []
    for l in range(L):
        c = expert_copies(Ws[l], x[l], D)
        held, load = placement(Ws[l], c, A[l])
        slot_expert, off = layer_tables(held)
        mx = max(load)
        bal = 1.0 if mx == 0 else (sum(load) / D) / mx
        layers.append(dict(n_replicas=x[l], copies=c, slot_expert=slot_expert,
                           rank_slot_off=off, capacity=A[l], rank_load=load,
                           est_max_rank_load=mx, est_balancedness=bal))
    total = sum(x)
    out = dict(L=L, E=E, D=D, x=list(x), order=[], layers=layers, total_replicas=total,
               replication_factor=total / D,
               memory_saving_vs_uniform=(L * D / total) if total else float("inf"))
    out.update(extra)
    return out


def make_plan_paper(W, D: int, budget_replicas: int, auto_R: bool = False) -> dict:
    """The paper's pipeline (Sec. 4.2.1): benefit matrix by Alg. 1, the replica total
    (given, or R * D with R from choose_replication_factor, R * D <= budget), the
    per-layer counts by Alg. 2, then Alg. 3 and the greedy placement.

    Alg. 2 needs a selection that sums to the total exactly; when none does (a total
    no combination of 0, 1, 2, 4, .. per layer reaches) the largest reachable total
    below it is used."""
    Ws = aggregate_load(W)
    L = len(Ws)
    counts, base, T = replication_benefit(W, D)
    if not counts:                       # a single rank: nothing to replicate onto
        return _finish_plan(Ws, D, [0] * L, dict(benefit_counts=[], benefit_base=base,
                                                 benefit={}, total_gain=0.0))
    cap = min(int(budget_replicas), L * max(counts))
    if auto_R:
        R = choose_replication_factor(T, D, cap // D)
        cap = R * D
    tab = mckp_table(T, cap)
    while tab[cap] is None:
        cap -= 1
    x = mckp_allocation(T, cap) if cap > 0 else [0] * L
    return _finish_plan(Ws, D, x, dict(benefit_counts=counts, benefit_base=base, benefit=T,
                                       total_gain=tab[cap]))


def make_plan_uniform(W, D: int, n: int) -> dict:
    """Comparison plans (Sec. 5 setups): n = 0 is placement only, n = D the uniform
    replication baseline (one replica per layer per rank); every layer gets n."""
    Ws = aggregate_load(W)
    return _finish_plan(Ws, D, [int(n)] * len(Ws), {})


def plan_diff(old_layer: dict, new_layer: dict, g: int) -> Tuple[List[int], int, int]:
    """Sec. 4.3 step 3 for one rank of one layer: which of its new slots keep weights the
    rank already holds.  Plain multiset matching: every old slot can be reused once, by a new
    slot of the same expert; equal experts pair up in slot order.  Returns (reuse[new local
    slot] = old local slot or -1, slots to fetch, old slots dropped)."""
    old = old_layer["slot_expert"][old_layer["rank_slot_off"][g]:old_layer["rank_slot_off"][g + 1]]
    new = new_layer["slot_expert"][new_layer["rank_slot_off"][g]:new_layer["rank_slot_off"][g + 1]]
    used = [False] * len(old)
    reuse = []
    for e in new:
        hit = -1
        for i, oe in enumerate(old):
            if oe == e and not used[i]:
                hit = i
                break
        if hit >= 0:
            used[hit] = True
        reuse.append(hit)
    return reuse, sum(1 for r in reuse if r < 0), used.count(False)


def realized_rank_rows(slot_cnt: Sequence[int], rank_slot_off: Sequence[int]) -> List[int]:
    """Rows each rank executes for a dispatched batch (sum of its slots' counts)."""
    return [sum(slot_cnt[rank_slot_off[g]:rank_slot_off[g + 1]])
            for g in range(len(rank_slot_off) - 1)]


def heaviest_rank(rows: Sequence[int]) -> int:
    """The rank with the most rows; the lowest-numbered one on ties."""
    best = 0
    for g in range(1, len(rows)):
        if rows[g] > rows[best]:
            best = g
    return best
