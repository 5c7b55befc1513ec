"""The paper's scheduling layer, written out plainly.  Test infrastructure only.

  expand()       T(G, rho): pointer matrix -> stages            (Sec. III-B Eqs. 3-6, Sec. III-C Eq. 8)
  issue_order()  order in which the main thread launches a stage (Sec. III-D, BFS vs DFS)
  coordinate_descent(), random_search()                          (Sec. III-C, Alg. 1)

Readings where the paper is silent:
  * A pointer is the 1-based index of the last operator of a stage, inclusive
    (Eq. 3: (3,5,7) over [1..10] gives [1,2,3],[4,5],[6,7],[8,9,10]); the last
    stage takes the remainder; 0 means "nothing yet"; equal neighbours give an
    empty slice, which Eq. 5 allows ("S3(None)").
  * Per-stage concurrency c: the tenants with a non-empty slice are ranked in
    tenant order; rank j runs on the stream of the tenant of rank j mod c, after
    the lower-ranked tenants mapped to the same stream.
  * Candidate rows of Alg. 1 are P draws, uniform on [0, len_i], sorted.  Random
    search draws every pointer independently and unsorted, and discards a matrix
    with a non-monotone row (the filtering of infeasible samples that Sec. IV-D mentions).
  * Random draws come from a counter-based generator so that an independent
    implementation can reproduce them: draw(seed, a, b, c, d) below.
"""
import math

M64 = (1 << 64) - 1


def mix64(z):
    z = (z + 0x9E3779B97F4A7C15) & M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M64
    return z ^ (z >> 31)


def draw(seed, a, b, c, d):
    h = mix64(seed & M64)
    for v in (a, b, c, d):
        h = mix64(h ^ (v & M64))
    return h


def validate(lens, rho):
    """rho: N rows of P pointers.  Returns None if valid, else a reason."""
    if len(rho) != len(lens):
        return "row count"
    for row, n in zip(rho, lens):
        prev = 0
        for v in row:
            if v < prev:
                return "non-monotone"
            if v > n:
                return "beyond sequence"
            prev = v
    return None


def expand(lens, rho):
    """T(G, rho): returns stages[s][i] = (begin, end), 0-based half-open slice of
    tenant i's operator list launched in stage s.  P pointers give P+1 stages."""
    assert validate(lens, rho) is None
    n_stages = (len(rho[0]) if rho else 0) + 1
    stages = []
    for s in range(n_stages):
        st = []
        for row, n in zip(rho, lens):
            begin = row[s - 1] if s > 0 else 0
            end = row[s] if s < n_stages - 1 else n
            st.append((begin, end))
        stages.append(st)
    return stages


def stream_map(stage, concurrency):
    """Host stream (a tenant index) of every tenant active in the stage: its own stream when there are enough
    streams (Sec. III-B, Eq. 2); otherwise streams 0 .. c-1, tenants taken longest slice first (ties: lower index),
    each to the stream carrying the fewest operators so far (ties: lowest stream)."""
    active = [i for i, (b, e) in enumerate(stage) if e > b]
    c = max(1, concurrency)
    if c >= len(active):
        return {t: t for t in active}
    size = {t: stage[t][1] - stage[t][0] for t in active}
    load = [0] * c
    out = {}
    for t in sorted(active, key=lambda t: (-size[t], t)):
        k = min(range(c), key=lambda k: (load[k], k))
        out[t] = k
        load[k] += size[t]
    return out


def issue_order(stage, concurrency, order="bfs"):
    """Launch sequence of one stage: list of (stream, tenant, op_index)."""
    smap = stream_map(stage, concurrency)
    queues = {}
    for t in sorted(smap):
        b, e = stage[t]
        queues.setdefault(smap[t], []).extend((t, i) for i in range(b, e))
    streams = sorted(queues)
    out = []
    if order == "dfs":
        for s in streams:
            out.extend((s, t, i) for t, i in queues[s])
        return out
    depth = 0
    while True:
        any_left = False
        for s in streams:
            if depth < len(queues[s]):
                t, i = queues[s][depth]
                out.append((s, t, i))
                any_left = True
        if not any_left:
            return out
        depth += 1


def even_split(lens, n_pointers):
    """Initial pointer matrix: stage boundaries at ceil(len * j / (P+1))."""
    return [[-(-n * (j + 1) // (n_pointers + 1)) for j in range(n_pointers)] for n in lens]


def sample_row(seed, rnd, model, cand, n_pointers, length):
    return sorted(draw(seed, rnd, model, cand, j) % (length + 1) for j in range(n_pointers))


def baseline_seeds(lens, n_pointers):
    """Extension to Alg. 1: matrices profiled and recorded before the search starts: everything in
    stage 1 (the stream-parallel baseline written as a pointer matrix) and the even split."""
    return [[[n] * n_pointers for n in lens], even_split(lens, n_pointers)]


def coordinate_descent(lens, n_pointers, rounds, n_cand, cost, seed, init=None, seed_baselines=False):
    """Alg. 1.  `cost(rho)` stands for the profiling step of the inner loop (the latency of the
    candidate schedule measured over several runs).
    Returns (best_rho, best_cost, records); records lists every evaluated
    (rho, cost) in evaluation order; the best is the earliest minimum."""
    rho = [list(r) for r in (init if init is not None else even_split(lens, n_pointers))]
    records = []
    if seed_baselines and n_pointers > 0:
        for m in baseline_seeds(lens, n_pointers):
            records.append((m, cost(m)))
    for r in range(rounds):
        for i in range(len(lens)):
            best_row, best_lat = None, None
            for m in range(n_cand):
                row = sample_row(seed, r, i, m, n_pointers, lens[i])
                cand = [list(x) for x in rho]
                cand[i] = row
                lat = cost(cand)
                records.append((cand, lat))
                if best_lat is None or lat < best_lat:
                    best_row, best_lat = row, lat
            rho[i] = best_row
    best = min(range(len(records)), key=lambda j: (records[j][1], j))
    return records[best][0], records[best][1], records


def random_search(lens, n_pointers, evaluations, cost, seed, seed_baselines=False):
    """Random search: whole matrices, independent unsorted draws, infeasible ones skipped."""
    records = []
    skipped = 0
    if seed_baselines and n_pointers > 0:
        for m in baseline_seeds(lens, n_pointers):
            records.append((m, cost(m)))
    for e in range(evaluations):
        rho = [[draw(seed, e, i, 0x52, j) % (lens[i] + 1) for j in range(n_pointers)]
               for i in range(len(lens))]
        if validate(lens, rho) is not None:
            skipped += 1
            continue
        records.append((rho, cost(rho)))
    if not records:
        return None, None, records, skipped
    best = min(range(len(records)), key=lambda j: (records[j][1], j))
    return records[best][0], records[best][1], records, skipped


def playoff(lens, n_pointers, records, top_k, final_cost):
    """Extension to Alg. 1 (its last step returns the best entry of the record memory as profiled once): the
    top_k distinct matrices of the record memory, lowest profiled cost first and earlier entry first on ties,
    followed by the matrix that puts every operator into stage 1 unless it is already among them, are measured
    again with `final_cost` (more runs); the lowest of these second measurements wins, the earlier candidate on
    ties.  Returns (rho, cost, candidates) with candidates = [(rho, final cost), ...] in evaluation order."""
    order = sorted(range(len(records)), key=lambda j: (records[j][1], j))
    cands = []
    for j in order:
        m = [list(r) for r in records[j][0]]
        if m not in cands:
            cands.append(m)
        if len(cands) >= max(1, top_k):
            break
    one_stage = [[n] * n_pointers for n in lens]
    if one_stage not in cands:
        cands.append(one_stage)
    scored = [(m, final_cost(m)) for m in cands]
    best = min(range(len(scored)), key=lambda j: (scored[j][1], j))
    return scored[best][0], scored[best][1], scored


def proportional_shares(weights, cu_count):
    """Extension: a disjoint start vector for the share descent.  Units are dealt out in eighths of cu_count;
    every tenant owns one eighth, the spare eighths follow the weights by largest remainder (lower index first
    on ties); with more than 8 tenants every share is one eighth."""
    n = len(weights)
    units = [1] * n
    spare = 8 - n
    total = 0.0
    for w in weights:
        total += float(w)
    if spare > 0 and total > 0:
        frac = []
        given = 0
        for i, w in enumerate(weights):
            quota = float(spare) * float(w) / total
            whole = int(math.floor(quota))
            units[i] += whole
            given += whole
            frac.append(quota - whole)
        while given < spare:
            pick = max(range(n), key=lambda i: (frac[i], -i))
            units[pick] += 1
            frac[pick] = -1.0
            given += 1
    elif spare > 0:
        for k in range(spare):
            units[k % n] += 1
    return [u * (cu_count // 8) for u in units]


def cu_share_descent(n_tenants, cu_count, rounds, cost, start_cost, start=None):
    """Extension: per-tenant CU share as one more coordinate.  Start with the given vector (default: all
    shares 0 = every unit); per round and tenant, try k * cu_count // 8 for k = 1..7 with the other shares
    fixed; a candidate replaces the tenant's share when its cost is lower than the best so far."""
    cur = list(start) if start is not None else [0] * n_tenants
    best = start_cost
    for _ in range(rounds):
        for i in range(n_tenants):
            for k in range(1, 8):
                cand = list(cur)
                cand[i] = k * cu_count // 8
                if cand[i] == cur[i]:
                    continue
                c = cost(cand)
                if c < best:
                    best, cur = c, cand
    return cur, best


def wave_priority_descent(n_tenants, rounds, cost, start_cost, start=None):
    """Extension: per-tenant wave priority as one more coordinate.  Start with the given vector (default: all 0);
    per round and tenant, try the values -1, 0, 1, 2, 3 other than the current one with the other entries fixed; a
    value replaces the tenant's entry when its cost is lower than the best so far; a round that changes nothing
    ends the search."""
    cur = list(start) if start is not None else [0] * n_tenants
    best = start_cost
    for _ in range(rounds):
        changed = False
        for i in range(n_tenants):
            for v in (-1, 0, 1, 2, 3):
                if v == cur[i]:
                    continue
                cand = list(cur)
                cand[i] = v
                c = cost(cand)
                if c < best:
                    best, cur, changed = c, cand, True
        if not changed:
            break
    return cur, best
