"""Independent checkers written from the problem's definition (Sec. III-C), in pure Python
integers.  They use no prefix sums, no tables and no recurrence, and import neither the
oracle nor the HIP path: they are what the oracle is pinned against, and what plan validity
is judged by at any size."""
from itertools import combinations

INF = (1 << 63) - 1


def cdiv(x, r):
    return -((-x) // r)


def stage_time(t, i, j, r, comm=None):
    """Time of the stage holding blocks i+1..j (1-based) at r replicas.  comm = (o, w): a stage
    that is followed by another one (j < N) also sends its replica's share of the o[j-1] bytes
    that cross the cut after block j, at w bytes per microsecond; times are nanoseconds."""
    h = cdiv(sum(int(x) for x in t[i:j]), r)
    if comm is not None and j < len(t):
        o, w = comm
        h += cdiv(1000 * int(o[j - 1]), r * int(w))
    return h


def stage_mem(p, a, i, j, r):
    return sum(int(x) for x in p[i:j]) + cdiv(sum(int(x) for x in a[i:j]), r)


def plan_value(t, p, a, M, bounds, reps, comm=None):
    """(feasible, max stage time) of the plan with stage ends bounds[1:] and replicas reps."""
    worst = 0
    for u in range(len(reps)):
        i, j, r = bounds[u], bounds[u + 1], reps[u]
        if stage_mem(p, a, i, j, r) > M:
            return False, INF
        worst = max(worst, stage_time(t, i, j, r, comm))
    return True, worst


def brute_force(t, p, a, D, S, M, comm=None):
    """Enumerate every plan: s stages, every set of s-1 cut points, every way to give the
    stages positive replica counts that sum to D.  Returns (opt, smallest s attaining it,
    number of feasible plans); opt = INF and s = 0 when nothing is feasible."""
    N = len(t)
    best, best_s, n_feasible = INF, 0, 0
    for s in range(1, min(S, N, D) + 1):
        for cuts in combinations(range(1, N), s - 1):
            bounds = (0,) + cuts + (N,)
            for dc in combinations(range(1, D), s - 1):
                dd = (0,) + dc + (D,)
                reps = [dd[u + 1] - dd[u] for u in range(s)]
                ok, v = plan_value(t, p, a, M, bounds, reps, comm)
                if ok:
                    n_feasible += 1
                    if v < best:
                        best, best_s = v, s
    return best, best_s, n_feasible


def brute_force_prefix(t, p, a, s, j, d, M, comm=None):
    """Best value over plans of exactly s stages covering blocks 1..j with exactly d devices."""
    best = INF
    if s > j or s > d:
        return best
    for cuts in combinations(range(1, j), s - 1):
        bounds = (0,) + cuts + (j,)
        for dc in combinations(range(1, d), s - 1):
            dd = (0,) + dc + (d,)
            reps = [dd[u + 1] - dd[u] for u in range(s)]
            ok, v = plan_value(t, p, a, M, bounds, reps, comm)
            if ok and v < best:
                best = v
    return best


def check_plan(t, p, a, D, S, M, opt, n_stages, stage_end, replicas, comm=None):
    """Validity of a reported plan, from the definition: contiguous cover of 1..N, replicas
    positive and summing to D, every stage fits, and the slowest stage equals opt."""
    N = len(t)
    if opt == INF:
        assert n_stages == 0
        assert all(int(x) == -1 for x in stage_end) and all(int(x) == -1 for x in replicas)
        return
    assert 1 <= n_stages <= min(S, N, D)
    se = [int(x) for x in stage_end[:n_stages]]
    rp = [int(x) for x in replicas[:n_stages]]
    assert all(int(x) == -1 for x in stage_end[n_stages:])
    assert all(int(x) == -1 for x in replicas[n_stages:])
    bounds = [0] + se
    assert all(bounds[u] < bounds[u + 1] for u in range(n_stages)) and bounds[-1] == N
    assert all(r >= 1 for r in rp) and sum(rp) == D
    ok, v = plan_value(t, p, a, M, bounds, rp, comm)
    assert ok, "a stage of the plan does not fit memory"
    assert v == opt, (v, opt)


def check_cells(t, p, a, D, M, V, arg_i, arg_d, comm=None):
    """Per-cell check of the value table and of the canonical argmin.

    For every cell (s, j, d), s >= 1: list the admissible candidates (i, d') in
    lexicographic order, each valued max(V[s-1][i][d'], stage time); the cell must hold their
    minimum and the FIRST candidate attaining it, or INF / (-1,-1) if there is none.
    Level 0 must be 0 at (0,0) and INF elsewhere."""
    n_levels, N = V.shape[0] - 1, V.shape[1] - 1
    for j in range(N + 1):
        for d in range(D + 1):
            assert int(V[0, j, d]) == (0 if (j == 0 and d == 0) else INF)
    for s in range(1, n_levels + 1):
        for j in range(N + 1):
            for d in range(D + 1):
                best, arg = INF, (-1, -1)
                for i in range(0, j):
                    for dp in range(0, d):
                        prev = int(V[s - 1, i, dp])
                        if prev == INF:
                            continue
                        r = d - dp
                        if stage_mem(p, a, i, j, r) > M:
                            continue
                        v = max(prev, stage_time(t, i, j, r, comm))
                        if v < best:
                            best, arg = v, (i, dp)
                assert int(V[s, j, d]) == best, (s, j, d)
                assert (int(arg_i[s, j, d]), int(arg_d[s, j, d])) == arg, (s, j, d)


def linear_partition(t, s):
    """Textbook problem: split the sequence into s non-empty contiguous parts so that the
    largest part sum is minimal; solved by bisection on the answer with a greedy count."""
    t = [int(x) for x in t]
    assert 1 <= s <= len(t)

    def parts_needed(limit):
        cnt, cur = 1, 0
        for x in t:
            if x > limit:
                return len(t) + 1
            if cur + x > limit:
                cnt, cur = cnt + 1, x
            else:
                cur += x
        return cnt

    lo, hi = max(t), sum(t)
    while lo < hi:
        mid = (lo + hi) // 2
        if parts_needed(mid) <= s:
            hi = mid
        else:
            lo = mid + 1
    return lo


# ---- split objective of Algorithm 1: largest forward time + largest backward time -------------
def plan_value_split(tf, tb, p, a, M, bounds, reps, comm=None):
    """(feasible, max forward stage time, max backward stage time) of a plan; the communication
    term, if any, belongs to the forward pass."""
    mf = mb = 0
    for u in range(len(reps)):
        i, j, r = bounds[u], bounds[u + 1], reps[u]
        if stage_mem(p, a, i, j, r) > M:
            return False, INF, INF
        mf = max(mf, stage_time(tf, i, j, r, comm))
        mb = max(mb, stage_time(tb, i, j, r))
    return True, mf, mb


def brute_force_prefix_split(tf, tb, p, a, s, j, d, M, comm=None):
    """Exact minimum of (max forward + max backward) over the plans of exactly s stages covering
    blocks 1..j with exactly d devices."""
    best = INF
    if s > j or s > d:
        return best
    for cuts in combinations(range(1, j), s - 1):
        bounds = (0,) + cuts + (j,)
        for dc in combinations(range(1, d), s - 1):
            dd = (0,) + dc + (d,)
            reps = [dd[u + 1] - dd[u] for u in range(s)]
            ok, mf, mb = plan_value_split(tf, tb, p, a, M, bounds, reps, comm)
            if ok and mf + mb < best:
                best = mf + mb
    return best


def walk_back(arg_i, arg_d, s, j, d):
    """Stage bounds and replica counts of the plan stored behind cell (s, j, d)."""
    ends, reps = [], []
    while s >= 1:
        i, dp = int(arg_i[s, j, d]), int(arg_d[s, j, d])
        assert 0 <= i < j and 0 <= dp < d
        ends.append(j)
        reps.append(d - dp)
        s, j, d = s - 1, i, dp
    assert (j, d) == (0, 0)
    return [0] + ends[::-1], reps[::-1]


def split_steps(tf, tb, p, a, D, M, n_levels, comm=None):
    """Algorithm 1's steps with the separate maxima, written out cell by cell in plain Python
    (a second, separately written run of the same steps: a cross-check against slips, not a pin)."""
    N = len(tf)
    cells = {(0, 0, 0): (0, 0, 0, -1, -1)}
    for s in range(1, n_levels + 1):
        for j in range(s, N + 1):
            for d in range(s, D + 1):
                best = None
                for i in range(s - 1, j):
                    for dp in range(s - 1, d):
                        prev = cells.get((s - 1, i, dp))
                        if prev is None:
                            continue
                        r = d - dp
                        if stage_mem(p, a, i, j, r) > M:
                            continue
                        f = max(prev[1], stage_time(tf, i, j, r, comm))
                        b = max(prev[2], stage_time(tb, i, j, r))
                        if best is None or f + b < best[0]:
                            best = (f + b, f, b, i, dp)
                if best is not None:
                    cells[(s, j, d)] = best
    return cells


# ---- compaction step of the block-level phase on a chain (Sec. III-B) ----------------------------
def compact_steps(t, p, a, k, M, max_passes=0):
    """The compaction procedure written out with Python lists of groups (a second, separately
    written run of the same steps).  Returns the ends of the resulting groups."""
    groups = [{"lo": g, "hi": g + 1, "t": int(t[g]), "m": int(p[g]) + int(a[g])} for g in range(len(t))]
    walks = 0
    while len(groups) > k and (max_passes <= 0 or walks < max_passes):
        walks += 1
        # the list of this walk: (lo, hi) names a group as it stood when listed
        listing = sorted(((gr["t"], gr["lo"], gr["hi"]) for gr in groups))
        before = len(groups)
        for _, lo, hi in listing:
            if len(groups) <= k:
                break
            pos = next((x for x, gr in enumerate(groups) if gr["lo"] == lo and gr["hi"] == hi), None)
            if pos is None:
                continue  # absorbed or grown since it was listed
            left = pos - 1 if pos > 0 else None
            right = pos + 1 if pos + 1 < len(groups) else None
            if left is None and right is None:
                break
            if left is None:
                w = right
            elif right is None:
                w = left
            else:
                w = right if groups[right]["t"] < groups[left]["t"] else left
            if groups[pos]["m"] + groups[w]["m"] > M:
                continue
            x, y = min(pos, w), max(pos, w)
            groups[x] = {"lo": groups[x]["lo"], "hi": groups[y]["hi"], "t": groups[x]["t"] + groups[y]["t"],
                         "m": groups[x]["m"] + groups[y]["m"]}
            del groups[y]
        if len(groups) == before:
            break
    return [gr["hi"] for gr in groups]
