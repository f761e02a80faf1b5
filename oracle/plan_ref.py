"""Reference of the Strand-Interleaving plan search (Sec. 4.2) in plain Python.

TEST INFRASTRUCTURE ONLY -- never imported by the product path.

  * oef()            -- the Overlap Effectiveness Factor, Eq. 1.
  * pair_dp()        -- the pairing recurrence, Eq. 2, for given segments and cost tables.
  * segment_cost()   -- cost P of co-running a forward segment with a backward segment, derived
                        from pairwise profiling results.  The paper only says P is "calculated from
                        the offline profiling results"; the reading used here is a two-queue fluid
                        model: each strand runs its segment's operators in order, and while forward
                        operator a and backward operator b are both active they progress at the
                        profiled rates rate_f[a][b] and rate_b[a][b] (1 = undisturbed).  A lone
                        operator runs at rate 1.  The pair ends when both queues are empty (barrier).
  * search_cuts()    -- for fixed operator sequences, the best placement of barriers: Eq. 2 applied
                        over operator prefixes, where a step may consume any contiguous run of
                        forward operators together with any contiguous run of backward operators.
  * topo_orders()    -- all topological orders of an operator DAG ("operator sequencing").
  * search()         -- minimum over all sequence pairs of search_cuts().
"""
import itertools


def oef(t_i, t_j, p_ij):
    """Eq. 1: how much of the shorter operator's time the overlap hides."""
    return (t_i + t_j - p_ij) / min(t_i, t_j)


def pair_dp(p_f, p_b, p_fb):
    """Eq. 2.  p_f[i] = P(i, empty), p_b[j] = P(empty, j), p_fb[i][j] = P(i, j), 0-based segments.
    Returns T_opt(N_f, N_b) and the chosen steps as a list of (i or None, j or None).
    Index ranges follow the recurrence (prefixes of length 0..N), base T(0,0) = 0."""
    nf, nb = len(p_f), len(p_b)
    INF = float("inf")
    T = [[INF] * (nb + 1) for _ in range(nf + 1)]
    back = [[None] * (nb + 1) for _ in range(nf + 1)]
    T[0][0] = 0.0
    for i in range(nf + 1):
        for j in range(nb + 1):
            if i == 0 and j == 0:
                continue
            cands = []
            if i > 0 and j > 0:
                cands.append((T[i - 1][j - 1] + p_fb[i - 1][j - 1], (i - 1, j - 1)))
            if i > 0:
                cands.append((T[i - 1][j] + p_f[i - 1], (i - 1, j)))
            if j > 0:
                cands.append((T[i][j - 1] + p_b[j - 1], (i, j - 1)))
            best = min(cands, key=lambda c: c[0])
            T[i][j], back[i][j] = best
    steps = []
    i, j = nf, nb
    while (i, j) != (0, 0):
        pi, pj = back[i][j]
        steps.append((i - 1 if pi < i else None, j - 1 if pj < j else None))
        i, j = pi, pj
    return T[nf][nb], steps[::-1]


def segment_cost(seg_f, seg_b, t_f, t_b, rate_f, rate_b):
    """Fluid co-run time of forward operators seg_f (ids, in order) with backward operators seg_b."""
    fi = bi = 0
    rem_f = t_f[seg_f[0]] if seg_f else 0.0
    rem_b = t_b[seg_b[0]] if seg_b else 0.0
    now = 0.0
    while fi < len(seg_f) and bi < len(seg_b):
        a, b = seg_f[fi], seg_b[bi]
        ra, rb = rate_f[a][b], rate_b[a][b]
        da, db = rem_f / ra, rem_b / rb      # time each would still need if the other stayed active
        dt = min(da, db)
        now += dt
        rem_f -= ra * dt
        rem_b -= rb * dt
        if da <= db:
            fi += 1
            rem_f = t_f[seg_f[fi]] if fi < len(seg_f) else 0.0
        if db <= da:
            bi += 1
            rem_b = t_b[seg_b[bi]] if bi < len(seg_b) else 0.0
    if fi < len(seg_f):
        now += rem_f + sum(t_f[o] for o in seg_f[fi + 1:])
    if bi < len(seg_b):
        now += rem_b + sum(t_b[o] for o in seg_b[bi + 1:])
    return now


def search_cuts(seq_f, seq_b, t_f, t_b, rate_f, rate_b, barrier_cost=0.0):
    """Best barrier placement for fixed sequences.  T(i,j) = min over (i',j') < (i,j) of
    T(i',j') + P(seq_f[i':i], seq_b[j':j]) + barrier_cost.  Returns (makespan, pairs) with
    pairs = [(f_begin, f_end, b_begin, b_end), ...] half-open ranges covering both sequences."""
    nf, nb = len(seq_f), len(seq_b)
    INF = float("inf")
    T = [[INF] * (nb + 1) for _ in range(nf + 1)]
    back = [[None] * (nb + 1) for _ in range(nf + 1)]
    T[0][0] = 0.0
    for i in range(nf + 1):
        for j in range(nb + 1):
            if i == 0 and j == 0:
                continue
            for ip in range(i + 1):
                for jp in range(j + 1):
                    if ip == i and jp == j:
                        continue
                    c = T[ip][jp] + segment_cost(seq_f[ip:i], seq_b[jp:j], t_f, t_b, rate_f, rate_b) + barrier_cost
                    if c < T[i][j]:
                        T[i][j], back[i][j] = c, (ip, jp)
    pairs = []
    i, j = nf, nb
    while (i, j) != (0, 0):
        ip, jp = back[i][j]
        pairs.append((ip, i, jp, j))
        i, j = ip, jp
    return T[nf][nb], pairs[::-1]


def topo_orders(n, deps):
    """All orderings of nodes 0..n-1 in which src precedes dst for every (src, dst) in deps."""
    out = []
    for perm in itertools.permutations(range(n)):
        pos = {v: p for p, v in enumerate(perm)}
        if all(pos[s] < pos[d] for s, d in deps):
            out.append(list(perm))
    return out


def search(kinds_f, deps_f, kinds_b, deps_b, t_f, t_b, rate_f, rate_b, barrier_cost=0.0):
    """Minimum makespan over all topological orders of both DAGs and all barrier placements.
    kinds_x[node] is the operator id used to index the profile tables."""
    best = (float("inf"), None, None, None)
    for of in topo_orders(len(kinds_f), deps_f):
        for ob in topo_orders(len(kinds_b), deps_b):
            m, pairs = search_cuts([kinds_f[n] for n in of], [kinds_b[n] for n in ob],
                                   t_f, t_b, rate_f, rate_b, barrier_cost)
            if m < best[0]:
                best = (m, of, ob, pairs)
    return best


def rates_from_corun(t_a, t_b, end_a, end_b):
    """Invert the fluid model for one profiled pair: operators with solo times t_a, t_b were started
    together and finished at end_a, end_b.  Returns (rate_a, rate_b) while both were active."""
    t1 = min(end_a, end_b)
    if end_a <= end_b:
        return t_a / t1, (t_b - (end_b - t1)) / t1
    return (t_a - (end_a - t1)) / t1, t_b / t1
