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
  * lane_cost()      -- cost of a segment pair with more than two participants: the executor's streams as lanes
                        (two strands, communication stream(s), cross-node stream).  The paper's P(segment pair) is
                        "calculated from the offline profiling results" (Sec. 4.2) and its executor puts computation,
                        local and cross-node communication on streams of their own (Sec. 5); the reading: replay the
                        issue order of the executor as a dependency graph (a stream runs its operators in issue order;
                        a stand-in on a stream of its own starts behind what its strand has issued so far and is
                        awaited only by the operators that consume its result, or at the end of the pair; an operator
                        flagged to run beside its strand goes to the other strand's stream behind what its own strand
                        has issued) and integrate it as a fluid in which every active operator advances at the product
                        of its pairwise profiled rates against the other active operators.  Two operators of one
                        direction have no profiled pair: one of them is replaced by the operator of the other
                        direction that runs the same kernel (`like`), and counts as undisturbed if there is none.
                        With no separate lanes and nothing beside the strand this is segment_cost().
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


def lane_cost(seg_f, seg_b, t_f, t_b, rate_f, rate_b, deps_f=(), deps_b=(), comm_f=None, comm_b=None, lanes=(0, 0, 0),
              side=(), like_f=None, like_b=None):
    """Fluid co-run time of one segment pair on the executor's streams.
    comm_x[op]: 0 compute, 1 collective stand-in, 2 cross-node transfer.  lanes = (comm_alpha, comm_beta, cross):
    comm_alpha 0/1 = alpha's collectives in alpha's stream / on the communication stream; comm_beta 0/1/2 = in beta's
    stream / on the shared communication stream / on beta's own communication stream; cross 1 = cross-node transfers on
    the cross-node stream.  side: backward operators that run beside their strand (in alpha's stream).
    like_x[op]: id of the like operator in the other direction (or absent)."""
    comm_f, comm_b = comm_f or {}, comm_b or {}
    like_f, like_b = like_f or {}, like_b or {}
    A, B, COMM, COMM_B, CROSS = "alpha", "beta", "comm", "comm_beta", "cross"

    def stream_of(direction, kind):
        if kind == 2 and lanes[2]:
            return CROSS
        if kind == 0:
            return A if direction == "f" else B
        if direction == "f":
            return COMM if lanes[0] else A
        return {0: B, 1: COMM, 2: COMM_B}[lanes[1]]

    # ---- issue: operators alternate between the strands, every stream keeps its issue order
    jobs = []                       # dicts: dir, op, stream, work, after (set of job indices)
    queue = {s: [] for s in (A, B, COMM, COMM_B, CROSS)}
    waits = {A: set(), B: set()}    # events a strand's stream has been told to wait for, taken up by its next job
    pending = {"f": {}, "b": {}}    # stand-ins their strand has not waited for yet: op -> job

    def submit(direction, op, stream, after):
        after = set(after)
        if stream in waits:
            after |= waits[stream]
            waits[stream] = set()
        if queue[stream]:
            after.add(queue[stream][-1])
        jobs.append(dict(dir=direction, op=op, stream=stream, work=(t_f if direction == "f" else t_b)[op], after=after))
        queue[stream].append(len(jobs) - 1)
        return len(jobs) - 1

    def strand_waits_for_inputs(direction, op, deps, strand):
        for src, dst in deps:
            if dst == op and src in pending[direction]:
                waits[strand].add(pending[direction].pop(src))

    fi = bi = 0
    while fi < len(seg_f) or bi < len(seg_b):
        if fi < len(seg_f):
            op = seg_f[fi]; fi += 1
            strand_waits_for_inputs("f", op, deps_f, A)
            st = stream_of("f", comm_f.get(op, 0))
            if st != A:
                pending["f"][op] = submit("f", op, st, queue[A][-1:] )
            else:
                submit("f", op, A, ())
        if bi < len(seg_b):
            op = seg_b[bi]; bi += 1
            strand_waits_for_inputs("b", op, deps_b, B)
            if op in side:
                submit("b", op, A, set(queue[B][-1:]) | waits[B])   # behind beta's issued work and what beta waits for
                continue
            st = stream_of("b", comm_b.get(op, 0))
            if st != B:
                pending["b"][op] = submit("b", op, st, queue[B][-1:])
            else:
                submit("b", op, B, ())

    # ---- fluid integration
    def slowdown(x, y):            # rate of job x while job y runs
        xd, xo, yd, yo = x["dir"], x["op"], y["dir"], y["op"]
        if xd == yd:
            like = like_f if xd == "f" else like_b
            if yo in like:
                yd, yo = ("b" if yd == "f" else "f"), like[yo]
            elif xo in like:
                xd, xo = ("b" if xd == "f" else "f"), like[xo]
            else:
                return 1.0
        return rate_f[xo][yo] if xd == "f" else rate_b[yo][xo]

    left = [j["work"] for j in jobs]
    finished = [False] * len(jobs)
    now = 0.0
    while not all(finished):
        running = []
        for s, q in queue.items():
            head = next((k for k in q if not finished[k]), None)
            if head is not None and all(finished[a] for a in jobs[head]["after"]):
                running.append(head)
        assert running, "dependency cycle"
        speed = {}
        for k in running:
            r = 1.0
            for o in running:
                if o != k:
                    r *= slowdown(jobs[k], jobs[o])
            speed[k] = r
        dt = min(left[k] / speed[k] for k in running)
        now += dt
        for k in running:
            left[k] -= speed[k] * dt
            if left[k] <= 1e-12 * max(jobs[k]["work"], 1e-300) or left[k] / speed[k] <= 1e-12 * dt:
                finished[k] = True
    return now


def plan_cost_lanes(plan_pairs, seq_f, seq_b, t_f, t_b, rate_f, rate_b, barrier_cost=0.0, **kw):
    """Sum of lane_cost over the segment pairs of a plan plus a barrier per pair."""
    return sum(lane_cost(seq_f[a:b], seq_b[c:d], t_f, t_b, rate_f, rate_b, **kw) + barrier_cost for a, b, c, d in plan_pairs)


def search_cuts_lanes(seq_f, seq_b, t_f, t_b, rate_f, rate_b, barrier_cost=0.0, **kw):
    """search_cuts with lane_cost as P."""
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
                    c = T[ip][jp] + lane_cost(seq_f[ip:i], seq_b[jp:j], t_f, t_b, rate_f, rate_b, **kw) + barrier_cost
                    if c < T[i][j]:
                        T[i][j], back[i][j] = c, (ip, jp)
    pairs = []
    i, j = nf, nb
    while (i, j) != (0, 0):
        ip, jp = back[i][j]
        pairs.append((ip, i, jp, j))
        i, j = ip, jp
    return T[nf][nb], pairs[::-1]
