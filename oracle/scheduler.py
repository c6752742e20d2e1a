"""Oracle for the wavefront sample scheduler (Sec. 3.4, Algorithm 1).  TEST INFRASTRUCTURE ONLY:
only tests/, the smoke check and the CPU-baseline leg of the benchmark may import this package.

A sample is the 6-tuple (t_f_bc, t_f_c, t_f_ac, t_b_bc, t_b_c, t_b_ac) of Sec. 3.4: forward time before,
within and after the critical section, then backward time before (i.e. in the sections that FOLLOW the
critical one in forward order), within, and after (the sections that PRECEDE it in forward order) the
critical section.  The timeline is simulated as a discrete-event system with three serial servers:

  PRE   runs the forward of the sections in front of the critical one (t_f_bc) and, later, their
        backward (t_b_ac);
  CRIT  runs the critical section's forward (t_f_c) and backward (t_b_c);
  POST  runs the sections behind the critical one: forward (t_f_ac) immediately followed by backward (t_b_bc).

Readings (the paper prints the greedy loop and a figure, not the timeline rules):
  * a server never pre-empts and serves the jobs of one kind in schedule order;
  * PRE prefers forward jobs (they have no predecessors, so all of them are ready at time 0) to backward
    jobs: the critical section must not wait for a forward input (critical-section-first principle);
  * CRIT, `interleave` = True: sample by sample, forward then backward (gradient accumulation over
    micro-batches); False: all forwards in order, then all backwards in order;
  * a job becomes ready when its predecessor on the sample's path finished:
    PRE.f -> CRIT.f -> POST.(f+b) -> CRIT.b -> PRE.b;
  * makespan = the time the last server goes idle;
  * Algorithm 1's insertion is done once per sample, after all positions were tried (the printed listing
    has it inside the position loop, which would insert a sample once per position); ties (makespans
    equal to within 1e-9 relative) keep the first (lowest) position because the comparison is strict.
"""
import heapq
import itertools

TIE = 1e-9   # makespans closer than this (relative) count as equal: sums taken in different orders differ by rounding


def simulate(samples, order, interleave=True):
    """Event simulation.  Returns dict(makespan, critical_idle, critical_busy): critical_idle is the time the
    critical server spends waiting between its first start and its last finish."""
    n = len(order)
    if n == 0:
        return dict(makespan=0.0, critical_idle=0.0, critical_busy=0.0)
    t = [tuple(float(x) for x in samples[i]) for i in order]          # in schedule order
    # job kinds on each server, each a FIFO in schedule order; ready[kind][k] = time job k may start (None: not yet)
    ready = {kind: [None] * n for kind in ("pre_f", "crit_f", "post", "crit_b", "pre_b")}
    for k in range(n):
        ready["pre_f"][k] = 0.0
    dur = {"pre_f": [x[0] for x in t], "crit_f": [x[1] for x in t], "post": [x[2] + x[3] for x in t],
           "crit_b": [x[4] for x in t], "pre_b": [x[5] for x in t]}
    succ = {"pre_f": "crit_f", "crit_f": "post", "post": "crit_b", "crit_b": "pre_b", "pre_b": None}
    nxt = {kind: 0 for kind in ready}                                   # next job index of each FIFO
    free = {"PRE": 0.0, "CRIT": 0.0, "POST": 0.0}
    busy_crit, first_crit, last_crit = 0.0, None, 0.0
    done = 0
    events = []                                                          # (time, seq, kind, k) completions
    seq = itertools.count()
    running = {"PRE": False, "CRIT": False, "POST": False}

    def candidates(server, now):
        if server == "PRE":
            kinds = ["pre_f", "pre_b"]                                   # forward first
        elif server == "POST":
            kinds = ["post"]
        elif interleave:
            # sample by sample: the backward of sample k precedes the forward of sample k + 1
            kinds = ["crit_b", "crit_f"] if nxt["crit_b"] < nxt["crit_f"] else ["crit_f"]
        else:
            kinds = ["crit_f"] if nxt["crit_f"] < n else ["crit_b"]
        for kind in kinds:
            k = nxt[kind]
            if k < n and ready[kind][k] is not None and ready[kind][k] <= now:
                return kind, k
            if server == "CRIT":
                return None                                              # the critical server keeps its order
        return None

    def try_start(server, now):
        nonlocal busy_crit, first_crit
        if running[server]:
            return
        c = candidates(server, now)
        if c is None:
            return
        kind, k = c
        nxt[kind] += 1
        running[server] = True
        if server == "CRIT":
            busy_crit += dur[kind][k]
            if first_crit is None:
                first_crit = now
        heapq.heappush(events, (now + dur[kind][k], next(seq), kind, k, server))

    now = 0.0
    for s in ("PRE", "CRIT", "POST"):
        try_start(s, now)
    # zero-length jobs complete at once; the loop below handles them through the event queue as well
    while events:
        now, _, kind, k, server = heapq.heappop(events)
        running[server] = False
        free[server] = now
        if server == "CRIT":
            last_crit = now
        if succ[kind] is not None:
            ready[succ[kind]][k] = now
        else:
            done += 1
        for s in ("PRE", "CRIT", "POST"):
            try_start(s, now)
    assert done == n, "simulation stalled"
    makespan = max(free.values())
    span = last_crit - (first_crit or 0.0)
    return dict(makespan=makespan, critical_idle=max(span - busy_crit, 0.0) + (first_crit or 0.0), critical_busy=busy_crit)


def makespan(samples, order, interleave=True):
    return simulate(samples, order, interleave)["makespan"]


def schedule(samples, interleave=True):
    """Algorithm 1: stable sort by t_f_bc, then greedy insertion at the position of least simulated makespan."""
    n = len(samples)
    if n == 0:
        return []
    initial = sorted(range(n), key=lambda i: samples[i][0])           # Python's sort is stable
    result = [initial[0]]
    for s in initial[1:]:
        best_pos, best = 0, float("inf")
        for pos in range(len(result) + 1):
            cand = result[:pos] + [s] + result[pos:]
            m = makespan(samples, cand, interleave)
            if m < best * (1.0 - TIE):
                best, best_pos = m, pos
        result.insert(best_pos, s)
    return result


def brute_force_best(samples, interleave=True):
    """Least makespan over all orders (small n only)."""
    return min(makespan(samples, list(p), interleave) for p in itertools.permutations(range(len(samples))))
