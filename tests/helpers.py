"""Independent reference pieces used to pin the oracle (pure Python, tiny inputs).

Nothing here is shared with oracle/ or with the GPU path: the partition
optimum is found by enumerating every contiguous partition, and the schedule
by a heap-driven discrete-event simulation whose per-resource order comes from
the closed form 'block j serves microbatch m in sweep m + j - 1'.
"""
import heapq
import itertools


def stage_costs(P, X, cuts, L):
    """Per-resource per-microbatch times of the partition with the given cuts.
    P: prefix of fwd+bwd (len L+1); X[n][k] = channel n (1-based) cost at cut k."""
    edges = [0] + list(cuts) + [L]
    comp = [P[edges[i + 1]] - P[edges[i]] for i in range(len(edges) - 1)]
    chan = [X[n][edges[n]] for n in range(1, len(edges) - 1)]
    return comp, chan


def brute_optimum(P, X, S, l):
    """min over all partitions of layers [0,l) into S non-empty contiguous stages of the
    largest per-stage / per-channel time; X[n][k] as above for channels 1..S-1."""
    best = None
    for cuts in itertools.combinations(range(1, l), S - 1):
        comp, chan = stage_costs(P, X, cuts, l)
        w = max(comp + chan)
        if best is None or w < best:
            best = w
    return best


def brute_plan(P, X, S, L):
    """The tie-broken plan: the last cut is the smallest k for which the optimum of the
    first k layers in S-1 stages, the channel at k and the last stage [k,L) together reach
    the optimum; then the same rule on the prefix with its own optimum."""
    bounds = [L]
    l = L
    for n in range(S - 1, 0, -1):
        target = brute_optimum(P, X, n + 1, l)
        for k in range(n, l):
            w = max(brute_optimum(P, X, n, k), X[n][k], P[l] - P[k])
            if w == target:
                bounds.append(k)
                l = k
                break
        else:
            raise AssertionError("no split reaches the optimum")
    return list(reversed(bounds))


def channel_table(XF, XB, D, L, order):
    """X[n][k] for n = 1..S-1 along an ordering, from flat tables indexed (u*D+v)*L + k-1."""
    X = [None]
    for n in range(1, len(order)):
        u, v = int(order[n - 1]), int(order[n])
        base = (u * D + v) * L
        X.append([None] + [int(XF[base + k - 1]) + int(XB[base + k - 1]) for k in range(1, L)])
    return X


def event_sim(F, B, cf, cb, M):
    """Discrete-event simulation of a flushed synchronous pipeline.
    Resources r = 1..R (odd: stages, even: channels); blocks j = 1..2R-1.
    Returns (T, start[j][m]) with 1-based j and m in dicts."""
    S = len(F)
    R = 2 * S - 1
    J = 2 * R - 1

    def res(j):
        return j if j <= R else 2 * R - j

    def dur(j):
        r = res(j)
        n = (r - 1) // 2 if r % 2 else r // 2
        if j == R:
            return F[S - 1] + B[S - 1]
        if r % 2:
            return F[n] if j < R else B[n]
        return cf[n] if j < R else cb[n]

    # service order per resource: sweep t = m + j - 1 ascending, then block ascending
    order = {r: [] for r in range(1, R + 1)}
    for j in range(1, J + 1):
        for m in range(1, M + 1):
            order[res(j)].append((m + j - 1, j, m))
    for r in order:
        order[r].sort()
    pos = {r: 0 for r in order}
    busy_until = {r: None for r in order}     # None = idle
    done = {}
    start = {}
    now = 0
    events = []  # (finish time, resource, j, m)

    def try_start(r):
        if busy_until[r] is not None or pos[r] >= len(order[r]):
            return
        _, j, m = order[r][pos[r]]
        if j > 1 and (j - 1, m) not in done:
            return
        start[(j, m)] = now
        busy_until[r] = now + dur(j)
        heapq.heappush(events, (now + dur(j), r, j, m))
        pos[r] += 1

    try_start(1)
    while events:
        now = events[0][0]
        # retire everything finishing now, then let every idle resource look at its head;
        # zero-length work finishes at the same instant, so repeat until nothing moves
        while True:
            moved = False
            while events and events[0][0] == now:
                _, r, j, m = heapq.heappop(events)
                done[(j, m)] = now
                busy_until[r] = None
                moved = True
            before = len(start)
            for r in order:
                try_start(r)
            if len(start) != before:
                moved = True
            if not moved:
                break
    assert len(done) == J * M, "simulation stalled"
    T = max(done[(J, m)] for m in range(1, M + 1))
    return T, start


def fifo_sim(F, B, cf, cb, M):
    """Clock-driven simulation of Alg. 1 read strictly: stages follow their lists (sweep
    m + j - 1, then block), a channel that is idle takes, of the transfers waiting for it, the
    one that has waited longest (equal: earlier in list order).  Positive durations only (with
    zero-length work "the same instant" is ambiguous).  Returns T."""
    S = len(F)
    R = 2 * S - 1
    J = 2 * R - 1
    res = lambda j: j if j <= R else 2 * R - j
    dur = {}
    for n in range(S):
        r = 2 * n + 1
        if n == S - 1:
            dur[R] = F[n] + B[n]
        else:
            dur[r], dur[2 * R - r] = F[n], B[n]
        if n:
            dur[r - 1], dur[2 * R - (r - 1)] = cf[n], cb[n]
    assert all(d >= 1 for d in dur.values())
    stage_list = {r: sorted((m + j - 1, j, m) for j in range(1, J + 1) if res(j) == r for m in range(1, M + 1))
                  for r in range(1, R + 1, 2)}
    pos = {r: 0 for r in stage_list}
    waiting = {r: [] for r in range(2, R + 1, 2)}   # (arrival time, list key, j, m)
    arrived = {}                                     # (j, m) -> time its microbatch reached block j
    for m in range(1, M + 1):
        arrived[(1, m)] = 0
    free_at = {r: 0 for r in range(1, R + 1)}
    running = []                                     # heap of (finish, r, j, m)
    finished = 0
    T = 0
    now = 0
    while finished < J * M:
        progressed = True
        while progressed:
            progressed = False
            for r in range(1, R + 1):
                if free_at[r] > now or any(x[1] == r for x in running):
                    continue
                if r % 2:
                    if pos[r] >= len(stage_list[r]):
                        continue
                    _, j, m = stage_list[r][pos[r]]
                    if (j, m) not in arrived:
                        continue
                    pos[r] += 1
                else:
                    if not waiting[r]:
                        continue
                    waiting[r].sort()
                    _, _, j, m = waiting[r].pop(0)
                heapq.heappush(running, (now + dur[j], r, j, m))
                free_at[r] = now + dur[j]
                progressed = True
        now = running[0][0]
        while running and running[0][0] == now:
            _, r, j, m = heapq.heappop(running)
            finished += 1
            T = max(T, now)
            if j < J:
                arrived[(j + 1, m)] = now
                if res(j + 1) % 2 == 0:
                    waiting[res(j + 1)].append((now, (m + j, j + 1), j + 1, m))
    return T


def list_sim(blocks, M):
    """Heap-driven simulation of serial resources that follow explicit service lists.
    blocks: list of (resource id, duration, key) in the order a microbatch passes them, where
    key(m) sorts the item (block, microbatch m) within its resource's list.
    Returns (T, finish) with finish[(j, m)] for 0-based block j and 1-based m."""
    J = len(blocks)
    order = {}
    for j, (r, d, key) in enumerate(blocks):
        for m in range(1, M + 1):
            order.setdefault(r, []).append((key(m), j, m))
    for r in order:
        order[r].sort()
    pos = {r: 0 for r in order}
    busy = {r: False for r in order}
    done = {}
    now = 0
    events = []

    def try_start(r):
        if busy[r] or pos[r] >= len(order[r]):
            return False
        _, j, m = order[r][pos[r]]
        if j > 0 and (j - 1, m) not in done:
            return False
        busy[r] = True
        heapq.heappush(events, (now + blocks[j][1], r, j, m))
        pos[r] += 1
        return True

    while True:
        moved = True
        while moved:
            moved = False
            while events and events[0][0] == now:
                _, r, j, m = heapq.heappop(events)
                done[(j, m)] = now
                busy[r] = False
                moved = True
            for r in order:
                if try_start(r):
                    moved = True
        if not events:
            break
        now = events[0][0]
    assert len(done) == J * M, "simulation stalled"
    return max(done[(J - 1, m)] for m in range(1, M + 1)), done


def variant_blocks(variant, F, B, cf, cb):
    """Block list of a schedule variant for list_sim.  'pe' and 'duplex': blocks of the PE
    scheduler (last stage merged), served by (sweep, block) with sweep = m + j; 'duplex' gives
    the backward transfers their own channels.  'gpipe': last stage's F and B separate, every
    resource serves all forward items, then all backward items, microbatches in order.
    'additive': 2S-1 stage blocks (last stage merged), transfers added to the stage they lead into,
    served by (sweep, block) on that shorter list."""
    S = len(F)
    blocks = []
    merged = variant != "gpipe"

    def add(res, dur, fwd):
        j = len(blocks)
        if variant == "gpipe":
            blocks.append((res, dur, (lambda m, fwd=fwd, j=j: (0 if fwd else 1, j, m))))
        else:
            blocks.append((res, dur, (lambda m, j=j: (m + j, j))))

    if variant == "additive":
        # stages only; a stage's passes include the transfers over its inbound link
        for n in range(S):
            d = F[n] + (cf[n] if n else 0)
            if n == S - 1:
                d += B[n] + (cb[n] if n else 0)
            add(("s", n), d, True)
        for n in range(S - 2, -1, -1):
            add(("s", n), B[n] + (cb[n] if n else 0), False)
        return blocks
    for n in range(S):
        if n:
            add(("c", n), cf[n], True)
        add(("s", n), F[n] + B[n] if (n == S - 1 and merged) else F[n], True)
    for n in range(S - 1, -1, -1):
        if not (n == S - 1 and merged):
            add(("s", n), B[n], False)
        if n:
            add(("cb", n) if variant == "duplex" else ("c", n), cb[n], False)
    return blocks
