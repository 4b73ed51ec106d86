"""Independent checkers used to pin the oracle (and to validate schedules from either side).

Nothing here knows about lags, graphs or longest paths.  A periodic schedule is *expanded*
into absolute start times of concrete blocks (type, micro-batch) over a few windows and the
three constraints of the paper's Eq. 1 are tested literally on that finite set:
[1] blocks sharing a device do not overlap, [2] per-device running memory sum in start order
stays within M, [3] every data dependency inside a micro-batch is respected.
"""
import itertools


def devices_of(problem, i):
    return [d for d in range(problem["D"]) if problem["dev_mask"][i] >> d & 1]


def slot_of_type_in_orders(problem, orders):
    """occurrence numbers: for each device order, the q of every position (Property 1)."""
    out = []
    for seq in orders:
        cnt = {}
        qs = []
        for g in seq:
            qs.append(cnt.get(g, 0))
            cnt[g] = cnt.get(g, 0) + 1
        out.append(qs)
    return out


def expand_periodic(problem, leads, orders, starts, T, windows):
    """absolute (type, mu) -> start for windows 0..windows-1; starts[type][q] (None = not set)."""
    NR = problem["NR"]
    blocks = {}
    for k in range(windows):
        for i in range(problem["K"]):
            for q in range(NR):
                if starts[i][q] is not None:
                    blocks[(i, leads[i] + q + NR * k)] = starts[i][q] + k * T
    return blocks


def check_periodic(problem, leads, orders, starts, T, windows=4):
    """True iff the rigid repetition of the window with period T violates nothing among the
    blocks whose start is set: device order as given (window after window), no overlap,
    dependencies between blocks that are both present.  Dependencies whose producer lies
    before window 0 cannot be looked at and are skipped -- the same constraint reappears one
    window later."""
    NR, t = problem["NR"], problem["t"]
    blocks = expand_periodic(problem, leads, orders, starts, T, windows)
    if any(s < 0 for s in blocks.values()):
        return False
    for (a, b) in problem["deps"]:
        for (i, mu), s in blocks.items():
            if i == b and (a, mu) in blocks and blocks[(a, mu)] + t[a] > s:
                return False
    qs = slot_of_type_in_orders(problem, orders)
    for d, seq in enumerate(orders):
        timeline = []
        for k in range(windows):
            for g, q in zip(seq, qs[d]):
                key = (g, leads[g] + q + NR * k)
                if key in blocks:
                    timeline.append((blocks[key], t[g]))
        for (s0, t0), (s1, _) in zip(timeline, timeline[1:]):
            if s0 + t0 > s1:
                return False
    return True


def exists_periodic_schedule(problem, leads, orders, T, box):
    """Brute force: is there any integer start vector in [0, box]^n that check_periodic
    accepts?  Depth-first over the nodes; a partial vector that already violates something
    is abandoned."""
    K, NR = problem["K"], problem["NR"]
    starts = [[None] * NR for _ in range(K)]
    nodes = [(i, q) for q in range(NR) for i in range(K)]

    def rec(k):
        if k == len(nodes):
            return True
        g, q = nodes[k]
        for s in range(box + 1):
            starts[g][q] = s
            if check_periodic(problem, leads, orders, starts, T, windows=3) and rec(k + 1):
                return True
        starts[g][q] = None
        return False

    return rec(0)


def memory_peaks_from_times(problem, blocks_by_device):
    """Eq. 1 [2] literally: sort a device's blocks by start time, running sum of m."""
    peaks = []
    for blocks in blocks_by_device:
        cur, peak = 0, None
        for _, m in sorted(blocks, key=lambda x: x[0]):
            cur += m
            peak = cur if peak is None else max(peak, cur)
        peaks.append(peak)
    return peaks


def check_flat_schedule(problem, N, start, dev_order):
    """Eq. 1 on a complete schedule of N micro-batches: start[type][mu]; dev_order[d] is the
    list of type*N+mu in execution order.  Returns (ok, makespan, peaks)."""
    K, t, m = problem["K"], problem["t"], problem["m"]
    for i in range(K):
        for mu in range(N):
            if start[i][mu] < 0:
                return False, None, None
    for (a, b) in problem["deps"]:
        for mu in range(N):
            if start[a][mu] + t[a] > start[b][mu]:
                return False, None, None
    peaks = []
    seen = set()
    for d in range(problem["D"]):
        mine = [(i, mu) for i in range(K) if problem["dev_mask"][i] >> d & 1 for mu in range(N)]
        if sorted(mine) != sorted((x // N, x % N) for x in dev_order[d]):
            return False, None, None
        tl = sorted((start[i][mu], t[i], m[i]) for (i, mu) in mine)
        for (s0, t0, _), (s1, _, _) in zip(tl, tl[1:]):
            if s0 + t0 > s1:
                return False, None, None
        # the reported device order must be the start-time order
        if [start[x // N][x % N] for x in dev_order[d]] != sorted(start[x // N][x % N] for x in dev_order[d]):
            return False, None, None
        cur, peak = 0, 0
        for _, _, mm in tl:
            cur += mm
            peak = max(peak, cur)
        peaks.append(peak)
        seen.update(mine)
    makespan = max(start[i][mu] + t[i] for i in range(K) for mu in range(N))
    return True, makespan, peaks


def check_instantiation(problem, N, start, ops):
    """Properties Sec. IV-D asks of the global operation sequence of a complete schedule.
    ops: (kind, block, src, dst, aux); kind 0 = block (src = device mask, dst = start time),
    kind 1 = send/receive pair (block = producer, src = sender, dst = receiver, aux = consumer).
    Returns (ok, reason)."""
    K, D, masks, deps = problem["K"], problem["D"], problem["dev_mask"], problem["deps"]
    pos_of_block, last_start = {}, -1
    for k, (kind, blk, src, dst, aux) in enumerate(ops):
        if kind == 0:
            if blk in pos_of_block or src != masks[blk // N] or dst != start[blk // N][blk % N] or dst < last_start:
                return False, "block order"
            pos_of_block[blk] = k
            last_start = dst
    if len(pos_of_block) != K * N:
        return False, "missing blocks"
    # every tensor a consumer needs on a device where the producer did not run arrives exactly once,
    # from a device that has it, after the producer and before the consumer
    want = set()
    for (a, b) in deps:
        for mu in range(N):
            for v in range(D):
                if masks[b] >> v & 1 and not masks[a] >> v & 1:
                    want.add((a * N + mu, b * N + mu, v))
    seen = set()
    for k, (kind, blk, src, dst, aux) in enumerate(ops):
        if kind != 1:
            continue
        key = (blk, aux, dst)
        if key not in want or key in seen or not masks[blk // N] >> src & 1:
            return False, "unexpected pair"
        seen.add(key)
        if not pos_of_block[blk] < k < pos_of_block[aux]:
            return False, "pair outside (producer, consumer)"
    if seen != want:
        return False, "missing pairs"
    # blocking execution: every device runs its share of the sequence in order; a block on several devices and a
    # send/receive pair need all their devices to have arrived.  It must run to the end.
    prog = [[] for _ in range(D)]
    for k, (kind, blk, src, dst, aux) in enumerate(ops):
        devs = [d for d in range(D) if src >> d & 1] if kind == 0 else [src, dst]
        for d in devs:
            prog[d].append((k, tuple(devs)))
    at = [0] * D
    progress = True
    while progress:
        progress = False
        for d in range(D):
            if at[d] >= len(prog[d]):
                continue
            k, devs = prog[d][at[d]]
            if all(at[e] < len(prog[e]) and prog[e][at[e]][0] == k for e in devs):
                for e in devs:
                    at[e] += 1
                progress = True
    if any(at[d] != len(prog[d]) for d in range(D)):
        return False, "deadlock"
    return True, ""
