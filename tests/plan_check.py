"""Host-side checks of the schedule the single-launch kernels build on the device (paper Section 4.3: a task
waits for one event counter to reach a static threshold; thresholds equal producer counts; queue order is a
topological order of the DAG, consumed in order, hence no deadlock).  Pure Python on a copy of the workspace:
decode the task tables, check coverage / thresholds / order, and interpret the queues with counters."""
import dataclasses

import numpy as np

PERMUTE, GEMM1, GEMM2 = 0, 1, 2
NARROW = 0x80    # flag in the type byte: a 128-column half of a wide GEMM-2 tile (a queue's halved last round)


@dataclasses.dataclass
class Plan:
    n_mtiles: int
    rows: np.ndarray            # rows per M tile
    queues: list                # per queue: list of (type, index, m, dep_event, threshold)
    gemm2_total: int
    ev_per_tile: int
    max_mtiles: int
    expert: np.ndarray = None   # local expert per M tile
    row0: np.ndarray = None     # first row (in the permuted order) per M tile


def decode_plan(ws: np.ndarray, lay) -> Plan:
    """ws: the workspace as uint8; lay: the integers of moe_ffn_debug_layout."""
    i32 = lambda off, n: ws[off: off + 4 * n].view(np.int32)
    meta = i32(lay[0], 16)
    max_m, max_q, n_q = lay[7], lay[8], lay[15]
    n_m = int(meta[lay[12]])
    rows = i32(lay[3], max_m)[:n_m].copy()
    queues = []
    for q in range(n_q):
        n = int(meta[lay[13] + q])
        assert 0 <= n <= max_q, (q, n)
        td = i32(lay[6] + q * max_q * lay[22], 4 * n).reshape(n, 4)
        queues.append([(int(t & 0xFF), int(t >> 8), int(m), int(d), int(th)) for t, m, d, th in td])   # type keeps its NARROW flag
    return Plan(n_m, rows, queues, int(meta[lay[14]]), lay[10], max_m,
                i32(lay[1], max_m)[:n_m].copy(), i32(lay[2], max_m)[:n_m].copy())


def check_tile_map(plan: Plan, counts, wide_rows, tall_rows, n_queues=8):
    """The M-tile map behind a plan: the tiles of every expert cover its rows of the permuted order exactly once,
    in tiles of at most wide_rows rows (tall_rows for a tile that owns its pair slot), and the XCDs' shares are
    even: slot j (entries 2j, 2j+1) belongs to XCD j % 8, and no XCD holds more than one tile more than another
    apart from what the tall tiles (which cannot share a slot) add.  Returns tiles per XCD."""
    counts = np.asarray(counts)
    offsets = np.concatenate([[0], np.cumsum(counts)])
    covered = np.zeros(int(offsets[-1]), dtype=np.int32)
    per_xcd = [0] * n_queues
    n_tall = 0
    for m in range(plan.n_mtiles):
        r = int(plan.rows[m])
        if r <= 0:
            continue
        e, r0 = int(plan.expert[m]), int(plan.row0[m])
        assert offsets[e] <= r0 and r0 + r <= offsets[e + 1], f"M tile {m}: rows {r0}..{r0 + r} outside expert {e}"
        if r > wide_rows:
            assert r <= tall_rows and m % 2 == 0 and int(plan.rows[m + 1]) == 0, f"M tile {m}: {r} rows need a slot of their own"
            n_tall += 1
        covered[r0: r0 + r] += 1
        per_xcd[(m // 2) % n_queues] += 1
    assert (covered == 1).all(), f"{int((covered != 1).sum())} rows are not covered exactly once"
    assert max(per_xcd) - min(per_xcd) <= 1 + min(n_tall, 1), f"tiles per XCD {per_xcd}"
    return per_xcd


def expected_tiles(plan: Plan, n1_wide, n1_tall, n2_wide, n2_tall, wide_rows, perm_rows, permute):
    """Per M tile with rows: (PERMUTE parts, GEMM-1 N tiles, GEMM-2 N tiles, 128-column halves of the GEMM-2 extent
    if the tile is wide, else 0)."""
    exp = {}
    for m in range(plan.n_mtiles):
        r = int(plan.rows[m])
        if r <= 0:
            continue
        tall = r > wide_rows
        exp[m] = ((r + perm_rows - 1) // perm_rows if permute else 0, n1_tall if tall else n1_wide,
                  n2_tall if tall else n2_wide, 0 if tall else n2_tall)
    return exp


def check_plan(plan: Plan, exp: dict, n_queues=8, workers_per_queue=None):
    """Raises AssertionError naming the first violated property.  A wide GEMM-2 tile (m, nt) may appear as ONE task
    or, in a queue's halved last round, as its 128-column halves (NARROW tasks 2nt and, if that half exists,
    2nt + 1).  workers_per_queue given: the halving must be exactly what the rule says (a last round of GEMM-2
    tasks that is at most half full, and nothing else)."""
    seen = {}
    for q, tasks in enumerate(plan.queues):
        for pos, (ty, idx, m, dep, thr) in enumerate(tasks):
            assert m in exp, f"queue {q} pos {pos}: task on M tile {m} that has no rows"
            assert (m // 2) % n_queues == q, f"M tile {m} in queue {q}: its pair belongs to queue {(m // 2) % n_queues}"
            key = (ty, m, idx)
            assert key not in seen, f"task {key} appears twice"
            seen[key] = (q, pos, dep, thr)
    n_g2 = n_tasks = 0
    for m, (parts, n1, n2, halves) in exp.items():
        for ty, n in ((PERMUTE, parts), (GEMM1, n1)):
            for idx in range(n):
                assert (ty, m, idx) in seen, f"task {(ty, m, idx)} is missing"
        n_tasks += parts + n1
        for nt in range(n2):
            whole = (GEMM2, m, nt) in seen
            lo, hi = (GEMM2 | NARROW, m, 2 * nt) in seen, (GEMM2 | NARROW, m, 2 * nt + 1) in seen
            if halves == 0:
                assert whole and not lo and not hi, f"GEMM-2 task {(m, nt)} of a tall tile must be one task"
                n_g2 += 1
            else:
                want_hi = 2 * nt + 1 < halves
                assert whole != lo, f"GEMM-2 tile {(m, nt)}: once as a whole or as halves"
                assert whole or hi == want_hi, f"GEMM-2 tile {(m, nt)}: second half {'missing' if want_hi else 'past the last column'}"
                assert not (whole and hi), f"GEMM-2 tile {(m, nt)}: a half beside the whole tile"
                n_g2 += 1 if whole else 1 + int(want_hi)
    n_tasks += n_g2
    assert len(seen) == n_tasks, "tasks beyond the expected index ranges"
    # thresholds = producer counts, dependent events = the producers' trigger events, producers precede consumers
    for (ty, m, idx), (q, pos, dep, thr) in seen.items():
        parts, n1, n2, halves = exp[m]
        base = ty & ~NARROW
        if base == PERMUTE or (base == GEMM1 and parts == 0):
            assert dep == -1, f"{(ty, m, idx)} must not wait"
            continue
        want_dep, want_thr, prod = ((plan.ev_per_tile + m, parts, PERMUTE) if base == GEMM1
                                    else (plan.ev_per_tile + plan.max_mtiles + m, n1, GEMM1))
        assert dep == want_dep, f"{(ty, m, idx)} waits on event {dep}, producers trigger {want_dep}"
        assert thr == want_thr, f"{(ty, m, idx)} threshold {thr} != {want_thr} producer tasks"
        for pi in range(want_thr):
            pq, ppos, _, _ = seen[(prod, m, pi)]
            assert pq == q and ppos < pos, f"producer {(prod, m, pi)} does not precede {(ty, m, idx)} in queue {q}"
    assert plan.gemm2_total == n_g2, f"GEMM-2 total {plan.gemm2_total} != {n_g2} GEMM-2 tasks"
    if workers_per_queue:
        for q, tasks in enumerate(plan.queues):
            g2 = [t for t in tasks if t[0] & ~NARROW == GEMM2]
            narrow = [t for t in g2 if t[0] & NARROW]
            wide_equiv = len(g2) - sum(1 for t in narrow if t[1] & 1)     # tasks before any halving
            tail = wide_equiv % workers_per_queue
            if 0 < tail <= workers_per_queue // 2:
                assert narrow, f"queue {q}: last round of {tail} GEMM-2 tiles is not halved"
                assert len({(t[2], t[1] // 2) for t in narrow}) <= tail and all(t in g2[-(2 * tail):] for t in narrow), \
                    f"queue {q}: halved tasks outside the last round of {tail}"
            else:
                assert not narrow, f"queue {q}: {len(narrow)} halved GEMM-2 tasks, but its last round is {tail} of {workers_per_queue}"


def simulate(plan: Plan, workers_per_queue=1):
    """In-order interpretation of the queues with event counters: every worker takes the next ticket of its
    queue and may only run the task once its event has reached the threshold; a finished task bumps its
    trigger event.  Returns the number of steps; raises AssertionError on deadlock."""
    events = {}
    heads = [0] * len(plan.queues)
    running = [[] for _ in plan.queues]     # tasks held by workers (waiting or runnable)
    done, total, steps = 0, sum(len(t) for t in plan.queues), 0
    while done < total:
        progressed = False
        for q, tasks in enumerate(plan.queues):
            while len(running[q]) < workers_per_queue and heads[q] < len(tasks):
                running[q].append(tasks[heads[q]])
                heads[q] += 1
            still = []
            for (ty, idx, m, dep, thr) in running[q]:
                if dep == -1 or events.get(dep, 0) >= thr:
                    trig = {PERMUTE: plan.ev_per_tile + m, GEMM1: plan.ev_per_tile + plan.max_mtiles + m, GEMM2: "g2"}[ty & ~NARROW]
                    events[trig] = events.get(trig, 0) + 1
                    done += 1
                    progressed = True
                else:
                    still.append((ty, idx, m, dep, thr))
            running[q] = still
        steps += 1
        assert progressed, f"deadlock after {done} of {total} tasks: waiting {[r[:1] for r in running if r]}"
    assert events.get("g2", 0) == plan.gemm2_total, "COMBINE would wait for a GEMM-2 total that is never reached"
    return steps
