"""CPU tests of the schedule checker itself (tests/plan_check.py) on a hand-made plan: it accepts a legal
schedule and names each planted mistake (paper Section 4.3: thresholds, topological queue order, progress)."""
import copy

import numpy as np
import pytest

from plan_check import GEMM1, GEMM2, PERMUTE, Plan, check_plan, expected_tiles, simulate

EV, MAXM = 2, 6


def hand_plan():
    # M tiles 0, 1 (pair 0 -> queue 0): 40 and 20 rows; M tile 2 (pair 1 -> queue 1): 300 rows (tall); tile 3 unused
    rows = np.array([40, 20, 300, 0], dtype=np.int32)
    q0 = [(PERMUTE, 0, 0, -1, 0), (PERMUTE, 1, 0, -1, 0), (PERMUTE, 0, 1, -1, 0),
          (GEMM1, 0, 0, EV + 0, 2), (GEMM1, 0, 1, EV + 1, 1), (GEMM1, 1, 0, EV + 0, 2), (GEMM1, 1, 1, EV + 1, 1),
          (GEMM2, 0, 0, EV + MAXM + 0, 2), (GEMM2, 0, 1, EV + MAXM + 1, 2)]
    q1 = [(PERMUTE, i, 2, -1, 0) for i in range(10)]
    q1 += [(GEMM1, i, 2, EV + 2, 10) for i in range(3)]
    q1 += [(GEMM2, i, 2, EV + MAXM + 2, 3) for i in range(2)]
    return Plan(4, rows, [q0, q1] + [[] for _ in range(6)], 4, EV, MAXM)


def exp_of(plan):
    return expected_tiles(plan, n1_wide=2, n1_tall=3, n2_wide=1, n2_tall=2, wide_rows=256, perm_rows=32, permute=True)


def test_legal_plan_passes_and_runs_to_completion():
    plan = hand_plan()
    check_plan(plan, exp_of(plan))
    assert simulate(plan, 1) > 0 and simulate(plan, 4) > 0


def _mutations():
    def thr_up(p): p.queues[0][3] = (GEMM1, 0, 0, EV + 0, 3)
    def thr_down(p): p.queues[1][10] = (GEMM1, 0, 2, EV + 2, 9)
    def wrong_event(p): p.queues[0][7] = (GEMM2, 0, 0, EV + MAXM + 1, 2)
    def consumer_first(p): p.queues[0].insert(2, p.queues[0].pop(7))           # GEMM-2 ahead of its GEMM-1 tiles
    def dropped(p): p.queues[1].pop(4)
    def doubled(p): p.queues[0].append(p.queues[0][4])
    def wrong_queue(p): p.queues[2].append(p.queues[1].pop())
    def total_off(p): p.gemm2_total += 1
    def phantom(p): p.queues[3].append((GEMM1, 0, 3, -1, 0))                   # task on a tile without rows
    return [thr_up, thr_down, wrong_event, consumer_first, dropped, doubled, wrong_queue, total_off, phantom]


@pytest.mark.parametrize("mutate", _mutations(), ids=lambda f: f.__name__)
def test_planted_mistake_is_named(mutate):
    plan = copy.deepcopy(hand_plan())
    mutate(plan)
    with pytest.raises(AssertionError):
        check_plan(plan, exp_of(hand_plan()))


def test_interpreter_reports_deadlock():
    plan = copy.deepcopy(hand_plan())
    plan.queues[0][3] = (GEMM1, 0, 0, EV + 0, 3)       # waits for a third PERMUTE part that does not exist
    with pytest.raises(AssertionError, match="deadlock"):
        simulate(plan, 1)
    plan = copy.deepcopy(hand_plan())
    plan.queues[0].insert(0, plan.queues[0].pop(7))    # a consumer at the head of an in-order queue with one worker
    with pytest.raises(AssertionError, match="deadlock"):
        simulate(plan, 1)


def _map_plan(tiles):
    """tiles: list of (expert, row0, rows) per map entry."""
    from plan_check import Plan
    return Plan(len(tiles), np.array([t[2] for t in tiles]), [[] for _ in range(8)], 0, 0, len(tiles),
                np.array([t[0] for t in tiles]), np.array([t[1] for t in tiles]))


def test_tile_map_check_accepts_a_legal_map_and_names_planted_mistakes():
    from plan_check import check_tile_map
    counts = [300, 700, 350]          # one wide tile, three siblings, one tall tile (wide 320, tall 384)
    legal = [(2, 1000, 350), (2, 1000, 0),                   # slot 0: the tall tile owns it
             (1, 300, 256), (1, 556, 256),                   # slot 1: siblings
             (0, 0, 300), (0, 0, 0),                         # slot 2: a single
             (1, 812, 188), (0, 0, 0)]                       # slot 3: the third sibling
    assert check_tile_map(_map_plan(legal), counts, 320, 384) == [1, 2, 1, 1, 0, 0, 0, 0]
    gap = list(legal); gap[6] = (1, 812, 187)                # a row nobody computes
    with pytest.raises(AssertionError, match="not covered exactly once"):
        check_tile_map(_map_plan(gap), counts, 320, 384)
    twice = list(legal); twice[3] = (1, 500, 312)            # rows 500..555 in two tiles
    with pytest.raises(AssertionError, match="not covered exactly once"):
        check_tile_map(_map_plan(twice), counts, 320, 384)
    stray = list(legal); stray[4] = (0, 100, 300)            # runs into the next expert's rows
    with pytest.raises(AssertionError, match="outside expert"):
        check_tile_map(_map_plan(stray), counts, 320, 384)
    shared = list(legal); shared[1] = (0, 0, 300); shared[4] = (0, 0, 0)   # a tall tile must not share its slot
    with pytest.raises(AssertionError, match="slot of their own"):
        check_tile_map(_map_plan(shared), counts, 320, 384)
    lopsided = [(0, 0, 256), (0, 256, 44), (1, 300, 256), (1, 556, 0)] + [(0, 0, 0)] * 12 + [(1, 556, 256), (1, 812, 188)]
    with pytest.raises(AssertionError, match="tiles per XCD"):   # slots 0 and 8 both belong to XCD 0
        check_tile_map(_map_plan(lopsided), [300, 700], 320, 384)


def test_halved_last_round_of_gemm2_tasks():
    """A queue whose last round of GEMM-2 tasks is at most half full carries those tiles as 128-column halves."""
    from plan_check import NARROW
    rows = np.array([200, 100], dtype=np.int32)          # one pair in queue 0, both wide
    # 3 GEMM-2 N tiles per M tile (5 halves: the last tile has only its first half) -> 6 wide tasks; 4 workers: tail 2
    g1 = [(GEMM1, 0, 0, -1, 0), (GEMM1, 0, 1, -1, 0)]
    whole = [(GEMM2, nt, m, EV + MAXM + m, 1) for nt in range(3) for m in range(2)]
    halved = whole[:4] + [(GEMM2 | NARROW, 4, 0, EV + MAXM, 1), (GEMM2 | NARROW, 4, 1, EV + MAXM + 1, 1)]
    def plan_of(g2):
        return Plan(2, rows, [g1 + g2] + [[] for _ in range(7)], len(g2), EV, MAXM)
    exp = lambda p: expected_tiles(p, n1_wide=1, n1_tall=1, n2_wide=3, n2_tall=5, wide_rows=256, perm_rows=32, permute=False)
    p = plan_of(halved)
    check_plan(p, exp(p), workers_per_queue=4)
    simulate(p, 4)
    with pytest.raises(AssertionError, match="not halved"):
        check_plan(plan_of(whole), exp(p), workers_per_queue=4)       # the rule asks for halves here
    check_plan(plan_of(whole), exp(p), workers_per_queue=3)           # 6 tasks on 3 workers: two full rounds
    with pytest.raises(AssertionError, match="halved GEMM-2 tasks, but"):
        check_plan(p, exp(p), workers_per_queue=3)
    both = plan_of(halved + [(GEMM2, 2, 0, EV + MAXM, 1)])            # a tile as halves AND as a whole
    with pytest.raises(AssertionError, match="once as a whole or as halves"):
        check_plan(both, exp(p))
    past = plan_of(halved + [(GEMM2 | NARROW, 5, 0, EV + MAXM, 1)])   # a half past the last column
    with pytest.raises(AssertionError, match="past the last column"):
        check_plan(past, exp(p))
    # a middle tile (nt = 1) halved but with its second half missing
    lone = plan_of([t for t in whole if t[1] != 1 or t[2] != 0] + [(GEMM2 | NARROW, 2, 0, EV + MAXM, 1)])
    with pytest.raises(AssertionError, match="second half missing"):
        check_plan(lone, exp(p))
