"""Timing checks of the planner, apart from the parity suite: the structure the library picks for a
shape (block tile, number of K slices) is compared with a search by timing over all of them.  These
are the only tests whose verdict depends on a clock; a measurement disturbed by another tenant of the
machine is taken again before it decides."""
import pytest

pytestmark = pytest.mark.gpu


def test_planning_rule_is_close_to_the_timed_search():
    """The fixed split-K rule against a search by timing (paper: structure first, counters later): for a
    few shapes the library's choice is within 25 % of the fastest slice count found."""
    from paper_2604_01489_amd import tune
    for M, N, K in [(256, 256, 8192), (1024, 2048, 4096), (2048, 2048, 2048)]:
        for attempt in range(3):            # launches of 15 us: one disturbed measurement must not decide
            best, auto, table = tune.sweep_split_k(M, N, K, reps=20)
            times = dict(table)
            print(f"{M}x{N}x{K}: auto {auto}, fastest {best}, table {[(s, round(t, 1)) for s, t in table]}", flush=True)
            if times[auto] <= 1.25 * times[best]:
                break
        assert times[auto] <= 1.25 * times[best], (M, N, K, auto, best, table)


def test_planning_rules_against_the_search_over_tile_and_slices():
    """Both structural choices together (block tile and K slices): the library's own plan is within 25 % of
    the fastest structure the timed search finds, on shapes from one tile row to many rounds of tiles."""
    from paper_2604_01489_amd import tune
    for M, N, K in [(512, 512, 16384), (1024, 1024, 1024), (4096, 4096, 1024), (384, 8192, 2048)]:
        for attempt in range(3):            # as above
            best, own, table = tune.sweep_structure(M, N, K, reps=15)
            print(f"{M}x{N}x{K}: own {own[0]} {own[1]:.1f} us, fastest {best}", flush=True)
            if own[1] <= 1.25 * best[2]:
                break
        assert own[1] <= 1.25 * best[2], (M, N, K, own, best, table)
