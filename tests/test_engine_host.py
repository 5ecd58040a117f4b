"""Host logic of the engine that needs no GPU: the choice of streams from a table of pairwise clashes."""
import itertools
import random

from paper_2504_14775_amd.engine import pick_independent


def table(total, queue_of):
    """Two candidates clash when they sit on the same hardware queue."""
    return {(i, j): queue_of[i] == queue_of[j] for i, j in itertools.combinations(range(total), 2)}


def test_picks_candidates_on_different_queues():
    queues = [0, 1, 1, 0, 2, 3]                       # the pattern measured on the box: 0-3 and 1-2 collide
    clash = table(6, queues)
    for n in (1, 2, 3, 4):
        got = pick_independent(n, 0, 6, clash)
        assert len(got) == n == len(set(got))
        assert len({queues[k] for k in got}) == n    # pairwise different queues


def test_respects_the_streams_already_in_use():
    queues = [2, 0, 2, 1, 2, 3]                       # candidate 0 is the caller's stream, on queue 2
    clash = table(6, queues)
    got = pick_independent(2, 1, 6, clash)
    assert all(k >= 1 for k in got) and len(set(got)) == 2
    assert 2 not in {queues[k] for k in got} and len({queues[k] for k in got}) == 2


def test_falls_back_when_there_are_not_enough_queues():
    queues = [0, 0, 1, 1, 0]
    got = pick_independent(3, 0, 5, table(5, queues))
    assert len(got) == 3 == len(set(got))
    assert len({queues[k] for k in got}) == 2          # the best there is: both queues used, the rest filled up
    assert pick_independent(0, 0, 5, table(5, queues)) == []


def test_random_tables_give_valid_and_maximal_answers():
    rng = random.Random(3)
    for _ in range(200):
        total, nq = rng.randint(2, 9), rng.randint(1, 4)
        queues = [rng.randrange(nq) for _ in range(total)]
        fixed = rng.randint(0, min(2, total - 1))
        n = rng.randint(1, total - fixed)
        got = pick_independent(n, fixed, total, table(total, queues))
        assert len(got) == n == len(set(got)) and all(fixed <= k < total for k in got)
        free = {queues[k] for k in range(fixed, total)} - {queues[k] for k in range(fixed)}
        want = min(n, len(free))                        # as many distinct free queues as can be had
        used = [queues[k] for k in got if queues[k] in free]
        assert len(set(used)) >= want
