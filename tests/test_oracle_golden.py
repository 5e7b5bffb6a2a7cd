"""The oracle against the values the paper prints (Tables 1-5 and the skips in their captions)."""
import numpy as np
import pytest

from conftest import load_table
from bcast_sim import simulate, ScheduleError

TABLES = ["table1_p20", "table2_p33", "table3_p32", "table4_p31", "table5_left_p9"]

# captions of Tables 1-4
PRINTED_SKIPS = {
    20: [1, 2, 3, 5, 10, 20],
    33: [1, 2, 3, 5, 9, 17, 33],
    32: [1, 2, 4, 8, 16, 32],
    31: [1, 2, 4, 8, 16, 31],
}


@pytest.mark.parametrize("p", sorted(PRINTED_SKIPS))
def test_skips_match_captions(oracle, p):
    assert oracle.skips(p).tolist() == PRINTED_SKIPS[p]


@pytest.mark.parametrize("name", TABLES)
def test_definition_level_matches_table(oracle, name):
    p, q, bb, recv, send = load_table(name)
    obb, orecv, osend = oracle.sched_definition(p)
    assert (obb[1:] == bb[1:]).all()            # the root cell is not a baseblock
    assert (orecv == recv).all()
    assert (osend == send).all()


@pytest.mark.parametrize("name", TABLES)
def test_per_rank_level_matches_table(oracle, name):
    p, q, bb, recv, send = load_table(name)
    for r in range(1, p):
        assert oracle.baseblock(p, r) == bb[r]
    orecv, osend = oracle.sched_range(p)
    assert (orecv == recv).all()
    assert (osend == send).all()
    for r in range(p):                          # Alg. 4 / Alg. 5 one rank at a time
        assert (oracle.recvsched(p, r) == recv[r]).all()
        assert (oracle.sendsched(p, r) == send[r]).all()


@pytest.mark.parametrize("name", TABLES + ["table5_right_p9"])
@pytest.mark.parametrize("n", [1, 2, 3, 4, 5, 8, 13])
def test_printed_tables_pass_the_simulator(name, n):
    p, q, bb, recv, send = load_table(name)
    assert simulate(p, n, recv, send) == n - 1 + q


def test_alternative_p9_schedule_differs_in_its_four_bold_cells(oracle):
    """Table 5 right is valid but is not what the construction emits."""
    p, q, bb, recv, send = load_table("table5_right_p9")
    orecv, osend = oracle.sched_range(p)
    dr = sorted((int(r), int(k)) for r, k in zip(*np.nonzero(orecv != recv)))
    ds = sorted((int(r), int(k)) for r, k in zip(*np.nonzero(osend != send)))
    assert dr == [(8, 1), (8, 2)]
    assert ds == [(5, 2), (6, 1)]


def test_simulator_rejects_broken_schedules():
    """The checker is not vacuous: one wrong cell anywhere must be caught."""
    p, q, bb, recv, send = load_table("table1_p20")
    rng = np.random.default_rng(7)
    caught = 0
    trials = 60
    for _ in range(trials):
        r2, s2 = recv.copy(), send.copy()
        tab = r2 if rng.integers(2) else s2
        r, k = int(rng.integers(p)), int(rng.integers(q))
        old = tab[r, k]
        new = old
        while new == old:
            new = int(rng.integers(-q, q))
        tab[r, k] = new
        try:
            simulate(p, 6, r2, s2)
        except ScheduleError:
            caught += 1
    assert caught == trials
