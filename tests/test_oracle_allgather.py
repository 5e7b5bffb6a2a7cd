"""Alg. 9's index arithmetic in the oracle: replayed as a whole allgather, and tied to the broadcast tables."""
import numpy as np
import pytest

from allgather_sim import simulate_allgather, AllgatherError


def all_tables(oracle, p, n):
    tabs = [oracle.allgather_tables(p, n, r) for r in range(p)]
    return np.array([t[0] for t in tabs]), np.array([t[1] for t in tabs])


@pytest.mark.parametrize("p", [2, 3, 4, 5, 7, 9, 16, 20, 31, 33, 48, 65])
def test_allgather_completes_for_every_process(oracle, p):
    q = oracle.q_of(p)
    for n in sorted({1, 2, 3, q - 1, q, q + 1, 2 * q + 1} - {0, -1}):
        pack, unpack = all_tables(oracle, p, n)
        assert simulate_allgather(p, n, pack, unpack) == n - 1 + q


def test_allgather_tables_are_rotated_broadcast_tables(oracle):
    """Process r treats root j as the virtual rank (r - j + p) mod p of a broadcast rooted at 0 (Section 2.5)."""
    for p, n in [(9, 4), (20, 7), (33, 2), (100, 11)]:
        recv, send = oracle.sched_range(p)
        er, es = oracle.expand(p, n, recv), oracle.expand(p, n, send)
        for r in (0, 1, p // 2, p - 1):
            pack, unpack = oracle.allgather_tables(p, n, r)
            rows = (r - np.arange(p)) % p
            assert np.array_equal(pack, es[rows].T)
            assert np.array_equal(unpack, er[rows].T)


def test_simulator_rejects_a_broken_table(oracle):
    p, n = 20, 6
    pack, unpack = all_tables(oracle, p, n)
    rng = np.random.default_rng(3)
    caught = 0
    for _ in range(30):
        a, b = pack.copy(), unpack.copy()
        tab = a if rng.integers(2) else b
        r, j, root = int(rng.integers(p)), int(rng.integers(tab.shape[1])), int(rng.integers(p))
        tab[r, j, root] = (tab[r, j, root] + 1 + int(rng.integers(n))) % (n + 1) - 1
        if np.array_equal(a, pack) and np.array_equal(b, unpack):
            caught += 1
            continue
        try:
            simulate_allgather(p, n, a, b)
        except AllgatherError:
            caught += 1
    assert caught == 30


def test_degenerate_sizes(oracle):
    pack, unpack = oracle.allgather_tables(1, 4, 0)
    assert pack.shape == (3, 1) and (pack == -1).all() and (unpack == -1).all()
    pack, unpack = oracle.allgather_tables(2, 1, 1)
    assert pack.tolist() == [[-1, 0]] and unpack.tolist() == [[0, -1]]
