"""The oracle's tables replayed round by round, and its expansion against the replay's own round arithmetic."""
import numpy as np
import pytest

from bcast_sim import simulate, _round_blocks


def test_sweep_every_p_to_1024_n_1_to_8(oracle):
    """Every p in 2..1024, every rank, n = 1..8 blocks: correct and finished in exactly n-1+q rounds."""
    for p in range(2, 1025):
        recv, send = oracle.sched_range(p)
        q = recv.shape[1]
        for n in range(1, 9):
            assert simulate(p, n, recv, send) == n - 1 + q


@pytest.mark.parametrize("p", [1025, 1535, 2047, 2048, 2049, 4097, 65537, 99999, 100003, 131071])
def test_sampled_larger_p(oracle, p):
    recv, send = oracle.sched_range(p, threads=4)
    q = recv.shape[1]
    for n in (1, 2, 3, q - 1, q, q + 1, 2 * q + 3):
        simulate(p, n, recv, send)


def test_one_million_ranks_non_power_of_two(oracle):
    p = (1 << 20) + 1
    recv, send = oracle.sched_range(p, threads=8)
    for n in (1, 2, 5):
        simulate(p, n, recv, send)


def test_rooted_schedule_broadcasts_from_that_root(oracle):
    """Rows under root rho, read in the renumbered order, are a valid broadcast from rank rho."""
    for p, root in [(20, 7), (33, 32), (1000, 999), (4097, 1)]:
        recv, send = oracle.sched_range(p, root=root)
        order = (np.arange(p) + root) % p               # virtual rank v lives at real rank (v + root) mod p
        for n in (1, 4, 9):
            simulate(p, n, recv[order], send[order])


@pytest.mark.parametrize("p,n", [(2, 1), (2, 5), (3, 1), (9, 4), (20, 1), (20, 6), (33, 7), (33, 12), (1000, 37),
                                 (65537, 3), (1, 4)])
def test_expand_equals_replay_arithmetic(oracle, p, n):
    recv, send = oracle.sched_range(p)
    q = oracle.q_of(p)
    R = n - 1 + q
    er, es = oracle.expand(p, n, recv), oracle.expand(p, n, send)
    assert er.shape == (p, R) and es.shape == (p, R)
    if q == 0:
        assert (er == -1).all() and (es == -1).all()
        return
    x = (q - R % q) % q
    assert (x + R) % q == 0
    assert (er == _round_blocks(recv, n, q, x)).all()
    assert (es == _round_blocks(send, n, q, x)).all()


def test_expand_structure(oracle):
    """Alg. 6 caption and the text under it: the x dummy rounds never show; every real block is in [0, n-1];
    a non-root rank's receive row lists every block exactly once; the root sends blocks 0, 1, ..., n-1 and
    then repeats n-1.  (The root keeps a receive row too: its neighbours' send rows are read off it.)"""
    for p, n in [(20, 1), (20, 3), (20, 11), (33, 6), (33, 20), (257, 9), (1000, 64)]:
        recv, send = oracle.sched_range(p)
        q = oracle.q_of(p)
        R = n - 1 + q
        er, es = oracle.expand(p, n, recv), oracle.expand(p, n, send)
        assert er.min() >= -1 and er.max() == n - 1 and es.min() >= -1 and es.max() == n - 1
        assert es[0].tolist() == [min(j, n - 1) for j in range(R)]
        for r in range(1, p):
            got = er[r][er[r] >= 0]
            assert sorted(got.tolist()) == list(range(n)), (p, n, r)
