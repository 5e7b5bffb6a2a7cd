"""Alg. 7 (regular allgather) and Alg. 8 (census) plans: the oracle's and the library's host functions, replayed for
all processes against the definitions of the two collectives."""
import numpy as np
import pytest


def run_regular_allgather(p, plan_of):
    """Every process starts with its own block in buffer[0]; afterwards buffer[i] must be the block of (r+i) mod p."""
    plans = [plan_of(p, r) for r in range(p)]
    q = (p - 1).bit_length()
    buf = np.full((p, p), -1, dtype=np.int64)
    buf[:, 0] = np.arange(p)
    have = np.ones(p, dtype=np.int64)                       # blocks held so far
    for k in range(q):
        new = buf.copy()
        for r in range(p):
            to, frm, cnt, first = (plans[r][i][k] for i in range(4))
            assert plans[frm][0][k] == r and plans[to][1][k] == r          # the pattern is symmetric
            assert cnt <= have[frm] and first == have[r]                   # sends what it has, appends at the end
            new[r, first:first + cnt] = buf[frm, 0:cnt]
        buf = new
        have = have + np.array([plans[r][2][k] for r in range(p)])
    for r in range(p):
        assert np.array_equal(buf[r], (r + np.arange(p)) % p), (p, r)


def run_census(p, plan_of):
    """x_r = 3^r mod a prime; afterwards every process must hold the sum of all x."""
    plans = [plan_of(p, r) for r in range(p)]
    q = (p - 1).bit_length()
    x = np.array([pow(3, r, 1000003) for r in range(p)], dtype=np.int64)
    S = np.zeros(p, dtype=np.int64)
    for k in range(q):
        out = np.array([S[r] + (x[r] if plans[r][2][k] else 0) for r in range(p)])
        newS = S.copy()
        for r in range(p):
            to, frm = plans[r][0][k], plans[r][1][k]
            assert plans[frm][0][k] == r and plans[to][1][k] == r
            newS[r] = S[r] + out[frm]
        S = newS
    assert (S + x == x.sum()).all(), p


PS = list(range(1, 70)) + [100, 127, 128, 129, 255, 257, 1000]


def test_oracle_plans_realise_the_collectives(oracle):
    for p in PS:
        run_regular_allgather(p, oracle.allgather_plan)
        run_census(p, oracle.census_plan)


def test_library_plans_equal_the_oracle_and_realise_the_collectives(oracle):
    import paper_2205_10072_amd as bcs
    for p in PS:
        run_regular_allgather(p, bcs.bcs_allgather_plan)
        run_census(p, bcs.bcs_census_plan)
    rng = np.random.default_rng(5)
    for p in [1, 2, 3, 20, 33, 1048577, 134217727, 2**31 - 1] + [int(v) for v in rng.integers(2, 2**31 - 1, 50)]:
        for r in {0, p - 1, p // 2, int(rng.integers(0, p))}:
            assert [list(a) for a in oracle.allgather_plan(p, r)] == bcs.bcs_allgather_plan(p, r)
            assert [list(a) for a in oracle.census_plan(p, r)] == bcs.bcs_census_plan(p, r)
    L = bcs.lib()
    assert L.bcs_allgather_plan(0, 0, None, None, None, None) == bcs.EINVAL
    assert L.bcs_census_plan(5, 5, None, None, None) == bcs.EINVAL
