"""The tensor-operation replay (tests/bcast_sim_torch.py) against the numpy one on the CPU: same verdicts on
correct tables and on tables with planted mistakes."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

import bcast_sim
import bcast_sim_torch


def _both(p, n, recv, send):
    verdicts = []
    for sim, conv in ((bcast_sim.simulate, lambda a: a), (bcast_sim_torch.simulate, torch.from_numpy)):
        try:
            verdicts.append(sim(p, n, conv(recv.copy()), conv(send.copy())))
        except bcast_sim.ScheduleError:
            verdicts.append("error")
    assert verdicts[0] == verdicts[1], (p, n, verdicts)
    return verdicts[0]


def test_same_verdict_on_correct_tables(oracle):
    for p in (2, 3, 5, 9, 20, 31, 32, 33, 100, 257, 1000):
        recv, send = oracle.sched_range(p, 0, 0, p)
        for n in (1, 2, 3, 7, 12):
            assert _both(p, n, recv, send) == n - 1 + recv.shape[1]


def test_same_verdict_on_planted_mistakes(oracle):
    rng = np.random.default_rng(5)
    caught = 0
    for p in (9, 20, 33, 100, 257):
        recv, send = oracle.sched_range(p, 0, 0, p)
        q = recv.shape[1]
        for trial in range(12):
            r2, s2 = recv.copy(), send.copy()
            r, k = int(rng.integers(0, p)), int(rng.integers(0, q))
            kind = trial % 4
            if kind == 0:                                  # one receive entry changed (and its sender's, consistently)
                r2[r, k] = r2[r, k] - 1 if r2[r, k] > -q else r2[r, k] + 1
                skips = bcast_sim.closed_form_skips(p)
                s2[(r - skips[k]) % p, k] = r2[r, k]
            elif kind == 1:                                # send and receive sides disagree
                s2[r, k] += 1
            elif kind == 2:                                # two slots of a row exchanged on both sides
                k2 = (k + 1) % q
                if q < 2:
                    continue
                r2[:, [k, k2]] = r2[:, [k2, k]]
                s2[:, [k, k2]] = s2[:, [k2, k]]
            else:                                          # a whole row replaced by the root's
                r2[r] = r2[0]
            for n in (1, 3, q + 2):
                if _both(p, n, r2, s2) == "error":
                    caught += 1
    assert caught > 100
