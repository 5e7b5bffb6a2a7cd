"""The oracle against cross-check values of an independent implementation (tests/golden/crosscheck_independent.txt):
hashes of whole tables for eleven p, and single rows at p = 2^20+1 and p = 2^27-1.  Not the paper's values."""
import os

import numpy as np

from conftest import GOLDEN


def _fnv1a32(a):
    h = 0x811C9DC5
    for byte in np.ascontiguousarray(a, dtype="<i4").tobytes():
        h = ((h ^ byte) * 0x01000193) & 0xFFFFFFFF
    return h


def _lines(kind):
    with open(os.path.join(GOLDEN, "crosscheck_independent.txt")) as f:
        for line in f:
            tok = line.split()
            if tok and tok[0] == kind:
                yield tok[1:]


def test_whole_table_hashes(oracle):
    seen = 0
    for p, q, h_recv, h_send, total in _lines("hash"):
        p, q = int(p), int(q)
        recv, send = oracle.sched_range(p, 0, 0, p)
        assert recv.shape == (p, q)
        assert "%08x" % _fnv1a32(recv) == h_recv, p
        assert "%08x" % _fnv1a32(send) == h_send, p
        assert int(recv.sum(dtype=np.int64)) == int(total) == int(send.sum(dtype=np.int64)), p
        seen += 1
    assert seen == 11


def test_single_rows_at_large_p(oracle):
    seen = 0
    for tok in _lines("row"):
        p, r, which = int(tok[0]), int(tok[1]), tok[2]
        want = np.array([int(v) for v in tok[3:]], dtype=np.int32)
        got = oracle.recvsched(p, r) if which == "recv" else oracle.sendsched(p, r)
        assert np.array_equal(np.asarray(got), want), (p, r, which)
        seen += 1
    assert seen == 10
