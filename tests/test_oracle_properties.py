"""The oracle against what the paper and plain mathematics fix: closed forms, lemmas,
brute force on small p, and the structure of a schedule row."""
import numpy as np
import pytest

from bcast_sim import closed_form_skips


def test_skips_closed_form_and_lemma1(oracle):
    """Alg. 1 halves with rounding up, so skips[k] = ceil(p / 2^(q-k)); Lemma 1."""
    rng = np.random.default_rng(1)
    ps = list(range(1, 3000)) + [int(v) for v in rng.integers(3000, 2**31 - 1, 3000)] + [2**31 - 1, 2**30, 2**30 + 1]
    for p in ps:
        s = oracle.skips(p).tolist()
        q = len(s) - 1
        assert q == (p - 1).bit_length()
        assert s == closed_form_skips(p)
        assert s[0] == 1 and s[q] == p
        if q >= 1:
            assert s[1] == 2
        acc = 0
        for k in range(q):
            assert 2 * s[k] >= s[k + 1] and 2 * s[k] - s[k + 1] in (0, 1)      # Lemma 1, first claim
            acc += s[k]
            assert acc >= s[k + 1] - 1                                        # Lemma 1, second claim
        assert sum(s[k + 1] - s[k] for k in range(q)) == p - 1                # Lemma 1, third claim


def test_baseblock_alg2_equals_linear_recipe(oracle):
    for p in list(range(2, 700)) + [1000, 1023, 1024, 1025, 2047, 2048, 2049, 4097]:
        bb = oracle.baseblocks_linear(p)
        assert bb[0] == -1
        got = [oracle.baseblock(p, r) for r in range(1, p)]
        assert got == bb[1:].tolist(), p
        # neighbours never share a baseblock (argument under Lemma 2)
        assert (bb[1:-1] != bb[2:]).all()


def test_power_of_two_baseblock_is_trailing_zero_count(oracle):
    """For p = 2^q the skips are powers of two and the first q rounds are a binomial tree."""
    for q in range(1, 13):
        p = 1 << q
        bb = oracle.baseblocks_linear(p)
        want = [(r & -r).bit_length() - 1 for r in range(1, p)]
        assert bb[1:].tolist() == want


def test_rangeblocks_fast_equals_scan(oracle):
    rng = np.random.default_rng(2)
    for p in list(range(2, 130)) + [255, 256, 257, 511, 513, 777, 1000, 1024, 1025, 2047]:
        bb = oracle.baseblocks_linear(p)
        if p < 40:
            pairs = [(a, b) for a in range(-p - 2, p + 3) for b in range(a - 1, a + p + 2)]
        else:
            a = rng.integers(-2 * p, 2 * p, 400)
            ln = rng.integers(0, p + 3, 400)
            pairs = [(int(x), int(x + l - 1)) for x, l in zip(a, ln)]
        for a, b in pairs:
            assert oracle.rangeblocks(p, a, b) == oracle.rangeblocks_scan(p, bb, a, b), (p, a, b)


def test_lemma2_distinct_blocks_in_any_range(oracle):
    """Lemma 2: any range of skips[k] ranks holds >= k baseblocks; 1 + sum_{i<k} skips[i] ranks hold >= k+1.
    Ranges may run past p-1 ("virtually doubling" the ranks); the root, which owns every block, then counts
    as one more distinct entry."""
    for p in list(range(2, 200)) + [255, 256, 257, 500]:
        bb = oracle.baseblocks_linear(p)
        s = oracle.skips(p).tolist()
        q = len(s) - 1
        seq = np.concatenate([bb[1:], bb])              # ranks 1..p-1, then 0 (marked -1), 1..p-1
        for k in range(1, q + 1):
            for size, need in ((s[k], k), (1 + sum(s[:k]), k + 1)):
                if size > p - 1:
                    continue
                for a in range(p - 1):
                    assert len(set(seq[a:a + size].tolist())) >= need, (p, k, size, a)


@pytest.mark.parametrize("general_only", [False, True])
def test_per_rank_equals_definition_small_p(oracle, general_only):
    """Alg. 2 + the O(q) range routine + Alg. 4 per rank == linear recipe + range scanning."""
    ps = list(range(1, 400)) + [511, 512, 513, 767, 1000, 1023, 1024, 1025, 1535, 2047, 2048]
    for p in ps:
        bb, recv, send = oracle.sched_definition(p, general_only=general_only)
        frecv, fsend = oracle.sched_range(p)
        assert (frecv == recv).all(), p
        assert (fsend == send).all(), p


def test_printed_special_cases_equal_general_rule(oracle):
    """The i = 0 and i = q-1 cases of Alg. 4 are the range rule in disguise."""
    rng = np.random.default_rng(3)
    for p in range(2, 1200):
        for r in range(p) if p < 300 else rng.integers(0, p, 40):
            r = int(r)
            assert (oracle.recvsched(p, r) == oracle.recvsched(p, r, general_only=True)).all(), (p, r)
    for p in [4097, 65537, 99999, 1048577, 134217727, 2**31 - 1, 2**30 + 12345]:
        for r in [0, 1, 2, p - 1, p // 2, p // 3] + [int(v) for v in rng.integers(0, p, 200)]:
            assert (oracle.recvsched(p, r) == oracle.recvsched(p, r, general_only=True)).all(), (p, r)


def test_recv_prefixes_are_stable(oracle):
    """recvsched(r, k) is the first k+1 entries of the full row (needed by Alg. 5)."""
    for p in [9, 20, 33, 100, 1000]:
        for r in range(p):
            full = oracle.recvsched(p, r)
            for k in range(len(full)):
                assert (oracle.recvsched(p, r, k) == full[:k + 1]).all()


def _check_rows(p, q, ranks, recv, send, bbs):
    for r, rr, ss, bb in zip(ranks, recv, send, bbs):
        if r == 0:
            assert sorted(rr.tolist()) == list(range(-q, 0))          # root row: a permutation of -q..-1
            assert ss.tolist() == list(range(q))                      # root sends block k in round k
            continue
        nonneg = rr[rr >= 0]
        assert nonneg.tolist() == [bb]                                 # the baseblock, once
        assert sorted((rr[rr < 0] + q).tolist()) == [b for b in range(q) if b != bb]
        for k in range(q):                                             # a sent block was received earlier,
            assert ss[k] in rr[:k] or ss[k] == bb - q                  # or is last phase's baseblock


def test_row_structure_all_ranks_small_p(oracle):
    """Section 2, end: a receive row is the baseblock once plus q-1 different earlier-phase blocks."""
    for p in list(range(2, 300)) + [1000, 1024, 1025, 4097]:
        recv, send = oracle.sched_range(p)
        q = recv.shape[1]
        bbs = [-1] + [oracle.baseblock(p, r) for r in range(1, p)]
        _check_rows(p, q, range(p), recv, send, bbs)


def test_row_structure_sampled_large_p(oracle):
    rng = np.random.default_rng(4)
    for p in [65537, 1048577, 134217727, 2**31 - 1, 2**30, 1500000001]:
        q = oracle.q_of(p)
        ranks = [0, 1, 2, 3, p - 1, p - 2, p // 2, p // 2 + 1] + [int(v) for v in rng.integers(0, p, 150)]
        recv = np.array([oracle.recvsched(p, r) for r in ranks])
        send = np.array([oracle.sendsched(p, r) for r in ranks])
        bbs = [oracle.baseblock(p, r) if r else -1 for r in ranks]
        _check_rows(p, q, ranks, recv, send, bbs)


def _pow2_recv(q, r):
    """Closed form for p = 2^q, read off the structure of Table 3: the home round (top bit) takes the
    baseblock; a round whose bit is set in r takes the next set bit above it; other rounds take their own index."""
    if r == 0:
        return [i - q for i in range(q)]
    h = r.bit_length() - 1
    row = []
    for i in range(q):
        if i == h:
            row.append((r & -r).bit_length() - 1)
        elif i < h and (r >> i) & 1:
            above = r >> (i + 1)
            row.append(i + 1 + (above & -above).bit_length() - 1 - q)
        else:
            row.append(i - q)
    return row


def test_power_of_two_closed_form(oracle):
    for q in range(1, 12):
        p = 1 << q
        recv, send = oracle.sched_range(p)
        want = np.array([_pow2_recv(q, r) for r in range(p)])
        assert (recv == want).all(), q
        for k in range(q):
            assert (send[:, k] == np.roll(want[:, k], -(1 << k))).all()
    rng = np.random.default_rng(5)
    for q in (20, 27, 30):
        p = 1 << q
        for r in [0, 1, p - 1, p // 2] + [int(v) for v in rng.integers(0, p, 300)]:
            assert oracle.recvsched(p, r).tolist() == _pow2_recv(q, r)
            want_send = [_pow2_recv(q, (r + (1 << k)) % p)[k] for k in range(q)]
            assert oracle.sendsched(p, r).tolist() == want_send


def test_alg5_equals_neighbour_lookup(oracle):
    """Send rows of a partial rank range (Alg. 5) equal the rows of the all-ranks look-up (Alg. 9)."""
    for p in [2, 3, 9, 20, 33, 100, 257, 1000, 4097]:
        recv, send = oracle.sched_range(p)
        lo, hi = p // 3, min(p, p // 3 + 50)
        precv, psend = oracle.sched_range(p, r0=lo, r1=hi)
        assert (precv == recv[lo:hi]).all()
        assert (psend == send[lo:hi]).all()


def test_rooted_rows_are_rotations(oracle):
    """Another root: renumber the ranks by subtracting the root mod p (Section 2, after Alg. 2)."""
    for p, root in [(9, 4), (20, 19), (33, 1), (1000, 123), (4097, 4096)]:
        recv, send = oracle.sched_range(p)
        rrecv, rsend = oracle.sched_range(p, root=root)
        assert (rrecv == np.roll(recv, root, axis=0)).all()
        assert (rsend == np.roll(send, root, axis=0)).all()
        lo, hi = 2, min(p, 40)
        precv, psend = oracle.sched_range(p, root=root, r0=lo, r1=hi)
        assert (precv == rrecv[lo:hi]).all() and (psend == rsend[lo:hi]).all()


def test_batch_rows_and_padding(oracle):
    rng = np.random.default_rng(6)
    ps = np.array([1, 2, 3, 9, 20, 33, 1000, 65537, 2**31 - 1, 1048577], dtype=np.int32)
    rs = np.array([int(rng.integers(0, p)) for p in ps], dtype=np.int32)
    roots = np.array([int(rng.integers(0, p)) for p in ps], dtype=np.int32)
    recv, send, qv = oracle.sched_batch(ps, rs, roots)
    for i, (p, r, root) in enumerate(zip(ps.tolist(), rs.tolist(), roots.tolist())):
        q = oracle.q_of(p)
        assert qv[i] == q
        v = (r - root) % p
        assert recv[i, :q].tolist() == oracle.recvsched(p, v).tolist()
        assert send[i, :q].tolist() == oracle.sendsched(p, v).tolist()
        assert (recv[i, q:] == oracle.PAD).all() and (send[i, q:] == oracle.PAD).all()


def test_degenerate_p(oracle):
    """p = 1: no rounds, empty rows.  p = 2: both special cases of Alg. 4 apply at once."""
    recv, send = oracle.sched_range(1)
    assert recv.shape == (1, 0) and send.shape == (1, 0)
    recv, send = oracle.sched_range(2)
    assert recv.tolist() == [[-1], [0]]
    assert send.tolist() == [[0], [-1]]
