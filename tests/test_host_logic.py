"""CPU tests of the product's host-side logic: the C ABI's symbols and argument checks (no GPU work is
enqueued), and the GPU lanes' construction code compiled for the host, against the oracle."""
import ctypes
import os
import re

import numpy as np
import pytest

import hostcheck

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    import paper_2205_10072_amd as bcs
    header = open(os.path.join(ROOT, "include", "bcsched.h")).read()
    declared = set(re.findall(r"\b(bcs_[a-z_0-9]+)\s*\(", header))
    assert declared == set(bcs.SYMBOLS)
    L = bcs.lib()
    for name in declared:
        assert hasattr(L, name), name


def test_host_helpers_and_argument_checks(oracle):
    import paper_2205_10072_amd as bcs
    L = bcs.lib()
    for p in [1, 2, 3, 20, 31, 32, 33, 1000, 1048577, 134217727, 2**31 - 1]:
        assert bcs.bcs_q(p) == oracle.q_of(p)
        assert bcs.bcs_skips(p) == oracle.skips(p).tolist()
    assert bcs.bcs_rounds(65537, 4096) == 4112
    assert L.bcs_q(0) == bcs.EINVAL and L.bcs_rounds(5, 0) == bcs.EINVAL
    assert L.bcs_skips(0, None) == bcs.EINVAL and L.bcs_skips(5, None) == bcs.EINVAL
    fake = ctypes.c_void_p(256)                 # never dereferenced: every call below must fail first
    bad = [(0, 0, 0, 0), (5, 5, 0, 5), (5, -1, 0, 5), (5, 0, -1, 5), (5, 0, 3, 2), (5, 0, 0, 6)]
    for p, root, r0, r1 in bad:
        assert L.bcs_sched_rooted(p, root, r0, r1, fake, fake, None) == bcs.EINVAL
        assert L.bcs_sched_rooted_ws(p, root, r0, r1, fake, fake, None, 0, None) == bcs.EINVAL
    assert L.bcs_sched(5, 0, 5, None, None, None) == bcs.EINVAL
    assert L.bcs_sched_rooted_ws(5, 0, 0, 5, fake, fake, None, 0, None) == bcs.ENOMEM
    assert L.bcs_sched_workspace_bytes(5, 0, 5, 1) == 3 * 256 + 256  # q rows of one byte an entry, padded to 256; a word a rank
    assert L.bcs_sched_workspace_bytes(5, 0, 1, 1) == 0 and L.bcs_sched_workspace_bytes(5, 0, 5, 0) == 0
    assert L.bcs_sched_workspace_bytes(5, 0, 4, 1) == 0 and L.bcs_sched_workspace_bytes(9, 0, 8, 1) == 256   # 8 * 16 >= 8 * 9
    assert L.bcs_sched_workspace_bytes(1 << 20, 5, 105, 1) == 0
    assert L.bcs_sched_workspace_bytes(5, 0, 6, 1) == bcs.EINVAL
    assert L.bcs_sched_batch(-1, fake, fake, fake, fake, fake, fake, None) == bcs.EINVAL
    assert L.bcs_sched_batch(4, None, fake, fake, fake, fake, fake, None) == bcs.EINVAL
    assert L.bcs_sched_batch(4, fake, fake, fake, None, None, None, None) == bcs.EINVAL
    assert L.bcs_expand(5, 0, 0, 5, fake, fake, fake, fake, None) == bcs.EINVAL
    assert L.bcs_expand(5, 3, 0, 5, fake, None, None, fake, None) == bcs.EINVAL
    assert L.bcs_expand(5, 3, 0, 5, None, None, None, None, None) == bcs.EINVAL
    assert L.bcs_expand_ws(5, 0, 0, 5, fake, fake, fake, fake, None, 0, None) == bcs.EINVAL
    assert L.bcs_expand_ws(5, 3, 0, 6, fake, fake, fake, fake, None, 0, None) == bcs.EINVAL
    assert L.bcs_expand_ws(5, 300, 0, 5, None, None, None, None, fake, 1 << 20, None) == bcs.EINVAL
    assert L.bcs_expand_workspace_bytes(5, 300, 0, 5) == 256         # 6 rows of 12 bytes, padded
    assert L.bcs_expand_workspace_bytes(5, 30, 0, 5) == 0 and L.bcs_expand_workspace_bytes(2, 300, 0, 2) == 0
    assert L.bcs_expand_workspace_bytes(5, 0, 0, 5) == bcs.EINVAL
    assert L.bcs_sched_expand_workspace_bytes(5, 300) == 3 * 256 + 256 + 2 * 256
    assert L.bcs_sched_expand_workspace_bytes(5, 3) == 3 * 256 + 256
    for p, root, n in [(0, 0, 3), (5, 5, 3), (5, -1, 3), (5, 0, 0), (5, 0, 2**31 - 1)]:
        assert L.bcs_sched_expand(p, root, n, fake, fake, fake, fake, None) == bcs.EINVAL
        assert L.bcs_sched_expand_ws(p, root, n, fake, fake, fake, fake, None, 0, None) == bcs.EINVAL
    assert L.bcs_sched_expand(5, 0, 3, None, fake, fake, fake, None) == bcs.EINVAL
    assert L.bcs_sched_expand(5, 0, 3, fake, fake, fake, None, None) == bcs.EINVAL
    assert L.bcs_sched_expand_ws(5, 0, 3, fake, fake, fake, fake, None, 0, None) == bcs.ENOMEM
    assert L.bcs_sched_expand(1, 0, 1, None, None, None, None, None) == bcs.OK      # nothing to write
    for p, n, r in [(0, 3, 0), (5, 0, 0), (5, 3, 5), (5, 3, -1)]:
        assert L.bcs_allgather_tables(p, n, r, fake, fake, None) == bcs.EINVAL
    assert L.bcs_allgather_tables(5, 3, 0, None, None, None) == bcs.EINVAL
    assert L.bcs_pack_plan_rounds(0, 3, 4, fake, fake, fake, fake, None) == bcs.EINVAL
    assert L.bcs_pack_plan_rounds(5, 0, 4, fake, fake, fake, fake, None) == bcs.EINVAL
    assert L.bcs_pack_plan_rounds(5, 3, -1, fake, fake, fake, fake, None) == bcs.EINVAL
    assert L.bcs_pack_plan_rounds(5, 3, 4, fake, fake, None, fake, None) == bcs.EINVAL
    assert L.bcs_pack_plan_rounds(5, 3, 4, fake, fake, ctypes.c_void_p(260), fake, None) == bcs.EINVAL   # misaligned
    assert L.bcs_pack_plan_rounds(5, 3, 0, fake, fake, fake, fake, None) == bcs.OK
    assert L.bcs_pack_round_planned(5, fake, fake, fake, None, 8, None) == bcs.EINVAL
    assert L.bcs_pack_round_planned(5, fake, None, fake, fake, 8, None) == bcs.EINVAL
    assert L.bcs_pack_round_planned(5, fake, fake, fake, fake, 0, None) == bcs.OK
    assert L.bcs_unpack_round_planned(5, fake, fake, fake, fake, -1, None) == bcs.EINVAL
    assert L.bcs_unpack_round_planned(5, fake, fake, fake, None, 0, None) == bcs.OK
    for fn in (L.bcs_allgather_partners, L.bcs_census_partners):
        for p, r0, r1 in [(0, 0, 0), (10, 3, 2), (10, 0, 11), (10, -1, 4)]:
            assert fn(p, r0, r1, fake, fake, None) == bcs.EINVAL
        assert fn(10, 0, 4, None, None, None) == bcs.EINVAL
        assert fn(1, 0, 1, None, None, None) == bcs.OK               # q = 0: no entries
        assert fn(10, 4, 4, fake, None, None) == bcs.OK
    # p = 1 and empty ranges succeed without touching the device
    assert L.bcs_sched(1, 0, 1, fake, fake, None) == bcs.OK
    assert L.bcs_sched(9, 4, 4, fake, fake, None) == bcs.OK
    assert L.bcs_sched_batch(0, fake, fake, fake, fake, fake, fake, None) == bcs.OK
    assert L.bcs_strerror(bcs.EINVAL) == b"invalid argument"
    assert L.bcs_strerror(-99) is not None


def test_binding_refuses_host_tensors():
    import torch
    import paper_2205_10072_amd as bcs
    t = torch.zeros(10, dtype=torch.int32)
    with pytest.raises(TypeError):
        bcs.bcs_sched(2, 0, 2, t, t)


def test_binding_size_checks():
    """The kernels trust the sizes they are given, so the binding must stop a table that is too small.  The check
    itself needs no device; the sizes it is given per call are covered on the GPU (test_gpu_parity)."""
    import torch
    import paper_2205_10072_amd as bcs
    t = torch.zeros(10, dtype=torch.int32)
    bcs._need(t, 10, "t")
    bcs._need(None, 10**12, "absent")
    with pytest.raises(ValueError):
        bcs._need(t, 11, "t")
    assert bcs._rows(3, 9) == 6 and bcs._rows(9, 3) == 0
    assert bcs._expand_sizes(65537, 4096, 65537) == (65537 * 17, 65537 * 4112)
    assert bcs._expand_sizes(1, 5, 1) == (0, 4)
    assert bcs._ws(None) == (None, 0) and bcs._ws(torch.zeros(0)) == (None, 0)
    with pytest.raises(TypeError):
        bcs._ws(torch.zeros(4))                  # host memory is no workspace


def test_misaligned_workspaces_are_refused():
    import paper_2205_10072_amd as bcs
    L = bcs.lib()
    fake = ctypes.c_void_p(4096)
    odd = ctypes.c_void_p(4096 + 64)             # 64-byte aligned only; never dereferenced
    big = 1 << 30
    assert L.bcs_sched_rooted_ws(5, 0, 0, 5, fake, fake, odd, big, None) == bcs.EINVAL
    assert L.bcs_sched_expand_ws(5, 0, 3, fake, fake, fake, fake, odd, big, None) == bcs.EINVAL
    assert L.bcs_allgather_tables_ws(5, 3, 0, fake, fake, odd, big, None) == bcs.EINVAL
    assert L.bcs_allgather_tables_ws(5, 3, 0, fake, fake, None, 0, None) == bcs.ENOMEM


def test_lane_code_range_blocks_equals_scan(oracle):
    rng = np.random.default_rng(11)
    for p in list(range(2, 80)) + [127, 128, 129, 255, 257, 1000, 1023, 1025]:
        bb = oracle.baseblocks_linear(p)
        if p < 40:
            pairs = [(a, b) for a in range(1, p) for b in range(1, p)]
        else:
            pairs = [(int(a), int(b)) for a, b in rng.integers(1, p, (600, 2))]
        for a, b in pairs:
            want = oracle.rangeblocks_scan(p, bb, a, b) if a <= b else 0
            assert hostcheck.range_blocks(p, a, b) == want, (p, a, b)


def test_lane_code_rows_equal_oracle_small_p(oracle):
    for p in list(range(2, 600)) + [1000, 1023, 1024, 1025, 2047, 2049, 4097]:
        recv, _ = oracle.sched_range(p)
        q = recv.shape[1]
        for v in range(p):
            assert (hostcheck.recv_row(p, v)[:q] == recv[v]).all(), (p, v)


def test_lane_code_all_rows_every_p_to_3000(oracle):
    """The digit form's closed expressions are not proved in general: every rank of every p up to 3000
    (BCS_EXHAUSTIVE_P_MAX in the environment raises the limit; 40000 takes eleven minutes on 8 cores)."""
    for p in range(2, int(os.environ.get("BCS_EXHAUSTIVE_P_MAX", "3000")) + 1):
        recv, _ = oracle.sched_range(p, want_send=False, threads=4)
        assert np.array_equal(hostcheck.recv_rows_all(p), recv), p


@pytest.mark.slow
def test_lane_code_all_rows_every_p_to_40000(oracle):
    """The same for every rank of every p up to 40 000 (about eleven minutes on 8 cores)."""
    for p in range(3001, 40001):
        recv, _ = oracle.sched_range(p, want_send=False, threads=8)
        assert np.array_equal(hostcheck.recv_rows_all(p), recv), p


def _p_from_bits(q, shape6, low_clear_levels):
    """p with ceil(log2 p) = q whose top seven bits of p - 1 are 1 and the six bits of shape6 (they fix skips[7]
    and the odd levels below 7) and whose levels >= 7 in low_clear_levels are odd (level k is odd exactly when bit
    q-1-k of p - 1 is clear)."""
    pm1 = (1 << (q - 1)) | (shape6 << (q - 7)) | ((1 << (q - 7)) - 1)
    for k in low_clear_levels:
        assert 7 <= k < q
        pm1 &= ~(1 << (q - 1 - k))
    return pm1 + 1


def test_lane_code_every_table_shape_and_odd_level_pattern(oracle):
    """Structural check of the closed forms on digit masks.  What they depend on: the shape of the seven lowest
    levels (64 values of the top bits of p - 1), which levels from 7 up are odd, and, for a window, the digits of
    its lower end point: the top level k where the end points differ, whether digits 7..k-1 are all set (then the
    table row `odd levels passed` is read with the seven low digits) and the low digits themselves.  For q from 8 to
    31, every shape, and odd-level patterns none / all / single / pairs / random: ranks are built from such digit
    patterns and shifted by skips so that the patterns become window end points of their receive rows; rows from
    both code paths of the lane code must equal the oracle's."""
    rng = np.random.default_rng(20221005)
    total = 0
    for q in (8, 9, 11, 14, 17, 21, 25, 28, 31):
        levels = list(range(7, q))
        patterns = [[], levels]
        patterns += [[k] for k in levels[::max(1, len(levels) // 4)]]
        patterns += [sorted(rng.choice(levels, size=min(2, len(levels)), replace=False).tolist()) for _ in range(2)]
        patterns += [[k for k in levels if rng.random() < 0.5] for _ in range(3)]
        for pi, pat in enumerate(patterns):
            shapes = range(64) if pi < 2 else rng.choice(64, size=6, replace=False).tolist()
            for shape6 in shapes:
                p = _p_from_bits(q, int(shape6), pat)
                if p > 2**31 - 1:
                    continue
                skips = oracle.skips(p).astype(np.int64)
                assert len(skips) == q + 1
                ranks = {0, 1, p - 1}
                for k in range(7, q + 1):
                    ones = sum(int(skips[j]) for j in range(7, k))             # digits 7..k-1 all set
                    for L in rng.integers(0, 128, size=4).tolist() + [0, 127]:
                        low = sum(int(skips[j]) for j in range(7) if L >> j & 1)
                        above = sum(int(skips[j]) for j in range(k + 1, q) if rng.random() < 0.5)
                        y1 = (above + ones + low) % p
                        for i in (k - 1, k):
                            if 0 <= i <= q:
                                ranks.add(int((y1 + skips[i]) % p))
                                ranks.add(int((y1 + skips[i] - 1) % p))
                v = np.array(sorted(ranks), dtype=np.int32)
                want, _, _ = oracle.sched_batch(np.full(len(v), p, np.int32), v, np.zeros(len(v), np.int32),
                                                want_send=False, threads=8)
                assert np.array_equal(hostcheck.recv_rows_list(p, v), want[:, :q]), (p, q, shape6, pat)
                assert np.array_equal(hostcheck.recv_rows_list(p, v, perlane=True), want[:, :q]), (p, q, shape6, pat)
                total += len(v)
    assert total > 100000


def test_lane_code_send_rows_every_p_to_1500(oracle):
    """Send rows the way the batch kernel builds them (entries that need none of the to-neighbour's rounds taken
    directly, the rest by Alg. 5 on the lane code) against the oracle's look-up table: every entry of every rank of
    every p up to 1500, with the wave's bound at q and above it."""
    taken = total = 0
    for p in range(1, 1501):
        _, send = oracle.sched_range(p, threads=4)
        got, direct = hostcheck.send_rows_list(p, np.arange(p), want_direct=True)
        assert np.array_equal(got, send), p
        if p % 97 == 0:
            assert np.array_equal(hostcheck.send_rows_list(p, np.arange(p), wave_q=31), send), p
        total += send.size
        taken += int(np.unpackbits(direct.view(np.uint8)).sum())
    assert taken > 0.6 * total                  # the direct rule must carry most entries, or it is not exercised


@pytest.mark.slow
def test_lane_code_send_rows_every_p_to_40000(oracle):
    for p in range(1501, 40001):
        _, send = oracle.sched_range(p, threads=8)
        assert np.array_equal(hostcheck.send_rows_list(p, np.arange(p)), send), p


def test_lane_code_send_rows_large_p_structured(oracle):
    """The direct send rule where it could break: additions r + skips[k] whose carries meet odd levels.  For q up
    to 31, table shapes and odd-level patterns as in the receive test; ranks whose digits from k up form carry
    chains of every length up to four, with lower parts empty, small, largest possible and one below, and on both
    sides of the margin from which the rule takes an entry without looking at the neighbour's digits; every entry
    against Alg. 5 of the oracle."""
    rng = np.random.default_rng(2205100)
    total = 0
    for q in (8, 10, 13, 17, 21, 25, 28, 31):
        levels = list(range(7, q))
        patterns = [[], levels, [k for k in levels if rng.random() < 0.5], [k for k in levels if rng.random() < 0.5]]
        patterns += [[k] for k in levels[::max(1, len(levels) // 2)]]
        for pi, pat in enumerate(patterns):
            for shape6 in (range(0, 64, 7) if pi < 2 else rng.choice(64, size=3, replace=False).tolist()):
                p = _p_from_bits(q, int(shape6), pat)
                if p > 2**31 - 1:
                    continue
                skips = oracle.skips(p).astype(np.int64)
                ranks = {0, 1, 2, p - 1, p - 2}
                for k in range(q):
                    sk = int(skips[k])
                    m = 2 * sum(1 for j in range(k + 1) if 2 * int(skips[j]) - int(skips[j + 1]) == 1) + 2
                    lows = {0, 1, 2, sk - 1, sk - 2, int(rng.integers(0, sk)), m, m + 1, m + 2, sk - 1 - m, sk - 2 - m, sk - 3 - m,
                            m // 2, sk - 1 - m // 2}
                    for chain in range(5):
                        top = sum(int(skips[j]) for j in range(k, min(k + chain, q)))
                        above = sum(int(skips[j]) for j in range(min(k + chain + 1, q), q) if rng.random() < 0.5)
                        for low in lows:
                            if 0 <= low < sk:
                                ranks.add(int((above + top + low) % p))
                ranks |= {int(x) for x in rng.integers(0, p, 24)}
                v = np.array(sorted(ranks), dtype=np.int32)
                if len(v) > 400:
                    v = np.sort(rng.choice(v, size=400, replace=False)).astype(np.int32)
                _, want, _ = oracle.sched_batch(np.full(len(v), p, np.int32), v, np.zeros(len(v), np.int32), threads=8)
                assert np.array_equal(hostcheck.send_rows_list(p, v, wave_q=min(q + 1, 31)), want[:, :q]), (p, q, shape6, pat)
                total += len(v)
    assert total > 20000


def test_lane_code_rows_from_the_digit_table(oracle):
    """The path of the whole-range kernels: one digit walk per rank into a table, every window's end points read
    from it.  Every rank of every p up to 1200 and of a few larger p."""
    for p in list(range(2, 1201)) + [4097, 65537, 99991]:
        recv, _ = oracle.sched_range(p, want_send=False, threads=4)
        assert np.array_equal(hostcheck.recv_rows_all_tab(p), recv), p
    # prefixes of rows, as Alg. 5 asks for them
    rng = np.random.default_rng(5)
    for p in [2, 3, 5, 17, 100, 1000, 4097, 99991]:
        recv, _ = oracle.sched_range(p, want_send=False, threads=4)
        _, dtab = hostcheck.recv_rows_all_tab(p, want_table=True)
        q = recv.shape[1]
        for v in [0, 1, p - 1] + [int(x) for x in rng.integers(0, p, 60)]:
            for last in {0, q - 1, int(rng.integers(0, q))}:
                assert np.array_equal(hostcheck.recv_row_tab(p, dtab, v, last)[:last + 1], recv[v, :last + 1]), (p, v, last)


def test_lane_code_rows_equal_oracle_large_p(oracle):
    rng = np.random.default_rng(12)
    ps = [65537, 1048577, 134217727, 2**31 - 1, 2**30, 2**30 + 1, 1500000001] + \
         [int(v) for v in rng.integers(2, 2**31 - 1, 60)]
    for p in ps:
        q = oracle.q_of(p)
        for v in [0, 1, 2, p - 1, p - 2, p // 2] + [int(x) for x in rng.integers(0, p, 120)]:
            want = oracle.recvsched(p, v)
            assert (hostcheck.recv_row(p, v)[:q] == want).all(), (p, v)
            assert (hostcheck.recv_row(p, v, perlane=True, wave_q=31)[:q] == want).all(), (p, v)
            k = int(rng.integers(0, q))          # a prefix, as Alg. 5 asks for
            assert (hostcheck.recv_row(p, v, last=k)[:k + 1] == want[:k + 1]).all()


def test_lane_code_rows_that_read_the_high_rows_of_the_low_table(oracle):
    """The rows of the low-level table for many odd levels passed (14 and up) are reached only when q >= 22 and p
    lies just above a power of two; ranks at and around skips and sums of skips are where windows straddle them."""
    rng = np.random.default_rng(1417)
    for k in range(17, 31):
        for p in [2**k + 1, 2**k + 2, 2**k + 3, 2**(k + 1) - 1, int(rng.integers(2**k + 1, 2**k + 2**(k - 8)))]:
            skips = oracle.skips(p).astype(np.int64)
            q = len(skips) - 1
            ranks = {0, 1, p - 1}
            for i in range(q + 1):
                for d in (-3, -2, -1, 0, 1, 2, 3):
                    ranks.add(int(skips[i]) + d)
            for _ in range(24):
                pick = rng.random(q) < 0.5
                ranks.add(int(skips[:q][pick].sum()) + int(rng.integers(-3, 4)))
            ranks |= {int(x) for x in rng.integers(0, p, 16)}
            for v in sorted(r for r in ranks if 0 <= r < p):
                want = oracle.recvsched(p, v)
                assert (hostcheck.recv_row(p, v)[:q] == want).all(), (p, v)
                assert (hostcheck.recv_row(p, v, perlane=True, wave_q=min(q + 2, 31))[:q] == want).all(), (p, v)


def test_lane_code_perlane_small_p_and_padding_lanes(oracle):
    """Per-lane path: a lane whose q is below the wave's bound must leave entries >= q alone."""
    for p in [1, 2, 3, 5, 9, 20, 33, 100, 1000]:
        q = oracle.q_of(p)
        for v in range(p):
            got = hostcheck.recv_row(p, v, last=30, perlane=True, wave_q=31)
            assert (got[:q] == oracle.recvsched(p, v)).all() if q else True
            assert (got[q:] == 12345).all()


def _greedy_digits(skips, ranks):
    """Alg. 2's walk kept as a digit mask, for an array of ranks: bit k set when skips[k] is taken."""
    rest = ranks.astype(np.int64).copy()
    digits = np.zeros(len(ranks), dtype=np.int64)
    for k in range(len(skips) - 2, -1, -1):
        take = rest >= skips[k]
        rest -= take * int(skips[k])
        digits |= take.astype(np.int64) << k
    return digits


def test_taking_a_digit_out_of_a_greedy_sum_leaves_a_greedy_sum(oracle):
    """What the kernels rest on when they skip the walk for an end point v - skips[n]: if skips[n] is one of the
    digits of v, the digits of v - skips[n] are those of v without digit n.  Every rank of every p below 700, and
    sampled ranks of large p of every bit length."""
    rng = np.random.default_rng(2205)
    cases = [(p, np.arange(p)) for p in range(2, 700)]
    for bits in range(11, 32):
        for p in {2**bits - 1, 2**(bits - 1) + 1, int(rng.integers(2**(bits - 1) + 1, 2**bits))}:
            cases.append((p, rng.integers(0, p, size=400)))
    for p, ranks in cases:
        skips = oracle.skips(p)
        d = _greedy_digits(skips, ranks)
        # the lowest digit is the baseblock (Alg. 2), which pins the digit walk itself to the oracle
        for idx in range(min(40, len(ranks))):
            r, dr = int(ranks[idx]), int(d[idx])
            if r > 0:
                assert (dr & -dr).bit_length() - 1 == oracle.baseblock(p, r), (p, r)
        for n in range(len(skips) - 1):
            has = ((d >> n) & 1) == 1
            if not has.any():
                continue
            lower = _greedy_digits(skips, ranks[has] - int(skips[n]))
            assert np.array_equal(lower, d[has] & ~(1 << n)), (p, n)
