"""Parity of the HIP library (through its C ABI) with the CPU oracle, bit for bit, on an MI355X."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def bcs():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2205_10072_amd as lib
    lib.lib()                                  # raises if libbcsched.so is missing: no fallback
    return lib


def dev_tables(rows, cols, fill=777):
    return (torch.full((rows, cols), fill, dtype=torch.int32, device="cuda"),
            torch.full((rows, cols), fill, dtype=torch.int32, device="cuda"))


def gpu_sched(bcs, p, root=0, r0=0, r1=None, want_recv=True, want_send=True):
    r1 = p if r1 is None else r1
    q = bcs.bcs_q(p)
    recv, send = dev_tables(r1 - r0, q)
    bcs.bcs_sched_rooted(p, root, r0, r1, recv if want_recv else None, send if want_send else None)
    torch.cuda.synchronize()
    return recv.cpu().numpy(), send.cpu().numpy()


def test_binding_refuses_tables_that_are_too_small(bcs):
    """Sizes are checked before the C call: a kernel writing past a short table would fault the device."""
    p, n = 1000, 40
    q, R = bcs.bcs_q(p), bcs.bcs_rounds(p, n)
    ok, short = dev_tables(p, q)[0], dev_tables(p - 1, q)[0]
    blocks, blocks_short = dev_tables(p, R)[0], dev_tables(p, R - 1)[0]
    ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    calls = [
        lambda: bcs.bcs_sched(p, 0, p, short, ok),
        lambda: bcs.bcs_sched_rooted(p, 3, 0, p, ok, short),
        lambda: bcs.bcs_sched_rooted_ws(p, 3, 0, p, short, ok, ws),
        lambda: bcs.bcs_sched_rooted_static(p, 3, 0, p, ok, short),
        lambda: bcs.bcs_expand(p, n, 0, p, short, None, blocks, None),
        lambda: bcs.bcs_expand(p, n, 0, p, ok, None, blocks_short, None),
        lambda: bcs.bcs_expand_ws(p, n, 0, p, None, ok, None, blocks_short, ws),
        lambda: bcs.bcs_sched_expand(p, 0, n, ok, ok, blocks, blocks_short),
        lambda: bcs.bcs_sched_expand_ws(p, 0, n, ok, short, blocks, blocks, ws),
        lambda: bcs.bcs_allgather_tables(p, n, 5, blocks_short, blocks),
        lambda: bcs.bcs_allgather_tables_ws(p, n, 5, blocks, blocks_short, ws),
    ]
    trip = torch.ones(8, dtype=torch.int32, device="cuda")
    calls += [
        lambda: bcs.bcs_sched_batch(trip, trip[:7], trip, dev_tables(8, 32)[0], None, None),
        lambda: bcs.bcs_sched_batch(trip, trip, trip, dev_tables(7, 32)[0], None, None),
        lambda: bcs.bcs_sched_batch(trip, trip, trip, None, None, trip[:7]),
    ]
    for i, call in enumerate(calls):
        with pytest.raises(ValueError):
            call()
    # a sub-range needs its rows only
    bcs.bcs_sched(p, 10, 20, short[:10], ok[:10])
    torch.cuda.synchronize()


def test_sweep_every_p_to_1024(bcs, oracle):
    """Config 1: every p in 2..1024, every rank, root 0; then the GPU's own tables are replayed."""
    from bcast_sim import simulate
    for p in range(2, 1025):
        recv, send = gpu_sched(bcs, p)
        orecv, osend = oracle.sched_range(p)
        assert np.array_equal(recv, orecv), p
        assert np.array_equal(send, osend), p
        for n in ((1, 2, 3, 4, 5, 6, 7, 8) if p % 16 == 0 or p < 70 else (1 + p % 8,)):
            simulate(p, n, recv, send)


def test_sweep_as_one_batch(bcs, oracle):
    """Config 1 again as a single batch call (per-lane p, mixed q in one wave)."""
    ps = np.concatenate([np.full(p, p, dtype=np.int32) for p in range(1, 1025)])
    rs = np.concatenate([np.arange(p, dtype=np.int32) for p in range(1, 1025)])
    roots = np.zeros_like(ps)
    count = ps.shape[0]
    recv, send = dev_tables(count, bcs.BATCH_STRIDE)
    qv = torch.full((count,), 99, dtype=torch.int32, device="cuda")
    bcs.bcs_sched_batch(torch.from_numpy(ps).cuda(), torch.from_numpy(rs).cuda(), torch.from_numpy(roots).cuda(),
                        recv, send, qv)
    torch.cuda.synchronize()
    orecv, osend, oq = oracle.sched_batch(ps, rs, roots, threads=8)
    assert np.array_equal(qv.cpu().numpy(), oq)
    assert np.array_equal(recv.cpu().numpy(), orecv)
    assert np.array_equal(send.cpu().numpy(), osend)


def test_one_million_and_one_ranks(bcs, oracle):
    """Config 2: p = 2^20 + 1, all ranks, root 0."""
    p = (1 << 20) + 1
    recv, send = gpu_sched(bcs, p)
    orecv, osend = oracle.sched_range(p, threads=16)
    assert np.array_equal(recv, orecv)
    assert np.array_equal(send, osend)


def test_sub_ranges_roots_and_single_tables(bcs, oracle):
    """Ragged ranges that start and end inside a tile, other roots, one table only, caller workspace."""
    for p, root in [(2, 0), (2, 1), (3, 2), (9, 4), (20, 19), (33, 1), (1000, 123), (4097, 4096), (65537, 40000),
                    (1048577, 77)]:
        q = bcs.bcs_q(p)
        orecv, osend = oracle.sched_range(p, root=root, threads=8)
        recv, send = gpu_sched(bcs, p, root=root)
        assert np.array_equal(recv, orecv) and np.array_equal(send, osend), (p, root)
        recv, _ = gpu_sched(bcs, p, root=root, want_send=False)
        assert np.array_equal(recv, orecv)
        _, send = gpu_sched(bcs, p, root=root, want_recv=False)
        assert np.array_equal(send, osend)
        # caller-provided workspace
        ws = torch.empty(bcs.bcs_sched_workspace_bytes(p, 0, p) + 256, dtype=torch.uint8, device="cuda")
        recv_d, send_d = dev_tables(p, q)
        bcs.bcs_sched_rooted_ws(p, root, 0, p, recv_d, send_d, ws)
        torch.cuda.synchronize()
        assert np.array_equal(recv_d.cpu().numpy(), orecv) and np.array_equal(send_d.cpu().numpy(), osend)
        # partial ranges: send rows are recomputed (Alg. 5) and must equal the looked-up ones
        for r0, r1 in [(0, min(p, 1)), (p - 1, p), (p // 3, min(p, p // 3 + 300)), (max(0, p - 259), p), (1, p)]:
            if p > 70000 and r1 - r0 > 1000:
                continue
            recv, send = gpu_sched(bcs, p, root=root, r0=r0, r1=r1)
            assert np.array_equal(recv, orecv[r0:r1]), (p, root, r0, r1)
            assert np.array_equal(send, osend[r0:r1]), (p, root, r0, r1)
    # an empty range and p = 1 succeed and leave the outputs untouched
    recv, send = dev_tables(3, 4)
    bcs.bcs_sched(9, 4, 4, recv, send)
    bcs.bcs_sched(1, 0, 1, recv, send)
    torch.cuda.synchronize()
    assert bool((recv == 777).all()) and bool((send == 777).all())


def test_receive_rows_with_and_without_the_digit_table(bcs, oracle):
    """Receive rows of all ranks: by digit walks (no workspace) and from the table of all ranks' digit masks (a
    workspace of a word a rank), at a small p and at two large ones.  The two agree everywhere; sampled rows are
    the oracle's."""
    rng = np.random.default_rng(24)
    for p, root in [(70001, 69), (1 << 24, 5), ((1 << 25) + 12345, 1 << 25)]:
        q = bcs.bcs_q(p)
        walked = torch.full((p, q), 777, dtype=torch.int32, device="cuda")
        tabled = torch.full((p, q), 778, dtype=torch.int32, device="cuda")
        ws = torch.empty(4 * p + 256, dtype=torch.uint8, device="cuda")
        bcs.bcs_sched_rooted_ws(p, root, 0, p, walked, None, None)
        bcs.bcs_sched_rooted_ws(p, root, 0, p, tabled, None, ws)
        torch.cuda.synchronize()
        assert torch.equal(walked, tabled), p
        for r in [0, 1, root, p - 1, p // 2] + [int(x) for x in rng.integers(0, p, 150)]:
            want = oracle.recvsched(p, (r - root) % p)
            assert np.array_equal(tabled[r].cpu().numpy(), want), (p, r)
        del walked, tabled, ws


def test_sched_random_ranges(bcs, oracle):
    """Seeded random p, roots, rank ranges (whole, ragged, short) and choices of tables, through the plain call and the
    one with a caller workspace: every kernel variant behind bcs_sched_rooted (digit walks, digit table, look-up,
    recomputation) gets its share."""
    rng = np.random.default_rng(2205_10072)
    tabled_parts = 0
    for case in range(400):
        bits = int(rng.integers(1, 18))
        p = int(rng.integers(max(2, 1 << (bits - 1)), (1 << bits) + 2))
        root = int(rng.integers(0, p))
        q = bcs.bcs_q(p)
        kind = int(rng.integers(0, 4))
        if kind == 0:
            r0, r1 = 0, p
        elif kind == 1:
            r0 = int(rng.integers(0, p))
            r1 = int(rng.integers(r0, p + 1))
        elif kind == 2:
            r0 = int(rng.integers(0, max(1, p // 8)))
            r1 = p - int(rng.integers(0, max(1, p // 8)))
        else:
            r0 = int(rng.integers(0, p))
            r1 = min(p, r0 + int(rng.integers(1, 700)))
        if r1 <= r0:
            continue
        want = int(rng.integers(1, 4))
        recv = torch.full((r1 - r0, q), 777, dtype=torch.int32, device="cuda") if want & 1 else None
        send = torch.full((r1 - r0, q), 778, dtype=torch.int32, device="cuda") if want & 2 else None
        need = bcs.bcs_sched_workspace_bytes(p, r0, r1, 1 if send is not None else 0)
        tabled_parts += need > 0 and not (r0 == 0 and r1 == p)
        if rng.integers(0, 2):
            ws = torch.empty(need + (4 * p + 512) * int(rng.integers(0, 2)), dtype=torch.uint8, device="cuda")
            bcs.bcs_sched_rooted_ws(p, root, r0, r1, recv, send, ws if ws.numel() else None)
        else:
            bcs.bcs_sched_rooted(p, root, r0, r1, recv, send)
        torch.cuda.synchronize()
        orecv, osend = oracle.sched_range(p, root=root, r0=r0, r1=r1, threads=8)
        if recv is not None:
            assert np.array_equal(recv.cpu().numpy(), orecv), ("recv", p, root, r0, r1, want)
        if send is not None:
            assert np.array_equal(send.cpu().numpy(), osend), ("send", p, root, r0, r1, want)
    assert tabled_parts > 20


def test_every_q_from_1_to_31(bcs, oracle):
    """One kernel instance exists per q: each is run on two p of that bit length (one random, one 2^q or 2^(q-1)+1),
    over all ranks when that is cheap and over ragged chunks otherwise, with both ways of making send rows."""
    rng = np.random.default_rng(31)
    for q in range(1, 32):
        lo, hi = (1 << (q - 1)) + 1, min(1 << q, 2**31 - 1)
        for p in {int(rng.integers(lo, hi + 1)), hi, lo}:
            assert bcs.bcs_q(p) == q
            root = int(rng.integers(0, p))
            if p <= 300000:
                recv, send = gpu_sched(bcs, p, root=root)
                orecv, osend = oracle.sched_range(p, root=root, threads=16)
                assert np.array_equal(recv, orecv), (p, root)
                assert np.array_equal(send, osend), (p, root)
            starts = [0, max(0, p - 700)] + [int(v) for v in rng.integers(0, max(1, p - 700), 2)]
            for r0 in starts:
                r1 = min(p, r0 + 700)
                recv, send = gpu_sched(bcs, p, root=root, r0=r0, r1=r1)
                orecv, osend = oracle.sched_range(p, root=root, r0=r0, r1=r1, threads=16)
                assert np.array_equal(recv, orecv), (p, root, r0)
                assert np.array_equal(send, osend), (p, root, r0)


def test_largest_p_sampled_chunks(bcs, oracle):
    """Config 3 (p = 2^27 - 1, q = 27): chunks at both ends and inside, and p = 2^31 - 1."""
    for p in (134217727, 2**31 - 1):
        q = bcs.bcs_q(p)
        for r0 in (0, p // 2 - 1000, 87654321, p - 3001):
            r1 = r0 + 3001
            recv, send = gpu_sched(bcs, p, r0=r0, r1=r1)
            orecv, osend = oracle.sched_range(p, r0=r0, r1=r1, threads=16)
            assert np.array_equal(recv, orecv), (p, r0)
            assert np.array_equal(send, osend), (p, r0)


def test_largest_p_all_ranks_in_full(bcs, oracle):
    """Config 3 in the all-ranks launch configuration (send by look-up), compared in full: every receive row
    against the oracle, chunk by chunk, and every send entry against its definition
    send[r][k] = recv[(r + skips[k]) mod p][k] (Alg. 9's look-up; Alg. 5) on the verified receive table."""
    p = 134217727
    q = 27
    recv = torch.empty((p, q), dtype=torch.int32, device="cuda")
    send = torch.empty((p, q), dtype=torch.int32, device="cuda")
    bcs.bcs_sched(p, 0, p, recv, send)
    torch.cuda.synchronize()
    # any size: a non-root receive row holds exactly one non-negative entry b and the other q-1 blocks
    # as c - q, so it sums to -q(q-1)/2 whatever b is; the root's row sums to -q(q+1)/2
    nonneg = (recv >= 0).sum(dim=1)
    assert int(nonneg[0]) == 0 and bool((nonneg[1:] == 1).all())
    rowsum = recv.sum(dim=1, dtype=torch.int64)
    assert bool((rowsum[1:] == -(q * (q - 1)) // 2).all())
    assert int(rowsum[0]) == -(q * (q + 1)) // 2
    del nonneg, rowsum
    chunk = 1 << 24
    for r0 in range(0, p, chunk):
        r1 = min(p, r0 + chunk)
        orecv, _ = oracle.sched_range(p, r0=r0, r1=r1, want_send=False, threads=16)
        assert np.array_equal(recv[r0:r1].cpu().numpy(), orecv), r0
        del orecv
    skips = bcs.bcs_skips(p)
    for k in range(q):
        assert torch.equal(send[:, k], torch.roll(recv[:, k], -int(skips[k]))), k
    rng = np.random.default_rng(21)                      # and a few send chunks by the oracle's Alg. 5
    for r0 in [0, p - 2048] + [int(v) for v in rng.integers(0, p - 2048, 2)]:
        _, osend = oracle.sched_range(p, r0=r0, r1=r0 + 2048, threads=16)
        assert np.array_equal(send[r0:r0 + 2048].cpu().numpy(), osend), r0
    del recv, send
    bcs.bcs_release()
    torch.cuda.empty_cache()


def test_largest_p_whole_table_replayed(bcs):
    """Config 3 without the oracle: the tables the GPU builds for all 2^27 - 1 ranks are played round by round
    (tests/bcast_sim_torch.py, on the device) and must broadcast n = 1, 2, 3 and q + 2 blocks correctly in
    n - 1 + q rounds.  The same for p = 2^20 + 1 under another root."""
    import bcast_sim_torch
    p, q = 134217727, 27
    recv = torch.empty((p, q), dtype=torch.int32, device="cuda")
    send = torch.empty((p, q), dtype=torch.int32, device="cuda")
    bcs.bcs_sched(p, 0, p, recv, send)
    torch.cuda.synchronize()
    for n in (1, 2, 3, q + 2):
        assert bcast_sim_torch.simulate(p, n, recv, send) == n - 1 + q
    del recv, send
    bcs.bcs_release()
    torch.cuda.empty_cache()
    p, root = (1 << 20) + 1, 777777
    q = bcs.bcs_q(p)
    recv, send = dev_tables(p, q)
    bcs.bcs_sched_rooted(p, root, 0, p, recv, send)
    torch.cuda.synchronize()
    # a schedule rooted at `root` is the root-0 schedule of the ranks renumbered from the root
    recv0, send0 = torch.roll(recv, -root, 0), torch.roll(send, -root, 0)
    for n in (1, 5, 64):
        assert bcast_sim_torch.simulate(p, n, recv0, send0) == n - 1 + q


def test_expand_p65537_n4096(bcs, oracle):
    """Config 4: 2 x 65 537 x 4112 int32."""
    p, n = 65537, 4096
    q = bcs.bcs_q(p)
    R = bcs.bcs_rounds(p, n)
    orecv, osend = oracle.sched_range(p, threads=16)
    recv, send = dev_tables(p, q)
    bcs.bcs_sched(p, 0, p, recv, send)
    rb = torch.full((p, R), 12345, dtype=torch.int32, device="cuda")
    sb = torch.full((p, R), 12345, dtype=torch.int32, device="cuda")
    bcs.bcs_expand(p, n, 0, p, recv, send, rb, sb)
    torch.cuda.synchronize()
    assert np.array_equal(recv.cpu().numpy(), orecv)
    assert np.array_equal(rb.cpu().numpy(), oracle.expand(p, n, orecv))
    assert np.array_equal(sb.cpu().numpy(), oracle.expand(p, n, osend))


def test_expand_with_workspace(bcs, oracle):
    """bcs_expand_ws: the caller's tables rewritten as byte rows in the workspace, then expanded from there; the
    same results as bcs_expand whatever path the sizes take."""
    for p, n, r0, r1 in [(65537, 4096, 0, 65537), (65537, 300, 1000, 50001), (5, 700, 0, 5), (1000, 247, 0, 1000),
                         (1000, 246, 3, 999), (33, 251, 0, 33), (4097, 521, 4000, 4097), (1048577, 256, 0, 1048577),
                         (9, 3, 0, 9), (2, 400, 0, 2), ((1 << 22) + 1, 300, 5, (1 << 22) - 2)]:   # the last: three chunks
        q, R = bcs.bcs_q(p), bcs.bcs_rounds(p, n)
        orecv, osend = oracle.sched_range(p, r0=r0, r1=r1, threads=16)
        recv, send = torch.from_numpy(orecv).cuda(), torch.from_numpy(osend).cuda()
        want_r, want_s = oracle.expand(p, n, orecv, threads=16), oracle.expand(p, n, osend, threads=16)
        need = bcs.bcs_expand_workspace_bytes(p, n, r0, r1)
        assert (need > 0) == (q >= 3 and R >= 256), (p, n)
        for ws_bytes, both in [(need, True), (need, False), (max(0, need - 16), True)]:
            ws = torch.empty(max(16, ws_bytes), dtype=torch.uint8, device="cuda")[:ws_bytes]
            rb, sb = dev_tables(r1 - r0, R, fill=4242)
            bcs.bcs_expand_ws(p, n, r0, r1, recv, send if both else None, rb, sb if both else None, ws)
            torch.cuda.synchronize()
            assert np.array_equal(rb.cpu().numpy(), want_r), (p, n, r0, r1, ws_bytes, both)
            if both:
                assert np.array_equal(sb.cpu().numpy(), want_s), (p, n, r0, r1, ws_bytes)
            else:
                assert bool((sb == 4242).all())
            del rb, sb


def test_expand_small_and_ragged(bcs, oracle):
    for p, n in [(1, 1), (1, 5), (2, 1), (2, 7), (3, 2), (9, 4), (20, 1), (20, 6), (33, 12), (33, 300), (1000, 37),
                 (4097, 1), (4097, 521)]:
        q = bcs.bcs_q(p)
        R = bcs.bcs_rounds(p, n)
        orecv, osend = oracle.sched_range(p)
        if R == 0:                       # p = 1, n = 1: no rounds, empty rows, nothing to hand over
            continue
        for r0, r1 in [(0, p), (p // 2, p), (0, max(1, p // 3))]:
            recv = torch.from_numpy(orecv[r0:r1].copy()).cuda()
            send = torch.from_numpy(osend[r0:r1].copy()).cuda()
            rb, sb = dev_tables(r1 - r0, R, fill=4242)
            bcs.bcs_expand(p, n, r0, r1, recv, send, rb, sb)
            bcs.bcs_expand(p, n, r0, r1, recv, None, rb, None)       # one table only
            torch.cuda.synchronize()
            assert np.array_equal(rb.cpu().numpy(), oracle.expand(p, n, orecv[r0:r1])), (p, n, r0, r1)
            assert np.array_equal(sb.cpu().numpy(), oracle.expand(p, n, osend[r0:r1])), (p, n, r0, r1)


def _check_blocks_on_device(p, n, sched, blocks, oracle, osched, seed):
    """`blocks` (device, [p][R]) against the index arithmetic of Alg. 6 applied to `sched` (device, [p][q]) with
    tensor operations, chunk by chunk, and sampled rows against the oracle's expansion of its own rows."""
    q = sched.shape[1]
    R = n - 1 + q
    x = (q - R % q) % q
    j = torch.arange(R, device="cuda")
    k = (x + j) % q
    shift = (j - k).to(torch.int32)
    step = max(1, (1 << 28) // R)
    for r0 in range(0, p, step):
        want = (sched[r0:r0 + step][:, k] + shift).clamp_(min=-1, max=n - 1)
        assert torch.equal(blocks[r0:r0 + step], want), r0
        del want
    rng = np.random.default_rng(seed)
    rows = np.unique(np.concatenate([[0, 1, p - 1], rng.integers(0, p, 3000)]))
    got = blocks[torch.from_numpy(rows).cuda()].cpu().numpy()
    assert np.array_equal(got, oracle.expand(p, n, osched[rows]))


def test_tables_of_more_than_2_to_32_entries(bcs, oracle):
    """Flat indices beyond 32 bits in the expansion (both store variants) and in the one-call entry point."""
    for p, n in [((1 << 22) + 1, 1100), ((1 << 23) + 1, 500)]:        # rows above / below 640 rounds
        q, R = bcs.bcs_q(p), bcs.bcs_rounds(p, n)
        assert p * R > 1 << 32
        orecv, _ = oracle.sched_range(p, want_send=False, threads=16)
        recv = torch.from_numpy(orecv).cuda()
        rb = torch.full((p, R), 4242, dtype=torch.int32, device="cuda")
        bcs.bcs_expand(p, n, 0, p, recv, None, rb, None)
        torch.cuda.synchronize()
        _check_blocks_on_device(p, n, recv, rb, oracle, orecv, seed=p)
        del recv, rb, orecv
        torch.cuda.empty_cache()
    p, n, root = (1 << 25) + 1, 103, 31415926                          # fused kernels, R = 128
    q, R = bcs.bcs_q(p), bcs.bcs_rounds(p, n)
    assert R == 128 and p * R > 1 << 32
    recv, send = dev_tables(p, q)
    rb = torch.full((p, R), 4242, dtype=torch.int32, device="cuda")
    sb = torch.full((p, R), 4242, dtype=torch.int32, device="cuda")
    bcs.bcs_sched_expand(p, root, n, recv, send, rb, sb)
    torch.cuda.synchronize()
    orecv, osend = oracle.sched_range(p, root=root, threads=16)
    assert np.array_equal(recv.cpu().numpy(), orecv)
    assert np.array_equal(send.cpu().numpy(), osend)
    _check_blocks_on_device(p, n, recv, rb, oracle, orecv, seed=1)
    _check_blocks_on_device(p, n, send, sb, oracle, osend, seed=2)
    del recv, send, rb, sb, orecv, osend
    torch.cuda.empty_cache()
    p, n, root = 1300001, 3400, 1234567                               # expansion from byte rows, R = 3421
    q, R = bcs.bcs_q(p), bcs.bcs_rounds(p, n)
    assert p * R > 1 << 32 and bcs.bcs_sched_expand_workspace_bytes(p, n) > bcs.bcs_sched_workspace_bytes(p, 0, p)
    recv, send = dev_tables(p, q)
    rb = torch.full((p, R), 4242, dtype=torch.int32, device="cuda")
    sb = torch.full((p, R), 4242, dtype=torch.int32, device="cuda")
    bcs.bcs_sched_expand(p, root, n, recv, send, rb, sb)
    torch.cuda.synchronize()
    orecv, osend = oracle.sched_range(p, root=root, threads=16)
    assert np.array_equal(recv.cpu().numpy(), orecv)
    assert np.array_equal(send.cpu().numpy(), osend)
    _check_blocks_on_device(p, n, recv, rb, oracle, orecv, seed=3)
    _check_blocks_on_device(p, n, send, sb, oracle, osend, seed=4)
    del recv, send, rb, sb
    bcs.bcs_release()
    torch.cuda.empty_cache()


def test_expand_largest_n(bcs, oracle):
    """n = BCS_MAX_N (2^31 - 65): rounds and blocks at the top of int32, rows of 8.6 GB, checked on the device
    against the index arithmetic of Alg. 6 piece by piece (p = 2: the entry-by-entry kernel; p = 5: the staged one)."""
    n = bcs.MAX_N
    for p, both in [(2, True), (5, False)]:
        q, R = bcs.bcs_q(p), bcs.bcs_rounds(p, n)
        assert R == n - 1 + q and R < 2**31
        orecv, osend = oracle.sched_range(p)
        x = (q - R % q) % q
        for table in ([orecv, osend] if both else [orecv]):
            sched = torch.from_numpy(table).cuda()
            blocks = torch.full((p, R), 4242, dtype=torch.int32, device="cuda")
            bcs.bcs_expand(p, n, 0, p, sched, None, blocks, None)
            torch.cuda.synchronize()
            step = 1 << 27
            for j0 in range(0, R, step):
                j = torch.arange(j0, min(R, j0 + step), device="cuda", dtype=torch.int64)
                k = (x + j) % q
                want = (sched.long()[:, k] + (j - k)).clamp_(min=-1, max=n - 1).to(torch.int32)
                assert torch.equal(blocks[:, j0:j0 + step], want), (p, j0)
                del want, j, k
            assert int(blocks[:, -1].max()) == n - 1
            del blocks
            torch.cuda.empty_cache()


def test_irregular_batch(bcs, oracle):
    """Config 5: 2^20 seeded (p, r, root) triples, p log-uniform up to 2^31 - 1."""
    from paper_2205_10072_amd import synth
    count = 1 << 20
    p, r, root = synth.batch_triples(count)
    recv, send = dev_tables(count, bcs.BATCH_STRIDE)
    qv = torch.full((count,), 99, dtype=torch.int32, device="cuda")
    bcs.bcs_sched_batch(torch.from_numpy(p).cuda(), torch.from_numpy(r).cuda(), torch.from_numpy(root).cuda(),
                        recv, send, qv)
    torch.cuda.synchronize()
    orecv, osend, oq = oracle.sched_batch(p, r, root, threads=16)
    assert np.array_equal(qv.cpu().numpy(), oq)
    assert np.array_equal(recv.cpu().numpy(), orecv)
    assert np.array_equal(send.cpu().numpy(), osend)


def test_batch_send_rows_where_the_direct_rule_is_at_its_limits(bcs, oracle):
    """Send rows of the batch kernel (entries taken from the rank's own digits where that is exact, Alg. 5 otherwise)
    on triples built to sit at the rule's limits: p with chosen odd levels for q up to 31, ranks whose additions
    r + skips[k] carry through odd levels, with lower parts empty, largest possible and on both sides of the rule's
    margin; every entry against Alg. 5 of the oracle.  A second call takes the same ranks as a range of one p
    (the kernel for parts of the ranks uses the same rule)."""
    from test_host_logic import _p_from_bits
    rng = np.random.default_rng(310522)
    ps, rs = [], []
    for q in (9, 12, 16, 20, 24, 27, 29, 31):
        levels = list(range(7, q))
        for pat in ([], levels, [k for k in levels if rng.random() < 0.5], [k for k in levels if rng.random() < 0.3]):
            p = _p_from_bits(q, int(rng.integers(0, 64)), pat)
            if p > 2**31 - 1:
                continue
            skips = oracle.skips(p).astype(np.int64)
            for k in range(q):
                sk = int(skips[k])
                m = 2 * sum(1 for j in range(k + 1) if 2 * int(skips[j]) - int(skips[j + 1]) == 1) + 2
                for chain in range(4):
                    top = sum(int(skips[j]) for j in range(k, min(k + chain, q)))
                    above = sum(int(skips[j]) for j in range(min(k + chain + 1, q), q) if rng.random() < 0.5)
                    for low in (0, 1, sk - 1, sk - 2, m, m + 1, sk - 1 - m, sk - 2 - m, int(rng.integers(0, sk))):
                        if 0 <= low < sk:
                            ps.append(p)
                            rs.append((above + top + low) % p)
    p_arr = np.array(ps, dtype=np.int32)
    v_arr = np.array(rs, dtype=np.int32)
    root = (rng.integers(0, 2**31 - 1, len(p_arr)) % p_arr).astype(np.int32)
    r_arr = ((v_arr.astype(np.int64) + root) % p_arr).astype(np.int32)      # so that the virtual rank is v
    print("structured batch: %d triples" % len(p_arr), flush=True)
    orecv, osend, oq = oracle.sched_batch(p_arr, r_arr, root, threads=16)
    d = [torch.from_numpy(a).cuda() for a in (p_arr, r_arr, root)]
    recv, send = dev_tables(len(p_arr), 32)
    qv = torch.empty(len(p_arr), dtype=torch.int32, device="cuda")
    bcs.bcs_sched_batch(d[0], d[1], d[2], recv, send, qv)
    torch.cuda.synchronize()
    assert np.array_equal(qv.cpu().numpy(), oq)
    assert np.array_equal(recv.cpu().numpy(), orecv)
    assert np.array_equal(send.cpu().numpy(), osend)
    # the kernel for a part of the ranks of one p uses the same rule: ranges around sums of skips
    for q, pat in ((27, list(range(7, 27))), (31, [k for k in range(7, 31) if k % 2]), (21, [9, 14])):
        p = _p_from_bits(q, int(rng.integers(0, 64)), pat)
        skips = oracle.skips(p).astype(np.int64)
        for _ in range(5):
            pick = rng.random(q) < 0.4
            centre = int(skips[:q][pick].sum()) % p
            v0, v1 = max(0, centre - 330), min(p, centre + 310)
            root = int(rng.integers(0, p - v1 + 1))                 # ranks root + v0 .. root + v1 - 1 play virtual ranks v0 .. v1 - 1
            r0, r1 = v0 + root, v1 + root
            _, want = oracle.sched_range(p, root=root, r0=r0, r1=r1, want_recv=False, threads=16)
            _, got = gpu_sched(bcs, p, root=root, r0=r0, r1=r1, want_recv=False)
            assert np.array_equal(got, want), (p, root, r0, r1)


def test_batch_with_more_left_over_send_entries_than_the_work_list_holds(bcs, oracle):
    """The batch kernel works the send entries that need Alg. 5 off as a list of the workgroup, 4096 entries at a
    time.  Triples picked (with the host build of the same lane code) so that every workgroup of 1024 has more than
    that: ranks of p = 2^16+1 and 2^20+1 with seven or more such entries each."""
    import hostcheck
    rng = np.random.default_rng(77)
    ps, vs = [], []
    for p, span in ((2**16 + 1, 2**16 + 1), (2**20 + 1, 300000)):
        q = (p - 1).bit_length()
        ranks = np.arange(span, dtype=np.int32)
        _, direct = hostcheck.send_rows_list(p, ranks, want_direct=True)
        left = q - np.array([bin(int(x) & ((1 << q) - 1)).count("1") for x in direct])
        many = ranks[left >= 7]
        assert len(many) >= 2048
        pick = rng.choice(many, 2048, replace=False)
        assert left[pick].reshape(2, 1024).sum(axis=1).min() > 4096 + 1024     # more than one filling of the list
        ps += [p] * 2048
        vs += pick.tolist()
    p_arr = np.array(ps, dtype=np.int32)
    v_arr = np.array(vs, dtype=np.int64)
    root = (rng.integers(0, 2**31 - 1, len(p_arr)) % p_arr).astype(np.int32)
    r_arr = ((v_arr + root) % p_arr).astype(np.int32)
    orecv, osend, oq = oracle.sched_batch(p_arr, r_arr, root, threads=16)
    d = [torch.from_numpy(a).cuda() for a in (p_arr, r_arr, root)]
    recv, send = dev_tables(len(p_arr), 32)
    qv = torch.empty(len(p_arr), dtype=torch.int32, device="cuda")
    bcs.bcs_sched_batch(d[0], d[1], d[2], recv, send, qv)
    torch.cuda.synchronize()
    assert np.array_equal(recv.cpu().numpy(), orecv)
    assert np.array_equal(send.cpu().numpy(), osend)


def test_send_rule_against_the_look_up_for_every_rank_of_large_p(bcs):
    """Send rows of parts of the ranks (taken from the ranks' own digits where the rule applies, Alg. 5 otherwise)
    against send rows of all ranks by look-up in the receive table, which is their definition (Alg. 9, second loop):
    every rank of 40 values of p of 12 to 27 bits, random and with chosen odd levels, each under a random root and cut
    into two ranges at a random rank.  Then p of 30 and 31 bits, whose tables do not fit: slices of 2^20 ranks
    against entry k of the receive rows of their to-neighbours.  (The receive rows themselves are compared with the
    oracle elsewhere in this file.)"""
    from test_host_logic import _p_from_bits
    rng = np.random.default_rng(20220510)
    ps = [(1 << 20) + 1, (1 << 23) + 1, (1 << 24) + 12345, (1 << 26) - 3, (1 << 27) - 1]
    while len(ps) < 40:
        q = int(rng.integers(12, 27))
        if rng.random() < 0.5:
            ps.append(int(rng.integers(2**(q - 1) + 1, 2**q)))
        else:
            pr = rng.choice([0.1, 0.5, 0.9, 1.0])
            ps.append(_p_from_bits(q, int(rng.integers(0, 64)), [k for k in range(7, q) if rng.random() < pr]))
    for p in ps:
        q = bcs.bcs_q(p)
        full = torch.empty((p, q), dtype=torch.int32, device="cuda")
        part = torch.full((p, q), 99, dtype=torch.int32, device="cuda")
        root, cut = int(rng.integers(0, p)), int(rng.integers(1, p))
        bcs.bcs_sched_rooted(p, root, 0, p, None, full)
        bcs.bcs_sched_rooted(p, root, 0, cut, None, part[:cut])
        bcs.bcs_sched_rooted(p, root, cut, p, None, part[cut:])
        torch.cuda.synchronize()
        assert torch.equal(full, part), (p, root, cut)
        del full, part
    bcs.bcs_release()
    torch.cuda.empty_cache()
    W = 1 << 20
    big = [2**31 - 1, 2**30 + 1, 2**30, _p_from_bits(31, 5, [k for k in range(7, 31) if k % 3]),
           _p_from_bits(30, 60, list(range(7, 30))), int(rng.integers(2**30 + 1, 2**31 - 1))]
    for p in big:
        q = bcs.bcs_q(p)
        skips = bcs.bcs_skips(p)
        pick = rng.random(q) < 0.4
        centres = [int(rng.integers(0, p)), int(sum(s for s, f in zip(skips[:q], pick) if f) % p), 0, p - 1]
        for c in centres:
            r0 = max(0, min(c - W // 2, p - W))
            send = torch.full((W, q), 99, dtype=torch.int32, device="cuda")
            nb = torch.empty((W, q), dtype=torch.int32, device="cuda")
            bcs.bcs_sched(p, r0, r0 + W, None, send)
            for k in range(q):
                a = (r0 + skips[k]) % p
                if a + W <= p:
                    bcs.bcs_sched(p, a, a + W, nb, None)
                else:
                    bcs.bcs_sched(p, a, p, nb[:p - a], None)
                    bcs.bcs_sched(p, 0, a + W - p, nb[p - a:], None)
                assert torch.equal(send[:, k], nb[:, k]), (p, r0, k)


def test_rows_from_digits_against_rows_from_windows(bcs):
    """The one-p kernels take most rounds above level 5 from the rank's own digits; the batch kernel takes every
    round from its windows.  Every rank of 40 values of p of 8 to 27 bits (random, and with chosen odd levels),
    each under a random root: the table by bcs_sched_rooted (all ranks: digit masks from the table) and a ragged
    part of it (digit walks) against bcs_sched_batch on the same ranks."""
    from test_host_logic import _p_from_bits
    rng = np.random.default_rng(20220511)
    ps = [(1 << 20) + 1, (1 << 23) + 1, (1 << 24) + 12345, (1 << 26) - 3, (1 << 27) - 1]
    while len(ps) < 40:
        q = int(rng.integers(8, 27))
        if rng.random() < 0.5:
            ps.append(int(rng.integers(2**(q - 1) + 1, 2**q)))
        else:
            pr = rng.choice([0.1, 0.5, 0.9, 1.0])
            ps.append(_p_from_bits(q, int(rng.integers(0, 64)), [k for k in range(7, q) if rng.random() < pr]))
    CH = 1 << 24
    brecv = torch.empty((CH, bcs.BATCH_STRIDE), dtype=torch.int32, device="cuda")
    qout = torch.empty(CH, dtype=torch.int32, device="cuda")
    for p in ps:
        q = bcs.bcs_q(p)
        root = int(rng.integers(0, p))
        full = torch.empty((p, q), dtype=torch.int32, device="cuda")
        bcs.bcs_sched_rooted(p, root, 0, p, full, None)
        a = int(rng.integers(0, p))
        b = min(p, a + int(rng.integers(1, 1 << 20)))
        part = torch.empty((b - a, q), dtype=torch.int32, device="cuda")
        bcs.bcs_sched_rooted(p, root, a, b, part, None)
        torch.cuda.synchronize()
        assert torch.equal(full[a:b], part), (p, root, a, b)
        for c0 in range(0, p, CH):
            n = min(p, c0 + CH) - c0
            pp = torch.full((n,), p, dtype=torch.int32, device="cuda")
            rr = torch.arange(c0, c0 + n, dtype=torch.int32, device="cuda")
            ro = torch.full((n,), root, dtype=torch.int32, device="cuda")
            bcs.bcs_sched_batch(pp, rr, ro, brecv[:n], None, qout[:n])
            torch.cuda.synchronize()
            assert torch.equal(full[c0:c0 + n], brecv[:n, :q]), (p, root, c0)
        del full, part
    bcs.bcs_release()
    torch.cuda.empty_cache()


def test_batch_edge_rows(bcs, oracle):
    """Invalid triples are flagged on the device; a ragged count; single outputs."""
    p = np.array([1, 2, 2, 0, 5, 5, 2**31 - 1, 7, -3, 9], dtype=np.int32)
    r = np.array([0, 1, 0, 0, 5, 2, 2**31 - 2, -1, 0, 3], dtype=np.int32)
    root = np.array([0, 0, 1, 0, 0, 6, 5, 0, 0, 8], dtype=np.int32)
    ok = np.array([1, 1, 1, 0, 0, 0, 1, 0, 0, 1], dtype=bool)
    recv, send = dev_tables(len(p), bcs.BATCH_STRIDE)
    qv = torch.full((len(p),), 99, dtype=torch.int32, device="cuda")
    args = [torch.from_numpy(a).cuda() for a in (p, r, root)]
    bcs.bcs_sched_batch(*args, recv, send, qv)
    torch.cuda.synchronize()
    orecv, osend, oq = oracle.sched_batch(p[ok], r[ok], root[ok])
    assert np.array_equal(qv.cpu().numpy()[ok], oq) and (qv.cpu().numpy()[~ok] == -1).all()
    assert np.array_equal(recv.cpu().numpy()[ok], orecv) and np.array_equal(send.cpu().numpy()[ok], osend)
    assert (recv.cpu().numpy()[~ok] == bcs.BATCH_PAD).all() and (send.cpu().numpy()[~ok] == bcs.BATCH_PAD).all()
    recv2, _ = dev_tables(len(p), bcs.BATCH_STRIDE)
    bcs.bcs_sched_batch(*args, recv2, None, None)
    torch.cuda.synchronize()
    assert torch.equal(recv2, recv)


def gpu_allgather(bcs, p, n, r, want_pack=True, want_unpack=True, ws=None, misalign=False):
    R = bcs.bcs_rounds(p, n)
    if misalign:                                         # tables that start 4 bytes past a 16-byte boundary
        flat = [torch.full((R * p + 1,), 555, dtype=torch.int32, device="cuda") for _ in range(2)]
        pack, unpack = (t[1:].view(R, p) for t in flat)
    else:
        pack, unpack = dev_tables(R, p, fill=555)
    if ws is None:
        bcs.bcs_allgather_tables(p, n, r, pack if want_pack else None, unpack if want_unpack else None)
    else:
        bcs.bcs_allgather_tables_ws(p, n, r, pack if want_pack else None, unpack if want_unpack else None, ws)
    torch.cuda.synchronize()
    return pack.cpu().numpy(), unpack.cpu().numpy()


def test_allgather_tables_against_oracle(bcs, oracle):
    """Alg. 9's pack / unpack index tables for one process: ragged p, every kind of n, both outputs and one."""
    for p, n in [(1, 3), (2, 1), (2, 4), (3, 2), (9, 4), (20, 6), (33, 12), (257, 3), (1000, 37), (1025, 2), (4097, 300),
                 (65537, 9)]:
        for r in sorted({0, 1 % p, p // 2, p - 1}):
            opack, ounpack = oracle.allgather_tables(p, n, r)
            if opack.size == 0:
                continue
            for misalign in (False, True):               # 16-byte stores / the kernel for any alignment
                pack, unpack = gpu_allgather(bcs, p, n, r, misalign=misalign)
                assert np.array_equal(pack, opack), (p, n, r, misalign)
                assert np.array_equal(unpack, ounpack), (p, n, r, misalign)
        pack, unpack = gpu_allgather(bcs, p, n, p - 1, want_unpack=False)
        assert np.array_equal(pack, opack) and (unpack == 555).all()
        ws = torch.empty(bcs.bcs_allgather_workspace_bytes(p) + 256, dtype=torch.uint8, device="cuda")
        pack, unpack = gpu_allgather(bcs, p, n, p - 1, want_pack=False, ws=ws)
        assert np.array_equal(unpack, ounpack) and (pack == 555).all()


def test_allgather_tables_random_sizes(bcs, oracle):
    """Seeded random (p, n, r), aligned and unaligned outputs, one table or both, against the oracle."""
    rng = np.random.default_rng(9042)
    for case in range(50):
        p = int(2 ** rng.uniform(1, 16.5))
        n = int(2 ** rng.uniform(0, 7.5))
        r = int(rng.integers(0, p))
        if p * bcs.bcs_rounds(p, n) > 3e7:
            continue
        opack, ounpack = oracle.allgather_tables(p, n, r)
        which = case % 3
        pack, unpack = gpu_allgather(bcs, p, n, r, want_pack=which != 1, want_unpack=which != 2,
                                     misalign=bool(case % 2))
        if which != 1:
            assert np.array_equal(pack, opack), (p, n, r, case)
        if which != 2:
            assert np.array_equal(unpack, ounpack), (p, n, r, case)


def test_allgather_tables_replayed_for_all_processes(bcs):
    """The GPU's own tables, one call per process, replayed as a whole allgather."""
    from allgather_sim import simulate_allgather
    for p, n in [(5, 2), (20, 4), (33, 7), (64, 3)]:
        tabs = [gpu_allgather(bcs, p, n, r) for r in range(p)]
        simulate_allgather(p, n, np.array([t[0] for t in tabs]), np.array([t[1] for t in tabs]))


def test_allgather_tables_one_million_processes(bcs, oracle):
    p, n, r = (1 << 20) + 1, 5, 777777
    opack, ounpack = oracle.allgather_tables(p, n, r)
    pack, unpack = gpu_allgather(bcs, p, n, r)
    assert np.array_equal(pack, opack)
    assert np.array_equal(unpack, ounpack)


def test_bench_step_configuration(bcs, oracle):
    """The very calls bench.py times (p = 2^20+1, root 0, caller workspace, n = 256), compared in full."""
    p, n = (1 << 20) + 1, 256
    q, R = bcs.bcs_q(p), bcs.bcs_rounds(p, n)
    recv, send = dev_tables(p, q)
    rb = torch.full((p, R), 4242, dtype=torch.int32, device="cuda")
    sb = torch.full((p, R), 4242, dtype=torch.int32, device="cuda")
    ws = torch.empty(bcs.bcs_sched_expand_workspace_bytes(p, n), dtype=torch.uint8, device="cuda")
    for _ in range(2):                                    # twice: scratch and tables are reused across steps
        bcs.bcs_sched_expand_ws(p, 0, n, recv, send, rb, sb, ws)
    torch.cuda.synchronize()
    orecv, osend = oracle.sched_range(p, threads=16)
    oracle_rb, oracle_sb = oracle.expand(p, n, orecv, threads=16), oracle.expand(p, n, osend, threads=16)
    assert np.array_equal(recv.cpu().numpy(), orecv)
    assert np.array_equal(send.cpu().numpy(), osend)
    assert np.array_equal(rb.cpu().numpy(), oracle_rb)
    assert np.array_equal(sb.cpu().numpy(), oracle_sb)
    # the same step by the separate calls
    rb.fill_(4242)
    sb.fill_(4242)
    bcs.bcs_sched_rooted_ws(p, 0, 0, p, recv, send, ws)
    bcs.bcs_expand(p, n, 0, p, recv, send, rb, sb)
    torch.cuda.synchronize()
    assert np.array_equal(rb.cpu().numpy(), oracle_rb)
    assert np.array_equal(sb.cpu().numpy(), oracle_sb)


def _sched_expand_case(bcs, oracle, p, n, root, own_ws=False, misalign=False):
    q, R = bcs.bcs_q(p), bcs.bcs_rounds(p, n)
    recv, send = dev_tables(p, max(q, 1))
    recv, send = recv[:, :q].contiguous(), send[:, :q].contiguous()
    flat = [torch.full((p * R + 4,), 4242, dtype=torch.int32, device="cuda") for _ in range(2)]
    off = 1 if misalign else 0                          # one int32 off a 16-byte boundary
    rb, sb = (t[off:off + p * R].view(p, R) for t in flat)
    args = (p, root, n, recv if q else None, send if q else None, rb, sb)
    if own_ws:                                          # "small": enough for the schedules, not for the byte rows
        size = bcs.bcs_sched_workspace_bytes(p, 0, p) if own_ws == "small" else bcs.bcs_sched_expand_workspace_bytes(p, n)
        ws = torch.empty(max(1, size), dtype=torch.uint8, device="cuda")
        bcs.bcs_sched_expand_ws(*args, ws)
    else:
        bcs.bcs_sched_expand(*args)
    torch.cuda.synchronize()
    orecv, osend = oracle.sched_range(p, root, 0, p, threads=16)
    tag = (p, n, root)
    if q:
        assert np.array_equal(recv.cpu().numpy(), orecv), tag
        assert np.array_equal(send.cpu().numpy(), osend), tag
    if R:
        assert np.array_equal(rb.cpu().numpy(), oracle.expand(p, n, orecv, threads=16)), tag
        assert np.array_equal(sb.cpu().numpy(), oracle.expand(p, n, osend, threads=16)), tag
    for t in flat:                                      # nothing written outside the tables
        assert int(t[off + p * R:].min()) == 4242 and int(t[:off].sum()) == 4242 * off, tag


def test_sched_expand_one_call(bcs, oracle):
    """bcs_sched_expand: schedules and both block tables of all ranks in one call.  Short rows are expanded by
    the workgroup that built them (every q from 3 to 23 here; larger q would need more than 2^23 ranks at
    once), longer rows from byte rows kept in scratch memory, the rest by the separate kernels; all compared in full."""
    rng = np.random.default_rng(2205)
    for q in range(3, 22):                              # fused: R = n-1+q <= 96
        p = (1 << (q - 1)) + 1 + int(rng.integers(0, 1 << (q - 1)))
        _sched_expand_case(bcs, oracle, p, int(rng.integers(max(1, 17 - q), 60)), int(rng.integers(0, p)),
                           own_ws=bool(q & 1))
    _sched_expand_case(bcs, oracle, (1 << 21) + 77, 3, 5)               # q = 22
    _sched_expand_case(bcs, oracle, (1 << 22) + 1, 1, (1 << 22), own_ws=True)   # q = 23, n = 1
    for p, n, root in [(5, 14, 4), (255, 89, 0), (256, 89, 255), (257, 88, 1), (511, 9, 77), (513, 87, 512),
                       (1000, 37, 123), (65536, 113, 9), (70001, 100, 70000), (65535, 81, 3)]:
        _sched_expand_case(bcs, oracle, p, n, root)     # fused, tiles with ragged tails, both length classes
    for p, n, root in [(1, 1, 0), (1, 9, 0), (2, 40, 1), (3, 20, 2), (4, 33, 0), (9, 3, 8), (1000, 5, 1),
                       (1000, 200, 999), (4097, 100, 5), (65535, 145, 9), (70000, 1000, 7), (5, 700, 2), (33, 14, 32),
                       (1025, 641, 1024), (300001, 160, 7)]:
        # longer rows: expansion from the byte rows the schedule kernels leave behind (plain call, caller's
        # workspace of the full size), or the separate kernels (a workspace that only holds the schedules' scratch)
        for own_ws in (False, True, "small"):
            _sched_expand_case(bcs, oracle, p, n, root, own_ws=own_ws)
    _sched_expand_case(bcs, oracle, 1000, 37, 123, misalign=True)
    _sched_expand_case(bcs, oracle, 70001, 130, 1, own_ws=True, misalign=True)
    with pytest.raises(bcs.BcsError):
        bcs.bcs_sched_expand(1000, 1000, 5, *dev_tables(1000, 10), *dev_tables(1000, 14))
    with pytest.raises(bcs.BcsError):
        bcs.bcs_sched_expand(1000, 0, 5, None, None, *dev_tables(1000, 14))
    with pytest.raises(bcs.BcsError):                   # caller workspace too small
        r, s = dev_tables(1000, 10)
        rb, sb = dev_tables(1000, 46)
        bcs.bcs_sched_expand_ws(1000, 0, 37, r, s, rb, sb, torch.empty(64, dtype=torch.uint8, device="cuda"))


def test_sched_expand_random_sizes(bcs, oracle):
    """Seeded random (p, n, root) through the one-call entry point and through bcs_expand_ws: whatever kernels the
    sizes select, the four tables equal the oracle's."""
    rng = np.random.default_rng(20220510)
    for case in range(70):
        p = int(2 ** rng.uniform(1, 18.2))
        n = int(2 ** rng.uniform(0, 9.6))
        root = int(rng.integers(0, p))
        q, R = bcs.bcs_q(p), bcs.bcs_rounds(p, n)
        orecv, osend = oracle.sched_range(p, root=root, threads=16)
        want_r, want_s = oracle.expand(p, n, orecv, threads=16), oracle.expand(p, n, osend, threads=16)
        recv, send = dev_tables(p, q)
        rb, sb = dev_tables(p, R, fill=4242)
        if case % 2:
            bcs.bcs_sched_expand(p, root, n, recv, send, rb, sb)
        else:
            ws = torch.empty(max(1, bcs.bcs_sched_expand_workspace_bytes(p, n)), dtype=torch.uint8, device="cuda")
            bcs.bcs_sched_expand_ws(p, root, n, recv, send, rb, sb, ws)
        torch.cuda.synchronize()
        tag = (p, n, root)
        assert np.array_equal(recv.cpu().numpy(), orecv) and np.array_equal(send.cpu().numpy(), osend), tag
        assert np.array_equal(rb.cpu().numpy(), want_r) and np.array_equal(sb.cpu().numpy(), want_s), tag
        # a ragged range of the same tables through bcs_expand_ws
        r0 = int(rng.integers(0, p))
        r1 = int(rng.integers(r0, p + 1))
        if r1 > r0:
            ws = torch.empty(max(16, bcs.bcs_expand_workspace_bytes(p, n, r0, r1)), dtype=torch.uint8, device="cuda")
            rb2, sb2 = dev_tables(r1 - r0, R, fill=4242)
            bcs.bcs_expand_ws(p, n, r0, r1, recv[r0:r1], send[r0:r1], rb2, sb2, ws)
            torch.cuda.synchronize()
            assert np.array_equal(rb2.cpu().numpy(), want_r[r0:r1]) and np.array_equal(sb2.cpu().numpy(), want_s[r0:r1]), \
                (tag, r0, r1)


def _pack_case(rng, p, n, kind):
    if kind == "paper":
        from paper_2205_10072_amd import synth
        sizes, displs = synth.irregular_sizes(p, int(rng.integers(p, 40 * p)))
    elif kind == "tiny":
        sizes = rng.integers(0, 4, p).astype(np.int64)
        displs = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    else:
        sizes = rng.integers(0, 3000, p).astype(np.int64)
        sizes[rng.integers(0, p, max(1, p // 3))] = 0
        displs = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    data = rng.integers(0, 1 << 30, max(1, int(displs[-1]))).astype(np.int32)
    idx = rng.integers(-1, n, p).astype(np.int32)
    if kind == "tiny":
        idx[rng.integers(0, p, p // 2)] = -1
    return displs, data, idx


def test_pack_and_unpack_one_round(bcs, oracle):
    """Alg. 9's pack and unpack loops on irregular buffers: message, offsets and unpacked buffers, bit for bit."""
    rng = np.random.default_rng(77)
    for p, n in [(1, 1), (2, 3), (5, 2), (37, 6), (1000, 9), (1025, 4), (5000, 33), (70000, 5)]:
        for kind in ("paper", "tiny", "mixed"):
            displs, data, idx = _pack_case(rng, p, n, kind)
            omsg, ooff = oracle.pack_round(n, idx, displs, data)
            d_idx = torch.from_numpy(idx).cuda()
            d_displs = torch.from_numpy(displs).cuda()
            d_data = torch.from_numpy(data).cuda()
            cap = len(omsg) + 5
            d_msg = torch.full((cap,), -99, dtype=torch.int32, device="cuda")
            d_off = torch.full((p + 1,), -1, dtype=torch.int64, device="cuda")
            ws = torch.empty(bcs.bcs_pack_workspace_bytes(p), dtype=torch.uint8, device="cuda")
            bcs.bcs_pack_round(n, d_idx, d_displs, d_data, d_msg, d_off, ws)
            torch.cuda.synchronize()
            assert np.array_equal(d_off.cpu().numpy(), ooff), (p, n, kind)
            got = d_msg.cpu().numpy()
            assert np.array_equal(got[:len(omsg)], omsg), (p, n, kind)
            assert (got[len(omsg):] == -99).all()
            # a message buffer that is too small is filled and not overrun
            if len(omsg) > 3:
                small = torch.full((len(omsg) - 3 + 8,), -99, dtype=torch.int32, device="cuda")
                bcs.bcs_pack_round(n, d_idx, d_displs, d_data, small[:len(omsg) - 3], d_off, ws)
                torch.cuda.synchronize()
                s = small.cpu().numpy()
                assert np.array_equal(s[:len(omsg) - 3], omsg[:-3]) and (s[len(omsg) - 3:] == -99).all()
                assert int(d_off[p]) == len(omsg)
            # unpack into blank buffers, from a message at an odd address
            blank = np.full_like(data, -5)
            oracle.unpack_round(n, idx, displs, blank, omsg)
            shifted = torch.empty(len(omsg) + 1, dtype=torch.int32, device="cuda")
            shifted[1:] = torch.from_numpy(omsg).cuda()
            d_blank = torch.full((len(data),), -5, dtype=torch.int32, device="cuda")
            bcs.bcs_unpack_round(n, d_idx, d_displs, d_blank, shifted[1:], len(omsg), d_off, ws)
            torch.cuda.synchronize()
            assert np.array_equal(d_blank.cpu().numpy(), blank), (p, n, kind)
            assert np.array_equal(d_off.cpu().numpy(), ooff)


def test_pack_plans_of_all_rounds_and_planned_rounds(bcs, oracle):
    """Alg. 9's pack and unpack loops with the plans of all rounds made in one launch: every row of the plan and
    every round's message against the oracle's pack loop, the unpacked buffers against its unpack loop.  The last
    case has the paper's own shape (p = 1152, m = 10^8 elements, n = 1658 blocks from its block-size rule)."""
    from paper_2205_10072_amd import synth
    rng = np.random.default_rng(1152)
    for p, n, m, r in [(1, 3, 10, 0), (5, 2, 40, 3), (37, 6, 5000, 11), (1000, 9, 300000, 999), (9001, 4, 90000, 77),
                       (1152, 1658, 100000000, 0)]:
        print("plan rounds: p=%d n=%d m=%d" % (p, n, m), flush=True)
        sizes, displs = synth.irregular_sizes(p, m)
        R = bcs.bcs_rounds(p, n)
        pack_t = torch.empty((R, p), dtype=torch.int32, device="cuda")
        unpack_t = torch.empty((R, p), dtype=torch.int32, device="cuda")
        bcs.bcs_allgather_tables(p, n, r, pack_t, unpack_t)
        data = rng.integers(0, 1 << 30, max(1, int(displs[-1]))).astype(np.int32)
        d_data = torch.from_numpy(data).cuda()
        d_displs = torch.from_numpy(displs).cuda()
        offs = torch.full((R, p + 1), -1, dtype=torch.int64, device="cuda")
        srcs = torch.full((R, p), -1, dtype=torch.int64, device="cuda")
        bcs.bcs_pack_plan_rounds(n, pack_t, d_displs, offs, srcs)
        uoffs = torch.full((R, p + 1), -1, dtype=torch.int64, device="cuda")
        usrcs = torch.full((R, p), -1, dtype=torch.int64, device="cuda")
        bcs.bcs_pack_plan_rounds(n, unpack_t, d_displs, uoffs, usrcs)
        torch.cuda.synchronize()
        h_pack, h_unpack = pack_t.cpu().numpy(), unpack_t.cpu().numpy()
        h_offs, h_uoffs = offs.cpu().numpy(), uoffs.cpu().numpy()
        cap = int(h_offs[:, p].max()) + 8
        d_msg = torch.empty(cap, dtype=torch.int32, device="cuda")
        blank = np.full_like(data, -5)
        d_blank = torch.full((len(data),), -5, dtype=torch.int32, device="cuda")
        rounds = range(R) if R <= 300 else sorted(set(range(0, R, 7)) | {0, 1, R - 2, R - 1})
        for j in range(R):
            # the plan rows of every round against the oracle's pack loop (it also gives the offsets)
            if j in rounds or p <= 1152:
                omsg, ooff = oracle.pack_round(n, h_pack[j], displs, data)
                assert np.array_equal(h_offs[j], ooff), (p, n, j)
            if j not in rounds:
                continue
            d_msg.fill_(-99)
            bcs.bcs_pack_round_planned(offs[j], srcs[j], d_data, d_msg)
            torch.cuda.synchronize()
            got = d_msg.cpu().numpy()
            assert np.array_equal(got[:len(omsg)], omsg) and (got[len(omsg):] == -99).all(), (p, n, j)
            # what this process receives in round j has the lengths of its unpack row: take the data's own blocks
            umsg, uoff = oracle.pack_round(n, h_unpack[j], displs, data)
            assert np.array_equal(h_uoffs[j], uoff), (p, n, j)
            oracle.unpack_round(n, h_unpack[j], displs, blank, umsg)
            d_umsg = torch.from_numpy(umsg).cuda() if len(umsg) else torch.empty(0, dtype=torch.int32, device="cuda")
            bcs.bcs_unpack_round_planned(uoffs[j], usrcs[j], d_blank, d_umsg, len(umsg))
        torch.cuda.synchronize()
        assert np.array_equal(d_blank.cpu().numpy(), blank), (p, n)
        del pack_t, unpack_t, d_data, d_blank, offs, srcs, uoffs, usrcs, d_msg
        torch.cuda.empty_cache()


def test_allgather_tables_and_messages_beyond_32_bit_sizes(bcs, oracle):
    """Index tables of 2 x 4.4 G entries and a packed message of 4.1 G elements: the 64-bit paths, checked on the
    device against the defining index arithmetic (Alg. 9; Alg. 6 for the round shift) written with tensor operations."""
    p, n, r = (1 << 23) + 1, 500, 1234567
    q, R = bcs.bcs_q(p), bcs.bcs_rounds(p, n)
    assert R * p > 1 << 32
    skips = bcs.bcs_skips(p)
    recv, _ = dev_tables(p, q)
    bcs.bcs_sched(p, 0, p, recv, None)
    pack = torch.full((R, p), 4242, dtype=torch.int32, device="cuda")
    unpack = torch.full((R, p), 4242, dtype=torch.int32, device="cuda")
    bcs.bcs_allgather_tables(p, n, r, pack, unpack)
    torch.cuda.synchronize()
    orecv, _ = oracle.sched_range(p, want_send=False, threads=16)
    assert np.array_equal(recv.cpu().numpy(), orecv)
    del orecv
    x = (q - R % q) % q
    vr = (r - torch.arange(p, device="cuda")) % p                  # virtual rank of r towards each root
    cols = [recv[:, k].contiguous() for k in range(q)]
    for j in range(R):
        k = (x + j) % q
        assert torch.equal(unpack[j], (cols[k][vr] + (j - k)).clamp_(min=-1, max=n - 1)), j
        assert torch.equal(pack[j], (cols[k][(vr + int(skips[k])) % p] + (j - k)).clamp_(min=-1, max=n - 1)), j
    del pack, unpack, recv, cols, vr
    bcs.bcs_release()
    torch.cuda.empty_cache()

    from paper_2205_10072_amd import synth
    p, n = 1152, 2
    sizes, displs = synth.irregular_sizes(p, 1 << 33)
    total = int(displs[-1])
    rng = np.random.default_rng(9)
    idx = rng.integers(0, n, p).astype(np.int32)
    idx[rng.integers(0, p, 40)] = -1                                # some roots send nothing
    begin = np.where(idx >= 0, idx.astype(np.int64) * sizes // n, 0)
    length = np.where(idx >= 0, (idx.astype(np.int64) + 1) * sizes // n - begin, 0)
    offsets = np.concatenate([[0], np.cumsum(length)]).astype(np.int64)
    msg_len = int(offsets[-1])
    assert msg_len > 1 << 31                                       # element indices do not fit in int32
    data = torch.randint(0, 1 << 30, (total,), dtype=torch.int32, device="cuda")
    d_idx, d_displs = torch.from_numpy(idx).cuda(), torch.from_numpy(displs).cuda()
    d_msg = torch.full((msg_len + 4,), -99, dtype=torch.int32, device="cuda")
    d_off = torch.full((p + 1,), -1, dtype=torch.int64, device="cuda")
    ws = torch.empty(bcs.bcs_pack_workspace_bytes(p), dtype=torch.uint8, device="cuda")
    bcs.bcs_pack_round(n, d_idx, d_displs, data, d_msg[:msg_len], d_off, ws)
    torch.cuda.synchronize()
    assert np.array_equal(d_off.cpu().numpy(), offsets)
    assert bool((d_msg[msg_len:] == -99).all())
    for j in range(p):
        src = int(displs[j] + begin[j])
        assert torch.equal(d_msg[int(offsets[j]):int(offsets[j + 1])], data[src:src + int(length[j])]), j
    blank = torch.full((total,), -5, dtype=torch.int32, device="cuda")
    bcs.bcs_unpack_round(n, d_idx, d_displs, blank, d_msg[:msg_len], msg_len, d_off, ws)
    torch.cuda.synchronize()
    for j in range(p):
        lo, src = int(displs[j]), int(displs[j] + begin[j])
        assert torch.equal(blank[src:src + int(length[j])], data[src:src + int(length[j])]), j
        assert bool((blank[lo:src] == -5).all()) and bool((blank[src + int(length[j]):int(displs[j + 1])] == -5).all()), j
    del data, blank, d_msg
    torch.cuda.empty_cache()


def test_irregular_allgather_on_the_gpu_moves_all_the_data(bcs):
    """The whole allgather of Alg. 9 with payload, every process simulated on the one GPU with the library's own
    tables, pack and unpack: at the end every process holds every buffer."""
    from paper_2205_10072_amd import synth
    for p, n, m in [(5, 3, 170), (20, 5, 4001), (33, 6, 50000)]:
        sizes, displs = synth.irregular_sizes(p, m)
        total = int(displs[-1])
        truth = (np.arange(total, dtype=np.int64) * 2654435761 % 2147483647).astype(np.int32)
        q, R = bcs.bcs_q(p), bcs.bcs_rounds(p, n)
        skips = bcs.bcs_skips(p)
        x = (q - R % q) % q
        d_displs = torch.from_numpy(displs).cuda()
        tabs, data = [], []
        for r in range(p):
            pack, unpack = dev_tables(R, p)
            bcs.bcs_allgather_tables(p, n, r, pack, unpack)
            tabs.append((pack, unpack))
            mine = np.full(total, -7, dtype=np.int32)
            mine[displs[r]:displs[r + 1]] = truth[displs[r]:displs[r + 1]]
            data.append(torch.from_numpy(mine).cuda())
        ws = torch.empty(bcs.bcs_pack_workspace_bytes(p), dtype=torch.uint8, device="cuda")
        off = torch.empty(p + 1, dtype=torch.int64, device="cuda")
        for j in range(R):
            k = (x + j) % q
            msgs, lens = [], []
            for r in range(p):
                msg = torch.empty(total // n + p + 8, dtype=torch.int32, device="cuda")
                bcs.bcs_pack_round(n, tabs[r][0][j], d_displs, data[r], msg, off, ws)
                torch.cuda.synchronize()
                lens.append(int(off[p]))
                assert lens[-1] <= msg.numel()
                msgs.append(msg)
            for r in range(p):
                t = (r + skips[k]) % p
                bcs.bcs_unpack_round(n, tabs[t][1][j], d_displs, data[t], msgs[r], lens[r], off, ws)
            torch.cuda.synchronize()
        for r in range(p):
            assert np.array_equal(data[r].cpu().numpy(), truth), (p, n, r)
