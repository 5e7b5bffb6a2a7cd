"""Partner tables of the regular allgather (Alg. 7) and the census (Alg. 8) written on the device for ranges of
processes: against the oracle's per-process plans, and by running both collectives for all processes at once with
the device tables."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def bcs():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2205_10072_amd as lib
    lib.lib()
    return lib


def tables(bcs, fn, p, r0, r1, misalign=0):
    q = bcs.bcs_q(p)
    n = (r1 - r0) * q
    raw = [torch.full((n + 8,), 777, dtype=torch.int32, device="cuda") for _ in range(2)]
    to, frm = (t[misalign:misalign + n] for t in raw)
    fn(p, r0, r1, to, frm)
    torch.cuda.synchronize()
    for t in raw:                                         # nothing outside the table is touched
        assert (t[:misalign] == 777).all() and (t[misalign + n:] == 777).all()
    return to.view(r1 - r0, q), frm.view(r1 - r0, q)


def oracle_rows(plan_of, p, ranks):
    q = (p - 1).bit_length()
    plans = [plan_of(p, int(r)) for r in ranks]
    to = np.array([pl[0] for pl in plans], dtype=np.int32).reshape(len(plans), q)
    frm = np.array([pl[1] for pl in plans], dtype=np.int32).reshape(len(plans), q)
    return to, frm


SMALL = list(range(1, 70)) + [100, 127, 128, 129, 255, 257, 1000]


def test_partner_tables_equal_the_oracle(bcs, oracle):
    for name, fn, plan_of in (("allgather", bcs.bcs_allgather_partners, oracle.allgather_plan),
                              ("census", bcs.bcs_census_partners, oracle.census_plan)):
        for p in SMALL:
            to, frm = tables(bcs, fn, p, 0, p, misalign=p % 3)
            oto, ofrm = oracle_rows(plan_of, p, range(p))
            assert np.array_equal(to.cpu().numpy(), oto) and np.array_equal(frm.cpu().numpy(), ofrm), (name, p)
        rng = np.random.default_rng(78)
        big = [1048577, 134217727, 2**31 - 1, 2**30, 2**30 + 1] + [int(v) for v in rng.integers(2**20, 2**31 - 1, 6)]
        for p in big:
            # ragged ranges at both ends of the ring and in the middle; some rows of each against the oracle
            for r0, r1 in ((0, 70001), (p - 70003, p), (p // 2 - 5, p // 2 + 33333)):
                to, frm = tables(bcs, fn, p, r0, r1, misalign=int(rng.integers(0, 4)))
                pick = np.unique(np.concatenate([[0, 1, r1 - r0 - 2, r1 - r0 - 1], rng.integers(0, r1 - r0, 40)]))
                oto, ofrm = oracle_rows(plan_of, p, r0 + pick)
                assert np.array_equal(to.cpu().numpy()[pick], oto), (name, p, r0)
                assert np.array_equal(frm.cpu().numpy()[pick], ofrm), (name, p, r0)
                # and every row by what the two tables are: inverse permutations of the ring, round by round
                skips = np.array(bcs.bcs_skips(p), dtype=np.int64)
                dist = (frm.cpu().numpy().astype(np.int64) - (r0 + np.arange(r1 - r0))[:, None]) % p
                back = ((r0 + np.arange(r1 - r0))[:, None] - to.cpu().numpy().astype(np.int64)) % p
                assert np.array_equal(dist, back)
                assert (dist == dist[0]).all()
                odd = 2 * skips[:-1] > skips[1:]
                assert np.array_equal(dist[0], skips[:-1] - (odd if name == "census" else 0)), (name, p)


def test_partner_calls_check_their_arguments(bcs):
    t = torch.empty(64, dtype=torch.int32, device="cuda")
    L = bcs.lib()
    for fn in (L.bcs_allgather_partners, L.bcs_census_partners):
        assert fn(0, 0, 0, t.data_ptr(), t.data_ptr(), None) == bcs.EINVAL
        assert fn(10, 3, 2, t.data_ptr(), t.data_ptr(), None) == bcs.EINVAL
        assert fn(10, 0, 11, t.data_ptr(), t.data_ptr(), None) == bcs.EINVAL
        assert fn(10, -1, 4, t.data_ptr(), t.data_ptr(), None) == bcs.EINVAL
        assert fn(10, 0, 4, None, None, None) == bcs.EINVAL
        assert fn(1, 0, 1, t.data_ptr(), None, None) == 0          # q = 0: nothing to write
        assert fn(10, 4, 4, t.data_ptr(), None, None) == 0
    with pytest.raises(ValueError):
        bcs.bcs_allgather_partners(100, 0, 100, t, None)            # 700 entries needed
    torch.cuda.synchronize()


def test_device_tables_run_both_collectives_for_all_processes(bcs):
    """Alg. 7: every process starts with its own block in buffer[0] and must end with the block of (r + i) mod p in
    buffer[i].  Alg. 8: every process must end with the sum of all inputs.  All processes at once, one indexed
    copy / addition per round, with the partners taken from the device tables."""
    for p in [1, 2, 3, 5, 17, 20, 33, 100, 1000, 4097, 6000]:
        q = bcs.bcs_q(p)
        skips = bcs.bcs_skips(p)
        ranks = torch.arange(p, device="cuda")
        to, frm = (t.long() for t in tables(bcs, bcs.bcs_allgather_partners, p, 0, p))
        buf = torch.full((p, p), -1, dtype=torch.int64, device="cuda")
        buf[:, 0] = ranks
        for k in range(q):
            count, first = skips[k + 1] - skips[k], skips[k]
            assert torch.equal(to[frm[:, k], k], ranks) and torch.equal(frm[to[:, k], k], ranks)
            assert count <= first                                       # a process sends blocks it already holds
            buf[:, first:first + count] = buf[frm[:, k], 0:count]
        assert torch.equal(buf, (ranks[:, None] + ranks[None, :]) % p), p
        del buf
        to, frm = (t.long() for t in tables(bcs, bcs.bcs_census_partners, p, 0, p))
        own = bcs.bcs_census_plan(p, 0)[2]
        g = torch.Generator(device="cpu").manual_seed(p)
        x = torch.randint(-2**40, 2**40, (p,), generator=g).cuda()
        S = torch.zeros(p, dtype=torch.int64, device="cuda")
        for k in range(q):
            assert torch.equal(to[frm[:, k], k], ranks) and torch.equal(frm[to[:, k], k], ranks)
            out = S + x if own[k] else S
            S = S + out[frm[:, k]]
        assert (S + x == x.sum()).all(), p
