"""Runs before the other GPU tests (file name order), so that the library's low-level table has not been filled
yet: the first two calls go out on two different streams, the second of which must be made to wait for the fill
that the first one enqueued.  Then: calls on a non-default stream with their own workspace."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def test_first_calls_on_two_streams_and_side_stream_use(oracle):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2205_10072_amd as bcs
    bcs.lib()
    p = 100003
    q = bcs.bcs_q(p)
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    ra = torch.full((p, q), 1, dtype=torch.int32, device="cuda")
    rb = torch.full((p, q), 2, dtype=torch.int32, device="cuda")
    sbuf = torch.full((p, q), 3, dtype=torch.int32, device="cuda")
    ws = torch.empty(bcs.bcs_sched_workspace_bytes(p, 0, p), dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    bcs.bcs_sched_rooted_ws(p, 0, 0, p, ra, None, None, stream=sa)        # enqueues the table fill on stream a
    bcs.bcs_sched_rooted_ws(p, 5, 0, p, rb, sbuf, ws, stream=sb)          # must wait for it on the device
    torch.cuda.synchronize()
    o0, _ = oracle.sched_range(p, threads=8)
    o5r, o5s = oracle.sched_range(p, root=5, threads=8)
    assert np.array_equal(ra.cpu().numpy(), o0)
    assert np.array_equal(rb.cpu().numpy(), o5r)
    assert np.array_equal(sbuf.cpu().numpy(), o5s)
    # expansion and batch on a side stream
    n = 19
    R = bcs.bcs_rounds(p, n)
    eb = torch.empty((p, R), dtype=torch.int32, device="cuda")
    with torch.cuda.stream(sb):
        bcs.bcs_expand(p, n, 0, p, rb, None, eb, None)                    # binding picks up the current stream
    sb.synchronize()
    assert np.array_equal(eb.cpu().numpy(), oracle.expand(p, n, o5r, threads=8))


def test_plain_calls_on_two_streams_share_the_scratch_in_order(oracle):
    """Plain calls keep one scratch allocation per device.  Two of them on different streams, enqueued back to
    back with no synchronisation in between, must not overwrite each other's tables: the library makes the
    second wait for the first on the device."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2205_10072_amd as bcs
    bcs.lib()
    pa, pb = 300007, 299993                     # same q, different skips: a mixed-up scratch cannot go unnoticed
    q = bcs.bcs_q(pa)
    assert bcs.bcs_q(pb) == q
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    ra, xa = (torch.full((pa, q), 1, dtype=torch.int32, device="cuda") for _ in range(2))
    rb, xb = (torch.full((pb, q), 2, dtype=torch.int32, device="cuda") for _ in range(2))
    torch.cuda.synchronize()
    for _ in range(3):
        bcs.bcs_sched_rooted(pa, 11, 0, pa, ra, xa, stream=sa)
        bcs.bcs_sched_rooted(pb, 0, 0, pb, rb, xb, stream=sb)
    torch.cuda.synchronize()
    oar, oas = oracle.sched_range(pa, root=11, threads=8)
    obr, obs = oracle.sched_range(pb, threads=8)
    assert np.array_equal(ra.cpu().numpy(), oar) and np.array_equal(xa.cpu().numpy(), oas)
    assert np.array_equal(rb.cpu().numpy(), obr) and np.array_equal(xb.cpu().numpy(), obs)
