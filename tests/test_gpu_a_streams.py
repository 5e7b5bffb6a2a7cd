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
