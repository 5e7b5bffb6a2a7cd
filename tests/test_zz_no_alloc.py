"""Collected last (file name order): the entry point that allocates nothing (bcs_sched_rooted_static: scratch in a fixed array inside the library)
against bcs_sched_rooted, bit for bit, through the C ABI.  Two calls in a row, the second with a smaller input,
so that whatever the first left in the shared array is still there; then a part of the ranks with send rows by
Alg. 5 (which takes the table of digit masks from the same array), and a size beyond the array."""
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _both(bcs, p, root, r0, r1, want_recv=True, want_send=True):
    q = bcs.bcs_q(p)
    rows = r1 - r0
    got = [torch.full((rows, q), 777, dtype=torch.int32, device="cuda") for _ in range(2)]
    ref = [torch.full((rows, q), 555, dtype=torch.int32, device="cuda") for _ in range(2)]
    bcs.bcs_sched_rooted_static(p, root, r0, r1, got[0] if want_recv else None, got[1] if want_send else None)
    torch.cuda.synchronize()
    bcs.bcs_sched_rooted(p, root, r0, r1, ref[0] if want_recv else None, ref[1] if want_send else None)
    torch.cuda.synchronize()
    if want_recv:
        assert torch.equal(got[0], ref[0]), ("recv", p, root, r0, r1)
    if want_send:
        assert torch.equal(got[1], ref[1]), ("send", p, root, r0, r1)
    return got


def test_static_scratch_entry_point_equals_the_allocating_one(oracle):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import numpy as np
    import paper_2205_10072_amd as bcs
    bcs.lib()
    print("static: p=1048577 root=12345 all ranks", flush=True)
    _both(bcs, (1 << 20) + 1, 12345, 0, (1 << 20) + 1)
    print("static: p=1000 root=7 all ranks (smaller, right after)", flush=True)
    small = _both(bcs, 1000, 7, 0, 1000)
    orecv, osend = oracle.sched_range(1000, root=7)
    assert np.array_equal(small[0].cpu().numpy(), orecv) and np.array_equal(small[1].cpu().numpy(), osend)
    print("static: the largest p the array holds, send rows only", flush=True)
    _both(bcs, 1342016, 0, 0, 1342016, want_recv=False)
    print("static: p=65537, ranks 100..60100, send rows by Alg. 5 with the digit table", flush=True)
    assert bcs.bcs_sched_workspace_bytes(65537, 100, 60100) > 0
    _both(bcs, 65537, 3, 100, 60100)
    print("static: p=2 and p=1", flush=True)
    _both(bcs, 2, 1, 0, 2)
    bcs.bcs_sched_rooted_static(1, 0, 0, 1, small[0], small[1])
    print("static: beyond the array", flush=True)
    p = 1342017
    t = torch.empty((p, 21), dtype=torch.int32, device="cuda")
    with pytest.raises(bcs.BcsError) as err:
        bcs.bcs_sched_rooted_static(p, 0, 0, p, t, t)
    assert err.value.code == bcs.ETOOBIG
    bcs.bcs_sched_rooted_static(p, 0, 0, p, t, None)      # receive rows alone need no scratch at any size
    torch.cuda.synchronize()
