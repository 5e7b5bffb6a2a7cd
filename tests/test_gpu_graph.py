"""The calls that allocate nothing (the *_ws entry points, bcs_expand, bcs_sched_batch) recorded into a HIP graph and
replayed: every replay, with the outputs overwritten and other work in between, gives the oracle's tables."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def test_graph_replays_of_the_no_allocation_calls(oracle):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2205_10072_amd as bcs
    bcs.lib()
    p, root, n = 70001, 4242, 300          # byte-row path; the allgather tables and a pack round ride along
    q, R = bcs.bcs_q(p), bcs.bcs_rounds(p, n)
    recv = torch.zeros((p, q), dtype=torch.int32, device="cuda")
    send = torch.zeros_like(recv)
    rb = torch.zeros((p, R), dtype=torch.int32, device="cuda")
    sb = torch.zeros_like(rb)
    rb2 = torch.zeros_like(rb)
    ws = torch.empty(bcs.bcs_sched_expand_workspace_bytes(p, n), dtype=torch.uint8, device="cuda")
    ws2 = torch.empty(max(16, bcs.bcs_expand_workspace_bytes(p, n, 0, p)), dtype=torch.uint8, device="cuda")
    pa, n_ag, r_ag = 3001, 9, 17
    pack = torch.zeros((bcs.bcs_rounds(pa, n_ag), pa), dtype=torch.int32, device="cuda")
    unpack = torch.zeros_like(pack)
    ws3 = torch.empty(bcs.bcs_allgather_workspace_bytes(pa), dtype=torch.uint8, device="cuda")

    def work():
        bcs.bcs_sched_expand_ws(p, root, n, recv, send, rb, sb, ws)
        bcs.bcs_expand_ws(p, n, 0, p, recv, None, rb2, None, ws2)
        bcs.bcs_allgather_tables_ws(pa, n_ag, r_ag, pack, unpack, ws3)

    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        work()                              # eager once: the library's table is filled outside the capture
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            work()
    torch.cuda.synchronize()
    orecv, osend = oracle.sched_range(p, root=root, threads=16)
    want_r, want_s = oracle.expand(p, n, orecv, threads=16), oracle.expand(p, n, osend, threads=16)
    opack, ounpack = oracle.allgather_tables(pa, n_ag, r_ag)
    for replay in range(4):
        for t in (recv, send, rb, sb, rb2, pack, unpack):
            t.fill_(-77 - replay)           # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(recv.cpu().numpy(), orecv) and np.array_equal(send.cpu().numpy(), osend), replay
        assert np.array_equal(rb.cpu().numpy(), want_r) and np.array_equal(sb.cpu().numpy(), want_s), replay
        assert np.array_equal(rb2.cpu().numpy(), want_r), replay
        assert np.array_equal(pack.cpu().numpy(), opack) and np.array_equal(unpack.cpu().numpy(), ounpack), replay
