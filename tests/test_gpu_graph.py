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


def test_graph_replays_of_planned_pack_and_unpack_rounds(oracle):
    """Rounds of Alg. 9's pack / unpack loops with their plans made ahead are one copy kernel each and launch bound at
    the paper's sizes, which is what a HIP graph is for: twelve rounds (pack into a message, unpack the message into a
    second copy of the buffers) recorded once and replayed four times, every message and the buffers against the
    oracle's loops."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2205_10072_amd as bcs
    from paper_2205_10072_amd import synth
    bcs.lib()
    p, n, m, r = 1152, 40, 500000, 5
    sizes, displs = synth.irregular_sizes(p, m)
    R = bcs.bcs_rounds(p, n)
    pack_t = torch.empty((R, p), dtype=torch.int32, device="cuda")
    unpack_t = torch.empty((R, p), dtype=torch.int32, device="cuda")
    bcs.bcs_allgather_tables(p, n, r, pack_t, unpack_t)
    rng = np.random.default_rng(9)
    data = rng.integers(0, 1 << 30, int(displs[-1])).astype(np.int32)
    d_data = torch.from_numpy(data).cuda()
    d_displs = torch.from_numpy(displs).cuda()
    offs = torch.empty((R, p + 1), dtype=torch.int64, device="cuda")
    srcs = torch.empty((R, p), dtype=torch.int64, device="cuda")
    bcs.bcs_pack_plan_rounds(n, pack_t, d_displs, offs, srcs)
    torch.cuda.synchronize()
    h_pack, h_offs = pack_t.cpu().numpy(), offs.cpu().numpy()
    rounds = list(range(3, 15))
    cap = (int(h_offs[rounds, p].max()) + 15) // 4 * 4 + 4
    msgs = torch.zeros((len(rounds), cap), dtype=torch.int32, device="cuda")
    d_copy = torch.zeros_like(d_data)
    rows = [(offs[j], srcs[j], int(h_offs[j, p])) for j in rounds]

    def work():
        for i, (o, s, length) in enumerate(rows):
            bcs.bcs_pack_round_planned(o, s, d_data, msgs[i])
            bcs.bcs_unpack_round_planned(o, s, d_copy, msgs[i], length)

    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        work()
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            work()
    torch.cuda.synchronize()
    want_copy = np.full_like(data, -7)
    want_msgs = []
    for j in rounds:
        omsg, _ = oracle.pack_round(n, h_pack[j], displs, data)
        oracle.unpack_round(n, h_pack[j], displs, want_copy, omsg)
        want_msgs.append(omsg)
    for replay in range(4):
        msgs.fill_(-3 - replay)
        d_copy.fill_(-7)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = msgs.cpu().numpy()
        for i, omsg in enumerate(want_msgs):
            assert np.array_equal(got[i, :len(omsg)], omsg) and (got[i, len(omsg):] == -3 - replay).all(), (replay, i)
        assert np.array_equal(d_copy.cpu().numpy(), want_copy), replay
