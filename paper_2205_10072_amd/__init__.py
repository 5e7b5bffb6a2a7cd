"""Python binding of libbcsched (round-optimal broadcast schedules on MI355X).

Argument marshalling only: every function here hands device pointers and a
stream to the C ABI declared in ``include/bcsched.h`` and returns.  PyTorch is
used for device memory and streams, nothing else.  There is no CPU fallback:
if ``libbcsched.so`` is not built, importing the library functions raises.

Method: J. L. Traff, arXiv 2205.10072, Section 2.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbcsched.so")

OK, EINVAL, EHIP, ENOMEM, ETOOBIG = 0, -1, -2, -3, -4
STATIC_SCRATCH_BYTES = 32 << 20  # BCS_STATIC_SCRATCH_BYTES
MAX_Q = 31
BATCH_STRIDE = 32
BATCH_PAD = -(2 ** 31)
NO_BLOCK = -1
MAX_N = 2**31 - 1 - 64          # BCS_MAX_N

# every symbol include/bcsched.h declares
SYMBOLS = (
    "bcs_q", "bcs_skips", "bcs_rounds", "bcs_sched", "bcs_sched_rooted", "bcs_sched_workspace_bytes",
    "bcs_sched_rooted_ws", "bcs_sched_rooted_static", "bcs_sched_batch", "bcs_expand", "bcs_sched_expand", "bcs_sched_expand_ws",
    "bcs_sched_expand_workspace_bytes", "bcs_expand_ws", "bcs_expand_workspace_bytes",
    "bcs_release", "bcs_strerror",
    "bcs_last_hip_error", "bcs_timing_begin", "bcs_timing_end", "bcs_timing_stats", "bcs_kernel_name", "bcs_valu_peak_launch",
    "bcs_allgather_workspace_bytes", "bcs_allgather_tables", "bcs_allgather_tables_ws",
    "bcs_pack_workspace_bytes", "bcs_pack_round", "bcs_unpack_round", "bcs_allgather_plan", "bcs_census_plan",
    "bcs_pack_plan_rounds", "bcs_pack_round_planned", "bcs_unpack_round_planned",
    "bcs_allgather_partners", "bcs_census_partners",
)
KERNEL_COUNT = 16
VALU_PEAK_OPS_PER_ITER = 32

_lib = None


class BcsError(RuntimeError):
    def __init__(self, code, what):
        self.code = code
        msg = "%s: %s (code %d)" % (what, _strerror(code), code)
        if code == EHIP and _lib is not None:
            msg += ", hipError %d" % _lib.bcs_last_hip_error()
        super().__init__(msg)


def lib():
    """The loaded C library; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError("libbcsched.so is not built: run `python -m paper_2205_10072_amd.build` "
                          "(or __graft_entry__.build()); there is no fallback path")
    L = ctypes.CDLL(LIB_PATH)
    i32, i64, vp, sz = ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p, ctypes.c_size_t
    L.bcs_q.argtypes = [i32]
    L.bcs_skips.argtypes = [i32, vp]
    L.bcs_rounds.argtypes = [i32, i32]
    L.bcs_rounds.restype = i64
    L.bcs_sched.argtypes = [i32, i32, i32, vp, vp, vp]
    L.bcs_sched_rooted.argtypes = [i32, i32, i32, i32, vp, vp, vp]
    L.bcs_sched_workspace_bytes.argtypes = [i32, i32, i32, ctypes.c_int]
    L.bcs_sched_workspace_bytes.restype = i64
    L.bcs_sched_rooted_ws.argtypes = [i32, i32, i32, i32, vp, vp, vp, sz, vp]
    L.bcs_sched_rooted_static.argtypes = [i32, i32, i32, i32, vp, vp, vp]
    L.bcs_sched_batch.argtypes = [i64, vp, vp, vp, vp, vp, vp, vp]
    L.bcs_expand.argtypes = [i32, i32, i32, i32, vp, vp, vp, vp, vp]
    L.bcs_expand_workspace_bytes.argtypes = [i32, i32, i32, i32]
    L.bcs_expand_workspace_bytes.restype = i64
    L.bcs_expand_ws.argtypes = [i32, i32, i32, i32, vp, vp, vp, vp, vp, sz, vp]
    L.bcs_sched_expand_workspace_bytes.argtypes = [i32, i32]
    L.bcs_sched_expand_workspace_bytes.restype = i64
    L.bcs_sched_expand.argtypes = [i32, i32, i32, vp, vp, vp, vp, vp]
    L.bcs_sched_expand_ws.argtypes = [i32, i32, i32, vp, vp, vp, vp, vp, sz, vp]
    L.bcs_release.argtypes = []
    L.bcs_strerror.argtypes = [ctypes.c_int]
    L.bcs_strerror.restype = ctypes.c_char_p
    L.bcs_last_hip_error.argtypes = []
    L.bcs_timing_begin.argtypes = []
    L.bcs_timing_end.argtypes = [vp, vp]
    L.bcs_timing_stats.argtypes = [vp, vp, vp, vp]
    L.bcs_kernel_name.argtypes = [ctypes.c_int]
    L.bcs_kernel_name.restype = ctypes.c_char_p
    L.bcs_valu_peak_launch.argtypes = [ctypes.c_uint32, ctypes.c_uint32, vp, vp]
    L.bcs_allgather_workspace_bytes.argtypes = [i32]
    L.bcs_allgather_workspace_bytes.restype = i64
    L.bcs_allgather_tables.argtypes = [i32, i32, i32, vp, vp, vp]
    L.bcs_allgather_tables_ws.argtypes = [i32, i32, i32, vp, vp, vp, sz, vp]
    L.bcs_allgather_plan.argtypes = [i32, i32, vp, vp, vp, vp]
    L.bcs_census_plan.argtypes = [i32, i32, vp, vp, vp]
    L.bcs_allgather_partners.argtypes = [i32, i32, i32, vp, vp, vp]
    L.bcs_census_partners.argtypes = [i32, i32, i32, vp, vp, vp]
    L.bcs_pack_workspace_bytes.argtypes = [i32]
    L.bcs_pack_workspace_bytes.restype = i64
    L.bcs_pack_round.argtypes = [i32, i32, vp, vp, vp, vp, i64, vp, vp, sz, vp]
    L.bcs_unpack_round.argtypes = [i32, i32, vp, vp, vp, vp, i64, vp, vp, sz, vp]
    L.bcs_pack_plan_rounds.argtypes = [i32, i32, i64, vp, vp, vp, vp, vp]
    L.bcs_pack_round_planned.argtypes = [i32, vp, vp, vp, vp, i64, vp]
    L.bcs_unpack_round_planned.argtypes = [i32, vp, vp, vp, vp, i64, vp]
    _lib = L
    return L


def _strerror(code):
    try:
        return lib().bcs_strerror(code).decode()
    except Exception:  # library missing: still produce a message
        return "bcsched error"


def _check(code, what):
    if code < 0:
        raise BcsError(int(code), what)
    return code


def _need(t, numel, what):
    """Raises ValueError when tensor `t` (or None) holds fewer than `numel` elements: the kernels trust the sizes
    the C ABI is given, so a table that is too small must be stopped here."""
    if t is not None and t.numel() < numel:
        raise ValueError("%s: tensor of %d elements, %d needed" % (what, t.numel(), numel))


def _ptr(t, numel=0, what="tensor"):
    """Device pointer of an int32, contiguous CUDA/HIP tensor of at least `numel` elements (None -> NULL)."""
    if t is None:
        return None
    import torch
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.int32 and t.is_contiguous()):
        raise TypeError("expected a contiguous int32 tensor in device memory")
    _need(t, numel, what)
    return ctypes.c_void_p(t.data_ptr())


def _rows(r0, r1):
    return max(int(r1) - int(r0), 0)


def _ws(workspace):
    """(pointer, bytes) of a workspace tensor of any dtype (None or empty -> NULL, 0)."""
    if workspace is None or workspace.numel() == 0:
        return None, 0
    if not workspace.is_cuda or not workspace.is_contiguous():
        raise TypeError("expected a contiguous workspace tensor in device memory")
    return ctypes.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size()


def _stream(stream):
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def bcs_q(p):
    return _check(lib().bcs_q(p), "bcs_q")


def bcs_skips(p):
    """Alg. 1: list of the q+1 skips."""
    q = bcs_q(p)
    buf = (ctypes.c_int32 * (q + 1))()
    _check(lib().bcs_skips(p, ctypes.cast(buf, ctypes.c_void_p)), "bcs_skips")
    return list(buf)


def bcs_rounds(p, n):
    return _check(lib().bcs_rounds(p, n), "bcs_rounds")


def bcs_sched(p, r0, r1, recv_out, send_out, stream=None):
    need = _rows(r0, r1) * bcs_q(p)
    _check(lib().bcs_sched(p, r0, r1, _ptr(recv_out, need, "recv_out"), _ptr(send_out, need, "send_out"),
                           _stream(stream)), "bcs_sched")


def bcs_sched_rooted(p, root, r0, r1, recv_out, send_out, stream=None):
    need = _rows(r0, r1) * bcs_q(p)
    _check(lib().bcs_sched_rooted(p, root, r0, r1, _ptr(recv_out, need, "recv_out"), _ptr(send_out, need, "send_out"),
                                  _stream(stream)), "bcs_sched_rooted")


def bcs_sched_workspace_bytes(p, r0, r1, want_send=True):
    return _check(lib().bcs_sched_workspace_bytes(p, r0, r1, 1 if want_send else 0), "bcs_sched_workspace_bytes")


def bcs_sched_rooted_ws(p, root, r0, r1, recv_out, send_out, workspace, stream=None):
    """`workspace`: a device tensor of any dtype (or None when no scratch is needed)."""
    wp, wb = _ws(workspace)
    need = _rows(r0, r1) * bcs_q(p)
    _check(lib().bcs_sched_rooted_ws(p, root, r0, r1, _ptr(recv_out, need, "recv_out"),
                                     _ptr(send_out, need, "send_out"), wp, wb, _stream(stream)),
           "bcs_sched_rooted_ws")


def bcs_sched_rooted_static(p, root, r0, r1, recv_out, send_out, stream=None):
    """bcs_sched_rooted on the library's fixed scratch array: allocates nothing (raises ETOOBIG beyond its size)."""
    need = _rows(r0, r1) * bcs_q(p)
    _check(lib().bcs_sched_rooted_static(p, root, r0, r1, _ptr(recv_out, need, "recv_out"),
                                         _ptr(send_out, need, "send_out"), _stream(stream)),
           "bcs_sched_rooted_static")


def bcs_sched_batch(p, r, root, recv_out, send_out, q_out, stream=None):
    count = p.numel()
    rows = count * BATCH_STRIDE
    _check(lib().bcs_sched_batch(count, _ptr(p), _ptr(r, count, "r"), _ptr(root, count, "root"),
                                 _ptr(recv_out, rows, "recv_out"), _ptr(send_out, rows, "send_out"),
                                 _ptr(q_out, count, "q_out"), _stream(stream)), "bcs_sched_batch")


def _expand_sizes(p, n, rows):
    q = bcs_q(p)
    return rows * q, rows * (max(int(n), 1) - 1 + q)


def bcs_expand(p, n, r0, r1, recv, send, recv_blocks, send_blocks, stream=None):
    nq, nr = _expand_sizes(p, n, _rows(r0, r1))
    _check(lib().bcs_expand(p, n, r0, r1, _ptr(recv, nq, "recv"), _ptr(send, nq, "send"),
                            _ptr(recv_blocks, nr, "recv_blocks"), _ptr(send_blocks, nr, "send_blocks"),
                            _stream(stream)), "bcs_expand")


def bcs_expand_workspace_bytes(p, n, r0, r1):
    return _check(lib().bcs_expand_workspace_bytes(p, n, r0, r1), "bcs_expand_workspace_bytes")


def bcs_expand_ws(p, n, r0, r1, recv, send, recv_blocks, send_blocks, workspace, stream=None):
    """`workspace`: a device tensor of any dtype (or None)."""
    wp, wb = _ws(workspace)
    nq, nr = _expand_sizes(p, n, _rows(r0, r1))
    _check(lib().bcs_expand_ws(p, n, r0, r1, _ptr(recv, nq, "recv"), _ptr(send, nq, "send"),
                               _ptr(recv_blocks, nr, "recv_blocks"), _ptr(send_blocks, nr, "send_blocks"), wp, wb,
                               _stream(stream)), "bcs_expand_ws")


def bcs_sched_expand_workspace_bytes(p, n):
    return _check(lib().bcs_sched_expand_workspace_bytes(p, n), "bcs_sched_expand_workspace_bytes")


def bcs_sched_expand(p, root, n, recv_out, send_out, recv_blocks, send_blocks, stream=None):
    nq, nr = _expand_sizes(p, n, max(int(p), 0))
    _check(lib().bcs_sched_expand(p, root, n, _ptr(recv_out, nq, "recv_out"), _ptr(send_out, nq, "send_out"),
                                  _ptr(recv_blocks, nr, "recv_blocks"), _ptr(send_blocks, nr, "send_blocks"),
                                  _stream(stream)), "bcs_sched_expand")


def bcs_sched_expand_ws(p, root, n, recv_out, send_out, recv_blocks, send_blocks, workspace, stream=None):
    """`workspace`: a device tensor of any dtype (or None when no scratch is needed)."""
    wp, wb = _ws(workspace)
    nq, nr = _expand_sizes(p, n, max(int(p), 0))
    _check(lib().bcs_sched_expand_ws(p, root, n, _ptr(recv_out, nq, "recv_out"), _ptr(send_out, nq, "send_out"),
                                     _ptr(recv_blocks, nr, "recv_blocks"), _ptr(send_blocks, nr, "send_blocks"),
                                     wp, wb, _stream(stream)), "bcs_sched_expand_ws")


def bcs_release():
    _check(lib().bcs_release(), "bcs_release")


def bcs_timing_begin():
    _check(lib().bcs_timing_begin(), "bcs_timing_begin")


def bcs_timing_end():
    """{kernel name: (summed milliseconds, timed launches)} since bcs_timing_begin()."""
    ms = (ctypes.c_double * KERNEL_COUNT)()
    cnt = (ctypes.c_int64 * KERNEL_COUNT)()
    _check(lib().bcs_timing_end(ctypes.cast(ms, ctypes.c_void_p), ctypes.cast(cnt, ctypes.c_void_p)),
           "bcs_timing_end")
    return {lib().bcs_kernel_name(i).decode(): (ms[i], cnt[i]) for i in range(KERNEL_COUNT) if cnt[i]}


def bcs_timing_stats():
    """{kernel name: (summed ms, timed launches, shortest ms, longest ms)} since bcs_timing_begin()."""
    ms = (ctypes.c_double * KERNEL_COUNT)()
    cnt = (ctypes.c_int64 * KERNEL_COUNT)()
    lo = (ctypes.c_double * KERNEL_COUNT)()
    hi = (ctypes.c_double * KERNEL_COUNT)()
    _check(lib().bcs_timing_stats(*(ctypes.cast(a, ctypes.c_void_p) for a in (ms, cnt, lo, hi))), "bcs_timing_stats")
    return {lib().bcs_kernel_name(i).decode(): (ms[i], cnt[i], lo[i], hi[i]) for i in range(KERNEL_COUNT) if cnt[i]}


def bcs_valu_peak_launch(blocks, iters, sink, stream=None):
    """`sink`: int32 device tensor of at least blocks * 256 entries."""
    _check(lib().bcs_valu_peak_launch(blocks, iters, _ptr(sink, blocks * 256, "sink"), _stream(stream)),
           "bcs_valu_peak_launch")


def bcs_allgather_workspace_bytes(p):
    return _check(lib().bcs_allgather_workspace_bytes(p), "bcs_allgather_workspace_bytes")


def bcs_allgather_tables(p, n, r, pack_idx, unpack_idx, stream=None):
    need = _expand_sizes(p, n, max(int(p), 0))[1]                 # R x p entries
    _check(lib().bcs_allgather_tables(p, n, r, _ptr(pack_idx, need, "pack_idx"), _ptr(unpack_idx, need, "unpack_idx"),
                                      _stream(stream)), "bcs_allgather_tables")


def bcs_allgather_tables_ws(p, n, r, pack_idx, unpack_idx, workspace, stream=None):
    wp, wb = _ws(workspace)
    need = _expand_sizes(p, n, max(int(p), 0))[1]
    _check(lib().bcs_allgather_tables_ws(p, n, r, _ptr(pack_idx, need, "pack_idx"),
                                         _ptr(unpack_idx, need, "unpack_idx"), wp, wb, _stream(stream)),
           "bcs_allgather_tables_ws")


def _dev(t, dtype, numel=0, what="tensor"):
    """Device pointer of a contiguous device tensor of the given torch dtype and at least `numel` elements."""
    import torch
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError("expected a contiguous %s tensor in device memory" % dtype)
    _need(t, numel, what)
    return ctypes.c_void_p(t.data_ptr())


def bcs_pack_workspace_bytes(p):
    return _check(lib().bcs_pack_workspace_bytes(p), "bcs_pack_workspace_bytes")


def bcs_pack_round(n, idx, displs, data, packed, offsets, workspace, stream=None):
    """idx int32[p], displs int64[p+1], data int32, packed int32 (its numel is the capacity), offsets int64[p+1].
    `data` must hold displs[p] elements: that value lives on the device, so it is the caller's to guarantee."""
    import torch
    p = idx.numel()
    wp, wb = _ws(workspace)
    _check(lib().bcs_pack_round(p, n, _ptr(idx), _dev(displs, torch.int64, p + 1, "displs"), _ptr(data), _ptr(packed),
                                packed.numel(), _dev(offsets, torch.int64, p + 1, "offsets"), wp, wb,
                                _stream(stream)), "bcs_pack_round")


def bcs_unpack_round(n, idx, displs, data, packed, length, offsets, workspace, stream=None):
    import torch
    p = idx.numel()
    wp, wb = _ws(workspace)
    _check(lib().bcs_unpack_round(p, n, _ptr(idx), _dev(displs, torch.int64, p + 1, "displs"), _ptr(data),
                                  _ptr(packed, max(int(length), 0), "packed"), length,
                                  _dev(offsets, torch.int64, p + 1, "offsets"), wp, wb, _stream(stream)),
           "bcs_unpack_round")


def bcs_pack_plan_rounds(n, idx_table, displs, offsets_all, src_all, stream=None):
    """idx_table int32[rounds][p], displs int64[p+1] -> offsets_all int64[rounds][p+1], src_all int64[rounds][p]."""
    import torch
    rounds, p = idx_table.shape
    _check(lib().bcs_pack_plan_rounds(p, n, rounds, _ptr(idx_table), _dev(displs, torch.int64, p + 1, "displs"),
                                      _dev(offsets_all, torch.int64, rounds * (p + 1), "offsets_all"),
                                      _dev(src_all, torch.int64, rounds * p, "src_all"), _stream(stream)),
           "bcs_pack_plan_rounds")


def bcs_pack_round_planned(offsets, src, data, packed, stream=None):
    """One round from its plan rows: offsets int64[p+1], src int64[p]; packed's numel is the capacity."""
    import torch
    p = src.numel()
    _check(lib().bcs_pack_round_planned(p, _dev(offsets, torch.int64, p + 1, "offsets"), _dev(src, torch.int64),
                                        _ptr(data), _ptr(packed), packed.numel(), _stream(stream)),
           "bcs_pack_round_planned")


def bcs_unpack_round_planned(offsets, src, data, packed, length, stream=None):
    import torch
    p = src.numel()
    _check(lib().bcs_unpack_round_planned(p, _dev(offsets, torch.int64, p + 1, "offsets"), _dev(src, torch.int64),
                                          _ptr(data), _ptr(packed, max(int(length), 0), "packed"), length,
                                          _stream(stream)), "bcs_unpack_round_planned")


def _host_plan(fn, what, p, r, arrays):
    q = bcs_q(p)
    bufs = [(ctypes.c_int32 * max(q, 1))() for _ in range(arrays)]
    _check(fn(p, r, *[ctypes.cast(b, ctypes.c_void_p) for b in bufs]), what)
    return [list(b)[:q] for b in bufs]


def bcs_allgather_plan(p, r):
    """Alg. 7: lists (to, from, count, recv_first) of q entries."""
    return _host_plan(lib().bcs_allgather_plan, "bcs_allgather_plan", p, r, 4)


def bcs_census_plan(p, r):
    """Alg. 8: lists (to, from, own) of q entries."""
    return _host_plan(lib().bcs_census_plan, "bcs_census_plan", p, r, 3)


def _partners(fn, what, p, r0, r1, to, frm, stream):
    need = _rows(r0, r1) * bcs_q(p) if p >= 1 else 0
    _check(fn(p, r0, r1, _ptr(to, need, what + ": to"), _ptr(frm, need, what + ": from"), _stream(stream)), what)


def bcs_allgather_partners(p, r0, r1, to, frm, stream=None):
    """Alg. 7's to- and from-processes of the processes [r0, r1): int32 device tables [(r - r0) * q + k]."""
    _partners(lib().bcs_allgather_partners, "bcs_allgather_partners", p, r0, r1, to, frm, stream)


def bcs_census_partners(p, r0, r1, to, frm, stream=None):
    """Alg. 8's to- and from-processes of the processes [r0, r1): int32 device tables [(r - r0) * q + k]."""
    _partners(lib().bcs_census_partners, "bcs_census_partners", p, r0, r1, to, frm, stream)
