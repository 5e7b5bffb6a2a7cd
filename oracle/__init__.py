"""CPU oracle for the broadcast-schedule construction (arXiv 2205.10072, Section 2).

TEST INFRASTRUCTURE.  Only tests, the smoke check and the benchmark's
cpu_baseline leg may import this package; the product never does.  It is a
ctypes door onto ``bcs_oracle.c`` (plain C, built with gcc by ``build()``),
returning numpy arrays.  It shares nothing with the HIP library.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "bcs_oracle.c")
_LIB = os.path.join(_HERE, "libbcs_oracle.so")
BATCH_STRIDE = 32
PAD = np.iinfo(np.int32).min

_lib = None


def build(force=True):
    """Compile the oracle with gcc -O2 (no intrinsics, OpenMP for the rank loop)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build(force=False)
    lib = ctypes.CDLL(_LIB)
    i32p = ctypes.POINTER(ctypes.c_int32)
    lib.orc_q.argtypes = [ctypes.c_int32]
    lib.orc_skips.argtypes = [ctypes.c_int32, i32p]
    lib.orc_baseblock.argtypes = [ctypes.c_int32, ctypes.c_int32]
    lib.orc_baseblocks_linear.argtypes = [ctypes.c_int32, i32p]
    lib.orc_rangeblocks_scan.argtypes = [ctypes.c_int32, i32p, ctypes.c_int64, ctypes.c_int64]
    lib.orc_rangeblocks_scan.restype = ctypes.c_uint32
    lib.orc_rangeblocks.argtypes = [ctypes.c_int32, ctypes.c_int64, ctypes.c_int64]
    lib.orc_rangeblocks.restype = ctypes.c_uint32
    lib.orc_recvsched.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int, ctypes.c_int, i32p]
    lib.orc_sendsched.argtypes = [ctypes.c_int32, ctypes.c_int32, i32p]
    lib.orc_sched_definition.argtypes = [ctypes.c_int32, ctypes.c_int, i32p, i32p, i32p]
    lib.orc_sched_range.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                    i32p, i32p, ctypes.c_int]
    lib.orc_sched_batch.argtypes = [ctypes.c_int64, i32p, i32p, i32p, i32p, i32p, i32p, ctypes.c_int]
    lib.orc_expand.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int64, i32p, i32p, ctypes.c_int]
    lib.orc_allgather_tables.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, i32p, i32p]
    i64p = ctypes.POINTER(ctypes.c_int64)
    lib.orc_allgather_plan.argtypes = [ctypes.c_int32, ctypes.c_int32, i32p, i32p, i32p, i32p]
    lib.orc_census_plan.argtypes = [ctypes.c_int32, ctypes.c_int32, i32p, i32p, i32p]
    lib.orc_pack_round.argtypes = [ctypes.c_int32, ctypes.c_int32, i32p, i64p, i32p, i32p, ctypes.c_int64, i64p]
    lib.orc_pack_round.restype = ctypes.c_int64
    lib.orc_unpack_round.argtypes = [ctypes.c_int32, ctypes.c_int32, i32p, i64p, i32p, i32p, ctypes.c_int64, i64p]
    lib.orc_unpack_round.restype = ctypes.c_int64
    _lib = lib
    return lib


def _ptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)) if a is not None else None


def _check(rc, what):
    if rc < 0:
        raise RuntimeError("oracle %s failed with code %d" % (what, rc))
    return rc


def q_of(p):
    return _check(_load().orc_q(p), "q")


def skips(p):
    """Alg. 1: the q+1 skips of the p-processor circulant graph."""
    out = np.zeros(q_of(p) + 1, dtype=np.int32)
    _check(_load().orc_skips(p, _ptr(out)), "skips")
    return out


def baseblock(p, r):
    """Alg. 2."""
    return _check(_load().orc_baseblock(p, r), "baseblock")


def baseblocks_linear(p):
    """Linear recipe of Section 2 (after Alg. 2); entry 0 is -1."""
    out = np.zeros(p, dtype=np.int32)
    _check(_load().orc_baseblocks_linear(p, _ptr(out)), "baseblocks_linear")
    return out


def rangeblocks_scan(p, bb, a, b):
    bb = np.ascontiguousarray(bb, dtype=np.int32)
    return int(_load().orc_rangeblocks_scan(p, _ptr(bb), a, b))


def rangeblocks(p, a, b):
    return int(_load().orc_rangeblocks(p, a, b))


def recvsched(p, r, k=None, general_only=False, scan=False):
    """Alg. 4: entries 0..min(k, q-1) of the receive schedule of rank r."""
    q = q_of(p)
    if k is None:
        k = q
    n = min(k, q - 1) + 1 if q > 0 else 0
    out = np.zeros(max(q, 1), dtype=np.int32)
    mode = (1 if general_only else 0) | (2 if scan else 0)
    _check(_load().orc_recvsched(p, r, k, mode, _ptr(out)), "recvsched")
    return out[:n].copy()


def sendsched(p, r):
    """Alg. 5."""
    q = q_of(p)
    out = np.zeros(max(q, 1), dtype=np.int32)
    _check(_load().orc_sendsched(p, r, _ptr(out)), "sendsched")
    return out[:q].copy()


def sched_definition(p, general_only=False):
    """(baseblocks, recv[p][q], send[p][q]) from the definitions; small p only."""
    q = q_of(p)
    bb = np.zeros(p, dtype=np.int32)
    recv = np.zeros((p, q), dtype=np.int32)
    send = np.zeros((p, q), dtype=np.int32)
    _check(_load().orc_sched_definition(p, 1 if general_only else 0, _ptr(bb), _ptr(recv), _ptr(send)),
           "sched_definition")
    return bb, recv, send


def sched_range(p, root=0, r0=0, r1=None, want_recv=True, want_send=True, threads=1):
    """(recv, send) rows of ranks [r0, r1) under broadcast root `root`."""
    if r1 is None:
        r1 = p
    q = q_of(p)
    recv = np.zeros((r1 - r0, q), dtype=np.int32) if want_recv else None
    send = np.zeros((r1 - r0, q), dtype=np.int32) if want_send else None
    _check(_load().orc_sched_range(p, root, r0, r1, _ptr(recv), _ptr(send), threads), "sched_range")
    return recv, send


def sched_batch(p, r, root, want_send=True, threads=1):
    """(recv[count][32], send[count][32], q[count]) for unrelated (p, r, root) triples."""
    p = np.ascontiguousarray(p, dtype=np.int32)
    r = np.ascontiguousarray(r, dtype=np.int32)
    root = np.ascontiguousarray(root, dtype=np.int32)
    count = p.shape[0]
    recv = np.zeros((count, BATCH_STRIDE), dtype=np.int32)
    send = np.zeros((count, BATCH_STRIDE), dtype=np.int32) if want_send else None
    qv = np.zeros(count, dtype=np.int32)
    _check(_load().orc_sched_batch(count, _ptr(p), _ptr(r), _ptr(root), _ptr(recv), _ptr(send),
                                   _ptr(qv), threads), "sched_batch")
    return recv, send, qv


def expand(p, n, table, threads=1):
    """Alg. 6 index arithmetic: table[rows][q] -> blocks[rows][n-1+q] (-1 = nothing)."""
    q = q_of(p)
    table = np.ascontiguousarray(table, dtype=np.int32).reshape(-1, q) if q > 0 \
        else np.zeros((np.asarray(table).shape[0], 0), dtype=np.int32)
    rows = table.shape[0]
    out = np.zeros((rows, n - 1 + q), dtype=np.int32)
    _check(_load().orc_expand(p, n, rows, _ptr(table), _ptr(out), threads), "expand")
    return out


def allgather_tables(p, n, r):
    """Alg. 9 index arithmetic for process r: (pack[R][p], unpack[R][p]), -1 = nothing."""
    q = q_of(p)
    R = n - 1 + q
    pack = np.zeros((R, p), dtype=np.int32)
    unpack = np.zeros((R, p), dtype=np.int32)
    _check(_load().orc_allgather_tables(p, n, r, _ptr(pack), _ptr(unpack)), "allgather_tables")
    return pack, unpack


def _ptr64(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int64))


def pack_round(n, idx, displs, data):
    """Alg. 9 'Pack' loop of one round: (message, offsets[p+1])."""
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    displs = np.ascontiguousarray(displs, dtype=np.int64)
    data = np.ascontiguousarray(data, dtype=np.int32)
    p = idx.shape[0]
    offsets = np.zeros(p + 1, dtype=np.int64)
    probe = np.zeros(1, dtype=np.int32)
    total = _check(_load().orc_pack_round(p, n, _ptr(idx), _ptr64(displs), _ptr(data), _ptr(probe), 0,
                                          _ptr64(offsets)), "pack_round")
    packed = np.zeros(max(total, 1), dtype=np.int32)
    _check(_load().orc_pack_round(p, n, _ptr(idx), _ptr64(displs), _ptr(data), _ptr(packed), total,
                                  _ptr64(offsets)), "pack_round")
    return packed[:total], offsets


def unpack_round(n, idx, displs, data, packed):
    """Alg. 9 'Unpack' loop of one round, in place on `data` (int32, contiguous); returns offsets[p+1]."""
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    displs = np.ascontiguousarray(displs, dtype=np.int64)
    packed = np.ascontiguousarray(packed, dtype=np.int32)
    assert data.dtype == np.int32 and data.flags["C_CONTIGUOUS"]
    p = idx.shape[0]
    offsets = np.zeros(p + 1, dtype=np.int64)
    _check(_load().orc_unpack_round(p, n, _ptr(idx), _ptr64(displs), _ptr(data), _ptr(packed), packed.shape[0],
                                    _ptr64(offsets)), "unpack_round")
    return offsets


def allgather_plan(p, r):
    """Alg. 7: (to, from, count, recv_first), q entries each."""
    q = q_of(p)
    a = [np.zeros(max(q, 1), dtype=np.int32) for _ in range(4)]
    _check(_load().orc_allgather_plan(p, r, *[_ptr(x) for x in a]), "allgather_plan")
    return [x[:q] for x in a]


def census_plan(p, r):
    """Alg. 8: (to, from, own), q entries each."""
    q = q_of(p)
    a = [np.zeros(max(q, 1), dtype=np.int32) for _ in range(3)]
    _check(_load().orc_census_plan(p, r, *[_ptr(x) for x in a]), "census_plan")
    return [x[:q] for x in a]
