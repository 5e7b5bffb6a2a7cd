"""ctypes door onto the host build of the GPU lanes' construction code (bcs_core.h)."""
import ctypes
import os
import subprocess

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(HERE, "bcs_hostcheck.cpp")
CSRC = os.path.join(ROOT, "paper_2205_10072_amd", "csrc")
CORE = os.path.join(CSRC, "bcs_core.h")
LIB = os.path.join(HERE, "libbcs_hostcheck.so")

_lib = None


def build(lib=LIB, extra=(), force=True):
    """Compiles the host build of the lane code (g++); `extra` adds flags, e.g. sanitizers."""
    stale = (force or not os.path.exists(lib)
             or os.path.getmtime(lib) < max(os.path.getmtime(SRC), os.path.getmtime(CORE)))
    if stale:
        subprocess.run(["g++", "-O2", "-std=c++17", "-fPIC", "-shared", "-Wno-unknown-pragmas", "-I", CSRC]
                       + list(extra) + ["-o", lib, SRC], check=True)
    return lib


def load():
    global _lib
    if _lib is None:
        build(force=False)
        L = ctypes.CDLL(LIB)
        i32p = ctypes.POINTER(ctypes.c_int32)
        L.hc_recv_row.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int, i32p]
        L.hc_recv_row_perlane.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int, ctypes.c_int, i32p]
        L.hc_recv_rows_list.argtypes = [ctypes.c_int32, i32p, ctypes.c_int64, ctypes.c_int, i32p]
        L.hc_send_rows_list.argtypes = [ctypes.c_int32, i32p, ctypes.c_int64, ctypes.c_int, i32p,
                                        ctypes.POINTER(ctypes.c_uint32)]
        L.hc_range_blocks.argtypes = [ctypes.c_int32, ctypes.c_uint32, ctypes.c_uint32]
        L.hc_range_blocks.restype = ctypes.c_uint32
        L.hc_recv_rows_all.argtypes = [ctypes.c_int32, i32p]
        L.hc_recv_rows_all_tab.argtypes = [ctypes.c_int32, ctypes.POINTER(ctypes.c_uint32), i32p]
        L.hc_recv_row_tab.argtypes = [ctypes.c_int32, ctypes.POINTER(ctypes.c_uint32), ctypes.c_int32, ctypes.c_int, i32p]
        _lib = L
    return _lib


def recv_row(p, v, last=None, perlane=False, wave_q=None):
    q = (p - 1).bit_length()
    if last is None:
        last = q - 1
    out = np.full(32, 12345, dtype=np.int32)
    ptr = out.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
    if perlane:
        rc = load().hc_recv_row_perlane(p, v, last, q if wave_q is None else wave_q, ptr)
    else:
        rc = load().hc_recv_row(p, v, last, ptr)
    assert rc == 0
    return out


def range_blocks(p, a, b):
    return int(load().hc_range_blocks(p, a, b))


def recv_rows_all(p):
    q = (p - 1).bit_length()
    out = np.zeros((p, q), dtype=np.int32)
    assert load().hc_recv_rows_all(p, out.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))) == 0
    return out


def recv_rows_all_tab(p, want_table=False):
    """All receive rows through the table of every rank's digit mask (the path of the whole-range kernels)."""
    q = (p - 1).bit_length()
    out = np.zeros((p, q), dtype=np.int32)
    dtab = np.zeros(p, dtype=np.uint32)
    assert load().hc_recv_rows_all_tab(p, dtab.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32)),
                                       out.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))) == 0
    return (out, dtab) if want_table else out


def recv_row_tab(p, dtab, v, last):
    """Entries 0..last of one row from a filled table (the path Alg. 5's kernel takes for a neighbour's row)."""
    out = np.full(32, 12345, dtype=np.int32)
    assert load().hc_recv_row_tab(p, dtab.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32)), v, last,
                                  out.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))) == 0
    return out


def recv_rows_list(p, ranks, perlane=False):
    """Full receive rows of the listed virtual ranks: array [len(ranks)][q]."""
    q = (p - 1).bit_length()
    v = np.ascontiguousarray(ranks, dtype=np.int32)
    out = np.full((len(v), 32), 12345, dtype=np.int32)
    i32p = ctypes.POINTER(ctypes.c_int32)
    assert load().hc_recv_rows_list(p, v.ctypes.data_as(i32p), len(v), 1 if perlane else 0, out.ctypes.data_as(i32p)) == 0
    assert (out[:, q:] == 12345).all()
    return out[:, :q]


def send_rows_list(p, ranks, wave_q=0, want_direct=False):
    """Send rows of the listed virtual ranks the way the batch kernel builds them: array [len(ranks)][q]
    (and, on request, per rank the mask of the entries that took the direct rule)."""
    q = (p - 1).bit_length()
    v = np.ascontiguousarray(ranks, dtype=np.int32)
    out = np.full((len(v), 32), 12345, dtype=np.int32)
    direct = np.zeros(len(v), dtype=np.uint32)
    i32p = ctypes.POINTER(ctypes.c_int32)
    assert load().hc_send_rows_list(p, v.ctypes.data_as(i32p), len(v), wave_q, out.ctypes.data_as(i32p),
                                    direct.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32))) == 0
    assert (out[:, q:] == 12345).all()
    return (out[:, :q], direct) if want_direct else out[:, :q]
