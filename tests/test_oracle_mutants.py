"""Do the pins bite?  Each case plants one plausible mistake in a COPY of the oracle's source (a dropped term, a
wrong sign or index, smallest instead of largest, ...), builds it with gcc on the CPU and runs a short list of pins
against it: the paper's printed tables, the brute-force definition, the power-of-two closed form and the round
simulator.  Every mutant must fail at least one pin; the unmodified source must pass them all.  A mutant may
read out of bounds or never finish, so the pins run in a child process: a crash or a time-out counts as caught."""
import ctypes
import os
import subprocess
import sys
import tempfile

import numpy as np
import pytest

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
from conftest import load_table                      # noqa: E402
from bcast_sim import simulate, ScheduleError        # noqa: E402
from allgather_sim import simulate_allgather, AllgatherError   # noqa: E402

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(os.path.dirname(HERE), "oracle", "bcs_oracle.c")

MUTANTS = [
    # (name, text in the source, replacement)
    ("skips_floor_halving", "skips[k - 1] = (int32_t)(((int64_t)skips[k] + 1) / 2);", "skips[k - 1] = skips[k] / 2;"),
    ("baseblock_le_instead_of_lt", "if (skips[k] < r) r -= skips[k];", "if (skips[k] <= r) r -= skips[k];"),
    ("linear_recipe_skips_rank_1", "for (int32_t r = 1; r < skips[i]; r++) {", "for (int32_t r = 2; r < skips[i]; r++) {"),
    ("range_rec_shift_wrong_level", "return rangeblocks_rec(skips, a - skips[k], b - skips[k], k - 1);",
     "return rangeblocks_rec(skips, a - skips[k - 1], b - skips[k - 1], k - 1);"),
    ("range_rec_drops_node_block", "uint32_t m = (uint32_t)1 << k;\n    m |= rangeblocks_rec(skips, a, (int64_t)skips[k] - 1, k - 1);",
     "uint32_t m = 0;\n    m |= rangeblocks_rec(skips, a, (int64_t)skips[k] - 1, k - 1);"),
    ("range_prefix_one_short", "if (a == 1) return ((uint32_t)2 << k) - 1;", "if (a == 1) return ((uint32_t)1 << k) - 1;"),
    ("cyclic_range_counts_root", "if (lo == 0) lo = 1;\n        m = rangeblocks_rec(skips, lo, hi, q - 1);",
     "m = rangeblocks_rec(skips, lo == 0 ? 1 : lo, hi, q - 1) | (lo == 0 ? 1u : 0u);"),
    ("recv_B_starts_empty", "uint32_t B = (r > 0) ? ((uint32_t)1 << own) : 0;", "uint32_t B = 0;"),
    ("recv_smallest_instead_of_largest", "b = highest_bit(U);", "b = highest_bit(U & (~U + 1));"),
    ("recv_first_range_off_by_one", "int64_t a1 = (int64_t)r - skips[i + 1] + 1, b1 = (int64_t)r - skips[i];",
     "int64_t a1 = (int64_t)r - skips[i + 1], b1 = (int64_t)r - skips[i];"),
    ("recv_second_range_sum_to_i_minus_1", "int64_t a2 = (int64_t)r - prefix, b2 = (int64_t)r - skips[i + 1];",
     "int64_t a2 = (int64_t)r - (prefix - skips[i]), b2 = (int64_t)r - skips[i + 1];"),
    ("recv_no_second_range", "if (U == 0) {\n                int64_t a2", "if (0) {\n                int64_t a2"),
    ("recv_home_test_strict", "if (skips[i] <= r && r < skips[i + 1]) {", "if (skips[i] < r && r < skips[i + 1]) {"),
    ("recv_offset_q_minus_1", "out[i] = b - q;", "out[i] = b - q + 1;"),
    ("send_neighbour_minus", "int32_t t = (int32_t)(((int64_t)j + skips[k]) % p);\n                send[(size_t)j * q + k] = recv[(size_t)t * q + k];",
     "int32_t t = (int32_t)(((int64_t)j - skips[k] + p) % p);\n                send[(size_t)j * q + k] = recv[(size_t)t * q + k];"),
    ("send_lookup_wrong_slot", "row[k] = rtab[(size_t)t * q + k];", "row[k] = rtab[(size_t)t * q + (k + 1) % q];"),
    ("alg5_wrong_prefix_length", "int rc = recvsched_core(skips, q, t, i, NULL, 0, tmp);\n        if (rc) return rc;\n        out[i] = tmp[i];",
     "int rc = recvsched_core(skips, q, t, i, NULL, 0, tmp);\n        if (rc) return rc;\n        out[i] = tmp[i > 0 ? i - 1 : 0];"),
    ("rooted_adds_root", "int32_t v = (int32_t)(((int64_t)r - root + p) % p);\n            int rc = recvsched_core(skips, q, v, q - 1, NULL, 0, rtab",
     "int32_t v = (int32_t)(((int64_t)r + root) % p);\n            int rc = recvsched_core(skips, q, v, q - 1, NULL, 0, rtab"),
    ("expand_dummy_rounds_wrong", "int64_t x = (q - (n - 1 + q) % q) % q;\n    #pragma omp", "int64_t x = (n - 1 + q) % q;\n    #pragma omp"),
    ("expand_no_phase_bump_for_early_slots", "if (i < x) sched[i] = (int64_t)in[row * q + i] - x + q;",
     "if (i < x) sched[i] = (int64_t)in[row * q + i] - x;"),
    ("expand_clamp_to_n", "else if (blk > n - 1) blk = n - 1;", "else if (blk > n) blk = n;"),
    ("allgather_without_dummy_round_adjustment", "int64_t adj = (i < x) ? (q - x) : (-x);", "int64_t adj = 0;"),
    ("allgather_wrong_rotation", "int32_t rr = (int32_t)(((int64_t)r - j + p) % p);\n            int64_t blk = sendsched",
     "int32_t rr = (int32_t)(((int64_t)r + j) % p);\n            int64_t blk = sendsched"),
]


class Lib:
    """A build of the (possibly mutated) oracle source with the few calls the pins need."""

    def __init__(self, so):
        L = ctypes.CDLL(so)
        i32p = ctypes.POINTER(ctypes.c_int32)
        L.orc_sched_definition.argtypes = [ctypes.c_int32, ctypes.c_int, i32p, i32p, i32p]
        L.orc_sched_range.argtypes = [ctypes.c_int32] * 4 + [i32p, i32p, ctypes.c_int]
        L.orc_skips.argtypes = [ctypes.c_int32, i32p]
        L.orc_expand.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int64, i32p, i32p, ctypes.c_int]
        L.orc_baseblocks_linear.argtypes = [ctypes.c_int32, i32p]
        L.orc_rangeblocks_scan.argtypes = [ctypes.c_int32, i32p, ctypes.c_int64, ctypes.c_int64]
        L.orc_rangeblocks_scan.restype = ctypes.c_uint32
        L.orc_rangeblocks.argtypes = [ctypes.c_int32, ctypes.c_int64, ctypes.c_int64]
        L.orc_rangeblocks.restype = ctypes.c_uint32
        L.orc_allgather_tables.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, i32p, i32p]
        self.L = L

    @staticmethod
    def _p(a):
        return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))

    def definition(self, p):
        q = (p - 1).bit_length()
        bb = np.zeros(p, np.int32)
        recv = np.zeros((p, q), np.int32)
        send = np.zeros((p, q), np.int32)
        rc = self.L.orc_sched_definition(p, 0, self._p(bb), self._p(recv), self._p(send))
        return rc, bb, recv, send

    def per_rank(self, p, root=0, r0=0, r1=None):
        r1 = p if r1 is None else r1
        q = (p - 1).bit_length()
        recv = np.zeros((r1 - r0, q), np.int32)
        send = np.zeros((r1 - r0, q), np.int32)
        rc = self.L.orc_sched_range(p, root, r0, r1, self._p(recv), self._p(send), 1)
        return rc, recv, send

    def allgather(self, p, n):
        q = (p - 1).bit_length()
        pack = np.zeros((p, n - 1 + q, p), np.int32)
        unpack = np.zeros((p, n - 1 + q, p), np.int32)
        for r in range(p):
            if self.L.orc_allgather_tables(p, n, r, self._p(pack[r]), self._p(unpack[r])):
                return None, None
        return pack, unpack

    def expand(self, p, n, table):
        q = (p - 1).bit_length()
        out = np.zeros((table.shape[0], n - 1 + q), np.int32)
        self.L.orc_expand(p, n, table.shape[0], self._p(np.ascontiguousarray(table)), self._p(out), 1)
        return out


def _pow2_row(q, r):
    if r == 0:
        return [i - q for i in range(q)]
    h = r.bit_length() - 1
    row = []
    for i in range(q):
        if i == h:
            row.append((r & -r).bit_length() - 1)
        elif i < h and (r >> i) & 1:
            above = r >> (i + 1)
            row.append(i + 1 + (above & -above).bit_length() - 1 - q)
        else:
            row.append(i - q)
    return row


def pins_hold(lib):
    """True when this build passes the short pin list."""
    try:
        for name in ("table1_p20", "table2_p33", "table3_p32", "table4_p31", "table5_left_p9"):
            p, q, bb, recv, send = load_table(name)
            rc, obb, orecv, osend = lib.definition(p)
            if rc or not ((obb[1:] == bb[1:]).all() and (orecv == recv).all() and (osend == send).all()):
                return False
            rc, frecv, fsend = lib.per_rank(p)
            if rc or not ((frecv == recv).all() and (fsend == send).all()):
                return False
            rc, precv, psend = lib.per_rank(p, r0=2, r1=p - 1)               # Alg. 5 rows
            if rc or not ((precv == recv[2:p - 1]).all() and (psend == send[2:p - 1]).all()):
                return False
            rc, rrecv, rsend = lib.per_rank(p, root=3)                        # rooted rows are rotations
            if rc or not ((rrecv == np.roll(recv, 3, axis=0)).all() and (rsend == np.roll(send, 3, axis=0)).all()):
                return False
        skips = np.zeros(8, np.int32)
        lib.L.orc_skips(33, lib._p(skips))
        if skips[:7].tolist() != [1, 2, 3, 5, 9, 17, 33]:
            return False
        for p in (2, 3, 5, 6, 7, 9, 11, 13, 24, 57, 100, 129, 257, 600):
            rc, bb, recv, send = lib.definition(p)
            rc2, frecv, fsend = lib.per_rank(p)
            if rc or rc2 or not ((frecv == recv).all() and (fsend == send).all()):
                return False
            q = recv.shape[1]
            for n in (1, 2, q, q + 3):
                simulate(p, n, frecv, fsend)
        for p in (5, 9, 20, 33):                      # ranges by recursion == ranges by scanning, also through rank 0
            bb = np.zeros(p, np.int32)
            lib.L.orc_baseblocks_linear(p, lib._p(bb))
            for a in range(-p, p + 1):
                for b in range(a, a + p + 1):
                    if lib.L.orc_rangeblocks(p, a, b) != lib.L.orc_rangeblocks_scan(p, lib._p(bb), a, b):
                        return False
        for q in (3, 6, 9):
            rc, recv, send = lib.per_rank(1 << q)
            if rc or recv.tolist() != [_pow2_row(q, r) for r in range(1 << q)]:
                return False
        # expansion: dummy rounds never show, blocks stay in range, a non-root row lists every block once,
        # the root sends 0, 1, .., n-1, n-1, ..
        for p, n in ((20, 3), (20, 11), (33, 6)):
            rc, recv, send = lib.per_rank(p)
            q = recv.shape[1]
            er, es = lib.expand(p, n, recv), lib.expand(p, n, send)
            if es[0].tolist() != [min(j, n - 1) for j in range(n - 1 + q)] or er.max() > n - 1 or er.min() < -1:
                return False
            for r in range(1, p):
                if sorted(er[r][er[r] >= 0].tolist()) != list(range(n)):
                    return False
        for p, n in ((5, 2), (9, 3), (20, 4)):         # the allgather of Alg. 9, replayed for all processes
            pack, unpack = lib.allgather(p, n)
            if pack is None:
                return False
            simulate_allgather(p, n, pack, unpack)
    except (ScheduleError, AllgatherError, AssertionError):
        return False
    return True


def build(text, workdir, name):
    src = os.path.join(workdir, name + ".c")
    so = os.path.join(workdir, name + ".so")
    with open(src, "w") as f:
        f.write(text)
    subprocess.run(["gcc", "-O1", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-w", "-o", so, src], check=True)
    return so


def pins_hold_in_child(so):
    """Run the pin list on a built library in a fresh interpreter; False on failure, crash or time-out."""
    try:
        done = subprocess.run([sys.executable, os.path.abspath(__file__), so], timeout=120,
                              stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
    except subprocess.TimeoutExpired:
        return False
    return done.returncode == 0


@pytest.fixture(scope="module")
def workdir():
    with tempfile.TemporaryDirectory(prefix="bcs_mutants_") as d:
        yield d


def test_unmodified_source_passes_the_pins(workdir):
    assert pins_hold_in_child(build(open(SRC).read(), workdir, "pristine"))


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_mutant_is_caught(workdir, name, old, new):
    text = open(SRC).read()
    assert text.count(old) == 1, "mutation site not found exactly once: %s" % name
    assert not pins_hold_in_child(build(text.replace(old, new), workdir, name)), "mutant survived: %s" % name


if __name__ == "__main__":
    sys.exit(0 if pins_hold(Lib(sys.argv[1])) else 1)
