"""Round-by-round replay of the irregular allgather on the circulant graph (arXiv 2205.10072, Alg. 9).

An independent checker for the per-process pack / unpack tables.  It is handed, for every process r, the
tables pack_r[R][p] and unpack_r[R][p] (block of buffer j packed for sending / unpacked on receipt in each
round) and plays all p processes at once, asserting
  (a) a process only packs blocks it holds (its own buffer r from the start, others once received);
  (b) what r packs for (r + skips[k]) mod p is, root by root, what that process expects to unpack;
  (c) every process receives every block of every other root exactly once;
  (d) all processes hold all n blocks of all p buffers after exactly n-1+q rounds.
"""
import numpy as np

from bcast_sim import closed_form_skips


class AllgatherError(AssertionError):
    pass


def simulate_allgather(p, n, pack, unpack):
    """pack, unpack: arrays [p][R][p] (process, round, root).  Raises AllgatherError; returns rounds played."""
    pack = np.asarray(pack)
    unpack = np.asarray(unpack)
    q = (p - 1).bit_length()
    R = n - 1 + q
    if p == 1:
        return R
    if pack.shape != (p, R, p) or unpack.shape != (p, R, p):
        raise AllgatherError("table shapes %s / %s" % (pack.shape, unpack.shape))
    skips = closed_form_skips(p)
    x = (q - R % q) % q
    have = np.zeros((p, p, n), dtype=bool)              # process, root, block
    for r in range(p):
        have[r, r, :] = True
    got = np.zeros((p, p, n), dtype=np.int32)
    procs = np.arange(p)
    roots = np.arange(p)
    for j in range(R):
        k = (x + j) % q
        to = (procs + skips[k]) % p
        sent = pack[:, j, :]                               # [process][root]
        expect = unpack[to, j, :]
        if not np.array_equal(sent, expect):                                               # (b)
            r, root = (int(v[0]) for v in np.nonzero(sent != expect))
            raise AllgatherError("p=%d n=%d round %d: process %d packs %d for root %d, process %d expects %d"
                                 % (p, n, j, r, sent[r, root], root, to[r], expect[r, root]))
        pr, rt = np.nonzero(sent >= 0)
        blk = sent[pr, rt]
        if not have[pr, rt, blk].all():                                                    # (a)
            i = int(np.nonzero(~have[pr, rt, blk])[0][0])
            raise AllgatherError("p=%d n=%d round %d: process %d packs block %d of root %d it does not hold"
                                 % (p, n, j, pr[i], blk[i], rt[i]))
        dst = to[pr]
        keep = dst != rt                                   # a process never needs its own buffer back
        np.add.at(got, (dst[keep], rt[keep], blk[keep]), 1)
        if j == R - 1 and have.all():
            raise AllgatherError("p=%d n=%d: complete before the last round" % (p, n))
        have[dst[keep], rt[keep], blk[keep]] = True
    if not have.all():                                                                     # (d)
        r, root, b = (int(v[0]) for v in np.nonzero(~have))
        raise AllgatherError("p=%d n=%d: process %d lacks block %d of root %d" % (p, n, r, b, root))
    off = ~np.eye(p, dtype=bool)
    if not (got[off] == 1).all():                                                          # (c)
        raise AllgatherError("p=%d n=%d: some block was delivered more or less than once" % (p, n))
    return R
