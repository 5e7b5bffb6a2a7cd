"""Round-by-round replay of the n-block broadcast on the circulant graph.

An independent checker: it knows nothing of how a schedule was built.  It is
handed recv[p][q] and send[p][q] and plays the rounds of the broadcast
algorithm (arXiv 2205.10072, Alg. 6) for all p ranks at once, asserting what
Section 2 demands of a correct, round-optimal schedule:

  (a) a rank only sends a block it already holds (the root holds all n);
  (b) every non-root rank receives each of the n blocks exactly once;
  (c) what r sends to (r + skips[k]) mod p in a round is what that rank
      expects to receive in that round (same block, or both nothing);
  (d) all ranks hold all blocks after exactly n-1+q rounds, and not one
      round earlier.

The skips come from the closed form ceil(p / 2^(q-k)) rather than from the
halving loop, so that a slip in either shows up as a disagreement.
"""
import numpy as np


class ScheduleError(AssertionError):
    pass


def closed_form_skips(p):
    q = (p - 1).bit_length()
    return [-((-p) >> (q - k)) for k in range(q + 1)]          # ceil(p / 2^(q-k))


def _round_blocks(table, n, q, x):
    """Per-rank block of every real round: [p][R], -1 where nothing moves."""
    p = table.shape[0]
    R = n - 1 + q
    sched = table.astype(np.int64).copy()
    # x virtual rounds are over: slots below x were "used" once already
    sched[:, :x] += q
    sched -= x
    out = np.empty((p, R), dtype=np.int64)
    for j in range(R):
        k = (x + j) % q
        out[:, j] = sched[:, k]
        sched[:, k] += q
    out[out < 0] = -1
    out[out > n - 1] = n - 1
    return out


def simulate(p, n, recv, send):
    """Replay the broadcast; raise ScheduleError on the first violated condition.

    Returns the number of rounds played (n-1+q)."""
    recv = np.asarray(recv)
    send = np.asarray(send)
    q = (p - 1).bit_length()
    if p == 1:
        return n - 1
    if recv.shape != (p, q) or send.shape != (p, q):
        raise ScheduleError("table shape %s / %s, expected (%d, %d)" % (recv.shape, send.shape, p, q))
    skips = closed_form_skips(p)
    R = n - 1 + q
    x = (q - R % q) % q
    rblk = _round_blocks(recv, n, q, x)
    sblk = _round_blocks(send, n, q, x)
    have = np.zeros((p, n), dtype=bool)
    have[0, :] = True
    got = np.zeros((p, n), dtype=np.int32)            # deliveries per (rank, block)
    ranks = np.arange(p)
    for j in range(R):
        k = (x + j) % q
        to = (ranks + skips[k]) % p
        s = sblk[:, j]
        r_at_to = rblk[to, j]
        bad = np.nonzero(s != r_at_to)[0]
        if bad.size:                                                       # (c)
            r = int(bad[0])
            raise ScheduleError("p=%d n=%d round %d (slot %d): rank %d sends %d but rank %d expects %d"
                                % (p, n, j, k, r, s[r], to[r], r_at_to[r]))
        active = s >= 0
        src = ranks[active]
        blk = s[active]
        held = have[src, blk]
        if not held.all():                                                 # (a)
            i = int(np.nonzero(~held)[0][0])
            raise ScheduleError("p=%d n=%d round %d: rank %d sends block %d it does not hold"
                                % (p, n, j, src[i], blk[i]))
        dst = to[active]
        keep = dst != 0                      # deliveries to the root are ignored
        np.add.at(got, (dst[keep], blk[keep]), 1)
        if j == R - 1 and have.all():                                      # (d), "not earlier"
            raise ScheduleError("p=%d n=%d: complete before the last round" % (p, n))
        have[dst[keep], blk[keep]] = True     # one delivery per rank per round: no ordering issue
    if not have.all():                                                     # (d)
        r, b = (int(v[0]) for v in np.nonzero(~have))
        raise ScheduleError("p=%d n=%d: rank %d lacks block %d after %d rounds" % (p, n, r, b, R))
    if not (got[1:] == 1).all():                                           # (b)
        r, b = (int(v[0]) for v in np.nonzero(got[1:] != 1))
        raise ScheduleError("p=%d n=%d: rank %d received block %d %d times" % (p, n, r + 1, b, got[r + 1, b]))
    return R
