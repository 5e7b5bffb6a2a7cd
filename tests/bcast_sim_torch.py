"""The round-by-round replay of tests/bcast_sim.py written with torch tensor operations, so that it can run
where the tables are (a GPU holds the 29 GB of tables of p = 2^27 - 1).  Same four conditions (a)-(d); it reads
one slot column of each table per round and never materialises the expanded tables.  Test infrastructure only."""
import torch

from bcast_sim import ScheduleError, closed_form_skips


def simulate(p, n, recv, send):
    """recv, send: int32 tensors [p][q] on any device.  Raises ScheduleError; returns the rounds played."""
    q = (p - 1).bit_length()
    if p == 1:
        return n - 1
    if tuple(recv.shape) != (p, q) or tuple(send.shape) != (p, q):
        raise ScheduleError("table shape %s / %s, expected (%d, %d)" % (tuple(recv.shape), tuple(send.shape), p, q))
    skips = closed_form_skips(p)
    R = n - 1 + q
    x = (q - R % q) % q
    dev = recv.device
    have = torch.zeros((p, n), dtype=torch.bool, device=dev)
    have[0] = True
    got = torch.zeros((p, n), dtype=torch.int8, device=dev)
    for j in range(R):
        k = (x + j) % q
        s = skips[k]
        # slot k has been used floor((x+j)/q) times before: block = entry + q*floor((x+j)/q) - x = entry + j - k
        sblk = (send[:, k] + (j - k)).clamp_(min=-1, max=n - 1)
        rblk = (recv[:, k] + (j - k)).clamp_(min=-1, max=n - 1)
        if not torch.equal(sblk, torch.roll(rblk, -s)):                                        # (c)
            r = int(torch.nonzero(sblk != torch.roll(rblk, -s))[0])
            raise ScheduleError("p=%d n=%d round %d (slot %d): rank %d sends %d but rank %d expects another block"
                                % (p, n, j, k, r, int(sblk[r]), (r + s) % p))
        del rblk
        active = sblk >= 0
        held = have.gather(1, sblk.clamp(min=0).unsqueeze(1).long()).squeeze(1)
        if not bool((held | ~active).all()):                                                   # (a)
            r = int(torch.nonzero(active & ~held)[0])
            raise ScheduleError("p=%d n=%d round %d: rank %d sends block %d it does not hold" % (p, n, j, r, int(sblk[r])))
        del held, active
        incoming = torch.roll(sblk, s)                  # block arriving at each rank, -1 = none
        incoming[0] = -1                                # deliveries to the root are ignored
        arrives = (incoming >= 0).unsqueeze(1)
        where = incoming.clamp_(min=0).unsqueeze(1).long()
        got.scatter_add_(1, where, arrives.to(torch.int8))
        if j == R - 1 and bool(have.all()):                                                    # (d), "not earlier"
            raise ScheduleError("p=%d n=%d: complete before the last round" % (p, n))
        have.scatter_(1, where, have.gather(1, where) | arrives)
    if not bool(have.all()):                                                                   # (d)
        r, b = (int(v) for v in torch.nonzero(~have)[0])
        raise ScheduleError("p=%d n=%d: rank %d lacks block %d after %d rounds" % (p, n, r, b, R))
    if not bool((got[1:] == 1).all()):                                                         # (b)
        r, b = (int(v) for v in torch.nonzero(got[1:] != 1)[0])
        raise ScheduleError("p=%d n=%d: rank %d received block %d %d times" % (p, n, r + 1, b, int(got[r + 1, b])))
    return R
