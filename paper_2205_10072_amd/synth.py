"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke check.

Holds none of the method's arithmetic: only the recipe for the irregular batch
of (p, r, root) triples.  The paper's workloads are plain values of p and n, so
nothing here stands in for a dataset.
"""
import numpy as np

MASK64 = (1 << 64) - 1
BATCH_SEED = 0x220510072


def splitmix64_stream(seed, count):
    """`count` 64-bit outputs of the splitmix64 generator as Python ints."""
    out = []
    s = seed & MASK64
    for _ in range(count):
        s = (s + 0x9E3779B97F4A7C15) & MASK64
        z = s
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & MASK64
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & MASK64
        out.append(z ^ (z >> 31))
    return out


def _splitmix64_np(seed, count):
    """Same stream, vectorised (uint64 arithmetic wraps mod 2^64)."""
    with np.errstate(over="ignore"):
        idx = np.arange(1, count + 1, dtype=np.uint64)
        s = np.uint64(seed & MASK64) + idx * np.uint64(0x9E3779B97F4A7C15)
        z = s
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        return z ^ (z >> np.uint64(31))


def batch_triples(count, seed=BATCH_SEED):
    """(p, r, root) int32 arrays: bit length L uniform in [2, 31], p uniform in [2^(L-1), 2^L - 1]
    (an integer-exact log-uniform p in [2, 2^31 - 1]), r and root uniform in [0, p)."""
    u = _splitmix64_np(seed, 4 * count).reshape(count, 4)
    L = (u[:, 0] % np.uint64(30)).astype(np.int64) + 2
    lo = np.left_shift(np.int64(1), L - 1)
    p = lo + (u[:, 1] % lo.astype(np.uint64)).astype(np.int64)
    r = (u[:, 2] % p.astype(np.uint64)).astype(np.int64)
    root = (u[:, 3] % p.astype(np.uint64)).astype(np.int64)
    return p.astype(np.int32), r.astype(np.int32), root.astype(np.int32)


def irregular_sizes(p, m):
    """Buffer sizes of the paper's irregular allgather experiment (Section 3.2): m_r = (r mod 3) * floor(m / p)
    elements for r < p-1 and the remainder of m for the last process.  Returns (sizes, displs[p+1]) as int64."""
    sizes = (np.arange(p, dtype=np.int64) % 3) * (m // p)
    sizes[p - 1] = m - int(sizes[:p - 1].sum())
    assert sizes[p - 1] >= 0
    displs = np.zeros(p + 1, dtype=np.int64)
    np.cumsum(sizes, out=displs[1:])
    return sizes, displs
