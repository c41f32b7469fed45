"""Counter-based random numbers for the oracle (test infrastructure only).

The paper needs three kinds of random draws per agent: the initial weights
(Sec. 4.1: replicas start from different random weights), the uniform replay
sample (App. A) and TD3's target-policy smoothing noise (the algorithm cited
in Sec. 4.1).  It names no generator.  The reading taken here: Philox4x32 with
10 rounds (Salmon, Moraes, Dror, Shaw, SC'11 -- a published algorithm), keyed
by the agent's 64-bit seed, with the 128-bit counter laid out as

    (block, step, stream, sub)

so that every (agent seed, stream, step, element) owns its own 32-bit word and
nothing depends on the agent's position in the population or on P.

Streams: 0 replay indices, 1 TD3 smoothing noise, 2/3 SAC actor noise at s/s',
4 parameter init (sub = tensor id), 5 exploration noise for acting.

Pin status: structure (distinct counters give distinct blocks, streams do not
collide) and statistics only; conformance to published known-answer vectors is
"parity unpinned" (none available offline).
"""
import numpy as np

STREAM_INDEX = 0
STREAM_SMOOTH = 1
STREAM_SAC_S = 2
STREAM_SAC_S2 = 3
STREAM_INIT = 4
STREAM_EXPLORE = 5

_MASK = np.uint64(0xFFFFFFFF)
_MUL_A = np.uint64(0xD2511F53)   # multiplier applied to counter word 0
_MUL_B = np.uint64(0xCD9E8D57)   # multiplier applied to counter word 2
_WEYL_A = 0x9E3779B9             # key word 0 increment per round
_WEYL_B = 0xBB67AE85             # key word 1 increment per round
_SHIFT32 = np.uint64(32)


def mix64(seed, i):
    """Derive agent i's seed from a population seed when the caller gave none.

    splitmix64 finaliser (Steele, Lea, Flood 2014) of seed + (i+1)*golden.
    """
    m = (1 << 64) - 1
    z = (int(seed) + (int(i) + 1) * 0x9E3779B97F4A7C15) & m
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & m
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & m
    z = z ^ (z >> 31)
    return z if z != 0 else 1


def philox4x32(seed, block, step, stream, sub=0, rounds=10):
    """Return uint32 words of shape block.shape + (4,) for counters
    (block, step, stream, sub) under key (seed low word, seed high word)."""
    block = np.asarray(block, dtype=np.uint64)
    c0 = block & _MASK
    c1 = np.full_like(c0, np.uint64(int(step) & 0xFFFFFFFF))
    c2 = np.full_like(c0, np.uint64(int(stream) & 0xFFFFFFFF))
    c3 = np.full_like(c0, np.uint64(int(sub) & 0xFFFFFFFF))
    k0 = int(seed) & 0xFFFFFFFF
    k1 = (int(seed) >> 32) & 0xFFFFFFFF
    for r in range(rounds):
        if r > 0:
            k0 = (k0 + _WEYL_A) & 0xFFFFFFFF
            k1 = (k1 + _WEYL_B) & 0xFFFFFFFF
        pa = _MUL_A * c0            # 32x32 -> 64 bit products (no overflow in uint64)
        pb = _MUL_B * c2
        hi_a, lo_a = pa >> _SHIFT32, pa & _MASK
        hi_b, lo_b = pb >> _SHIFT32, pb & _MASK
        c0, c1, c2, c3 = (hi_b ^ c1 ^ np.uint64(k0), lo_b,
                          hi_a ^ c3 ^ np.uint64(k1), lo_a)
    return np.stack([c0, c1, c2, c3], axis=-1).astype(np.uint32)


def words(seed, n, step, stream, sub=0):
    """First n words of the (seed, stream, step, sub) stream: element e is word
    e & 3 of block e >> 2."""
    nblk = (int(n) + 3) // 4
    w = philox4x32(seed, np.arange(nblk, dtype=np.uint64), step, stream, sub)
    return w.reshape(-1)[:n]


def sample_indices(seed, step, batch, count):
    """Replay sample of one agent at one step (App. A: uniform sampling from
    the agent's own buffer).  Reading: with replacement, slot b takes word b
    of stream 0 and maps it to [0, count) by the high half of the 32x32-bit
    product word*count -- integer only, so both sides agree bit for bit."""
    if not (0 < count <= 0xFFFFFFFF):
        raise ValueError("count must be in [1, 2^32-1]")
    w = words(seed, batch, step, STREAM_INDEX).astype(np.uint64)
    return ((w * np.uint64(count)) >> _SHIFT32).astype(np.int64)


def uniform01(w):
    """Top 24 bits of each word as a multiple of 2^-24 in [0, 1)."""
    return (np.asarray(w, dtype=np.uint32) >> np.uint32(8)).astype(np.float64) * 2.0 ** -24


def normals(seed, n, step, stream, sub=0):
    """n standard normals in fp64: element e comes from block e >> 2; inside a
    block words (0,1) give elements 0,1 and words (2,3) give elements 2,3 by
    the Box-Muller transform with u1 in (0,1], u2 in [0,1)."""
    nblk = (int(n) + 3) // 4
    w = philox4x32(seed, np.arange(nblk, dtype=np.uint64), step, stream, sub)
    w = w.reshape(nblk, 2, 2)
    u1 = ((w[..., 0] >> np.uint32(8)).astype(np.float64) + 1.0) * 2.0 ** -24
    u2 = (w[..., 1] >> np.uint32(8)).astype(np.float64) * 2.0 ** -24
    rad = np.sqrt(-2.0 * np.log(u1))
    ang = 2.0 * np.pi * u2
    out = np.stack([rad * np.cos(ang), rad * np.sin(ang)], axis=-1)
    return out.reshape(-1)[:n]
