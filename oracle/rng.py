"""Counter-based random numbers drawn by the method (oracle side).

TEST INFRASTRUCTURE ONLY - see oracle/__init__.py.

The paper draws three things at random: how long a worker's Compute takes
(Section 7.3.1 slows every worker 6x with probability 1/n per iteration,
Section 7.3.5 slows one worker 4x deterministically), which samples form a
minibatch (Figure 1, "randomly selected samples"), and - in the synthetic
"mixing only" workload - the gradient itself.  The paper fixes no generator, so
every draw is a pure function of (seed, stream, a, b, c): a skipped iteration
never shifts a later draw, and any element can be regenerated anywhere.

The 64-bit mixer is the SplitMix64 output function (Steele, Lea, Flood 2014)
folded over the five words.  The 32-bit finaliser used per gradient element is
the two-multiply xorshift-multiply construction with the constants 0x7feb352d /
0x846ca68b (C. Wellons' published "lowbias32").
"""
import math

import numpy as np

M64 = (1 << 64) - 1

STREAM_DELAY = 1
STREAM_BATCH = 2
STREAM_SYNTHGRAD = 6
STREAM_LATENCY = 7

TICKS_PER_UNIT = 1 << 20          # one time unit of simulated Compute
TICKS_NEVER = 1 << 62             # a duration at or above this never completes

DELAY_NONE = 0        # every Compute takes one time unit
DELAY_EXP1 = 1        # Exp(1) time units
DELAY_BERNOULLI6 = 2  # 6 units with probability 1/N, else 1 (Section 7.3.1)
DELAY_TABLE = 3       # explicit ticks per (worker, iteration)


def sm64(z):
    z = (z + 0x9E3779B97F4A7C15) & M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M64
    return z ^ (z >> 31)


def mix(seed, stream, a, b, c):
    h = sm64(seed & M64)
    for w in (stream, a, b, c):
        h = sm64(h ^ (w & M64))
    return h


def uniform(u64):
    """53 random bits as a double in [0, 1)."""
    return (u64 >> 11) * (1.0 / 9007199254740992.0)


def duration_ticks(seed, kind, n_workers, mult_i, i, k, table=None):
    """Compute time of (worker i, iteration k) in integer ticks, at least 1."""
    if kind == DELAY_TABLE:
        return int(table[i][k])
    if mult_i >= float(TICKS_NEVER):
        return TICKS_NEVER
    u = uniform(mix(seed, STREAM_DELAY, i, k, 0))
    if kind == DELAY_NONE:
        base = 1.0
    elif kind == DELAY_EXP1:
        base = -math.log(1.0 - u)
    elif kind == DELAY_BERNOULLI6:
        base = 6.0 if u < 1.0 / n_workers else 1.0
    else:
        raise ValueError("unknown delay kind")
    t = base * mult_i
    t = t * float(TICKS_PER_UNIT)
    if t >= float(TICKS_NEVER):
        return TICKS_NEVER
    return max(1, int(math.floor(t)))


def latency_ticks(seed, max_latency, sender, receiver, tag):
    """Ticks an update needs from Send to the receiver's queue: 1, or uniform in 1..max_latency
    keyed by (sender, receiver, tag) - later updates can then overtake earlier ones."""
    if max_latency <= 1:
        return 1
    return 1 + mix(seed, STREAM_LATENCY, sender, receiver, tag) % max_latency


def batch_rows(seed, i, k, batch, rows):
    """Minibatch of (worker i, iteration k): iid row ids with replacement."""
    return np.array([mix(seed, STREAM_BATCH, i, k, m) % rows for m in range(batch)],
                    dtype=np.int64)


def _h32(x):
    x = x.astype(np.uint32, copy=True)
    x ^= x >> np.uint32(16)
    x *= np.uint32(0x7FEB352D)
    x ^= x >> np.uint32(15)
    x *= np.uint32(0x846CA68B)
    x ^= x >> np.uint32(16)
    return x


def _byte_sum(x):
    return ((x & np.uint32(0xFF)) + ((x >> np.uint32(8)) & np.uint32(0xFF))
            + ((x >> np.uint32(16)) & np.uint32(0xFF)) + (x >> np.uint32(24))).astype(np.int64)


SYNTH_TERMS = 12                       # bytes summed per element
SYNTH_MEAN = 1530                      # 12 * 127.5
SYNTH_VAR = 65535.0                    # 12 * (256^2 - 1) / 12


def synth_scale(variance):
    """fp32 factor that gives the byte sum the requested variance."""
    return np.float32(math.sqrt(variance / SYNTH_VAR))


def synth_keys(seed, i, k):
    ka = mix(seed, STREAM_SYNTHGRAD, i, k, 0)
    kb = mix(seed, STREAM_SYNTHGRAD, i, k, 1)
    return ka & 0xFFFFFFFF, ka >> 32, kb & 0xFFFFFFFF


def synth_grad(seed, i, k, cols, variance):
    """Synthetic gradient of (worker i, iteration k) at the given columns.

    Each element is a centred sum of 12 bytes (an Irwin-Hall approximation of
    a normal draw) times one fp32 scale: the bytes of two hashed words a, b of
    the column index and of (a + rotl(b, 16)) ^ k2, which is uniform and
    independent of a and of b taken singly, so the bytes are pairwise
    independent and the variance is exactly 12 (256^2 - 1) / 12.  Integer work
    plus a single correctly rounded multiply: every implementation agrees bit
    for bit.  Returns float32.
    """
    cols = np.asarray(cols, dtype=np.int64)
    c32 = (cols & 0xFFFFFFFF).astype(np.uint32)
    k0, k1, k2 = synth_keys(seed, i, k)
    a = _h32(c32 ^ np.uint32(k0))
    b = _h32(c32 ^ np.uint32(k1))
    t = (a + ((b << np.uint32(16)) | (b >> np.uint32(16)))) ^ np.uint32(k2)   # wraps modulo 2^32
    s = _byte_sum(a) + _byte_sum(b) + _byte_sum(t)
    centred = (s - SYNTH_MEAN).astype(np.float32)
    return centred * synth_scale(variance)
