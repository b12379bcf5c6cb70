"""Seeded synthetic inputs: payloads and failure scenarios.

This module serves BOTH the CPU oracle and the GPU library with the same
inputs.  It holds none of the method's arithmetic: no tree, no groups, no
reduction.  Quantities of the protocol that a recipe needs (the number of
rounds of one attempt) are passed in by the caller.

Counter-based generator: Philox4x32-10 (Salmon et al., "Parallel random
numbers: as easy as 1, 2, 3", SC'11), written from the published definition.
A draw is addressed by counter = (scenario, index, draw, stream) and key =
(seed_lo, seed_hi), so any scenario can be regenerated alone.  The GPU library
has a device generator that follows the same recipe (ftred_gen_failures,
ftred_gen_payload_int); tests compare the two bit for bit.

Recipes (shapes follow the five configurations of the benchmark definition):
  exhaustive_failure_sets  all subsets of size 0..f, failed before the operation
  random_failure_sets      k uniform in 0..f, ranks uniform without replacement
                           (redraw on duplicate), each failure during the
                           operation with probability inop_permille/1000 at a
                           round uniform in 1..(attempts * rounds_per_attempt)
  payload_int              two's-complement integers of `bits` random bits
  payload_normal           N(0,1) float64 from numpy's Philox bit generator
"""
from __future__ import annotations

import itertools
from concurrent.futures import ThreadPoolExecutor

import numpy as np

NO_RANK = 0xFFFFFFFF

STREAM_ROOT = 0
STREAM_COUNT = 1
STREAM_RANK = 2
STREAM_TIME = 3
STREAM_PAYLOAD = 4

_M0 = np.uint64(0xD2511F53)
_M1 = np.uint64(0xCD9E8D57)
_W0 = 0x9E3779B9
_W1 = 0xBB67AE85
_MASK = np.uint64(0xFFFFFFFF)
_SH = np.uint64(32)


def philox4x32(c0, c1, c2, c3, k0: int, k1: int):
    """Philox4x32 with 10 rounds.  c0..c3: uint32 arrays (broadcastable); k0, k1: ints.
    Returns four uint32 arrays."""
    c0, c1, c2, c3 = np.broadcast_arrays(*(np.asarray(c, dtype=np.uint32) for c in (c0, c1, c2, c3)))
    c0 = c0.astype(np.uint64)
    c1 = c1.astype(np.uint64)
    c2 = c2.astype(np.uint64)
    c3 = c3.astype(np.uint64)
    k0 &= 0xFFFFFFFF
    k1 &= 0xFFFFFFFF
    for _ in range(10):
        p0 = _M0 * c0
        p1 = _M1 * c2
        hi0, lo0 = p0 >> _SH, p0 & _MASK
        hi1, lo1 = p1 >> _SH, p1 & _MASK
        c0, c1, c2, c3 = (hi1 ^ c1 ^ np.uint64(k0), lo1, hi0 ^ c3 ^ np.uint64(k1), lo0)
        k0 = (k0 + _W0) & 0xFFFFFFFF
        k1 = (k1 + _W1) & 0xFFFFFFFF
    return (c0.astype(np.uint32), c1.astype(np.uint32), c2.astype(np.uint32), c3.astype(np.uint32))


def _key(seed: int):
    return seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF


def mulhi(u, n: int):
    """floor(u * n / 2^32): maps a uniform uint32 onto 0..n-1."""
    return ((np.asarray(u, dtype=np.uint64) * np.uint64(n)) >> _SH).astype(np.uint32)


# ----------------------------------------------------------------------------
# failure scenarios


def exhaustive_failure_sets(P: int, f: int):
    """Every subset of {0..P-1} of size 0..f, in order of size then lexicographic,
    all failed before the operation.  Returns (fail_rank[S][max(f,1)], fail_round)."""
    rows = []
    for k in range(f + 1):
        for comb in itertools.combinations(range(P), k):
            rows.append(list(comb) + [NO_RANK] * (max(f, 1) - k))
    fail_rank = np.array(rows, dtype=np.uint32).reshape(len(rows), max(f, 1))
    return fail_rank, np.zeros_like(fail_rank)


def random_roots(seed: int, S: int, P: int, scen0: int = 0):
    """One root per scenario, uniform over 0..P-1."""
    k0, k1 = _key(seed)
    s = np.arange(scen0, scen0 + S, dtype=np.uint32)
    u, _, _, _ = philox4x32(s, 0, 0, STREAM_ROOT, k0, k1)
    return mulhi(u, P)


def random_failure_sets(seed: int, S: int, P: int, f: int, *, inop_permille: int = 0,
                        rounds_per_attempt: int = 0, protected: int = 0, scen0: int = 0):
    """k uniform in 0..f failed ranks per scenario, uniform without replacement.

    inop_permille: chance (in 1/1000) that a failure happens during the operation;
    its round is then uniform in 1..A*rounds_per_attempt, where A = 1 + the number
    of leading ranks 0,1,2,.. (below `protected`) that are in the set: the number
    of attempts an allreduce that tries roots 0,1,2,.. will need.
    protected: ranks below it always fail before the operation (the allreduce's
    root candidates); 0 for a reduce.
    Unused slots hold NO_RANK / round 0.  Returns (fail_rank[S][max(f,1)], fail_round).
    """
    k0, k1 = _key(seed)
    F = max(f, 1)
    s = np.arange(scen0, scen0 + S, dtype=np.uint32)
    u, _, _, _ = philox4x32(s, 0, 0, STREAM_COUNT, k0, k1)
    count = mulhi(u, f + 1)
    fail_rank = np.full((S, F), NO_RANK, dtype=np.uint32)
    fail_round = np.zeros((S, F), dtype=np.uint32)
    for i in range(f):
        need = count > i
        draw = np.zeros(S, dtype=np.uint32)
        todo = need.copy()
        while todo.any():
            idx = np.nonzero(todo)[0]
            u, _, _, _ = philox4x32(s[idx], i, draw[idx], STREAM_RANK, k0, k1)
            r = mulhi(u, P)
            dup = np.zeros(idx.size, dtype=bool)
            for j in range(i):
                dup |= fail_rank[idx, j] == r
            ok = ~dup
            fail_rank[idx[ok], i] = r[ok]
            todo[idx[ok]] = False
            draw[idx[dup]] += 1
    if inop_permille > 0:
        attempts = np.ones(S, dtype=np.uint32)
        for c in range(protected):
            present = (fail_rank == c).any(axis=1)
            attempts = np.where(present & (attempts == c + 1), c + 2, attempts).astype(np.uint32)
        for i in range(f):
            u0, u1, _, _ = philox4x32(s, i, 0, STREAM_TIME, k0, k1)
            inop = (mulhi(u0, 1000) < inop_permille) & (fail_rank[:, i] != NO_RANK) \
                & (fail_rank[:, i] >= protected)
            span = (attempts.astype(np.uint64) * np.uint64(rounds_per_attempt))
            rnd = ((u1.astype(np.uint64) * span) >> _SH).astype(np.uint32) + np.uint32(1)
            fail_round[:, i] = np.where(inop, rnd, 0)
    return fail_rank, fail_round


# ----------------------------------------------------------------------------
# payloads

_NP = {"i64": np.int64, "u32": np.uint32, "f64": np.float64}


def payload_int(seed: int, S: int, P: int, elems: int, dtype: str, bits: int, scen0: int = 0):
    """Integers of `bits` random bits per element, payload[S][P][elems].

    dtype "i64": value = (r mod 2^bits) - 2^(bits-1), i.e. uniform in [-2^(bits-1), 2^(bits-1)).
    dtype "u32": value = r mod 2^bits (bits <= 32), uniform in [0, 2^bits).
    r = 64 random bits: element with flat index i = rank*elems + e takes words
    (0,1) of the Philox block with counter (scenario, i div 2, 0, STREAM_PAYLOAD)
    if i is even, words (2,3) if i is odd; r = word_lo | word_hi << 32.
    """
    k0, k1 = _key(seed)
    n = P * elems
    nblk = (n + 1) // 2
    out = np.empty((S, n), dtype=_NP[dtype])
    blk = np.arange(nblk, dtype=np.uint32)
    mask = np.uint64((1 << bits) - 1) if bits < 64 else np.uint64(0xFFFFFFFFFFFFFFFF)
    for si in range(S):
        w0, w1, w2, w3 = philox4x32(np.uint32(scen0 + si), blk, 0, STREAM_PAYLOAD, k0, k1)
        r = np.empty(2 * nblk, dtype=np.uint64)
        r[0::2] = w0.astype(np.uint64) | (w1.astype(np.uint64) << _SH)
        r[1::2] = w2.astype(np.uint64) | (w3.astype(np.uint64) << _SH)
        r = r[:n] & mask
        if dtype == "i64":
            out[si] = (r - np.uint64(1 << (bits - 1))).astype(np.int64) if bits < 64 else r.astype(np.int64)
        else:
            out[si] = r.astype(np.uint32)
    return out.reshape(S, P, elems)


def payload_normal(seed: int, S: int, P: int, elems: int, scen0: int = 0, threads: int = 8, out=None):
    """N(0,1) float64, payload[S][P][elems]; scenario s comes from numpy's
    Philox bit generator keyed (seed, s), so it can be regenerated alone."""
    if out is None:
        out = np.empty((S, P, elems), dtype=np.float64)

    def one(si):
        g = np.random.Generator(np.random.Philox(key=[seed, scen0 + si]))
        g.standard_normal(out=out[si].reshape(-1))

    if threads <= 1 or S < 4:
        for si in range(S):
            one(si)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(one, range(S)))
    return out
