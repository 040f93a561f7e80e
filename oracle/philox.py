"""ORACLE (test infrastructure only) -- counter-based random streams of the chains.

The paper asks for standard normal vectors Z and uniforms U on [0,1] and names no generator
(detailed algorithm of speculative sampling for DDMs, App. "Detailed implementation").  So that the CPU oracle and the
GPU library consume the *same* random numbers, both implement -- independently -- the published
Philox4x32-10 generator (Salmon, Moraes, Dror, Shaw, "Parallel random numbers: as easy as
1, 2, 3", SC'11) keyed by absolute coordinates:

    key     = (seed low 32 bits, seed high 32 bits)
    counter = (chain_id low, chain_id high, k, (stream << 28) | block)

``k`` is the index of the chain state the number is *for*: the noise that produces state k and
the uniform that tests state k carry k; the initial state carries 0.  ``stream``: 0 = Gaussian
noise, 1 = accept-test uniform, 2 = initial state.  One block yields four 32-bit words, i.e.
elements 4*block .. 4*block+3 of a d-vector.

32-bit word -> uniform: ``u = ((w >> 9) + 1/2) * 2^-23``, which lies strictly inside (0,1) and is
exactly representable in fp32 as well as fp64.  Words -> normals: Box-Muller on (w0,w1) and
(w2,w3): ``r = sqrt(-2 ln u(w_even))``, ``(z_even, z_odd) = r * (cos, sin)(2 pi u(w_odd))``.

Pinned by tests/test_oracle_rng.py: the SC'11 known-answer vectors, and moment / KS checks.
"""
from __future__ import annotations

import numpy as np

_M0 = np.uint64(0xD2511F53)
_M1 = np.uint64(0xCD9E8D57)
_W0 = 0x9E3779B9
_W1 = 0xBB67AE85
_MASK = np.uint64(0xFFFFFFFF)
_SH32 = np.uint64(32)

STREAM_NOISE = 0
STREAM_UNIFORM = 1
STREAM_INIT = 2


def philox4x32_10(c0, c1, c2, c3, k0: int, k1: int):
    """Ten rounds of Philox-4x32.  c0..c3: broadcastable integer arrays; k0, k1: Python ints.

    Returns four uint32 arrays.  One round: (hi0,lo0) = M0*c0, (hi1,lo1) = M1*c2,
    new counter = (hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0); the key is bumped by the Weyl
    constants between rounds.
    """
    c0, c1, c2, c3 = np.broadcast_arrays(*(np.asarray(c, dtype=np.uint64) & _MASK
                                           for c in (c0, c1, c2, c3)))
    k0 &= 0xFFFFFFFF
    k1 &= 0xFFFFFFFF
    for rnd in range(10):
        p0 = _M0 * c0
        p1 = _M1 * c2
        hi0, lo0 = p0 >> _SH32, p0 & _MASK
        hi1, lo1 = p1 >> _SH32, p1 & _MASK
        c0, c1, c2, c3 = (hi1 ^ c1 ^ np.uint64(k0), lo1, hi0 ^ c3 ^ np.uint64(k1), lo0)
        k0 = (k0 + _W0) & 0xFFFFFFFF
        k1 = (k1 + _W1) & 0xFFFFFFFF
    return tuple(c.astype(np.uint32) for c in (c0, c1, c2, c3))


def word_to_uniform(w) -> np.ndarray:
    """u = ((w >> 9) + 0.5) * 2^-23  in (0,1)."""
    return ((np.asarray(w, dtype=np.uint32) >> np.uint32(9)).astype(np.float64) + 0.5) * (2.0 ** -23)


def _blocks(seed: int, chain_id, k, stream: int, nblocks: int):
    """Philox words for blocks 0..nblocks-1; chain_id, k: arrays of a common shape S.
    Returns uint32 array [*S, nblocks, 4]."""
    chain_id = np.asarray(chain_id, dtype=np.uint64)
    k = np.asarray(k, dtype=np.uint64)
    chain_id, k = np.broadcast_arrays(chain_id, k)
    blk = np.arange(nblocks, dtype=np.uint64)
    c3 = (np.uint64(stream) << np.uint64(28)) | blk
    w = philox4x32_10((chain_id & _MASK)[..., None], (chain_id >> _SH32)[..., None],
                      k[..., None], c3, seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
    return np.stack(w, axis=-1)


def normals(seed: int, chain_id, k, d: int, stream: int = STREAM_NOISE) -> np.ndarray:
    """Standard normal d-vectors for each (chain_id, k): float64 [*S, d]."""
    nb = (d + 3) // 4
    w = _blocks(seed, chain_id, k, stream, nb)                # [*S, nb, 4]
    u = word_to_uniform(w)
    out = np.empty(u.shape, dtype=np.float64)
    for p in (0, 2):
        r = np.sqrt(-2.0 * np.log(u[..., p]))
        th = 2.0 * np.pi * u[..., p + 1]
        out[..., p] = r * np.cos(th)
        out[..., p + 1] = r * np.sin(th)
    return out.reshape(out.shape[:-2] + (4 * nb,))[..., :d]


def uniforms(seed: int, chain_id, k) -> np.ndarray:
    """The accept-test uniform of state k of each chain: word 0 of block 0 of stream 1."""
    w = _blocks(seed, chain_id, k, STREAM_UNIFORM, 1)
    return word_to_uniform(w[..., 0, 0])


def initial_state(seed: int, chain_id, d: int) -> np.ndarray:
    """The chain's start: Y_0 ~ N(0, Id), step index 0 (first line of Alg. "Speculative Sampling for DDM")."""
    return normals(seed, chain_id, np.zeros_like(np.asarray(chain_id)), d, STREAM_INIT)
