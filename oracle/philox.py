"""Counter-based random numbers and Gumbel-max sampling for the oracle (test
infrastructure; see package docstring).

The generator is Philox-4x32 with 10 rounds, implemented here from its published
definition (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as
1, 2, 3", SC'11): a 128-bit counter, a 64-bit key, ten rounds of two 32x32->64
multiplications with word permutation, the key bumped by the Weyl constants
between rounds.

Noise for vocabulary entry v of a sequence at absolute position p:
    key     = (seed mod 2^32, seed div 2^32)          per-sequence 64-bit seed
    counter = (v div 4, p, 0, 0)
    R       = output word (v mod 4)
    u       = (R + 0.5) * 2^-32   in (0, 1)
    g       = -log(-log(u))
so a draw depends only on (seed, position, vocabulary index), never on the batch
slot.  Gumbel noise is evaluated in float64.
"""
from __future__ import annotations

import numpy as np

_M0 = np.uint64(0xD2511F53)
_M1 = np.uint64(0xCD9E8D57)
_W0 = np.uint32(0x9E3779B9)
_W1 = np.uint32(0xBB67AE85)
_LO = np.uint64(0xFFFFFFFF)
_S32 = np.uint64(32)


def philox4x32_10(counter: np.ndarray, key: np.ndarray) -> np.ndarray:
    """counter: uint32 [..., 4]; key: uint32 [..., 2] (broadcastable) -> uint32 [..., 4]."""
    c = np.asarray(counter, dtype=np.uint32)
    k = np.asarray(key, dtype=np.uint32)
    c0, c1, c2, c3 = (c[..., i].astype(np.uint64) for i in range(4))
    k0 = np.broadcast_to(k[..., 0], c0.shape).astype(np.uint32)
    k1 = np.broadcast_to(k[..., 1], c0.shape).astype(np.uint32)
    with np.errstate(over="ignore"):
        for _ in range(10):
            p0 = _M0 * c0            # 64-bit products of 32-bit values: exact in uint64
            p1 = _M1 * c2
            n0 = (p1 >> _S32) ^ c1 ^ k0.astype(np.uint64)
            n1 = p1 & _LO
            n2 = (p0 >> _S32) ^ c3 ^ k1.astype(np.uint64)
            n3 = p0 & _LO
            c0, c1, c2, c3 = n0, n1, n2, n3
            k0 = (k0 + _W0).astype(np.uint32)
            k1 = (k1 + _W1).astype(np.uint32)
    return np.stack([c0, c1, c2, c3], axis=-1).astype(np.uint32)


def uniform_u32(seed: int, pos: int, vocab: int) -> np.ndarray:
    """The 32-bit words R[v], v = 0..vocab-1, for one (seed, position)."""
    nblk = (vocab + 3) // 4
    ctr = np.zeros((nblk, 4), dtype=np.uint32)
    ctr[:, 0] = np.arange(nblk, dtype=np.uint32)
    ctr[:, 1] = np.uint32(int(pos) & 0xFFFFFFFF)
    key = np.array([int(seed) & 0xFFFFFFFF, (int(seed) >> 32) & 0xFFFFFFFF], dtype=np.uint32)
    return philox4x32_10(ctr, key).reshape(-1)[:vocab]


def gumbel_noise(seed: int, pos: int, vocab: int) -> np.ndarray:
    """float64 Gumbel(0,1) noise g[v] = -log(-log(u[v]))."""
    u = (uniform_u32(seed, pos, vocab).astype(np.float64) + 0.5) * 2.0 ** -32
    return -np.log(-np.log(u))


def sample_gumbel_max(z: np.ndarray, temperature: float, seed: int, pos: int) -> int:
    """argmax_v(z_v / T + g_v) for the token that will sit at absolute position `pos`;
    ties to the smaller v.  T <= 0 means greedy argmax of z."""
    z = np.asarray(z)
    if temperature <= 0:
        return int(np.argmax(z))
    score = z.astype(np.float64) / float(temperature) + gumbel_noise(seed, pos, z.shape[-1])
    return int(np.argmax(score))
