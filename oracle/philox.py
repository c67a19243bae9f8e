"""Philox4x32-10 counter-based generator (Salmon, Moraes, Dror, Shaw, SC'11) and the
uniforms Algorithm 1 draws from it.

Test infrastructure only.  The paper's Algorithm 1 draws r_i ~ U(0,1) for the
acceptance tests and samples tokens from q and p'; it does not say how.  Reading
used here: every draw is a function of (seed, stream, batch, step, position), so the
GPU and this oracle consume identical numbers.

  key     = (seed & 0xffffffff, seed >> 32)
  counter = (position k, step j, batch b, stream)
  stream  : DRAFT = 1 -> word 0: unmask decision u_a, word 1: token sample u_b
            VERIFY = 2 -> word 0: acceptance r,      word 1: final-token sample u
            SPS = 3    -> word 1: token sample of the autoregressive drafter's step k (position k, step 0)
  uniform = (word >> 8) * 2**-24, in [0, 1), exactly representable in fp32
"""
import numpy as np

STREAM_DRAFT = 1
STREAM_VERIFY = 2
STREAM_SPS = 3

_M0 = np.uint64(0xD2511F53)
_M1 = np.uint64(0xCD9E8D57)
_W0 = 0x9E3779B9
_W1 = 0xBB67AE85
_MASK = np.uint64(0xFFFFFFFF)
_S32 = np.uint64(32)


def philox4x32_10(counter, key):
    """counter: (..., 4) integers < 2**32; key: (2,) integers < 2**32 -> (..., 4) uint32."""
    c = np.asarray(counter, dtype=np.uint64) & _MASK
    c0, c1, c2, c3 = (c[..., i].copy() for i in range(4))
    k0, k1 = int(key[0]) & 0xFFFFFFFF, int(key[1]) & 0xFFFFFFFF
    for _ in range(10):
        p0 = _M0 * c0          # 32x32 -> 64 bit products
        p1 = _M1 * c2
        hi0, lo0 = p0 >> _S32, p0 & _MASK
        hi1, lo1 = p1 >> _S32, p1 & _MASK
        c0 = hi1 ^ c1 ^ np.uint64(k0)
        c1 = lo1
        c2 = hi0 ^ c3 ^ np.uint64(k1)
        c3 = lo0
        k0 = (k0 + _W0) & 0xFFFFFFFF
        k1 = (k1 + _W1) & 0xFFFFFFFF
    return np.stack([c0, c1, c2, c3], axis=-1).astype(np.uint32)


def uniforms(seed, stream, batch, step, positions):
    """Two uniforms per position: returns (u_word0, u_word1), fp64 arrays of len(positions)."""
    pos = np.asarray(positions, dtype=np.uint64).reshape(-1)
    ctr = np.zeros((pos.size, 4), dtype=np.uint64)
    ctr[:, 0] = pos
    ctr[:, 1] = step
    ctr[:, 2] = batch
    ctr[:, 3] = stream
    seed = int(seed)
    out = philox4x32_10(ctr, (seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF))
    u = (out >> np.uint32(8)).astype(np.float64) * 2.0 ** -24
    return u[:, 0], u[:, 1]
