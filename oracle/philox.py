"""Counter-based random numbers for the CPU oracle (TEST INFRASTRUCTURE ONLY).

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this.

The paper only says that r_1..r_gamma are drawn from U(0,1) (Alg. 1, the line that
samples r) and that tokens are sampled from distributions (Eq. 1, Eq. 5).  To make a
GPU run comparable token by token, every random number is a pure function of
(seed, sequence, decode step, row, purpose, vocabulary index) through the public
Philox-4x32-10 generator (Salmon et al., "Parallel random numbers: as easy as 1, 2, 3",
SC'11).  The HIP library implements the same published algorithm separately.

Pins (tests/test_oracle_rng.py): the known-answer vectors of the Random123 distribution,
uniformity/independence chi-square, and the Gumbel-max law against softmax.
"""
import numpy as np

_M0 = np.uint64(0xD2511F53)
_M1 = np.uint64(0xCD9E8D57)
_W0 = 0x9E3779B9
_W1 = 0xBB67AE85
_MASK = np.uint64(0xFFFFFFFF)

PURPOSE_DRAFT = 0    # Gumbel noise used when the draft model samples y_i ~ q_i
PURPOSE_ACCEPT = 1   # the uniform r_i of Alg. 1
PURPOSE_NEXT = 2     # Gumbel noise for the residual / bonus sample


def philox4x32_10(ctr, key):
    """ctr: uint32 array [..., 4]; key: (k0, k1) python ints.  Returns uint32 [..., 4]."""
    c = np.asarray(ctr, dtype=np.uint64)
    c0, c1, c2, c3 = c[..., 0], c[..., 1], c[..., 2], c[..., 3]
    k0, k1 = int(key[0]) & 0xFFFFFFFF, int(key[1]) & 0xFFFFFFFF
    for rnd in range(10):
        p0 = _M0 * c0          # 32x32 -> 64 bit products
        p1 = _M1 * c2
        hi0, lo0 = p0 >> np.uint64(32), p0 & _MASK
        hi1, lo1 = p1 >> np.uint64(32), p1 & _MASK
        n0 = (hi1 ^ c1 ^ np.uint64(k0)) & _MASK
        n1 = lo1
        n2 = (hi0 ^ c3 ^ np.uint64(k1)) & _MASK
        n3 = lo0
        c0, c1, c2, c3 = n0, n1, n2, n3
        k0 = (k0 + _W0) & 0xFFFFFFFF
        k1 = (k1 + _W1) & 0xFFFFFFFF
    return np.stack([c0, c1, c2, c3], axis=-1).astype(np.uint32)


def u01(bits):
    """uint32 -> open-interval uniform that is exactly representable in fp32:
    ((bits >> 9) + 0.5) * 2^-23 (24 significant bits)."""
    return ((np.asarray(bits, dtype=np.uint32) >> np.uint32(9)).astype(np.float64) + 0.5) * (2.0 ** -23)


def _key(seed):
    seed = int(seed)
    return (seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)


def vocab_uniforms(seed, seq, step, row, purpose, vocab):
    """One uniform per vocabulary index v: word (v % 4) of Philox at counter
    (v // 4, row, step, purpose | seq << 8)."""
    nblk = (vocab + 3) // 4
    ctr = np.zeros((nblk, 4), dtype=np.uint32)
    ctr[:, 0] = np.arange(nblk, dtype=np.uint32)
    ctr[:, 1] = row
    ctr[:, 2] = step
    ctr[:, 3] = purpose | (seq << 8)
    out = philox4x32_10(ctr, _key(seed)).reshape(-1)[:vocab]
    return u01(out)


def scalar_uniform(seed, seq, step, row, purpose):
    return float(vocab_uniforms(seed, seq, step, row, purpose, 1)[0])


def gumbel(u):
    return -np.log(-np.log(u))
