"""Seeded, counter-based input generator (host side, numpy).

Normal deviates come from Philox4x32-10 (Salmon et al., "Parallel random numbers:
as easy as 1, 2, 3", SC'11) followed by the Box-Muller transform:

    key     = (seed low 32 bits, seed high 32 bits)
    counter = (block low, block high, step, stream)      block = element index // 4
    four 32-bit outputs x0..x3 -> uniforms u_k = ((x_k >> 9) + 0.5) * 2^-23
    (z0, z1) = sqrt(-2 ln u0) * (cos 2 pi u1, sin 2 pi u1), (z2, z3) likewise from u2, u3

so every element of every (stream, step) draw is addressable on its own.  The
device twin of this recipe is csrc/pier_inputs.hip; the two agree to float
rounding of log/sin/cos, not bit for bit, so a test never mixes them: inputs of
one case come from one side and are copied to the other.

Holds no optimizer arithmetic.
"""
import numpy as np

_M0 = np.uint64(0xD2511F53)
_M1 = np.uint64(0xCD9E8D57)
_W0 = 0x9E3779B9
_W1 = 0xBB67AE85
_MASK = np.uint64(0xFFFFFFFF)
_S32 = np.uint64(32)


def philox4x32_10(c0, c1, c2, c3, k0, k1):
    """Vectorised Philox4x32 with 10 rounds.  Counters are uint32 arrays (or
    scalars broadcast against them); keys are Python ints.  Returns 4 uint32 arrays."""
    c0, c1, c2, c3 = [np.asarray(c, dtype=np.uint32).astype(np.uint64) for c in (c0, c1, c2, c3)]
    c0, c1, c2, c3 = np.broadcast_arrays(c0, c1, c2, c3)
    k0 &= 0xFFFFFFFF
    k1 &= 0xFFFFFFFF
    for r in range(10):
        if r:
            k0 = (k0 + _W0) & 0xFFFFFFFF
            k1 = (k1 + _W1) & 0xFFFFFFFF
        p0 = _M0 * c0
        p1 = _M1 * c2
        hi0, lo0 = p0 >> _S32, p0 & _MASK
        hi1, lo1 = p1 >> _S32, p1 & _MASK
        c0, c1, c2, c3 = hi1 ^ c1 ^ np.uint64(k0), lo1, hi0 ^ c3 ^ np.uint64(k1), lo0
    return tuple(c.astype(np.uint32) for c in (c0, c1, c2, c3))


def _uniform(x):
    return ((x >> np.uint32(9)).astype(np.float32) + np.float32(0.5)) * np.float32(2.0 ** -23)


def _box_muller(xa, xb):
    ua, ub = _uniform(xa), _uniform(xb)
    r = np.sqrt(np.float32(-2.0) * np.log(ua)).astype(np.float32)
    ang = np.float32(2.0 * np.pi) * ub
    return r * np.cos(ang).astype(np.float32), r * np.sin(ang).astype(np.float32)


def normal_at(idx, *, seed, stream, step, std):
    """float32 N(0, std) deviates of draw (seed, stream, step) at element indices ``idx``."""
    idx = np.asarray(idx, dtype=np.int64)
    blk = idx >> 2
    x = philox4x32_10((blk & 0xFFFFFFFF).astype(np.uint32), (blk >> 32).astype(np.uint32),
                      np.uint32(step & 0xFFFFFFFF), np.uint32(stream & 0xFFFFFFFF),
                      seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
    z0, z1 = _box_muller(x[0], x[1])
    z2, z3 = _box_muller(x[2], x[3])
    lane = idx & 3
    z = np.where(lane == 0, z0, np.where(lane == 1, z1, np.where(lane == 2, z2, z3)))
    return (np.float32(std) * z).astype(np.float32)


def normal(n, *, seed, stream, step, std, offset=0):
    """The n consecutive elements [offset, offset + n) of draw (seed, stream, step)."""
    return normal_at(np.arange(offset, offset + n, dtype=np.int64),
                     seed=seed, stream=stream, step=step, std=std)


def to_bf16_bits(x):
    """float32 -> bfloat16 bit patterns (uint16), round to nearest even."""
    b = np.asarray(x, dtype=np.float32).view(np.uint32)
    rounded = b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(h):
    return (np.asarray(h, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)
