"""Counter-based seeded generators.

Every value is a pure function of (seed, element counter), so the same bits
come out whatever order, chunking or machine is used, and no library RNG state
is involved.  Recipe: a 64-bit mix of (seed, counter) gives 24 uniform bits;
uniforms are k * 2^-24; normals are Box-Muller on two such uniforms, computed
in float64 and rounded once to float32.  bf16 inputs are those float32 values
rounded once (to nearest, ties to even) and handed around as uint16 bit
patterns, so every consumer sees identical operands.
"""
import numpy as np

_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_GOLD = np.uint64(0x9E3779B97F4A7C15)


def _mix64(seed, stream, n):
    with np.errstate(over="ignore"):
        ctr = np.arange(n, dtype=np.uint64)
        z = ctr * _GOLD + np.uint64(seed) * _M1 + np.uint64(stream) * _M2
        z ^= z >> np.uint64(30)
        z *= _M1
        z ^= z >> np.uint64(27)
        z *= _M2
        z ^= z >> np.uint64(31)
    return z


def _u24(seed, stream, n):
    return (_mix64(seed, stream, n) >> np.uint64(40)).astype(np.float64)


def uniform_f32(seed, shape, lo=-1.0, hi=1.0):
    """i.i.d. uniform[lo, hi) float32 of the given shape."""
    n = int(np.prod(shape))
    u = _u24(seed, 0, n) * (2.0 ** -24)
    return (lo + (hi - lo) * u).astype(np.float32).reshape(shape)


def normal_f32(seed, shape, std=1.0):
    """i.i.d. N(0, std^2) float32 of the given shape (Box-Muller)."""
    n = int(np.prod(shape))
    u1 = (_u24(seed, 1, n) + 1.0) * (2.0 ** -24)      # (0, 1]
    u2 = _u24(seed, 2, n) * (2.0 ** -24)
    z = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    return (std * z).astype(np.float32).reshape(shape)


def small_ints_f32(seed, shape, lo=-4, hi=4):
    """i.i.d. integers in [lo, hi], stored as float32 (exact in bf16 too)."""
    n = int(np.prod(shape))
    k = _mix64(seed, 3, n) % np.uint64(hi - lo + 1)
    return (k.astype(np.int64) + lo).astype(np.float32).reshape(shape)


def f32_to_bf16_bits(x):
    """Round float32 to bf16 (nearest, ties to even; NaN kept quiet) -> uint16."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (b >> np.uint32(16)) & np.uint32(1)
    r = (b + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    nan = (b & np.uint32(0x7FFFFFFF)) > np.uint32(0x7F800000)
    r = np.where(nan, (b >> np.uint32(16)) | np.uint32(0x40), r)
    return r.astype(np.uint16)


def bf16_bits_to_f32(u):
    """Widen bf16 bit patterns (uint16) to the float32 they denote."""
    return (np.ascontiguousarray(u, dtype=np.uint16).astype(np.uint32)
            << np.uint32(16)).view(np.float32)


def special_bit_patterns(seed, shape, bits):
    """Raw words (uint16 or uint32) salted with NaN payloads, infinities,
    negative zero and denormals, for tests that must move bits untouched."""
    n = int(np.prod(shape))
    z = _mix64(seed, 4, n)
    if bits == 16:
        w = (z >> np.uint64(48)).astype(np.uint16)
        special = np.array([0x8000, 0x7FC1, 0xFFFF, 0x7F80, 0xFF80, 0x0001,
                            0x8001, 0x7F81], dtype=np.uint16)
    else:
        w = (z >> np.uint64(32)).astype(np.uint32)
        special = np.array([0x80000000, 0x7FC00001, 0xFFFFFFFF, 0x7F800000,
                            0xFF800000, 0x00000001, 0x80000001, 0x7F800001],
                           dtype=np.uint32)
    pick = (z % np.uint64(5)) == np.uint64(0)
    which = ((z >> np.uint64(8)) % np.uint64(len(special))).astype(np.int64)
    w = np.where(pick, special[which], w)
    return w.reshape(shape)
