"""Oracle: seeded synthetic intermediate labels (paper Sec. 2, Eq. 1).

TEST INFRASTRUCTURE ONLY (see the package docstring).

The paper asks for an ``N_P x M`` matrix whose entries are ``kappa * U(0,1)``,
one column per class (Sec. 2, Eq. 1; the experiment uses 60 x 47 with
kappa = 10, Sec. 3).  It names no generator.  The reading taken here, so that a
GPU and a CPU can agree bit for bit, is a counter-based generator: every table
entry is a pure function of (seed, class, index), computed with Philox4x32-10
(Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3",
SC'11) followed by a fixed sequence of individually rounded float32 operations.

Layout: tables are stored row = class, ``T[class, index]`` (the transpose of the
paper's ``SIL``; same numbers).

Counter / key convention (the method's definition, implemented independently by
the HIP library):

  key      = (seed & 0xffffffff, seed >> 32)
  labels   : counter = (index i, class j, 0, 0)
  weights  : counter = (input k, output o, 1, layer)    bias uses k = fan_in
  noise    : counter = (index i, n & 0xffffffff, 2, n >> 32), n = global sample

Word r0 (and r1 for the normal transform) of the 4-word Philox output is used;
one counter per element, so an entry never depends on the table's shape.

Transforms, all float32, every operation rounded on its own (no fused
multiply-add anywhere):

  u          = (r0 >> 8) * 2^-24                       in [0,1)   (exact)
  UNIFORM01  : kappa * u                               Eq. 1, read as [0,1)
  UNIFORM_PM1: 2u - 1                                  in [-1,1)  (exact)
  BINARY_PM1 : +1 if r0's top bit is set else -1
  NORMAL     : Box-Muller, cosine branch, with ln and cos written out as fixed
               polynomial sequences (``normal_from_words``) because library
               log/cos differ between a host libm and a device math library.

parity pins: tests/test_oracle_rng.py (published Philox known-answer vectors,
an arbitrary-precision second implementation, exact integer identities, the
normal transform against double-precision Box-Muller, distribution tests).
"""

import numpy as np

UNIFORM01, UNIFORM_PM1, NORMAL, BINARY_PM1 = 0, 1, 2, 3

STREAM_LABELS, STREAM_WEIGHTS, STREAM_NOISE = 0, 1, 2

_M0 = np.uint64(0xD2511F53)
_M1 = np.uint64(0xCD9E8D57)
_W0 = 0x9E3779B9
_W1 = 0xBB67AE85
_MASK = np.uint64(0xFFFFFFFF)
_SH32 = np.uint64(32)


def philox4x32_10(c0, c1, c2, c3, k0, k1):
    """Philox4x32 with 10 rounds on arrays of 32-bit words.

    One round maps (c0,c1,c2,c3) to (hi(M1*c2)^c1^k0, lo(M1*c2),
    hi(M0*c0)^c3^k1, lo(M0*c0)); the key is advanced by the Weyl constants
    between rounds (9 bumps for 10 rounds).  Arguments broadcast; returns four
    uint32 arrays.
    """
    c0, c1, c2, c3 = (np.asarray(c, dtype=np.uint64) & _MASK for c in (c0, c1, c2, c3))
    c0, c1, c2, c3 = np.broadcast_arrays(c0, c1, c2, c3)
    k0 = int(k0) & 0xFFFFFFFF
    k1 = int(k1) & 0xFFFFFFFF
    for rnd in range(10):
        p0 = _M0 * c0          # 32x32 -> 64 bit products, exact in uint64
        p1 = _M1 * c2
        hi0, lo0 = p0 >> _SH32, p0 & _MASK
        hi1, lo1 = p1 >> _SH32, p1 & _MASK
        n0 = hi1 ^ c1 ^ np.uint64(k0)
        n2 = hi0 ^ c3 ^ np.uint64(k1)
        c0, c1, c2, c3 = n0, lo1, n2, lo0
        if rnd != 9:
            k0 = (k0 + _W0) & 0xFFFFFFFF
            k1 = (k1 + _W1) & 0xFFFFFFFF
    return tuple(c.astype(np.uint32) for c in (c0, c1, c2, c3))


def _key(seed):
    seed = int(seed) & 0xFFFFFFFFFFFFFFFF
    return seed & 0xFFFFFFFF, seed >> 32


def uniform01_from_word(r0):
    """u = (r0 >> 8) * 2^-24, exact in float32, in [0,1)."""
    return (np.asarray(r0, np.uint32) >> np.uint32(8)).astype(np.float32) * np.float32(2.0 ** -24)


# float32 constants of the normal transform, given by their bit patterns.
def _f32(bits):
    return np.array([bits], dtype=np.uint32).view(np.float32)[0]


_SQRT2 = _f32(0x3FB504F3)       # fl(sqrt 2)
_LN2_HI = _f32(0x3F317200)      # upper bits of ln 2 (low 9 mantissa bits zero)
_LN2_LO = _f32(0x35BFBE8E)      # fl(ln 2 - LN2_HI)
_A3 = _f32(0x3F2AAAAB)          # fl(2/3)
_A5 = _f32(0x3ECCCCCD)          # fl(2/5)
_A7 = _f32(0x3E924925)          # fl(2/7)
_A9 = _f32(0x3E638E39)          # fl(2/9)
_PIO2 = _f32(0x3FC90FDB)        # fl(pi/2)
_S3 = _f32(0xBE2AAAAB)          # fl(-1/3!)
_S5 = _f32(0x3C088889)          # fl(1/5!)
_S7 = _f32(0xB9500D01)          # fl(-1/7!)
_S9 = _f32(0x3638EF1D)          # fl(1/9!)
_K2 = _f32(0xBF000000)          # -1/2!
_K4 = _f32(0x3D2AAAAB)          # fl(1/4!)
_K6 = _f32(0xBAB60B61)          # fl(-1/6!)
_K8 = _f32(0x37D00D01)          # fl(1/8!)
_K10 = _f32(0xB493F27E)         # fl(-1/10!)


def normal_from_words(r0, r1):
    """Standard normal from two Philox words: sqrt(-2 ln u1) * cos(2 pi u2).

    u1 = ((r0>>8)+1) * 2^-24 in (0,1],  u2 = (r1>>8) * 2^-24 in [0,1).

    ln u1: split u1 = m * 2^e with m in [1,2) from the float32 bit pattern; if
    m > fl(sqrt 2) halve m and bump e.  With s = (m-1)/(m+1),
    ln m = 2s + s*s^2 * (2/3 + s^2 (2/5 + s^2 (2/7 + s^2 * 2/9))) (Horner, each
    multiply and add rounded), and ln u1 = e*LN2_HI + (e*LN2_LO + ln m).

    cos(2 pi u2): with k = r1 >> 8 (24 bits) the quadrant is q = k >> 22 and the
    fraction f = (k & (2^22-1)) / 2^22.  If f > 1/2 it is reflected, t = 1 - f
    (sine and cosine swap), so x = t * fl(pi/2) lies in [0, pi/4]; sin x and
    cos x are the Taylor polynomials to x^9 and x^10 in Horner form; the
    quadrant picks +-sin or +-cos.

    Every arithmetic step is a single float32 operation.
    """
    f32 = np.float32
    r0 = np.asarray(r0, np.uint32)
    r1 = np.asarray(r1, np.uint32)
    j1 = (r0 >> np.uint32(8)) + np.uint32(1)
    u1 = j1.astype(f32) * f32(2.0 ** -24)
    bits = u1.view(np.uint32)
    e = (bits >> np.uint32(23)).astype(np.int32) - np.int32(127)
    m = ((bits & np.uint32(0x007FFFFF)) | np.uint32(0x3F800000)).view(f32)
    big = m > _SQRT2
    m = np.where(big, m * f32(0.5), m).astype(f32)
    e = np.where(big, e + 1, e).astype(np.int32)
    s = (m - f32(1.0)) / (m + f32(1.0))
    s2 = s * s
    p = s2 * _A9 + _A7
    p = p * s2 + _A5
    p = p * s2 + _A3
    lnm = s * f32(2.0) + (s * s2) * p
    ef = e.astype(f32)
    ln_u = ef * _LN2_HI + (ef * _LN2_LO + lnm)
    radius = np.sqrt(f32(-2.0) * ln_u)

    k = r1 >> np.uint32(8)
    q = k >> np.uint32(22)
    fi = k & np.uint32(0x3FFFFF)
    swap = fi > np.uint32(1 << 21)
    ti = np.where(swap, np.uint32(1 << 22) - fi, fi).astype(np.uint32)
    t = ti.astype(f32) * f32(2.0 ** -22)
    x = t * _PIO2
    x2 = x * x
    sp = x2 * _S9 + _S7
    sp = sp * x2 + _S5
    sp = sp * x2 + _S3
    sinx = x + (x * x2) * sp
    cp = x2 * _K10 + _K8
    cp = cp * x2 + _K6
    cp = cp * x2 + _K4
    cp = cp * x2 + _K2
    cosx = f32(1.0) + x2 * cp
    cf = np.where(swap, sinx, cosx)     # cos(pi f / 2)
    sf = np.where(swap, cosx, sinx)     # sin(pi f / 2)
    c = np.where(q == 0, cf, np.where(q == 1, -sf, np.where(q == 2, -cf, sf))).astype(f32)
    z = radius * c
    assert z.dtype == np.float32
    return z


def transform(dist, kappa, r0, r1):
    """Apply one of the four label distributions to Philox words."""
    if dist == UNIFORM01:
        return (np.float32(kappa) * uniform01_from_word(r0)).astype(np.float32)
    if dist == UNIFORM_PM1:
        return (np.float32(2.0) * uniform01_from_word(r0) - np.float32(1.0)).astype(np.float32)
    if dist == BINARY_PM1:
        top = np.asarray(r0, np.uint32) >> np.uint32(31)
        return np.where(top == 1, np.float32(1.0), np.float32(-1.0)).astype(np.float32)
    if dist == NORMAL:
        return normal_from_words(r0, r1)
    raise ValueError("unknown distribution %r" % (dist,))


def make_synthetic_labels(seed, classes, dim, dist, kappa=1.0):
    """Label table ``T[classes, dim]`` float32 (paper Eq. 1, transposed)."""
    k0, k1 = _key(seed)
    i = np.arange(dim, dtype=np.uint64)[None, :]
    j = np.arange(classes, dtype=np.uint64)[:, None]
    r0, r1, _, _ = philox4x32_10(i, j, STREAM_LABELS, 0, k0, k1)
    return transform(dist, kappa, r0, r1)


def make_segment_inputs(seed, table, y, first_sample, sigma):
    """Inputs of an interior segment in the simultaneous variant (paper Sec. 2,
    the paragraph on training every partition at once): the previous cut's label
    of the sample's class plus Gaussian noise,
    ``X[n, i] = T[y_n, i] + sigma * N(0,1)`` (float32 multiply, then add).
    The noise counter is the global sample index ``first_sample + n``.
    """
    table = np.asarray(table, np.float32)
    y = np.asarray(y, np.int64)
    k0, k1 = _key(seed)
    dim = table.shape[1]
    n = np.uint64(first_sample) + np.arange(len(y), dtype=np.uint64)
    i = np.arange(dim, dtype=np.uint64)[None, :]
    r0, r1, _, _ = philox4x32_10(i, (n & _MASK)[:, None], STREAM_NOISE, (n >> _SH32)[:, None], k0, k1)
    z = normal_from_words(r0, r1)
    return (table[y] + np.float32(sigma) * z).astype(np.float32)


def init_weights(seed, layer, fan_out, fan_in):
    """Initial ``W[fan_out, fan_in]`` and ``b[fan_out]``, both
    U(-1/sqrt(fan_in), +1/sqrt(fan_in)) -- the documented default of the
    framework the paper names for its demonstration network (Sec. 2).
    value = (2u - 1) * (1 / sqrt(fan_in)), bound computed in float32.
    """
    k0, k1 = _key(seed)
    bound = np.float32(1.0) / np.sqrt(np.float32(fan_in))
    kk = np.arange(fan_in + 1, dtype=np.uint64)[None, :]
    oo = np.arange(fan_out, dtype=np.uint64)[:, None]
    r0, _, _, _ = philox4x32_10(kk, oo, STREAM_WEIGHTS, layer, k0, k1)
    v = (np.float32(2.0) * uniform01_from_word(r0) - np.float32(1.0)) * bound
    v = v.astype(np.float32)
    return np.ascontiguousarray(v[:, :fan_in]), np.ascontiguousarray(v[:, fan_in])


def round_to_bf16(x):
    """Round float32 to the nearest bfloat16 (ties to even); returns float32
    holding the bf16 value.  NaN stays NaN."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    b = x.view(np.uint32).astype(np.uint64)
    lsb = (b >> np.uint64(16)) & np.uint64(1)
    r = (b + np.uint64(0x7FFF) + lsb) & np.uint64(0xFFFF0000)
    out = r.astype(np.uint32).view(np.float32).reshape(x.shape).copy()
    nan = np.isnan(x)
    if nan.any():
        out[nan] = np.float32(np.nan)
    return out
