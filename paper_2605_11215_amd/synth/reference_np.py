"""Seeded synthetic inputs, NumPy side.

This module only makes INPUTS (gradient streams and initial parameters); it holds none of
the arithmetic of the gradient path.  Both the CPU oracle's tests and the HIP library's
tests draw their inputs from it (or from its device twin, `synth.hip`, which is written to
return the same bits), so that both sides see identical numbers.

Stream definition (counter-based, random access by element index i):

  Philox4x32-10 (Salmon et al., SC'11): key = (seed, tag), counter = (c0, mb_id, iter, kind)
    tag  0 gradients, 1 initial parameters, 2 failure schedule
    kind 0 Gaussian: c0 = i >> 2, element i takes lane i & 3 of the four normals below
    kind 1 Student-t(3): c0 = i, one draw per element
  uniforms  u_j = (2 * (x_j >> 9) + 1) / 2**24            (odd 24-bit numerators, never 0 or 1)
  normals   (z0, z1) = Box-Muller(u0, u1), (z2, z3) = Box-Muller(u2, u3) with
            z_even = sqrt(-2 ln u_a) * cos(2 pi u_b), z_odd = sqrt(-2 ln u_a) * sin(2 pi u_b)
  value     Gaussian: fp32(scale * z)            Student-t: fp32(scale * z0 / sqrt((z1^2+z2^2+z3^2)/3))
  bf16      round-to-nearest-even of that fp32 value

ln, cos and sin are evaluated with the fixed fp64 operation sequences below (+, -, *, /
and sqrt only, no fused multiply-add), so any IEEE-754 implementation that follows the
same sequence returns the same bits.
"""
import numpy as np

_M0 = np.uint64(0xD2511F53)
_M1 = np.uint64(0xCD9E8D57)
_W0 = 0x9E3779B9
_W1 = 0xBB67AE85
_MASK = np.uint64(0xFFFFFFFF)
_S32 = np.uint64(32)

TAG_GRAD, TAG_PARAM, TAG_SCHEDULE = 0, 1, 2
KIND_NORMAL, KIND_STUDENT_T3 = 0, 1

LN2 = 0.6931471805599453
SQRT2 = 1.4142135623730951
HALF_PI = 1.5707963267948966
_LOG_COEF = [2.0 / (2 * k + 1) for k in range(13)]          # 2, 2/3, 2/5, ...
_SIN_COEF = [1.0, -1.0 / 6, 1.0 / 120, -1.0 / 5040, 1.0 / 362880, -1.0 / 39916800,
             1.0 / 6227020800, -1.0 / 1307674368000, 1.0 / 355687428096000]
_COS_COEF = [1.0, -1.0 / 2, 1.0 / 24, -1.0 / 720, 1.0 / 40320, -1.0 / 3628800,
             1.0 / 479001600, -1.0 / 87178291200, 1.0 / 20922789888000,
             -1.0 / 6402373705728000]


def philox4x32_10(c0, c1, c2, c3, k0, k1):
    """Vectorised Philox4x32 with 10 rounds.  Inputs broadcastable uint32-valued arrays or
    ints; returns four uint64 arrays holding 32-bit words."""
    c0, c1, c2, c3 = (np.asarray(c, np.uint64) & _MASK for c in (c0, c1, c2, c3))
    c0, c1, c2, c3 = np.broadcast_arrays(c0, c1, c2, c3)
    k0, k1 = int(k0) & 0xFFFFFFFF, int(k1) & 0xFFFFFFFF
    for _ in range(10):
        p0 = _M0 * c0                        # 32x32 -> 64 products
        p1 = _M1 * c2
        n0 = (p1 >> _S32) ^ c1 ^ np.uint64(k0)
        n1 = p1 & _MASK
        n2 = (p0 >> _S32) ^ c3 ^ np.uint64(k1)
        n3 = p0 & _MASK
        c0, c1, c2, c3 = n0, n1, n2, n3
        k0 = (k0 + _W0) & 0xFFFFFFFF
        k1 = (k1 + _W1) & 0xFFFFFFFF
    return c0, c1, c2, c3


def _numerator(x):
    """Odd 24-bit numerator n of u = n / 2**24 from a 32-bit word."""
    return ((x >> np.uint64(9)) << np.uint64(1)) | np.uint64(1)


def _ln_u(n):
    """ln(n / 2**24) for odd integers 1 <= n < 2**24, fixed fp64 sequence."""
    nf = n.astype(np.float64)
    m, e = np.frexp(nf)                                     # nf = m * 2**e, m in [0.5, 1), exact
    m = m * 2.0                                             # [1, 2)
    e = e.astype(np.int64) - 1
    big = m > SQRT2
    m = np.where(big, m * 0.5, m)
    e = np.where(big, e + 1, e)
    s = (m - 1.0) / (m + 1.0)
    s2 = s * s
    acc = np.full_like(s, _LOG_COEF[12])
    for k in range(11, -1, -1):
        acc = acc * s2 + _LOG_COEF[k]
    return (e - 24).astype(np.float64) * LN2 + s * acc


def _cos_sin_2pi_u(n):
    """(cos, sin) of 2*pi*n / 2**24 for odd integers n < 2**24, fixed fp64 sequence."""
    q = (n >> np.uint64(22)).astype(np.int64)               # quadrant
    r = (n & np.uint64((1 << 22) - 1)).astype(np.int64)     # numerator of the quarter fraction
    flip = r > (1 << 21)
    r = np.where(flip, (1 << 22) - r, r)
    th = (r.astype(np.float64) * (1.0 / (1 << 22))) * HALF_PI        # (0, pi/4]
    t2 = th * th
    sp = np.full_like(th, _SIN_COEF[8])
    for k in range(7, -1, -1):
        sp = sp * t2 + _SIN_COEF[k]
    sp = sp * th
    cp = np.full_like(th, _COS_COEF[9])
    for k in range(8, -1, -1):
        cp = cp * t2 + _COS_COEF[k]
    c1 = np.where(flip, sp, cp)                             # within the first quadrant
    s1 = np.where(flip, cp, sp)
    c = np.where(q == 0, c1, np.where(q == 1, -s1, np.where(q == 2, -c1, s1)))
    s = np.where(q == 0, s1, np.where(q == 1, c1, np.where(q == 2, -s1, -c1)))
    return c, s


def _four_normals(x0, x1, x2, x3):
    ra = np.sqrt(-2.0 * _ln_u(_numerator(x0)))
    ca, sa = _cos_sin_2pi_u(_numerator(x1))
    rb = np.sqrt(-2.0 * _ln_u(_numerator(x2)))
    cb, sb = _cos_sin_2pi_u(_numerator(x3))
    return ra * ca, ra * sa, rb * cb, rb * sb


def values(idx, seed, tag, mb_id, it, scale, kind=KIND_NORMAL):
    """fp32 stream values at element indices `idx` (any integer array; below 2^34 for the Gaussian stream, which
    packs four elements per 32-bit counter word, below 2^32 for the Student-t stream)."""
    idx = np.asarray(idx, np.uint64)
    if idx.size and int(idx.max()) >= (1 << 34 if kind == KIND_NORMAL else 1 << 32):
        raise ValueError("element index beyond the stream's counter word")
    if kind == KIND_NORMAL:
        x = philox4x32_10(idx >> np.uint64(2), mb_id, it, KIND_NORMAL, seed, tag)
        lane = (idx & np.uint64(3)).astype(np.int64)
        second = lane >= 2                                  # lanes 2, 3 come from words 2, 3
        r = np.sqrt(-2.0 * _ln_u(_numerator(np.where(second, x[2], x[0]))))
        c, s = _cos_sin_2pi_u(_numerator(np.where(second, x[3], x[1])))
        zz = r * np.where((lane & 1) == 0, c, s)
        return (float(scale) * zz).astype(np.float32)
    if kind == KIND_STUDENT_T3:
        x = philox4x32_10(idx, mb_id, it, KIND_STUDENT_T3, seed, tag)
        z0, z1, z2, z3 = _four_normals(*x)
        den = np.sqrt(((z1 * z1 + z2 * z2) + z3 * z3) / 3.0)
        return ((float(scale) * z0) / den).astype(np.float32)
    raise ValueError("kind")


def fill(n, seed, tag, mb_id, it, scale, kind=KIND_NORMAL, start=0, chunk=1 << 20):
    """fp32 stream values for elements start .. start+n-1 (same bits as `values`)."""
    out = np.empty(n, np.float32)
    if kind != KIND_NORMAL:
        for lo in range(0, n, chunk):
            hi = min(n, lo + chunk)
            out[lo:hi] = values(np.arange(start + lo, start + hi, dtype=np.uint64),
                                seed, tag, mb_id, it, scale, kind)
        return out
    q0, q1 = start >> 2, (start + n + 3) >> 2               # one Philox call per four elements
    for lo in range(q0, q1, chunk):
        hi = min(q1, lo + chunk)
        x = philox4x32_10(np.arange(lo, hi, dtype=np.uint64), mb_id, it, KIND_NORMAL, seed, tag)
        z = np.stack(_four_normals(*x), axis=1).reshape(-1)
        v = (float(scale) * z).astype(np.float32)
        a, b = max(start, lo * 4), min(start + n, hi * 4)
        out[a - start:b - start] = v[a - lo * 4:b - lo * 4]
    return out


def f32_to_bf16_bits(x):
    """Round-to-nearest-even bf16 bit patterns (uint16) of fp32 values; a NaN keeps its sign and upper
    payload bits and gets the quiet bit, so it stays a NaN."""
    b = np.ascontiguousarray(x, np.float32).view(np.uint32)
    r = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    nan = (b & np.uint32(0x7FFFFFFF)) > np.uint32(0x7F800000)
    r = np.where(nan, (b >> np.uint32(16)) | np.uint32(0x40), r)
    return r.astype(np.uint16)


def bf16_bits_to_f32(h):
    return (np.asarray(h, np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def schedule_words(seed, it):
    """Four 32-bit words for drawing a failure (replica, offset) at iteration `it`."""
    x = philox4x32_10(it, 0, 0, 0, seed, TAG_SCHEDULE)
    return [int(np.asarray(w).reshape(-1)[0]) for w in x]
