"""Oracle: the perturbation stream z ~ N(0, I) regenerated from (seed, step, k).

TEST INFRASTRUCTURE ONLY - never imported by the product path.

Algorithm 1 (its seed-sampling and noise-drawing steps) only says that query i samples a seed s_i and draws z_i ~ N(0, I)
from it, and that s_i is stored instead of z_i (the seed trick of Section 2, "ZO LLM
Fine-Tuning").  The concrete generator is this build's own specification:

* words: Philox4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw, SC'11).  key = (seed low
  word, seed high word); counter = (j, tensor_id, step, k) where j indexes groups of four
  consecutive elements of a LoRA factor in row-major order, tensor_id =
  (layer*4 + target)*2 + factor, and k is the query index.  The stream therefore depends on
  neither q, E, S nor the perturbation sign, and any element can be regenerated alone.
* uniform: u = ((x >> 9) + 1/2) * 2^-23, exact in binary32, strictly inside (0, 1).
* normal: Box-Muller on the word pairs (x0, x1) and (x2, x3):
  rho = sqrt(-2 ln u_a), z_even = rho cos(2 pi u_b), z_odd = rho sin(2 pi u_b).
  ln, sin and cos are fixed sequences of binary32 multiplies and adds (each rounded to
  nearest-even, never fused) with the polynomial coefficients below, so that any IEEE-754
  machine produces the same bits; sqrt is the correctly rounded binary32 square root.
"""
from __future__ import annotations

import numpy as np

# ---- Philox4x32-10 -----------------------------------------------------------------------
_M0 = np.uint64(0xD2511F53)
_M1 = np.uint64(0xCD9E8D57)
_W0 = 0x9E3779B9
_W1 = 0xBB67AE85
_MASK = np.uint64(0xFFFFFFFF)
_SH32 = np.uint64(32)


def philox4x32_10(counter, key):
    """counter: four uint32 arrays (broadcastable); key: two python ints. Returns 4 uint32 arrays."""
    c0, c1, c2, c3 = [np.asarray(c, dtype=np.uint64) for c in np.broadcast_arrays(*counter)]
    k0, k1 = int(key[0]) & 0xFFFFFFFF, int(key[1]) & 0xFFFFFFFF
    for rnd in range(10):
        p0 = _M0 * c0                      # 32x32 -> 64-bit products, exact in uint64
        p1 = _M1 * c2
        hi0, lo0 = p0 >> _SH32, p0 & _MASK
        hi1, lo1 = p1 >> _SH32, p1 & _MASK
        c0, c1, c2, c3 = (hi1 ^ c1 ^ np.uint64(k0), lo1, hi0 ^ c3 ^ np.uint64(k1), lo0)
        k0 = (k0 + _W0) & 0xFFFFFFFF       # Weyl key schedule
        k1 = (k1 + _W1) & 0xFFFFFFFF
    return tuple(c.astype(np.uint32) for c in (c0, c1, c2, c3))


# ---- binary32 transform ------------------------------------------------------------------
_f = np.float32


def _h(s: str) -> np.float32:
    return np.float32(float.fromhex(s))


# ln(1+t) = t * P(t), t in [sqrt(1/2)-1, sqrt(2)-1]; coefficients of t^0..t^10
_LN_C = [_h(s) for s in (
    "0x1.000000p+0", "-0x1.000000p-1", "0x1.555540p-2", "-0x1.000010p-2", "0x1.99a71cp-3",
    "-0x1.555c8cp-3", "0x1.2312fep-3", "-0x1.fbdf42p-4", "0x1.e8676ep-4", "-0x1.e058eap-4",
    "0x1.141476p-4")]
_LN2_HI = _h("0x1.62e000p-1")     # ln 2 split so that e * LN2_HI is exact for |e| <= 24
_LN2_LO = _h("0x1.0bfbe8p-15")
# sin(pi/2 * y) = y * S(y^2), cos(pi/2 * y) = C(y^2), y in (0, 1/2]; coefficients of w^0..w^4
_SIN_C = [_h(s) for s in ("0x1.921fb6p+0", "-0x1.4abbcep-1", "0x1.466bbap-4", "-0x1.32ca9ep-8",
                          "0x1.4bc87ap-13")]
_COS_C = [_h(s) for s in ("0x1.000000p+0", "-0x1.3bd3ccp+0", "0x1.03c1dcp-2", "-0x1.55c57ap-6",
                          "0x1.d9c326p-11")]
_SQRT2_BITS = np.uint32(0x3FB504F3)   # binary32 just above sqrt(2)


def _horner(coefs, x):
    acc = np.full(x.shape, coefs[-1], dtype=np.float32)
    for c in coefs[-2::-1]:
        acc = acc * x          # rounded binary32 multiply
        acc = acc + c          # rounded binary32 add
    return acc


def uniform_from_word(x):
    """u = ((x >> 9) + 1/2) * 2^-23 as binary32 (exact)."""
    m = (np.asarray(x, dtype=np.uint32) >> np.uint32(9)).astype(np.float32)
    return (m + _f(0.5)) * _f(2.0 ** -23)


def neg2_ln(u):
    """-2 ln(u) for binary32 u in (0, 1), by exponent extraction and a fixed polynomial."""
    bits = np.asarray(u, dtype=np.float32).view(np.uint32)
    e = (bits >> np.uint32(23)).astype(np.int32) - 127
    fbits = (bits & np.uint32(0x007FFFFF)) | np.uint32(0x3F800000)       # f in [1, 2)
    big = fbits >= _SQRT2_BITS
    f = fbits.view(np.float32)
    f = np.where(big, f * _f(0.5), f)                                     # exact
    e = np.where(big, e + 1, e).astype(np.float32)
    t = f - _f(1.0)                                                       # exact (Sterbenz)
    lnf = _horner(_LN_C, t) * t
    ln_u = e * _LN2_HI + (e * _LN2_LO + lnf)
    return ln_u * _f(-2.0)


def sincos_2pi(x):
    """(cos, sin)(2 pi u) for the uniform u made from word x; octant folding on the 23-bit integer."""
    m = np.asarray(x, dtype=np.uint32) >> np.uint32(9)                    # 23 bits
    quad = (m >> np.uint32(21)).astype(np.int32)
    wq = m & np.uint32(0x1FFFFF)                                          # position in the quadrant
    flip = wq >= np.uint32(0x100000)
    wq = np.where(flip, np.uint32(0x1FFFFF) - wq, wq)                     # reflect about pi/4
    y = (wq.astype(np.float32) + _f(0.5)) * _f(2.0 ** -21)                # exact, in (0, 1/2)
    w = y * y
    s = _horner(_SIN_C, w) * y
    c = _horner(_COS_C, w)
    s, c = np.where(flip, c, s), np.where(flip, s, c)                     # first-quadrant sin, cos
    # rotate by quadrant: angle = quad * pi/2 + phi
    cos_out = np.where(quad == 0, c, np.where(quad == 1, -s, np.where(quad == 2, -c, s)))
    sin_out = np.where(quad == 0, s, np.where(quad == 1, c, np.where(quad == 2, -s, -c)))
    return cos_out.astype(np.float32), sin_out.astype(np.float32)


def normals_from_words(x0, x1, x2, x3):
    """Four binary32 standard normals from four Philox words (Box-Muller on two pairs)."""
    out = []
    for xa, xb in ((x0, x1), (x2, x3)):
        rho = np.sqrt(neg2_ln(uniform_from_word(xa)))                     # correctly rounded sqrt
        c, s = sincos_2pi(xb)
        out.append(rho * c)
        out.append(rho * s)
    return out


def noise_tensor(seed: int, step: int, k: int, tensor_id: int, numel: int) -> np.ndarray:
    """z for one LoRA factor (flat, row-major, binary32).  numel must be a multiple of 4."""
    assert numel % 4 == 0
    j = np.arange(numel // 4, dtype=np.uint32)
    ctr = (j, np.uint32(tensor_id), np.uint32(step), np.uint32(k))
    key = (seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
    z = normals_from_words(*philox4x32_10(ctr, key))
    return np.stack(z, axis=1).reshape(-1)
