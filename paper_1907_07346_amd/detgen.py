"""Bit-reproducible synthetic gradients: the same numbers on the host (numpy, here) and on the GPU
(`ds_workload_gradient` in libdsq), so that long free runs need no host-device traffic.

This is input generation, not part of DeepSqueeze: it holds none of the method's arithmetic.  Every value is a
pure function of (seed, tag, t, worker i, column j):

    words  = Philox4x32-10(counter = (c, i, t mod 2^32, tag), key = (seed low, seed high))
    u1, u2 = (word + 0.5) * 2^-32                       two uniforms in (0, 1) per pair of words
    z0, z1 = sqrt(-2 ln u1) * (cos 2 pi u2, sin 2 pi u2)        Box-Muller in double

with ln, sin and cos evaluated by fixed polynomials in plain IEEE double operations (+, -, *, /, sqrt, no fused
multiply-add), written out identically in the HIP kernel, so both sides round alike.

    'normal'     columns 4c..4c+3 take (z0, z1) of words (0,1) and (z0, z1) of words (2,3) of counter c;
                 g = fp32(scale * z), scale an fp32 number widened to double
    'student_t3' column j takes all four normals of counter c = j:  g = fp32(scale * z0 / sqrt((z1^2+z2^2+z3^2)/3))
    'quadratic'  g = fp32(fp32(x - c_ij) + fp32(fp32(scale) * xi)),  c_ij and xi 'normal' variates of the tags
                 'CENT' (t = 0) and 'GRAD'
"""
from __future__ import annotations

from fractions import Fraction
from math import factorial

import numpy as np

TAG_CENTRE, TAG_NOISE = 0x43454E54, 0x47524144          # 'CENT', 'GRAD'
GRAD_NORMAL, GRAD_STUDENT_T3, GRAD_QUADRATIC = 0, 1, 2
GRAD_KINDS = {"normal": GRAD_NORMAL, "student_t3": GRAD_STUDENT_T3, "quadratic": GRAD_QUADRATIC}

LN2 = float.fromhex("0x1.62e42fefa39efp-1")
HALF_PI = float.fromhex("0x1.921fb54442d18p+0")
SQRT_HALF = float.fromhex("0x1.6a09e667f3bcdp-1")
LOG_TERMS, TRIG_TERMS = 13, 14
LOG_COEF = [float(Fraction(1, 2 * k + 1)) for k in range(LOG_TERMS)]                         # atanh series
SIN_COEF = [float(Fraction((-1) ** k, factorial(2 * k + 1))) for k in range(TRIG_TERMS)]
COS_COEF = [float(Fraction((-1) ** k, factorial(2 * k))) for k in range(TRIG_TERMS)]


def philox4x32_10(c0, c1, c2, c3, k0, k1):
    """Vectorised Philox4x32-10 (Salmon et al., SC'11) on uint32 arrays; returns four uint32 arrays."""
    c0, c1, c2, c3 = (np.asarray(v, dtype=np.uint64) for v in np.broadcast_arrays(c0, c1, c2, c3))
    k0, k1 = np.uint64(k0), np.uint64(k1)
    M0, M1, MASK = np.uint64(0xD2511F53), np.uint64(0xCD9E8D57), np.uint64(0xFFFFFFFF)
    for _ in range(10):
        p0, p1 = M0 * c0, M1 * c2
        n0 = (p1 >> np.uint64(32)) ^ c1 ^ k0
        n2 = (p0 >> np.uint64(32)) ^ c3 ^ k1
        c1, c3, c0, c2 = p1 & MASK, p0 & MASK, n0 & MASK, n2 & MASK
        k0 = (k0 + np.uint64(0x9E3779B9)) & MASK
        k1 = (k1 + np.uint64(0xBB67AE85)) & MASK
    return c0.astype(np.uint32), c1.astype(np.uint32), c2.astype(np.uint32), c3.astype(np.uint32)


def det_log(u):
    """ln u for double u in (0, 1]: u = f 2^e with f in [sqrt(1/2), sqrt 2), ln f = 2 atanh((f-1)/(f+1))."""
    f, e = np.frexp(u)                                   # f in [0.5, 1)
    small = f < SQRT_HALF
    f = np.where(small, f * 2.0, f)
    e = np.where(small, e - 1, e).astype(np.float64)
    s = (f - 1.0) / (f + 1.0)
    z = s * s
    p = np.full_like(z, LOG_COEF[-1])
    for c in LOG_COEF[-2::-1]:
        p = p * z + c
    return e * LN2 + (2.0 * s) * p


def det_sincos_2pi(u):
    """(cos 2 pi u, sin 2 pi u) for double u in [0, 1): quadrant from 4u, Taylor polynomials on [0, pi/2)."""
    a = 4.0 * u
    q = np.floor(a)
    phi = (a - q) * HALF_PI
    z = phi * phi
    ps = np.full_like(z, SIN_COEF[-1])
    pc = np.full_like(z, COS_COEF[-1])
    for cs, cc in zip(SIN_COEF[-2::-1], COS_COEF[-2::-1]):
        ps = ps * z + cs
        pc = pc * z + cc
    s, c = phi * ps, pc
    qi = q.astype(np.int64)
    cos = np.where(qi == 0, c, np.where(qi == 1, -s, np.where(qi == 2, -c, s)))
    sin = np.where(qi == 0, s, np.where(qi == 1, c, np.where(qi == 2, -s, -c)))
    return cos, sin


def _pair(wa, wb):
    u1 = (wa.astype(np.float64) + 0.5) * 2.0 ** -32
    u2 = (wb.astype(np.float64) + 0.5) * 2.0 ** -32
    r = np.sqrt(-2.0 * det_log(u1))
    c, s = det_sincos_2pi(u2)
    return r * c, r * s


def normals4(seed: int, tag: int, t: int, rows, counters):
    """The four double normals of each (row, counter): arrays broadcast against each other."""
    w = philox4x32_10(np.asarray(counters, dtype=np.uint64) & np.uint64(0xFFFFFFFF), np.asarray(rows, dtype=np.uint64),
                      np.uint64(t & 0xFFFFFFFF), np.uint64(tag), seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
    z0, z1 = _pair(w[0], w[1])
    z2, z3 = _pair(w[2], w[3])
    return z0, z1, z2, z3


def normal_field(seed: int, tag: int, t: int, n: int, N: int) -> np.ndarray:
    """n x N double normals, columns 4c..4c+3 from counter c."""
    nc = (N + 3) // 4
    z = normals4(seed, tag, t, np.arange(n)[:, None], np.arange(nc)[None, :])
    return np.stack(z, axis=-1).reshape(n, 4 * nc)[:, :N]


def gradient(kind: str, n: int, N: int, scale: float, seed: int, t: int, x=None) -> np.ndarray:
    """The gradients of step t (n x N, fp32); 'quadratic' needs the current x (n x N, fp32)."""
    if kind == "normal":
        return (np.float64(np.float32(scale)) * normal_field(seed, TAG_NOISE, t, n, N)).astype(np.float32)
    if kind == "student_t3":
        z0, z1, z2, z3 = normals4(seed, TAG_NOISE, t, np.arange(n)[:, None], np.arange(N)[None, :])
        return (np.float64(np.float32(scale)) * z0 / np.sqrt((z1 * z1 + z2 * z2 + z3 * z3) / 3.0)).astype(np.float32)
    if kind == "quadratic":
        c = normal_field(seed, TAG_CENTRE, 0, n, N).astype(np.float32)
        xi = normal_field(seed, TAG_NOISE, t, n, N).astype(np.float32)
        d = np.asarray(x, dtype=np.float32) - c
        return d + np.float32(scale) * xi
    raise ValueError(kind)


def centres(n: int, N: int, seed: int) -> np.ndarray:
    """The minimisers c_i of the quadratic workload (fp32)."""
    return normal_field(seed, TAG_CENTRE, 0, n, N).astype(np.float32)
