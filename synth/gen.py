"""Counter-based fp32 Gaussian generator, host side (numpy).

value(seed, domain, row, col) is a pure function, so any column subset of any row can be
produced without generating the rest -- the parity tests rely on this to follow a few
thousand columns of a 25.6 M-column state.

Definition (the device kernel in fill.hip performs exactly the same operations):

  words  = Philox4x32-10(counter = (col // 4, row_lo, row_hi, domain), key = (seed_lo, seed_hi))
  (z0, z1) = box_muller(words[0], words[1]);  (z2, z3) = box_muller(words[2], words[3])
  value  = mean + sigma * z[col % 4]

box_muller uses only individually rounded fp32 +, -, *, /, sqrt and exact integer/bit
operations, in a fixed order, with polynomial logarithm / sine / cosine written out here, so
that host and device agree bit for bit (no libm, no fused multiply-add):

  u1 = ((w0 >> 9) + 0.5) * 2^-23                      in (0, 1), exact
  -ln u1:  u1 = m * 2^e, m in [1, 2); if m > sqrt(2): m /= 2, e += 1
           s = (m - 1) / (m + 1);  ln m = 2 s (1 + s^2/3 + s^4/5 + s^6/7 + s^8/9)
  r  = sqrt(2 * (-ln u1))
  angle = 2 pi * (w1 >> 8) / 2^24, reduced to a quadrant (top two bits) and an octant
          (reflection about pi/4), Taylor polynomials on [0, pi/4]
  z0 = r cos(angle), z1 = r sin(angle)
"""
import numpy as np

DOMAIN_INIT = 1   # row = worker index: initial parameters x_i(0)
DOMAIN_C = 2      # row = worker index: minimiser c_i of the local quadratic
DOMAIN_XI = 3     # row = serial event index: additive gradient noise of that event
DOMAIN_H = 5      # row = worker index: the normals behind the curvatures h_i of the local quadratic (4: straggler rates)

_M32 = np.uint64(0xFFFFFFFF)
_f = np.float32


def philox4x32_10(c0, c1, c2, c3, k0, k1):
    """Vectorised Philox4x32-10 (Salmon et al., SC'11).  Inputs broadcastable, values < 2^32.
    Returns four uint64 arrays holding 32-bit words."""
    c0, c1, c2, c3 = (np.asarray(v, np.uint64) & _M32 for v in (c0, c1, c2, c3))
    c0, c1, c2, c3 = np.broadcast_arrays(c0, c1, c2, c3)
    k0 = np.uint64(int(k0) & 0xFFFFFFFF)
    k1 = np.uint64(int(k1) & 0xFFFFFFFF)
    m0, m1 = np.uint64(0xD2511F53), np.uint64(0xCD9E8D57)
    w0, w1 = np.uint64(0x9E3779B9), np.uint64(0xBB67AE85)
    s32 = np.uint64(32)
    for _ in range(10):
        p0 = m0 * c0
        p1 = m1 * c2
        c0, c1, c2, c3 = ((p1 >> s32) ^ c1 ^ k0), (p1 & _M32), ((p0 >> s32) ^ c3 ^ k1), (p0 & _M32)
        k0 = (k0 + w0) & _M32
        k1 = (k1 + w1) & _M32
    return c0, c1, c2, c3


_LN2 = _f(0.693147182464599609375)
_SQRT2 = _f(1.41421353816986083984375)
_L3, _L5, _L7, _L9 = _f(1.0 / 3.0), _f(0.2), _f(1.0 / 7.0), _f(1.0 / 9.0)
_ANGLE_STEP = _f(np.pi / 2.0 * 2.0 ** -22)
_S3, _S5, _S7, _S9 = _f(-1.0 / 6.0), _f(1.0 / 120.0), _f(-1.0 / 5040.0), _f(1.0 / 362880.0)
_C2, _C4, _C6, _C8, _C10 = _f(-0.5), _f(1.0 / 24.0), _f(-1.0 / 720.0), _f(1.0 / 40320.0), _f(-1.0 / 3628800.0)


def box_muller(w0, w1):
    """Two fp32 standard normals from two 32-bit words (arrays of uint64 holding 32-bit values)."""
    w0 = np.asarray(w0, np.uint64); w1 = np.asarray(w1, np.uint64)
    one, half, two = _f(1.0), _f(0.5), _f(2.0)
    u1 = ((w0 >> np.uint64(9)).astype(np.float32) + half) * _f(2.0 ** -23)
    bits = u1.view(np.uint32)
    e = (bits >> np.uint32(23)).astype(np.int32) - np.int32(127)
    m = ((bits & np.uint32(0x007FFFFF)) | np.uint32(0x3F800000)).view(np.float32)
    big = m > _SQRT2
    m = np.where(big, m * half, m)
    e = np.where(big, e + np.int32(1), e)
    s = (m - one) / (m + one)
    z = s * s
    p = _L9 * z + _L7
    p = p * z + _L5
    p = p * z + _L3
    p = p * z + one
    ln = e.astype(np.float32) * _LN2 + (s + s) * p
    neg = -ln
    r = np.sqrt(neg + neg)

    w = (w1 >> np.uint64(8)).astype(np.uint32)
    quad = w >> np.uint32(22)
    fr = w & np.uint32(0x3FFFFF)
    swap = fr > np.uint32(0x200000)
    fr = np.where(swap, np.uint32(0x400000) - fr, fr)
    phi = fr.astype(np.float32) * _ANGLE_STEP
    y = phi * phi
    ps = _S9 * y + _S7
    ps = ps * y + _S5
    ps = ps * y + _S3
    ps = ps * y + one
    sn = phi * ps
    pc = _C10 * y + _C8
    pc = pc * y + _C6
    pc = pc * y + _C4
    pc = pc * y + _C2
    cs = pc * y + one
    sn, cs = np.where(swap, cs, sn), np.where(swap, sn, cs)
    # rotate by quad * pi/2
    c_out = np.where(quad == 0, cs, np.where(quad == 1, -sn, np.where(quad == 2, -cs, sn)))
    s_out = np.where(quad == 0, sn, np.where(quad == 1, cs, np.where(quad == 2, -sn, -cs)))
    return (r * c_out).astype(np.float32), (r * s_out).astype(np.float32)


def normal(seed, domain, row, cols, sigma=1.0, mean=0.0):
    """fp32 values of the generator at (row, cols) for an arbitrary integer array cols."""
    cols = np.asarray(cols, np.int64)
    q = (cols >> 2).astype(np.uint64)
    lane = (cols & 3)
    row = int(row)
    w = philox4x32_10(q, row & 0xFFFFFFFF, (row >> 32) & 0xFFFFFFFF, int(domain),
                      int(seed) & 0xFFFFFFFF, (int(seed) >> 32) & 0xFFFFFFFF)
    z0, z1 = box_muller(w[0], w[1])
    z2, z3 = box_muller(w[2], w[3])
    z = np.where(lane == 0, z0, np.where(lane == 1, z1, np.where(lane == 2, z2, z3)))
    return (_f(mean) + _f(sigma) * z).astype(np.float32)


def normal_rows(seed, domain, rows, cols, sigma=1.0, mean=0.0):
    """(len(rows), len(cols)) fp32 matrix: one generator row per entry of rows (numpy implementation)."""
    return np.stack([normal(seed, domain, r, cols, sigma, mean) for r in rows]) if len(rows) else \
        np.zeros((0, len(cols)), np.float32)


_clib = None


def _c_library():
    """gen_c.c compiled on first use (gcc, -ffp-contract=off): the same definition, ~100x faster."""
    global _clib
    if _clib is None:
        import ctypes as C
        import os
        import subprocess
        here = os.path.dirname(os.path.abspath(__file__))
        src, lib = os.path.join(here, "gen_c.c"), os.path.join(here, "libsynth_gen.so")
        if not os.path.exists(lib) or os.path.getmtime(lib) < os.path.getmtime(src):
            subprocess.run(["gcc", "-O2", "-ffp-contract=off", "-fno-fast-math", "-std=c11", "-shared", "-fPIC",
                            src, "-o", lib, "-lm"], check=True)
        _clib = C.CDLL(lib)
        i64 = np.ctypeslib.ndpointer(np.int64, flags="C_CONTIGUOUS")
        _clib.synth_normal_rows.argtypes = [C.c_uint64, C.c_uint32, i64, C.c_int64, i64, C.c_int64, C.c_float,
                                            C.c_float, np.ctypeslib.ndpointer(np.float32, flags="C_CONTIGUOUS")]
        _clib.synth_normal_rows.restype = None
    return _clib


def normal_rows_fast(seed, domain, rows, cols, sigma=1.0, mean=0.0):
    """Same values as normal_rows, computed by the C implementation of the same definition."""
    rows = np.ascontiguousarray(rows, np.int64)
    cols = np.ascontiguousarray(cols, np.int64)
    out = np.zeros((len(rows), len(cols)), np.float32)
    if out.size:
        _c_library().synth_normal_rows(int(seed), int(domain), rows, len(rows), cols, len(cols),
                                       float(sigma), float(mean), out)
    return out


def curvature(z):
    """Curvatures of a local quadratic from standard normals: h = 0.25 + 0.75 min(z^2, 4), in [0.25, 3.25] with mean
    about 0.96, every step an individually rounded fp32 operation (the device harness does the same three steps)."""
    z = np.asarray(z, np.float32)
    return (np.minimum(z * z, _f(4.0)) * _f(0.75) + _f(0.25)).astype(np.float32)
