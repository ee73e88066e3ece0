"""Parity rules between a device result and the fp64 oracle (test infrastructure).

Rules (floating point decides integers here, so the rules say where the two
sides may legitimately differ):

1. steps:  |s_dev - s_or| <= 1e-3 * s_or  (one fp16 ulp is < 9.8e-4 relative).
   When the two fp16 steps differ (the fp64 value sat on an fp16 rounding
   midpoint to within the device's fp32 error) the expected codes are
   recomputed by the oracle with the device's step.
2. codes:  bit-exact wherever the fp64 pre-round value u lies more than 1e-3
   away from a rounding boundary k + 0.5 that separates two representable
   codes; inside the band the device code must be one of the two neighbours.
3. de-quantized values: max |yhat_dev - yhat_or| <= 1e-2 * s on elements
   outside the band.
"""
from __future__ import annotations

import numpy as np

from . import flatquant_oracle as fo

BAND = 1e-3
SCALE_RTOL = 1e-3
DEQ_TOL = 1e-2


def _band_mask(u, lo, hi):
    """True where u is within BAND of a boundary between two codes of [lo, hi]."""
    d = np.abs(u - (np.floor(u) + 0.5))
    return (d <= BAND) & (u > lo) & (u < hi)


def check_sym(y_or, clip, codes_dev, scales_dev, deq_dev=None, rows=None):
    """y_or: fp64 [R, n] oracle transform of the checked rows; clip scalar or [R];
    codes_dev u8 [R, n/2]; scales_dev fp16 [R]; deq_dev optional fp32/64 [R, n]."""
    y_or = np.asarray(y_or, dtype=np.float64)
    scales_dev = np.asarray(scales_dev).view(np.float16).reshape(-1)
    q_or, s_or, u_or = fo.quantize_sym_int4(y_or, clip)
    s_or64, s_dev64 = fo.as_f64(s_or), fo.as_f64(scales_dev)
    assert np.all(np.isfinite(s_dev64)), "device step not finite"
    bad = np.abs(s_dev64 - s_or64) > SCALE_RTOL * s_or64
    assert not bad.any(), f"step mismatch at rows {np.nonzero(bad)[0][:8]}: dev {s_dev64[bad][:4]} oracle {s_or64[bad][:4]}"
    differ = s_dev64 != s_or64
    if differ.any():
        q2, _, u2 = fo.quantize_sym_int4(y_or[differ], None, scale_fp16=scales_dev[differ])
        q_or, u_or = q_or.copy(), u_or.copy()
        q_or[differ], u_or[differ] = q2, u2
    q_dev = fo.unpack_nibbles(codes_dev, signed=True)
    band = _band_mask(u_or, fo.QMIN_SYM, fo.QMAX_SYM)
    neq = q_dev != q_or
    hard = neq & ~band
    if hard.any():
        r, c = np.nonzero(hard)
        msg = [f"row {rows[i] if rows is not None else i} ch {j}: dev {q_dev[i, j]} oracle {q_or[i, j]} u {u_or[i, j]:.6f}"
               for i, j in list(zip(r, c))[:8]]
        raise AssertionError(f"{hard.sum()} code mismatches outside the band: " + "; ".join(msg))
    soft = neq & band
    if soft.any():
        ok = np.abs(q_dev[soft].astype(np.float64) - u_or[soft]) <= 0.5 + BAND
        assert ok.all(), "in-band code is not a neighbour of the pre-round value"
    rep = {"rows": int(y_or.shape[0]), "step_differs": int(differ.sum()), "in_band": int(band.sum()),
           "band_flips": int(soft.sum()), "max_step_rel": float(np.max(np.abs(s_dev64 - s_or64) / np.where(s_or64 == 0, 1, s_or64), initial=0.0))}
    if deq_dev is not None:
        yhat_or = s_dev64[:, None] * q_or.astype(np.float64)
        yhat_or0 = s_or64[:, None] * q_or.astype(np.float64)
        err = np.abs(np.asarray(deq_dev, dtype=np.float64) - yhat_or0)
        err[band] = 0.0
        lim = DEQ_TOL * s_or64[:, None]
        assert np.all(err <= lim), f"dequant error {np.max(err / np.where(lim == 0, 1, lim)):.3e} x limit"
        # the helper itself must reproduce s_dev * q_dev exactly (fp32 product of fp16 x small int is exact)
        exact = s_dev64[:, None] * q_dev.astype(np.float64)
        assert np.array_equal(np.asarray(deq_dev, dtype=np.float64), exact), "dequant helper is not s*q"
        rep["max_deq_err_over_s"] = float(np.max(err / np.where(s_or64[:, None] == 0, 1, s_or64[:, None]), initial=0.0))
        del yhat_or
    return rep


def band_flip_allowance(in_band: int) -> int:
    """How many of the `in_band` elements (pre-round value within BAND of a tie) may come out as the other neighbour.
    The kernels' arithmetic error is about 1e-5 code units (fp32 accumulation, hi + lo split of the intermediate,
    reciprocal of the step), a hundredth of the band, so about one in a hundred in-band elements lies close enough to
    its tie to flip.  A tenth of them (and never fewer than 2) is the ceiling: more means the error is ten times what the
    arithmetic explains."""
    return max(2, int(in_band) // 10)


def check_kv(y_or, clip, codes_dev, scales_dev, zeros_dev, deq_dev=None, bits=4):
    """y_or fp64 [G, D] (groups flattened); codes u8 [G, D*bits/8]; scales/zeros fp16 [G]."""
    qmax = (1 << int(bits)) - 1
    y_or = np.asarray(y_or, dtype=np.float64)
    G, D = y_or.shape
    scales_dev = np.asarray(scales_dev).view(np.float16).reshape(G)
    zeros_dev = np.asarray(zeros_dev).view(np.float16).reshape(G)
    q_or, s_or, z_or, u_or, zf_or = fo.kv_quantize_asym(y_or, clip, bits)
    s_or64, s_dev64 = fo.as_f64(s_or), fo.as_f64(scales_dev)
    z_dev64 = fo.as_f64(zeros_dev)
    assert np.all(np.isfinite(s_dev64)) and np.all(np.isfinite(z_dev64))
    assert np.all(z_dev64 == np.rint(z_dev64)) and np.all((z_dev64 >= 0) & (z_dev64 <= qmax)), "zero point not an integer on the grid"
    bad = np.abs(s_dev64 - s_or64) > SCALE_RTOL * s_or64
    assert not bad.any(), f"KV step mismatch at groups {np.nonzero(bad)[0][:8]}"
    sdiff = s_dev64 != s_or64
    # pre-round zero point with the step the device emitted
    a = float(clip)
    mn = a * np.minimum(np.min(y_or, axis=-1), 0.0)
    zf = np.zeros(G)
    np.divide(-mn, s_dev64, out=zf, where=(s_dev64 != 0))
    z_exp = np.clip(np.rint(zf), 0, qmax)
    zdiff = z_dev64 != z_exp
    if zdiff.any():
        near = np.abs(zf[zdiff] - (np.floor(zf[zdiff]) + 0.5)) <= BAND
        assert near.all() and np.all(np.abs(z_dev64[zdiff] - zf[zdiff]) <= 0.5 + BAND), \
            f"zero point mismatch at groups {np.nonzero(zdiff)[0][:8]}"
    q_exp, _, _, u, _ = fo.kv_quantize_asym(y_or, clip, bits, scale_fp16=scales_dev, zero=z_dev64)
    if bits == 4:
        q_dev = fo.unpack_nibbles(codes_dev, signed=False).astype(np.uint8)
    else:
        q_dev = fo.unpack_bits(np.asarray(codes_dev).reshape(G, D * bits // 8), bits, D)
    uz = u + z_dev64[:, None]
    band = _band_mask(uz, 0, qmax)
    neq = q_dev != q_exp
    hard = neq & ~band
    if hard.any():
        r, c = np.nonzero(hard)
        msg = [f"group {i} d {j}: dev {q_dev[i, j]} oracle {q_exp[i, j]} u+z {uz[i, j]:.6f}" for i, j in list(zip(r, c))[:8]]
        raise AssertionError(f"{hard.sum()} KV code mismatches outside the band: " + "; ".join(msg))
    soft = neq & band
    if soft.any():
        assert np.all(np.abs(q_dev[soft].astype(np.float64) - uz[soft]) <= 0.5 + BAND)
    rep = {"groups": int(G), "step_differs": int(sdiff.sum()), "zero_differs": int(zdiff.sum()),
           "in_band": int(band.sum()), "band_flips": int(soft.sum())}
    if deq_dev is not None:
        exact = s_dev64[:, None] * (q_dev.astype(np.float64) - z_dev64[:, None])
        assert np.array_equal(np.asarray(deq_dev, dtype=np.float64).reshape(G, D), exact), "KV dequant helper is not s*(q-z)"
        yhat_or = s_or64[:, None] * (q_or.astype(np.float64) - z_or.astype(np.float64)[:, None])
        err = np.abs(exact - yhat_or)
        # a legitimately different (s, z) pair moves the whole grid: allow the step change and one code of shift
        err[band] = 0.0
        plain = ~(sdiff | zdiff)
        lim = DEQ_TOL * s_or64[:, None]
        assert np.all(err[plain] <= np.broadcast_to(lim, err.shape)[plain]), "KV dequant error above 1e-2 * s"
    return rep


MX_BOUNDARIES = ((0.25, 0.5), (0.75, 0.5), (1.25, 0.5), (1.75, 0.5), (2.5, 1.0), (3.5, 1.0), (5.0, 2.0))   # (tie point, grid spacing there)


def check_mx(y_or, clip, codes_dev, exps_dev):
    """MXFP4 output against the oracle.  y_or fp64 [T, n]; codes u8 [T, n/2]; exps u8 [T, n/32].
    Shared exponents: identical, except where alpha * max|block| lies within 1e-3 (relative) of a power of two.
    Codes, taken with the exponent the device emitted: identical magnitude outside 1e-3 of a grid spacing around a
    tie point; the sign bit must match wherever the magnitude is not zero."""
    y_or = np.asarray(y_or, dtype=np.float64)
    T, n = y_or.shape
    exps_dev = np.asarray(exps_dev, dtype=np.uint8).reshape(T, n // fo.MX_BLOCK)
    e_or = fo.mx_scale_exponent(y_or, clip)
    assert np.all(exps_dev <= 254), "NaN scale emitted"
    ediff = exps_dev != e_or
    if ediff.any():
        alpha = np.asarray(clip, dtype=np.float64)
        if alpha.ndim:
            alpha = alpha[..., None]
        m = alpha * np.max(np.abs(y_or.reshape(T, n // fo.MX_BLOCK, fo.MX_BLOCK)), axis=-1)
        hi = np.maximum(exps_dev, e_or).astype(np.int64)
        edge = np.ldexp(1.0, hi - 127 + 2)                   # the power of two that separates the two exponents
        ok = (np.abs(exps_dev.astype(np.int64) - e_or.astype(np.int64)) == 1) & (np.abs(m - edge) <= SCALE_RTOL * edge)
        assert np.all(ok[ediff]), f"shared exponent mismatch at blocks {np.argwhere(ediff & ~ok)[:8].tolist()}"
    q_exp, _, u = fo.mx_quantize(y_or, clip, scale_exp=exps_dev)
    q_dev = fo.unpack_nibbles(codes_dev, signed=False).astype(np.uint8)
    au = np.abs(u)
    band = np.zeros(u.shape, dtype=bool)
    for tie, spacing in MX_BOUNDARIES:
        band |= np.abs(au - tie) <= BAND * spacing
    mag_neq = (q_dev & 7) != (q_exp & 7)
    hard = mag_neq & ~band
    if hard.any():
        r, c = np.nonzero(hard)
        msg = [f"token {i} ch {j}: dev {q_dev[i, j]} oracle {q_exp[i, j]} u {u[i, j]:.6f}" for i, j in list(zip(r, c))[:8]]
        raise AssertionError(f"{hard.sum()} MXFP4 code mismatches outside the band: " + "; ".join(msg))
    soft = mag_neq & band
    if soft.any():   # a flip inside the band must still be one of the two neighbours of the tie point
        assert np.all(np.abs(fo.e2m1_value(q_dev & 7)[soft] - au[soft]) <= np.abs(fo.e2m1_value(q_exp & 7)[soft] - au[soft]) + 2 * BAND * 2.0)
    sign_neq = ((q_dev ^ q_exp) & 8) != 0
    assert not np.any(sign_neq & ((q_dev & 7) != 0)), "sign bit differs on a non-zero code"
    return {"rows": int(T), "exp_differs": int(ediff.sum()), "in_band": int(band.sum()), "band_flips": int(soft.sum()),
            "zero_sign_differs": int(sign_neq.sum())}
