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
