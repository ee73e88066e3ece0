"""Plain fp64 CPU oracle of the FlatQuant online transform + quantization path.

TEST INFRASTRUCTURE ONLY.  This module is deliberately slow and literal: it
materialises the dense n x n matrix P = P1 (x) P2, multiplies, clips and rounds,
exactly in the order the method is stated in the paper.  It shares no code,
tables or helpers with the HIP library and must never be imported by it.

What each function follows
--------------------------
* kron_dense / affine_transform : Sec. 3.1 "Kronecker Product" -- P = P1 (x) P2
  and the product X P of Eq. (2)'s left factor, with X~ the row-major reshape
  of a token row to n1 x n2.
* quantize_sym_int4            : Sec. 2.1 (uniform quantizer s * Pi(W / s)),
  Sec. 4.1 "Quantization" (per-token symmetric for activations) and Sec. 3.1
  "Learnable Clipping Thresholds" (alpha in (0, 1], applied after the
  transform, shrinking the range that the grid covers).
* kv_quantize_asym(_int4)      : Sec. 4.1 "Quantization" and App. "KV Cache
  Quantization": group-wise asymmetric b-bit codes (b = 4 in the main results,
  b = 2 and 3 in the appendix tables on key / value bit widths), group =
  head_dim, on the unsigned grid {0 .. 2^b - 1} of Sec. 2.1.  The paper
  prints no formula for the asymmetric grid; the textbook min/max affine grid
  that contains zero is used, with the clipping threshold of Sec. 3.1
  multiplying both ends of the range.  The paper prints no value to compare
  with (PARITY UNPINNED by the paper); this reading is pinned in the CPU tests
  by hand-worked groups with and without clipping, an exact-rational scaling
  law, brute force over the levels and invariants.
* pack_bits / unpack_bits      : storage of b-bit codes (not fixed by the
  paper): code k of a group sits at bits [b k, b k + b) of the group's bytes
  read as one little-endian integer; for b = 4 this is pack_nibbles.
* kv_transform                 : Sec. 3.2 "Self-Attention": a dense per-head
  matrix P_h applied head by head (not decomposed).
* dequantize                   : Sec. 2.1, s * q (symmetric) or s * (q - z).
* inverse_transpose / weight_transform / weight_transform_quant /
  quantized_linear             : the right factor of Eq. (2),
  Q(P1^-1 x_1 W~ x_2 (P2^-1)^T), i.e. every weight row times (P1 (x) P2)^-T,
  with per-output-channel symmetric INT4 (Sec. 4.1 "Quantization") and the
  product of the two de-quantized factors that replaces X W^T (Eq. (1)).
* w4a4_gemm                    : the same product computed the way low-bit
  hardware does it (Sec. 3.2, Sec. 3.3): integer dot products of the codes,
  scaled by the activation step of the row and the weight step of the column.

* mx_* / transform_mxfp4 / mxfp4_gemm : the MXFP4 data type the paper's "Limitations"
  name as the next one to combine with the transform.  The paper defines
  nothing for it; the format is the published OCP Microscaling one: blocks of
  32 consecutive channels, one shared power-of-two scale per block stored as
  its biased exponent (E8M0, bias 127), elements in E2M1 (sign, 2 exponent
  bits, 1 mantissa bit: magnitudes 0, 0.5, 1, 1.5, 2, 3, 4, 6).  Conversion as
  that specification states it: scale = 2^(floor(log2(max|v|)) - 2), elements
  = v / scale rounded to the nearest E2M1 value (ties to the even code),
  saturating at +-6, sign kept.  The clipping threshold alpha multiplies the
  block maximum before the exponent is taken (alpha = 1 is the plain
  conversion).  PARITY UNPINNED by the paper; pinned by the format's value
  table and hand-worked cases in the CPU tests.

Conventions fixed where the paper is silent (all listed in the design notes):
row-major reshape (channel c = i * n2 + j); signed grid [-8, 7] with step
alpha * max|y| / 7; the step is rounded once to fp16 (round-to-nearest-even,
directly from fp64) and the *rounded* step divides; round-half-to-even; two
codes per byte, even channel in the low nibble, two's complement nibbles.
"""
from __future__ import annotations

import numpy as np

QMAX_SYM = 7          # largest positive symmetric INT4 code
QMIN_SYM = -8
QMAX_ASYM = 15        # unsigned INT4 grid of the KV-cache variant


def as_f64(a) -> np.ndarray:
    """fp16 (or any float) array -> fp64; exact for fp16/fp32 inputs."""
    return np.asarray(a).astype(np.float64)


def round_to_fp16(v) -> np.ndarray:
    """One correctly rounded fp64 -> fp16 conversion (no fp32 stop-over)."""
    return np.asarray(v, dtype=np.float64).astype(np.float16)


# --------------------------------------------------------------------------
# Sec. 3.1, Kronecker product and Eq. (2)
# --------------------------------------------------------------------------
def kron_dense(P1, P2) -> np.ndarray:
    """P = P1 (x) P2 as a dense fp64 matrix.

    Block convention: P[i*n2 + j, i'*n2 + j'] = P1[i, i'] * P2[j, j'].
    """
    P1 = as_f64(P1)
    P2 = as_f64(P2)
    n1, n2 = P1.shape[0], P2.shape[0]
    assert P1.shape == (n1, n1) and P2.shape == (n2, n2)
    return np.kron(P1, P2)


def affine_transform(x, P1, P2, P=None) -> np.ndarray:
    """y = x P for every token row of x ([T, n]), fp64.  `P` may be a
    pre-built kron_dense(P1, P2) to avoid rebuilding it."""
    x = as_f64(x)
    if P is None:
        P = kron_dense(P1, P2)
    assert x.ndim == 2 and x.shape[1] == P.shape[0]
    return x @ P


def affine_transform_factored(x, P1, P2) -> np.ndarray:
    """The same product in the factored form of Eq. (2), as printed: for every token, P1^T X~ P2 with X~ the
    row-major n1 x n2 reshape (two small contractions instead of one n x n product)."""
    x = as_f64(x)
    P1, P2 = as_f64(P1), as_f64(P2)
    n1, n2 = P1.shape[0], P2.shape[0]
    Xt = x.reshape(x.shape[0], n1, n2)
    return np.matmul(P1.T, np.matmul(Xt, P2)).reshape(x.shape[0], n1 * n2)


# --------------------------------------------------------------------------
# Sec. 2.1 / 3.1 / 4.1: per-token symmetric INT4 with a clipping ratio
# --------------------------------------------------------------------------
def sym_scale(y, clip) -> np.ndarray:
    """Per-row step s = fp16(alpha * max|y| / 7).  `clip` is a scalar or [T]."""
    y = as_f64(y)
    alpha = np.broadcast_to(as_f64(clip), (y.shape[0],))
    m = np.max(np.abs(y), axis=1) if y.shape[1] else np.zeros(y.shape[0])
    return round_to_fp16(alpha * m / QMAX_SYM)


def preround_sym(y, scale_fp16) -> np.ndarray:
    """u = y / s with the emitted (fp16) step; rows with s == 0 give u = 0."""
    y = as_f64(y)
    s = as_f64(scale_fp16).reshape(-1, 1)
    u = np.zeros_like(y)
    np.divide(y, s, out=u, where=(s != 0))
    return u


def round_clamp_sym(u) -> np.ndarray:
    """q = clamp(round_half_even(u), -8, 7) as int8."""
    return np.clip(np.rint(u), QMIN_SYM, QMAX_SYM).astype(np.int8)


def quantize_sym_int4(y, clip, scale_fp16=None):
    """Returns (q int8 [T, n], s fp16 [T], u fp64 [T, n]).

    If `scale_fp16` is given it replaces the step this function would compute
    (used by the comparator when two adjacent fp16 steps are both legitimate).
    """
    s = sym_scale(y, clip) if scale_fp16 is None else np.asarray(scale_fp16, dtype=np.float16)
    u = preround_sym(y, s)
    return round_clamp_sym(u), s, u


def pack_nibbles(q) -> np.ndarray:
    """Two 4-bit codes per byte: channel 2k -> low nibble, 2k+1 -> high nibble.
    Works for signed (two's complement) and unsigned codes alike."""
    q = np.asarray(q)
    assert q.shape[-1] % 2 == 0
    b = (q.astype(np.int16) & 0xF).astype(np.uint8)
    return (b[..., 0::2] | (b[..., 1::2] << 4)).astype(np.uint8)


def unpack_nibbles(packed, signed: bool) -> np.ndarray:
    packed = np.asarray(packed, dtype=np.uint8)
    lo = (packed & 0xF).astype(np.int8)
    hi = (packed >> 4).astype(np.int8)
    out = np.empty(packed.shape[:-1] + (packed.shape[-1] * 2,), dtype=np.int8)
    out[..., 0::2] = lo
    out[..., 1::2] = hi
    if signed:
        out = np.where(out >= 8, out - 16, out).astype(np.int8)
    return out


def transform_quant(x, P1, P2, clip, P=None):
    """The whole online path for activations: Q(x (P1 (x) P2)).

    Returns a dict with the packed codes (u8 [T, n/2]), the fp16 steps [T],
    and the fp64 intermediates the comparator needs: y (transformed), u
    (pre-round values), q (codes before packing).
    """
    y = affine_transform(x, P1, P2, P=P)
    q, s, u = quantize_sym_int4(y, clip)
    return {"codes": pack_nibbles(q), "scales": s, "q": q, "u": u, "y": y}


# --------------------------------------------------------------------------
# KV-cache variant (Sec. 3.2 per-head transform; Sec. 4.1 asymmetric groups)
# --------------------------------------------------------------------------
def kv_transform(kv, P) -> np.ndarray:
    """kv [T, H, D] times P [Hp, D, D] (Hp == 1: shared; Hp == H: per head)."""
    kv = as_f64(kv)
    P = as_f64(P)
    T, H, D = kv.shape
    assert P.shape[1:] == (D, D) and P.shape[0] in (1, H)
    y = np.empty_like(kv)
    for h in range(H):
        y[:, h, :] = kv[:, h, :] @ P[h if P.shape[0] == H else 0]
    return y


def head_transform_fp16(x, P) -> np.ndarray:
    """Transform only, kept in FP16 (Sec. 3.2: queries are not quantized):
    fp16(x[t, h, :] P_h), one rounding of the fp64 product."""
    return round_to_fp16(kv_transform(x, P))


def kv_scale_zero(y, clip, bits=4):
    """Per group (last axis): mx = max(y, 0), mn = min(y, 0) scaled by alpha;
    step s = fp16((mx - mn) / (2^b - 1)); zero point z = round(-mn / s) in
    [0, 2^b - 1].  Returns (s fp16, z int8, zf fp64 = pre-round zero point)."""
    y = as_f64(y)
    a = float(clip)
    qmax = (1 << int(bits)) - 1
    mx = a * np.maximum(np.max(y, axis=-1), 0.0)
    mn = a * np.minimum(np.min(y, axis=-1), 0.0)
    s = round_to_fp16((mx - mn) / qmax)
    s64 = as_f64(s)
    zf = np.zeros_like(s64)
    np.divide(-mn, s64, out=zf, where=(s64 != 0))
    z = np.clip(np.rint(zf), 0, qmax).astype(np.int8)
    return s, z, zf


def kv_preround(y, scale_fp16) -> np.ndarray:
    y = as_f64(y)
    s = as_f64(scale_fp16)[..., None]
    u = np.zeros_like(y)
    np.divide(y, s, out=u, where=(s != 0))
    return u


def kv_quantize_asym(y, clip, bits=4, scale_fp16=None, zero=None):
    """Returns (q uint8 in [0, 2^b - 1], s fp16, z int8, u fp64, zf fp64)."""
    qmax = (1 << int(bits)) - 1
    s0, z0, zf = kv_scale_zero(y, clip, bits)
    s = s0 if scale_fp16 is None else np.asarray(scale_fp16, dtype=np.float16)
    z = z0 if zero is None else np.asarray(zero).astype(np.int8)
    u = kv_preround(y, s)
    q = np.clip(np.rint(u) + z[..., None], 0, qmax).astype(np.uint8)
    return q, s, z, u, zf


def kv_quantize_asym_int4(y, clip, scale_fp16=None, zero=None):
    return kv_quantize_asym(y, clip, 4, scale_fp16, zero)


def pack_bits(q, bits) -> np.ndarray:
    """q [..., n] unsigned codes below 2^bits, n * bits a multiple of 8 ->
    u8 [..., n * bits / 8]: code k at bits [bits k, bits k + bits) of the row
    read as one little-endian integer."""
    q = np.asarray(q)
    bits = int(bits)
    n = q.shape[-1]
    assert (n * bits) % 8 == 0
    assert np.all((q >= 0) & (q < (1 << bits)))
    flat = q.reshape(-1, n)
    out = np.zeros((flat.shape[0], n * bits // 8), dtype=np.uint8)
    for r in range(flat.shape[0]):
        big = 0
        for k in range(n):
            big |= int(flat[r, k]) << (bits * k)
        out[r] = np.frombuffer(big.to_bytes(n * bits // 8, "little"), dtype=np.uint8)
    return out.reshape(q.shape[:-1] + (n * bits // 8,))


def unpack_bits(packed, bits, n) -> np.ndarray:
    """Inverse of pack_bits: u8 [..., n * bits / 8] -> uint8 [..., n]."""
    packed = np.asarray(packed, dtype=np.uint8)
    bits = int(bits)
    nb = n * bits // 8
    assert packed.shape[-1] == nb
    flat = packed.reshape(-1, nb)
    out = np.zeros((flat.shape[0], n), dtype=np.uint8)
    for r in range(flat.shape[0]):
        big = int.from_bytes(flat[r].tobytes(), "little")
        for k in range(n):
            out[r, k] = (big >> (bits * k)) & ((1 << bits) - 1)
    return out.reshape(packed.shape[:-1] + (n,))


def kv_transform_quant(kv, P, clip, bits=4):
    y = kv_transform(kv, P)
    q, s, z, u, zf = kv_quantize_asym(y, clip, bits)
    return {"codes": pack_bits(q, bits), "scales": s, "zeros": z, "q": q, "u": u, "y": y, "zf": zf}


# --------------------------------------------------------------------------
# MXFP4 output (named in the paper's "Limitations"; format: OCP Microscaling)
# --------------------------------------------------------------------------
MX_BLOCK = 32
E2M1_VALUES = (0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0)   # magnitude of codes 0..7; bit 3 is the sign


def e2m1_round(u) -> np.ndarray:
    """fp64 -> E2M1 code (uint8, sign-magnitude): nearest of the 8 magnitudes,
    a tie goes to the even code, anything beyond 6 saturates, the sign bit is
    the sign of the input (a negative value that rounds to zero is -0)."""
    u = as_f64(u)
    a = np.minimum(np.abs(u), max(E2M1_VALUES))          # saturating: beyond the largest magnitude is the largest magnitude
    grid = np.asarray(E2M1_VALUES)                       # (left unclamped, a value above 2^53 is equally far from all 8 in fp64)
    d = np.abs(a[..., None] - grid)                      # distance to each magnitude
    best = d.min(axis=-1, keepdims=True)
    cand = d == best                                     # one or (on a tie) two neighbours
    even = cand & (np.arange(8) % 2 == 0)
    pick = np.where(cand.sum(axis=-1, keepdims=True) > 1, even, cand)
    mag = np.argmax(pick, axis=-1).astype(np.uint8)
    return (mag | (np.signbit(u).astype(np.uint8) << 3)).astype(np.uint8)


def e2m1_value(code) -> np.ndarray:
    code = np.asarray(code, dtype=np.uint8)
    v = np.asarray(E2M1_VALUES)[code & 7]
    return np.where(code & 8, -v, v)


def mx_scale_exponent(y, clip) -> np.ndarray:
    """y [..., n], n a multiple of 32 -> biased exponents uint8 [..., n/32]:
    floor(log2(alpha * max|block|)) - 2 + 127, kept inside [0, 254]; an
    all-zero block gets exponent 0."""
    y = as_f64(y)
    blocks = y.reshape(y.shape[:-1] + (y.shape[-1] // MX_BLOCK, MX_BLOCK))
    alpha = np.asarray(clip, dtype=np.float64)
    if alpha.ndim:                                       # one threshold per token
        alpha = alpha[..., None]
    m = alpha * np.max(np.abs(blocks), axis=-1)
    e = np.zeros(m.shape, dtype=np.int64)
    nz = m > 0
    _, ex = np.frexp(m[nz])                              # m = f * 2^ex, f in [0.5, 1): floor(log2 m) = ex - 1
    e[nz] = (ex - 1) - 2 + 127
    return np.clip(e, 0, 254).astype(np.uint8)


def mx_quantize(y, clip, scale_exp=None):
    """Returns (codes uint8 [..., n] E2M1, exponents uint8 [..., n/32],
    u fp64 = y / 2^(e - 127))."""
    y = as_f64(y)
    e = mx_scale_exponent(y, clip) if scale_exp is None else np.asarray(scale_exp, dtype=np.uint8)
    x = np.ldexp(1.0, e.astype(np.int64) - 127)          # exact powers of two
    u = y / np.repeat(x, MX_BLOCK, axis=-1)
    return e2m1_round(u), e, u


def transform_mxfp4(x, P1, P2, clip, P=None):
    """Transform (Eq. (2), left factor), then MXFP4 per block of 32 channels.
    codes are packed two per byte, even channel in the low nibble."""
    y = affine_transform(x, P1, P2, P)
    q, e, u = mx_quantize(y, clip)
    return {"codes": pack_nibbles(q.astype(np.int8)), "scales": e, "q": q, "u": u, "y": y}


def dequantize_mxfp4(codes_packed, scale_exp) -> np.ndarray:
    q = unpack_nibbles(codes_packed, signed=False)
    x = np.ldexp(1.0, np.asarray(scale_exp).astype(np.int64) - 127)
    return e2m1_value(q) * np.repeat(x, MX_BLOCK, axis=-1)


def mx_tile_scales(e, fill=0) -> np.ndarray:
    """Row-major exponents [R, n/32] -> the tile order the MXFP4 product reads, as a flat byte array: rows in tiles of
    128 (padded with `fill`), blocks in groups of 8; byte of (row r, block k) = (((r // 128) * (n // 256) + k // 8) *
    128 + r % 128) * 8 + k % 8."""
    e = np.asarray(e, dtype=np.uint8)
    R, nb = e.shape
    assert nb % 8 == 0
    tiles, groups = (R + 127) // 128, nb // 8
    out = np.full((tiles, groups, 128, 8), fill, dtype=np.uint8)
    for r in range(R):
        for k in range(nb):
            out[r // 128, k // 8, r % 128, k % 8] = e[r, k]
    return out.reshape(-1)


def mx_untile_scales(tiled, rows, n) -> np.ndarray:
    """Inverse of mx_tile_scales (the padding rows are dropped)."""
    nb = n // 32
    t = np.asarray(tiled, dtype=np.uint8).reshape((rows + 127) // 128, nb // 8, 128, 8)
    out = np.zeros((rows, nb), dtype=np.uint8)
    for r in range(rows):
        for k in range(nb):
            out[r, k] = t[r // 128, k // 8, r % 128, k % 8]
    return out


def mxfp4_gemm(x_codes, x_exps, w_codes, w_exps):
    """Product of two MXFP4 factors, the low-bit matrix multiplication of
    Sec. 3.2 with the data type of the "Limitations": out[t, o] = sum_k x^[t, k]
    w^[o, k] with x^, w^ the de-quantized factors (element times the block's
    power of two).  Returns (y fp64, y rounded once to fp16, sum_k |x^ w^|,
    which bounds what any summation order can lose)."""
    xd = dequantize_mxfp4(x_codes, x_exps)
    wd = dequantize_mxfp4(w_codes, w_exps)
    y = xd @ wd.T
    return y, round_to_fp16(y), np.abs(xd) @ np.abs(wd).T


# --------------------------------------------------------------------------
# Sec. 2.1: de-quantization
# --------------------------------------------------------------------------
def dequantize(codes_packed, scales_fp16, zeros=None, bits=4) -> np.ndarray:
    """s * q (zeros is None: signed nibbles) or s * (q - z) (unsigned b-bit
    codes).  codes [..., n b / 8] u8, scales [...] fp16, zeros [...] -> fp64
    [..., n]."""
    if bits == 4:
        q = unpack_nibbles(codes_packed, signed=zeros is None).astype(np.float64)
    else:
        assert zeros is not None, "only the asymmetric grid has other widths"
        packed = np.asarray(codes_packed)
        q = unpack_bits(packed, bits, packed.shape[-1] * 8 // bits).astype(np.float64)
    s = as_f64(scales_fp16)[..., None]
    if zeros is not None:
        q = q - as_f64(zeros)[..., None]
    return s * q


# --------------------------------------------------------------------------
# Closed forms of the paper's cost analysis (App. "Overhead Analysis")
# --------------------------------------------------------------------------
# --------------------------------------------------------------------------
# Right factor of Eq. (2): the offline weight side
# --------------------------------------------------------------------------
def inverse_transpose(P) -> np.ndarray:
    """(P^-1)^T in fp64 (library LU inverse as the one step)."""
    return np.linalg.inv(as_f64(P)).T


def weight_transform(W, P1, P2) -> np.ndarray:
    """W [m, n] -> (P^-1 W^T)^T = W (P1 (x) P2)^-T, the weights that pair with
    X P in Eq. (1): the inverse of the dense Kronecker matrix is taken as it
    stands (no use of the factor structure)."""
    P = kron_dense(P1, P2)
    return as_f64(W) @ np.linalg.inv(P).T


def weight_transform_factored(W, A1, A2) -> np.ndarray:
    """Eq. (2), right factor, as printed: for every output channel o,
    A1^T W~_o A2 with A1^T = P1^-1 and A2 = (P2^-1)^T, W~_o the row-major
    n1 x n2 reshape of row o.  A1, A2 are passed in (e.g. fp16-rounded)."""
    W = as_f64(W)
    A1, A2 = as_f64(A1), as_f64(A2)
    n1, n2 = A1.shape[0], A2.shape[0]
    Wt = W.reshape(W.shape[0], n1, n2)
    return np.einsum("ia,oij,jb->oab", A1, Wt, A2).reshape(W.shape[0], n1 * n2)


def weight_transform_quant(W, A1, A2, clip_w):
    """Per-output-channel symmetric INT4 of the transformed weights, with the
    weight clipping ratio alpha_w (scalar or one per output channel)."""
    y = weight_transform_factored(W, A1, A2)
    q, s, u = quantize_sym_int4(y, clip_w)
    return {"codes": pack_nibbles(q), "scales": s, "q": q, "u": u, "y": y}


def quantized_linear(codes_x, scales_x, codes_w, scales_w) -> np.ndarray:
    """deq(Q(XP)) deq(Q(P^-1 W^T)): [T, n/2] x [m, n/2] packed codes -> [T, m] fp64."""
    return dequantize(codes_x, scales_x) @ dequantize(codes_w, scales_w).T


def w4a4_gemm(codes_x, scales_x, codes_w, scales_w):
    """The low-bit matrix multiplication that consumes the two quantized factors of Eq. (2) (Sec. 3.2: "low-bit
    matrix multiplications for all linear layers"): exact integer dot products of the 4-bit codes, then the two
    steps.  Returns (acc int64 [T, m], y fp64 [T, m], y rounded once to fp16)."""
    qx = unpack_nibbles(codes_x, signed=True).astype(np.int64)
    qw = unpack_nibbles(codes_w, signed=True).astype(np.int64)
    acc = qx @ qw.T
    y = acc.astype(np.float64) * as_f64(scales_x).reshape(-1, 1) * as_f64(scales_w).reshape(1, -1)
    return acc, y, round_to_fp16(y)


def choose_factors(n: int):
    """argmin (n1 + n2) s.t. n1 * n2 = n, n1 <= n2  (Sec. 3.1)."""
    best = None
    for n1 in range(1, int(np.sqrt(n)) + 1):
        if n % n1 == 0:
            best = (n1, n // n1)
    return best


def flops_per_token(n1: int, n2: int) -> int:
    """Multiply-adds counted as 2 flops: X~ P2 then P1^T (.)."""
    return 2 * n1 * n2 * n2 + 2 * n1 * n1 * n2


def extra_param_bytes_per_block(h_d: int, h_i: int, a: int) -> int:
    """fp16 bytes of the online transforms of one Transformer block with
    perfect-square factorizations (App. "Memory Consumption")."""
    return 2 * (4 * h_d + 2 * h_i + a * a + (h_d // a) ** 2)
