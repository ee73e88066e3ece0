"""Pins of the CPU oracle to facts that do not come from the oracle itself:
brute force, exact rational arithmetic, closed forms the paper prints, a
textbook transform, hand-worked cases and invariants of the method."""
import itertools
import os
import struct
from fractions import Fraction

import numpy as np
import pytest

from oracle import flatquant_oracle as fo
from oracle import parity
from paper_2410_09426_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def read_golden(name):
    out = {}
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if "=" in line:
                k, v = line.split("=", 1)
                out[k.strip()] = v.strip()
    return out


def rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def rand_fp16(r, shape, scale=1.0):
    return (r.standard_normal(shape) * scale).astype(np.float16)


# ---- exact helpers, independent of the oracle --------------------------------
def frac(v):
    return Fraction(float(v))


def exact_fp16_nearest(v: Fraction) -> float:
    """Nearest fp16 to an exact rational, ties to even, by exhaustive neighbour test."""
    if v == 0:
        return 0.0
    h = struct.unpack("<H", struct.pack("<e", float(v)))[0]
    best = None
    for cand in (h - 1, h, h + 1):
        if cand < 0 or (cand & 0x7FFF) >= 0x7C00:
            continue
        val = struct.unpack("<e", struct.pack("<H", cand))[0]
        d = abs(Fraction(val) - v)
        key = (d, cand & 1)
        if best is None or key < best[0]:
            best = (key, val)
    return best[1]


def exact_round_half_even(v: Fraction) -> int:
    fl = v.numerator // v.denominator
    r = v - fl
    if r > Fraction(1, 2):
        return fl + 1
    if r < Fraction(1, 2):
        return fl
    return fl if fl % 2 == 0 else fl + 1


def exact_sym_quant(row, alpha):
    """Per-token symmetric INT4 in exact rational arithmetic (Sec. 2.1 / 4.1)."""
    vals = [frac(v) for v in row]
    m = max(abs(v) for v in vals)
    s = exact_fp16_nearest(frac(alpha) * m / 7)
    if s == 0:
        return [0] * len(vals), 0.0
    return [max(-8, min(7, exact_round_half_even(v / Fraction(s)))) for v in vals], s


# ---- Sec. 3.1: Kronecker / vec identity ---------------------------------------
@pytest.mark.parametrize("n1,n2", [(1, 1), (1, 4), (4, 1), (3, 5), (5, 3), (4, 4), (2, 6), (16, 16)])
def test_kron_identity_bruteforce(n1, n2):
    r = rng(100 + 17 * n1 + n2)
    T = 3
    x = rand_fp16(r, (T, n1 * n2), 3.0)
    P1 = rand_fp16(r, (n1, n1))
    P2 = rand_fp16(r, (n2, n2))
    y = fo.affine_transform(x, P1, P2)
    # (a) four nested loops over the index definition, exact rationals
    for t in range(T):
        for ip, jp in itertools.product(range(n1), range(n2)):
            acc = Fraction(0)
            for i, j in itertools.product(range(n1), range(n2)):
                acc += frac(x[t, i * n2 + j]) * frac(P1[i, ip]) * frac(P2[j, jp])
            assert abs(float(acc) - y[t, ip * n2 + jp]) <= 1e-12 * max(1.0, abs(float(acc)))
    # (b) the factored form P1^T X~ P2 with a row-major reshape
    X = x.astype(np.float64).reshape(T, n1, n2)
    yf = np.einsum("ia,tij,jb->tab", P1.astype(np.float64), X, P2.astype(np.float64)).reshape(T, -1)
    np.testing.assert_allclose(y, yf, rtol=1e-12, atol=1e-12)


def test_factored_form_of_eq2_equals_the_dense_product():
    """vec(V)(P1 (x) P2) = vec(P1^T V P2) (the vectorisation identity the paper recalls in Sec. 3.1): the oracle's
    factored route and its dense route are two different computations of the same numbers."""
    r = rng(77)
    for n1, n2 in [(1, 6), (5, 3), (16, 16), (8, 32)]:
        x = rand_fp16(r, (9, n1 * n2), 3.0)
        P1, P2 = rand_fp16(r, (n1, n1)), rand_fp16(r, (n2, n2))
        assert np.allclose(fo.affine_transform_factored(x, P1, P2), fo.affine_transform(x, P1, P2), rtol=1e-12, atol=1e-12)


def test_kron_hand_worked_and_transpose_matters():
    g = read_golden("hand_worked.txt")
    P1 = np.array([[1, 2], [3, 4]], dtype=np.float16)
    P2 = np.array([[0, 1], [1, 0]], dtype=np.float16)
    x = np.array([[1, 10, 100, 1000]], dtype=np.float16)
    y = fo.affine_transform(x, P1, P2)
    assert y[0].tolist() == [float(v) for v in g["kron_2x2.y"].split()]
    # a transposed P1 or a column-major reshape gives something else on this input
    assert not np.array_equal(fo.affine_transform(x, P1.T, P2), y)
    assert not np.array_equal(fo.affine_transform(x[:, [0, 2, 1, 3]], P1, P2), y)


def test_unit_vector_closed_form():
    r = rng(7)
    n1, n2 = 5, 6
    P1, P2 = rand_fp16(r, (n1, n1)), rand_fp16(r, (n2, n2))
    for i, j in [(0, 0), (2, 3), (4, 5), (1, 0)]:
        x = np.zeros((1, n1 * n2), dtype=np.float16)
        x[0, i * n2 + j] = 1
        y = fo.affine_transform(x, P1, P2).reshape(n1, n2)
        np.testing.assert_array_equal(y, np.outer(P1[i].astype(np.float64), P2[j].astype(np.float64)))


def test_permutation_matrices_bit_exact():
    r = rng(11)
    n1, n2, T = 6, 8, 5
    p1, p2 = r.permutation(n1), r.permutation(n2)
    P1 = np.eye(n1, dtype=np.float16)[:, p1]      # P1[i, i'] = 1 iff i == p1[i']
    P2 = np.eye(n2, dtype=np.float16)[:, p2]
    x = rand_fp16(r, (T, n1 * n2), 4.0)
    res = fo.transform_quant(x, P1, P2, 1.0)
    xp = x.reshape(T, n1, n2)[:, p1][:, :, p2].reshape(T, -1)   # y[i', j'] = x[p1[i'], p2[j']]
    for t in range(T):
        q, s = exact_sym_quant(xp[t], 1.0)
        assert res["q"][t].tolist() == q
        assert float(res["scales"][t]) == s


def fwht(v):
    """Textbook in-place fast Walsh-Hadamard transform (Sylvester order), unnormalised."""
    v = list(v)
    h = 1
    while h < len(v):
        for i in range(0, len(v), 2 * h):
            for k in range(i, i + h):
                a, b = v[k], v[k + h]
                v[k], v[k + h] = a + b, a - b
        h *= 2
    return v


def sylvester(n):
    H = np.array([[1.0]])
    while H.shape[0] < n:
        H = np.block([[H, H], [H, -H]])
    return H


@pytest.mark.parametrize("n1,n2", [(4, 4), (16, 16), (4, 16)])
def test_hadamard_reduces_to_fwht(n1, n2):
    # Sec. 2.2: a Hadamard rotation is one member of the affine family; H_{n1} (x) H_{n2} = H_{n}
    r = rng(13)
    n = n1 * n2
    P1 = (sylvester(n1) / np.sqrt(n1)).astype(np.float16)   # +-2^-k: exact in fp16
    P2 = (sylvester(n2) / np.sqrt(n2)).astype(np.float16)
    x = rand_fp16(r, (4, n), 2.0)
    y = fo.affine_transform(x, P1, P2)
    for t in range(4):
        ref = np.array(fwht(x[t].astype(np.float64))) / np.sqrt(n)
        np.testing.assert_allclose(y[t], ref, rtol=0, atol=1e-12)


# ---- Sec. 2.1 / 4.1: quantizer ---------------------------------------------------
def test_fp16_rounding_is_single_and_to_even():
    v = 1.0 + 2.0 ** -11 + 2.0 ** -30          # just above a midpoint; via fp32 it would tie to 1.0
    assert fo.round_to_fp16(v).view(np.uint16) == 0x3C01
    assert fo.round_to_fp16(1.0 + 2.0 ** -11).view(np.uint16) == 0x3C00      # exact tie -> even
    assert fo.round_to_fp16(1.0 + 3 * 2.0 ** -11).view(np.uint16) == 0x3C02  # exact tie -> even
    r = rng(5)
    for v in r.uniform(1e-6, 6e4, 300):
        assert float(fo.round_to_fp16(v)) == exact_fp16_nearest(Fraction(v))


def test_hand_worked_symmetric():
    g = read_golden("hand_worked.txt")
    x = np.array([[float(v) for v in g["sym_identity.x"].split()]], dtype=np.float16)
    P1, P2 = np.eye(2, dtype=np.float16), np.eye(4, dtype=np.float16)
    for case, clip in (("sym_identity", 1.0), ("sym_clip_half", 0.5)):
        res = fo.transform_quant(x, P1, P2, clip)
        assert res["q"][0].tolist() == [int(v) for v in g[case + ".codes"].split()]
        assert bytes(res["codes"][0]).hex().upper() == g[case + ".bytes"].replace(" ", "")
        assert float(res["scales"][0]) == float(g[case + ".scale"])


@pytest.mark.parametrize("alpha", [1.0, 0.9, 0.61])
def test_identity_transform_is_plain_per_token_quant(alpha):
    r = rng(21)
    n1, n2, T = 4, 8, 12
    x = rand_fp16(r, (T, n1 * n2), 5.0)
    x[3] = 0                      # all-zero row
    x[4, 7] = 900                 # outlier row
    res = fo.transform_quant(x, np.eye(n1, dtype=np.float16), np.eye(n2, dtype=np.float16), alpha)
    for t in range(T):
        q, s = exact_sym_quant(x[t], alpha)
        assert res["q"][t].tolist() == q, t
        assert float(res["scales"][t]) == s
    assert not res["codes"][3].any() and float(res["scales"][3]) == 0.0


def test_ranges_and_error_bound():
    c = synth.tiny()
    for clip in (1.0, 0.8):
        res = fo.transform_quant(c.x, c.P1, c.P2, clip)
        q, s, y = res["q"], res["scales"].astype(np.float64), res["y"]
        assert q.min() >= -8 and q.max() <= 7
        if clip == 1.0:
            # s was rounded to fp16, so |u| may exceed 7 by the rounding error of s only
            assert np.all(np.max(np.abs(q), axis=1) == 7) and q.min() >= -7
        yc = np.clip(y, -8 * s[:, None], 7 * s[:, None])
        assert np.all(np.abs(fo.dequantize(res["codes"], res["scales"]) - yc) <= s[:, None] / 2 * (1 + 1e-12))


def test_pack_unpack_roundtrip_and_order():
    q = np.arange(-8, 8, dtype=np.int8).reshape(1, 16)
    p = fo.pack_nibbles(q)
    assert p[0, 0] == ((-8 & 15) | ((-7 & 15) << 4))
    np.testing.assert_array_equal(fo.unpack_nibbles(p, signed=True), q)
    qu = np.arange(16, dtype=np.uint8).reshape(1, 16)
    np.testing.assert_array_equal(fo.unpack_nibbles(fo.pack_nibbles(qu), signed=False), qu.astype(np.int8))


def test_equivariances():
    c = synth.generic(3, 9, 4, 8, sigma=0.2, clip_mode=0)
    base = fo.transform_quant(c.x, c.P1, c.P2, 1.0)
    # power-of-two input scaling: same codes, step scaled exactly
    up = fo.transform_quant((c.x.astype(np.float32) / 4).astype(np.float16), c.P1, c.P2, 1.0)
    np.testing.assert_array_equal(up["codes"], base["codes"])
    np.testing.assert_array_equal(up["scales"].astype(np.float64) * 4, base["scales"].astype(np.float64))
    # sign flip with alpha = 1: codes negate
    neg = fo.transform_quant(-c.x, c.P1, c.P2, 1.0)
    np.testing.assert_array_equal(neg["q"], -base["q"])
    # token permutation and row independence
    perm = rng(1).permutation(c.T)
    pr = fo.transform_quant(c.x[perm], c.P1, c.P2, 1.0)
    np.testing.assert_array_equal(pr["codes"], base["codes"][perm])
    one = fo.transform_quant(c.x[5:6], c.P1, c.P2, 1.0)
    np.testing.assert_array_equal(one["codes"][0], base["codes"][5])


def test_invertibility_recovers_input_within_quantization_bound():
    # Eq. (1)/(2): Q(X P) P^-1 ~ X; the residual is the rounding error pushed through P^-1
    c = synth.generic(4, 6, 8, 8, sigma=0.1, clip_mode=0, outlier_frac=0.05)
    res = fo.transform_quant(c.x, c.P1, c.P2, 1.0)
    P = fo.kron_dense(c.P1, c.P2)
    Pinv = np.linalg.inv(P)
    s = res["scales"].astype(np.float64)
    # rows whose |u| stays <= 7.5 are unclipped, so |yhat - y| <= s/2 elementwise
    assert np.all(np.abs(res["u"]) <= 7.5)
    xr = fo.dequantize(res["codes"], res["scales"]) @ Pinv
    bound = (s / 2)[:, None] * np.sum(np.abs(Pinv), axis=0)[None, :]
    assert np.all(np.abs(xr - c.x.astype(np.float64)) <= bound * (1 + 1e-9) + 1e-12)
    # and the Kronecker structure of the inverse: (P1 (x) P2)^-1 = P1^-1 (x) P2^-1
    np.testing.assert_allclose(Pinv, np.kron(np.linalg.inv(c.P1.astype(np.float64)), np.linalg.inv(c.P2.astype(np.float64))), rtol=1e-9, atol=1e-12)


# ---- closed forms of Sec. 3.1 and App. "Overhead Analysis" ------------------------
def test_closed_forms_from_the_paper():
    g = read_golden("closed_forms.txt")
    assert list(fo.choose_factors(8192)) == [int(v) for v in g["factors_8192"].split()]
    assert fo.choose_factors(4096) == (64, 64)
    total = 32 * fo.extra_param_bytes_per_block(4096, 11008, 32)
    assert total == int(g["extra_memory_7b_bytes"])
    assert round(total / 2 ** 20, 2) == float(g["extra_memory_7b_mib"])
    assert fo.flops_per_token(64, 64) == int(g["flops_per_token_sq_4096"])
    n = 4096
    assert n * n // (64 * 64 + 64 * 64) == int(g["memory_saving_sq_4096"])
    assert 2 * n * n // fo.flops_per_token(64, 64) == int(g["compute_saving_sq_4096"])
    for n1, n2 in [(64, 128), (86, 128), (112, 256)]:
        assert fo.flops_per_token(n1, n2) == 2 * n1 * n2 * (n1 + n2)


# ---- KV-cache variant ----------------------------------------------------------------
def test_kv_hand_worked():
    g = read_golden("hand_worked.txt")
    y = np.array([[[float(v) for v in g["kv_asym.y"].split()]]], dtype=np.float16)   # [T=1, H=1, D=4]
    res = fo.kv_transform_quant(y, np.eye(4, dtype=np.float16)[None], 1.0)
    assert res["q"][0, 0].tolist() == [int(v) for v in g["kv_asym.codes"].split()]
    assert float(res["scales"][0, 0]) == float(g["kv_asym.scale"]) and int(res["zeros"][0, 0]) == int(g["kv_asym.zero"])


@pytest.mark.parametrize("case", ["kv_clip_half", "kv_clip_half_3bit", "kv_clip_095", "kv_clip_075"])
def test_kv_hand_worked_with_clipping(case):
    """Sec. 3.1 "Learnable Clipping Thresholds" on the group-wise asymmetric grid of Sec. 4.1: the threshold scales both
    ends of the range.  Values derived on paper (tests/golden/hand_worked.txt), none of them by the oracle."""
    g = read_golden("hand_worked.txt")
    yv = [float(v) for v in g[case + ".y"].split()]
    clip, bits = float(g[case + ".clip"]), int(g[case + ".bits"])
    D = 8                                                    # pad the group with zeros: b-bit rows need D * b % 8 == 0
    y = np.zeros((1, 1, D), dtype=np.float16)
    y[0, 0, :len(yv)] = yv
    res = fo.kv_transform_quant(y, np.eye(D, dtype=np.float16)[None], clip, bits)
    want = [int(v) for v in g[case + ".codes"].split()]
    assert res["q"][0, 0, :len(yv)].tolist() == want
    assert float(res["scales"][0, 0]) == float(g[case + ".scale"])
    assert int(res["zeros"][0, 0]) == int(g[case + ".zero"])
    # zero inputs sit on the zero point, and the packed row holds the same codes
    assert np.all(res["q"][0, 0, len(yv):] == int(g[case + ".zero"]))
    assert fo.unpack_bits(res["codes"], bits, D)[0, 0, :len(yv)].tolist() == want


def test_kv_clip_scales_both_ends_exactly():
    """With a power-of-two threshold and power-of-two-friendly data the clipped grid is the unclipped grid of the
    scaled range: step(alpha) = alpha * step(1), same zero point; codes = clamp(rne(y / (alpha s)) + z)."""
    y = np.array([[[-3.0, 0.0, 4.5, 12.0, 1.0, -1.5, 6.0, 11.0]]], dtype=np.float16)
    eye = np.eye(8, dtype=np.float16)[None]
    full = fo.kv_transform_quant(y, eye, 1.0)
    for alpha in (0.5, 0.25):
        res = fo.kv_transform_quant(y, eye, alpha)
        assert float(res["scales"][0, 0]) == alpha * float(full["scales"][0, 0])
        assert int(res["zeros"][0, 0]) == int(full["zeros"][0, 0]) == 3
        want = [min(15, max(0, exact_round_half_even(frac(v) / frac(alpha)) + 3)) for v in y[0, 0].tolist()]
        assert res["q"][0, 0].tolist() == want


def test_kv_transform_index_by_index():
    """y[t, h, e] = sum_d kv[t, h, d] P[h, d, e], written out over every index in exact rationals, with a different
    matrix per head (so a head permutation or a transposed P_h cannot pass), and with distinct permutation matrices."""
    r = rng(77)
    T, H, D = 2, 3, 4
    kv = rand_fp16(r, (T, H, D))
    P = rand_fp16(r, (H, D, D))
    got = fo.kv_transform(kv, P)
    for t in range(T):
        for h in range(H):
            for e in range(D):
                acc = Fraction(0)
                for d in range(D):
                    acc += frac(kv[t, h, d]) * frac(P[h, d, e])
                assert abs(Fraction(float(got[t, h, e])) - acc) <= abs(acc) * Fraction(1, 2 ** 48) + Fraction(1, 2 ** 60)
    shared = fo.kv_transform(kv, P[1:2])
    for t in range(T):
        for h in range(H):
            for e in range(D):
                acc = sum(frac(kv[t, h, d]) * frac(P[1, d, e]) for d in range(D))
                assert abs(Fraction(float(shared[t, h, e])) - acc) <= abs(acc) * Fraction(1, 2 ** 48) + Fraction(1, 2 ** 60)
    # permutation matrices, a different one per head: P_h[d, perm_h[d]] = 1 sends input dim d to output dim perm_h[d]
    perms = [[1, 2, 3, 0], [3, 2, 1, 0], [2, 0, 3, 1]]
    Pp = np.zeros((H, D, D), dtype=np.float16)
    for h, pm in enumerate(perms):
        for d, e in enumerate(pm):
            Pp[h, d, e] = 1
    yp = fo.kv_transform(kv, Pp)
    for h, pm in enumerate(perms):
        for d, e in enumerate(pm):
            assert np.array_equal(yp[:, h, e], kv[:, h, d].astype(np.float64))


def test_kv_comparator_accepts_oracle_and_rejects_planted_mistakes():
    kv = synth.kv_cache(T=12)
    G = kv.T * kv.H
    clip = 0.95
    res = fo.kv_transform_quant(kv.k, kv.P, clip)
    y = res["y"].reshape(G, kv.D)
    codes, s, z = res["codes"].reshape(G, -1), res["scales"].reshape(G), res["zeros"].reshape(G).astype(np.float16)
    rep = parity.check_kv(y, clip, codes, s, z, deq_dev=fo.dequantize(codes, s, z))
    assert rep["band_flips"] == 0 and rep["step_differs"] == 0 and rep["zero_differs"] == 0
    yk = y.reshape(kv.T, kv.H, kv.D)

    def grid_with(mx_scale, mn_scale):
        """A planted variant of the grid (CPU only): the two range ends scaled separately."""
        mx = mx_scale * np.maximum(y.max(-1), 0.0)
        mn = mn_scale * np.minimum(y.min(-1), 0.0)
        sw = ((mx - mn) / 15).astype(np.float16)
        zw = np.clip(np.rint(-mn / sw.astype(np.float64)), 0, 15)
        qw = np.clip(np.rint(y / sw.astype(np.float64)[:, None]) + zw[:, None], 0, 15).astype(np.uint8)
        return fo.pack_bits(qw, 4), sw, zw.astype(np.float16)

    ok = grid_with(clip, clip)                                # the same construction with the right reading passes
    parity.check_kv(y, clip, *ok)
    with pytest.raises(AssertionError):                       # threshold on the upper end only
        parity.check_kv(y, clip, *grid_with(clip, 1.0))
    with pytest.raises(AssertionError):                       # threshold on the lower end only
        parity.check_kv(y, clip, *grid_with(1.0, clip))
    with pytest.raises(AssertionError):                       # no threshold at all
        parity.check_kv(y, clip, *grid_with(1.0, 1.0))
    with pytest.raises(AssertionError):                       # zero point off by one, codes consistent with it
        z1 = np.where(z.astype(np.float64) < 15, z.astype(np.float64) + 1, 14).astype(np.float16)
        q1, _, _, _, _ = fo.kv_quantize_asym(y, clip, 4, scale_fp16=s, zero=z1.astype(np.float64))
        parity.check_kv(y, clip, fo.pack_bits(q1, 4), s, z1)
    with pytest.raises(AssertionError):                       # zero point off by one, codes stale
        parity.check_kv(y, clip, codes, s, z1)
    with pytest.raises(AssertionError):                       # swapped nibbles
        parity.check_kv(y, clip, ((codes << 4) | (codes >> 4)).astype(np.uint8), s, z)
    with pytest.raises(AssertionError):                       # step one ulp off, codes stale (not re-derived with it)
        s_up = (s.view(np.uint16) + 1).view(np.float16)
        q_up, _, _, _, _ = fo.kv_quantize_asym(y, clip, 4, scale_fp16=s_up, zero=z.astype(np.float64))
        assert np.any(q_up != res["q"].reshape(G, kv.D))      # the case does separate the two
        parity.check_kv(y, clip, codes, s_up, z)
    with pytest.raises(AssertionError):                       # two heads' results exchanged
        perm = np.arange(kv.H); perm[[0, 1]] = [1, 0]
        cs = res["codes"][:, perm].reshape(G, -1); ss = res["scales"][:, perm].reshape(G); zs = res["zeros"][:, perm].reshape(G)
        parity.check_kv(y, clip, cs, ss, zs.astype(np.float16))
    with pytest.raises(AssertionError):                       # the transposed head matrix
        wrong = fo.kv_transform_quant(kv.k, np.ascontiguousarray(kv.P.transpose(0, 2, 1)), clip)
        parity.check_kv(y, clip, wrong["codes"].reshape(G, -1), wrong["scales"].reshape(G), wrong["zeros"].reshape(G).astype(np.float16))
    with pytest.raises(AssertionError):                       # truncation instead of rounding
        qt = np.clip(np.trunc(res["u"].reshape(G, kv.D)) + z.astype(np.float64)[:, None], 0, 15).astype(np.uint8)
        parity.check_kv(y, clip, fo.pack_bits(qt, 4), s, z)
    # an adjacent fp16 step with codes re-derived from it is legitimate
    q_ok, _, _, _, _ = fo.kv_quantize_asym(y, clip, 4, scale_fp16=s_up, zero=z.astype(np.float64))
    zf_up = -clip * np.minimum(y.min(-1), 0.0) / s_up.astype(np.float64)
    same_z = np.clip(np.rint(zf_up), 0, 15) == z.astype(np.float64)
    rep = parity.check_kv(y[same_z], clip, fo.pack_bits(q_ok, 4)[same_z], s_up[same_z], z[same_z])
    assert rep["step_differs"] == int(same_z.sum())
    del yk


def test_kv_invariants():
    kv = synth.kv_cache(T=24)
    eye = np.broadcast_to(np.eye(kv.D, dtype=np.float16), (kv.H, kv.D, kv.D))
    res = fo.kv_transform_quant(kv.k, eye, 1.0)
    q, s, z = res["q"], res["scales"].astype(np.float64), res["zeros"].astype(np.float64)
    assert q.min() >= 0 and q.max() <= 15
    # the group minimum lands on code 0 or the maximum on code 15 (the grid spans the range)
    assert np.all((q.min(axis=-1) == 0) | (q.max(axis=-1) == 15))
    yhat = fo.dequantize(res["codes"], res["scales"], res["zeros"])
    # |yhat - y| <= s/2, plus the shift the rounded zero point adds at the two range ends
    assert np.all(np.abs(yhat - res["y"]) <= s[..., None] * (1.0 + 1e-9))
    inner = (res["u"] + z[..., None] > 0.5) & (res["u"] + z[..., None] < 14.5)
    assert np.all(np.abs(yhat - res["y"])[inner] <= (s[..., None] / 2 * (1 + 1e-9) * np.ones_like(yhat))[inner])
    # all-positive group -> zero point 0 and codes = round(y / s)
    pos = np.abs(kv.k[:3]).astype(np.float16)
    rp = fo.kv_transform_quant(pos, eye, 1.0)
    assert not rp["zeros"].any()
    # per-head matrices really are applied head by head
    r2 = fo.kv_transform(kv.k[:2], kv.P)
    for h in range(kv.H):
        np.testing.assert_allclose(r2[:, h], kv.k[:2, h].astype(np.float64) @ kv.P[h].astype(np.float64), rtol=1e-13)
    shared = fo.kv_transform(kv.k[:2], kv.P[:1])
    np.testing.assert_allclose(shared[:, 3], kv.k[:2, 3].astype(np.float64) @ kv.P[0].astype(np.float64), rtol=1e-13)


def test_bit_packing_hand_set_bytes():
    # 3-bit: 1 | 2<<3 | 3<<6 | 4<<9 | 5<<12 | 6<<15 | 7<<18 | 0<<21 = 0x1F58D1, little-endian bytes D1 58 1F
    assert fo.pack_bits(np.array([1, 2, 3, 4, 5, 6, 7, 0]), 3).tolist() == [0xD1, 0x58, 0x1F]
    # 2-bit: 1 | 2<<2 | 3<<4 | 0<<6 = 0x39;   3 | 3<<2 | 0 | 2<<6 = 0x8F
    assert fo.pack_bits(np.array([1, 2, 3, 0, 3, 3, 0, 2]), 2).tolist() == [0x39, 0x8F]
    # 4-bit is the nibble layout of the rest of the library: even channel in the low nibble
    q = np.array([[1, 15, 0, 9, 7, 8]])
    assert fo.pack_bits(q, 4).tolist() == [[0xF1, 0x90, 0x87]]
    assert np.array_equal(fo.pack_bits(q, 4), fo.pack_nibbles(q.astype(np.int8)))
    rng = np.random.default_rng(5)
    for bits in (2, 3, 4):
        q = rng.integers(0, 1 << bits, size=(3, 5, 128)).astype(np.uint8)
        p = fo.pack_bits(q, bits)
        assert p.shape == (3, 5, 16 * bits) and p.dtype == np.uint8
        assert np.array_equal(fo.unpack_bits(p, bits, 128), q)
    # a code that crosses a byte boundary (3-bit code 2 occupies bits 6..8)
    assert fo.pack_bits(np.array([0, 0, 7, 0, 0, 0, 0, 0]), 3).tolist() == [0xC0, 0x01, 0x00]


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_kv_lower_bit_grid(bits):
    """App. "KV Cache Quantization", tables on key / value bit widths: the same asymmetric group-wise grid with
    2^b levels.  Pinned by what any such grid must do."""
    qmax = (1 << bits) - 1
    kv = synth.kv_cache(T=16)
    eye = np.broadcast_to(np.eye(kv.D, dtype=np.float16), (kv.H, kv.D, kv.D))
    res = fo.kv_transform_quant(kv.k, eye, 1.0, bits)
    q, s, z = res["q"], res["scales"].astype(np.float64), res["zeros"].astype(np.float64)
    assert res["codes"].shape == (16, kv.H, kv.D * bits // 8)
    assert q.min() >= 0 and q.max() <= qmax and z.min() >= 0 and z.max() <= qmax
    assert np.all((q.min(axis=-1) == 0) | (q.max(axis=-1) == qmax))
    # the step divides the (zero-containing) range into 2^b - 1 intervals
    rng_ = np.maximum(res["y"].max(-1), 0) - np.minimum(res["y"].min(-1), 0)
    np.testing.assert_allclose(s, rng_ / qmax, rtol=2.0 ** -11)
    # every value goes to the nearest level of its group's grid (brute force over the 2^b levels), except that a
    # tie or the clamped ends may pick a neighbour: the chosen level is never worse than the best by more than that
    levels = (np.arange(qmax + 1)[None, None, None, :] - z[..., None, None]) * s[..., None, None]
    best = np.min(np.abs(res["y"][..., None] - levels), axis=-1)
    yhat = fo.dequantize(res["codes"], res["scales"], res["zeros"], bits)
    assert np.all(np.abs(yhat - res["y"]) <= best + 1e-9 * s[..., None])
    # zero is on the grid: an exact 0.0 input comes back as exactly 0.0
    y0 = kv.k[:2].copy()
    y0[:, :, 5] = 0
    r0 = fo.kv_transform_quant(y0, eye, 1.0, bits)
    assert np.all(fo.dequantize(r0["codes"], r0["scales"], r0["zeros"], bits)[:, :, 5] == 0.0)
    # a group of exactly 2^b equally spaced values 0, d, 2d, ... is reproduced exactly (d a power of two)
    ramp = np.zeros((1, 1, 128), dtype=np.float16)
    ramp[0, 0, :qmax + 1] = 0.25 * np.arange(qmax + 1)
    rr = fo.kv_transform_quant(ramp, np.eye(128, dtype=np.float16)[None], 1.0, bits)
    assert float(rr["scales"][0, 0]) == 0.25 and int(rr["zeros"][0, 0]) == 0
    assert rr["q"][0, 0, :qmax + 1].tolist() == list(range(qmax + 1))
    # fewer bits never give a finer grid
    if bits < 4:
        finer = fo.kv_transform_quant(kv.k, eye, 1.0, bits + 1)
        assert np.all(finer["scales"].astype(np.float64) <= s * (1 + 2.0 ** -10))


# ---- MXFP4 output (format: OCP Microscaling; named by the paper's "Limitations") -------
def test_e2m1_values_follow_the_format_definition():
    # sign, 2 exponent bits (bias 1), 1 mantissa bit; exponent field 0 is subnormal: M * 0.5
    for code in range(16):
        sgn, e, m = code >> 3, (code >> 1) & 3, code & 1
        v = (m * 0.5) if e == 0 else (2.0 ** (e - 1)) * (1 + m / 2)
        assert float(fo.e2m1_value(np.uint8(code))) == (-v if sgn else v)
    assert max(fo.E2M1_VALUES) == 6.0 and fo.MX_BLOCK == 32


def test_e2m1_rounding_hand_cases_and_arithmetic_route():
    # ties go to the even code; beyond 6 saturates; the sign is kept, also on a zero result
    cases = {0.0: 0, 0.2: 0, 0.25: 0, 0.26: 1, 0.5: 1, 0.75: 2, 1.0: 2, 1.25: 2, 1.26: 3, 1.75: 4, 2.5: 4, 2.51: 5, 3.0: 5,
             3.5: 6, 4.0: 6, 5.0: 6, 5.01: 7, 6.0: 7, 7.0: 7, 1e9: 7, -0.1: 8, -0.25: 8, -0.75: 10, -5.0: 14, -100.0: 15}
    for v, code in cases.items():
        assert int(fo.e2m1_round(np.float64(v))) == code, v
    assert int(fo.e2m1_round(np.float64(-0.0))) == 8
    # saturation holds however large the value is (beyond 2^53 an fp64 distance no longer tells the magnitudes apart)
    for v, code in ((1e17, 7), (-1e17, 15), (1e30, 7), (-1e300, 15), (float(2 ** 60), 7)):
        assert int(fo.e2m1_round(np.float64(v))) == code, v
    # the same rounding done arithmetically: spacing 0.5 * 2^max(floor(log2 a), 0), round-half-even in units of it
    r = np.random.default_rng(11)
    u = np.concatenate([r.uniform(-8, 8, 20000), r.normal(0, 1.5, 20000), np.arange(-32, 33) / 4.0])
    a = np.abs(u)
    k = np.maximum(np.floor(np.log2(np.where(a > 0, a, 1.0))), 0)
    sp = 0.5 * 2.0 ** k
    val = np.minimum(np.rint(a / sp) * sp, 6.0)
    got = fo.e2m1_value(fo.e2m1_round(u))
    assert np.array_equal(np.abs(got), val) and np.array_equal(np.signbit(got) | (got == 0), np.signbit(u) | (got == 0))


def test_mx_shared_exponent_and_block_properties():
    blk = np.zeros((1, 64))
    for mx, e in [(6.0, 127), (5.99, 127), (7.9, 127), (8.0, 128), (4.0, 127), (3.99, 126), (1.0, 125), (0.9, 124), (2.0 ** -20, 105)]:
        blk[0, :32] = 0.0
        blk[0, 7] = -mx                       # the maximum is taken over magnitudes
        blk[0, 40] = 2 * mx                   # the second block has its own exponent
        ex = fo.mx_scale_exponent(blk, 1.0)
        assert ex.tolist() == [[e, e + 1]], (mx, ex)
    assert fo.mx_scale_exponent(np.zeros((2, 32)), 1.0).tolist() == [[0], [0]]
    c = synth.tiny()
    y = fo.affine_transform(c.x, c.P1, c.P2)
    y = np.concatenate([y, y], axis=-1)[:, :64] if y.shape[-1] < 64 else y[:, : (y.shape[-1] // 32) * 32]
    q, e, u = fo.mx_quantize(y, 1.0)
    ub = np.abs(u).reshape(u.shape[0], -1, 32)
    top = ub.max(-1)
    assert np.all((top >= 4.0) & (top < 8.0) | (top == 0))         # the block maximum lands in the top binade
    assert np.all(((q.reshape(ub.shape) & 7).max(-1) >= 6) | (top == 0))
    deq = fo.dequantize_mxfp4(fo.pack_nibbles(q.astype(np.int8)), e)
    x = np.repeat(np.ldexp(1.0, e.astype(np.int64) - 127), 32, axis=-1)
    au = np.abs(u)
    spacing = np.where(au < 2, 0.5, np.where(au < 4, 1.0, 2.0))
    bound = np.where(au <= 6, spacing / 2, au - 6) * x
    assert np.all(np.abs(deq - y) <= bound * (1 + 1e-12))
    # idempotent: what comes out is on the grid of its own block
    q2, e2, _ = fo.mx_quantize(deq, 1.0)
    assert np.array_equal(e2, e) and np.array_equal(q2 & 7, q & 7)
    # the clipping threshold multiplies the block maximum: alpha = 1/2 lowers every exponent by one
    assert np.array_equal(fo.mx_scale_exponent(y, 0.5).astype(int), e.astype(int) - 1)
    per_tok = np.full(y.shape[0], 0.5)
    assert np.array_equal(fo.mx_scale_exponent(y, per_tok), fo.mx_scale_exponent(y, 0.5))
    # the comparator accepts the oracle and rejects planted mistakes (CPU only)
    codes = fo.pack_nibbles(q.astype(np.int8))
    rep = parity.check_mx(y, 1.0, codes, e)
    assert rep["band_flips"] == 0 and rep["exp_differs"] == 0
    with pytest.raises(AssertionError):
        parity.check_mx(y, 1.0, codes, e + 1)
    with pytest.raises(AssertionError):
        parity.check_mx(y, 1.0, ((codes << 4) | (codes >> 4)).astype(np.uint8), e)
    trunc = (np.searchsorted(np.asarray(fo.E2M1_VALUES), np.minimum(np.abs(u), 6.0), side="right") - 1).astype(np.uint8) | (q & 8)
    with pytest.raises(AssertionError):
        parity.check_mx(y, 1.0, fo.pack_nibbles(trunc.astype(np.int8)), e)


def test_mx_tile_order_of_exponents():
    # byte of (row r, block k) = (((r // 128) * (n // 256) + k // 8) * 128 + r % 128) * 8 + k % 8, written out for a few entries
    R, n = 130, 512
    e = (np.arange(R * 16) % 251).astype(np.uint8).reshape(R, 16)
    t = fo.mx_tile_scales(e, fill=0xEE)
    assert t.shape == (2 * 2 * 128 * 8,)
    assert t[0] == e[0, 0] and t[7] == e[0, 7] and t[8] == e[1, 0]                      # rows of a group are 8 bytes apart
    assert t[128 * 8] == e[0, 8] and t[128 * 8 + 127 * 8 + 3] == e[127, 11]              # second group of the first tile
    assert t[3081] == e[129, 9] and t[2 * 128 * 8 + 0] == e[128, 0]                      # second tile
    assert t[2 * 128 * 8 + 2 * 8] == 0xEE                                                # padding row 130
    assert np.array_equal(fo.mx_untile_scales(t, R, n), e)


def test_mxfp4_product_hand_set_and_brute_force():
    # one token, one channel, n = 32: x = [1.0, 6.0, -0.5, 0...] * 2^1, w = [3.0, -1.5, 4.0, 0...] * 2^-2
    xc = np.zeros((1, 16), dtype=np.uint8); wc = np.zeros((1, 16), dtype=np.uint8)
    xc[0, 0] = 0x72; xc[0, 1] = 0x09          # codes 2 (1.0), 7 (6.0), 9 (-0.5), 0
    wc[0, 0] = 0xB5; wc[0, 1] = 0x06          # codes 5 (3.0), 11 (-1.5), 6 (4.0), 0
    y, y16, ab = fo.mxfp4_gemm(xc, np.array([[128]], dtype=np.uint8), wc, np.array([[125]], dtype=np.uint8))
    want = (1.0 * 3.0 + 6.0 * -1.5 + -0.5 * 4.0) * 2.0 * 0.25
    assert y[0, 0] == want == -4.0 and float(y16[0, 0]) == -4.0 and ab[0, 0] == (3.0 + 9.0 + 2.0) * 0.5
    r = np.random.default_rng(17)
    T, m, n = 5, 7, 96
    xc = r.integers(0, 256, size=(T, n // 2), dtype=np.uint8); wc = r.integers(0, 256, size=(m, n // 2), dtype=np.uint8)
    xe = r.integers(120, 132, size=(T, n // 32), dtype=np.uint8); we = r.integers(118, 130, size=(m, n // 32), dtype=np.uint8)
    y, _, _ = fo.mxfp4_gemm(xc, xe, wc, we)
    val = [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]
    for t in range(T):
        for o in range(m):
            acc = 0.0
            for k in range(n):
                a = (xc[t, k // 2] >> (4 * (k & 1))) & 15
                b = (wc[o, k // 2] >> (4 * (k & 1))) & 15
                av = (-1.0 if a & 8 else 1.0) * val[a & 7] * 2.0 ** (int(xe[t, k // 32]) - 127)
                bv = (-1.0 if b & 8 else 1.0) * val[b & 7] * 2.0 ** (int(we[o, k // 32]) - 127)
                acc += av * bv
            assert abs(acc - y[t, o]) <= 1e-12 * max(1.0, abs(acc))


# ---- the comparator itself -----------------------------------------------------------
def test_comparator_accepts_oracle_and_rejects_planted_mistakes():
    c = synth.tiny()
    res = fo.transform_quant(c.x, c.P1, c.P2, c.clip)
    deq = fo.dequantize(res["codes"], res["scales"])
    rep = parity.check_sym(res["y"], c.clip, res["codes"], res["scales"], deq_dev=deq)
    assert rep["band_flips"] == 0 and rep["step_differs"] == 0
    # mistakes planted in oracle copies (CPU only): transposed P1, swapped nibbles, truncation, unclipped step
    wrong = fo.transform_quant(c.x, c.P1.T.copy(), c.P2, c.clip)
    with pytest.raises(AssertionError):
        parity.check_sym(res["y"], c.clip, wrong["codes"], wrong["scales"])
    swapped = ((res["codes"] << 4) | (res["codes"] >> 4)).astype(np.uint8)
    with pytest.raises(AssertionError):
        parity.check_sym(res["y"], c.clip, swapped, res["scales"])
    trunc = fo.pack_nibbles(np.clip(np.trunc(res["u"]), -8, 7).astype(np.int8))
    with pytest.raises(AssertionError):
        parity.check_sym(res["y"], c.clip, trunc, res["scales"])
    with pytest.raises(AssertionError):
        parity.check_sym(res["y"], 0.9, res["codes"], res["scales"])
    # an adjacent fp16 step is legitimate when the oracle re-run with it agrees
    s2 = (res["scales"].view(np.uint16) + 1).view(np.float16)
    q2, _, _ = fo.quantize_sym_int4(res["y"], None, scale_fp16=s2)
    rep = parity.check_sym(res["y"], c.clip, fo.pack_nibbles(q2), s2)
    assert rep["step_differs"] == c.T


def test_synthetic_recipes_are_deterministic_and_shaped():
    a, b = synth.prefill_7b(32), synth.prefill_7b(32)
    assert a.x.dtype == np.float16 and a.x.shape == (32, 4096) and np.array_equal(a.x, b.x)
    assert np.array_equal(a.P1, b.P1) and a.clip.shape == (32,) and 0.8 < a.clip.min() and a.clip.max() < 0.96
    assert np.abs(a.x[0].astype(np.float32)).max() <= 30000 and np.abs(a.x[0].astype(np.float32)).mean() > 100
    assert np.all(np.isfinite(a.x.astype(np.float32)))
    d = synth.decode_7b(8, wide=True)
    assert (d.n1, d.n2, d.n) == (86, 128, 11008)


# ---- right factor of Eq. (2): the offline weight side -------------------------
def _invertible(r, n, noise=0.2):
    return (np.eye(n) + noise * r.standard_normal((n, n))).astype(np.float16)


def test_weight_side_keeps_the_layer_output_eq1():
    """Eq. (1): (X P)(P^-1 W^T) = X W^T.  The oracle's transformed weights, multiplied with the transformed
    activations, must give back the plain layer output; brute-force exact rationals on a tiny case."""
    r = rng(601)
    n1, n2, T, m = 2, 3, 2, 3
    P1 = np.array([[2, 1], [1, 1]], dtype=np.float16)              # unimodular: exact integer inverses
    P2 = np.array([[1, 1, 0], [0, 1, 1], [0, 0, 1]], dtype=np.float16)
    X = r.integers(-4, 5, size=(T, n1 * n2)).astype(np.float16)
    W = r.integers(-4, 5, size=(m, n1 * n2)).astype(np.float16)
    Wt = fo.weight_transform(W, P1, P2)
    Y = fo.affine_transform(X, P1, P2) @ Wt.T
    for t in range(T):
        for o in range(m):
            exact = sum(frac(X[t, c]) * frac(W[o, c]) for c in range(n1 * n2))
            assert abs(Y[t, o] - float(exact)) < 1e-9
    # a transposed or un-inverted factor must not pass (orientation pin)
    wrong = fo.weight_transform_factored(W, np.linalg.inv(P1.astype(np.float64)), np.linalg.inv(P2.astype(np.float64)))
    assert np.abs(fo.affine_transform(X, P1, P2) @ wrong.T - X.astype(np.float64) @ W.astype(np.float64).T).max() > 0.5


@pytest.mark.parametrize("n1,n2", [(1, 4), (3, 5), (8, 8), (16, 4)])
def test_weight_side_factored_form_equals_dense_inverse(n1, n2):
    """(P1 (x) P2)^-1 = P1^-1 (x) P2^-1 (textbook): the factored right factor of Eq. (2) with A1 = P1^-T,
    A2 = P2^-T must equal the weights obtained from the dense inverse."""
    r = rng(610 + n1 * 31 + n2)
    P1, P2 = _invertible(r, n1), _invertible(r, n2)
    W = rand_fp16(r, (7, n1 * n2))
    dense = fo.weight_transform(W, P1, P2)
    fact = fo.weight_transform_factored(W, fo.inverse_transpose(P1), fo.inverse_transpose(P2))
    assert np.allclose(dense, fact, rtol=1e-9, atol=1e-9)
    # inverse_transpose against the defining property, not against itself
    A1 = fo.inverse_transpose(P1)
    assert np.allclose(A1.T @ P1.astype(np.float64), np.eye(n1), atol=1e-10)


def test_weight_side_with_orthogonal_factors_is_the_activation_transform():
    """For orthogonal P (normalised Hadamard factors) P^-T = P: weights and activations get the same transform."""
    H = np.array([[1.0]])
    for _ in range(3):
        H = np.block([[H, H], [H, -H]])
    P1 = (H / np.sqrt(8)).astype(np.float64)     # 8 x 8, not exactly representable in fp16: keep fp64
    H2 = np.block([[H, H], [H, -H]])
    P2 = (H2 / 4.0).astype(np.float16)           # 16 x 16, entries +-1/4 exact
    r = rng(620)
    W = rand_fp16(r, (5, 128))
    assert np.allclose(fo.weight_transform(W, P1, P2), fo.affine_transform(W, P1, P2), atol=1e-12)


def test_quantized_layer_error_is_within_the_rounding_bound():
    """With alpha = 1 nothing clips, so |x^ - x'| <= s_x / 2 and |w^ - w'| <= s_w / 2 element-wise and
    |y^ - y| <= ||x'||_1 s_w / 2 + ||w'||_1 s_x / 2 + n s_x s_w / 4 for every output: a rigorous bound that a wrong
    scale, a wrong pairing of transformed factors or a wrong de-quantization breaks."""
    r = rng(630)
    n1, n2, T, m = 8, 16, 12, 9
    P1, P2 = _invertible(r, n1, 0.1), _invertible(r, n2, 0.1)
    X = rand_fp16(r, (T, n1 * n2), 2.0)
    X[:, 5] *= 30
    W = rand_fp16(r, (m, n1 * n2), 0.05)
    ax = fo.transform_quant(X, P1, P2, 1.0)
    aw = fo.weight_transform_quant(W, fo.inverse_transpose(P1), fo.inverse_transpose(P2), 1.0)
    Yq = fo.quantized_linear(ax["codes"], ax["scales"], aw["codes"], aw["scales"])
    Y = X.astype(np.float64) @ W.astype(np.float64).T
    sx, sw = fo.as_f64(ax["scales"]), fo.as_f64(aw["scales"])
    bound = (np.abs(ax["y"]).sum(1)[:, None] * sw[None, :] / 2 + np.abs(aw["y"]).sum(1)[None, :] * sx[:, None] / 2
             + n1 * n2 * sx[:, None] * sw[None, :] / 4)
    assert np.all(np.abs(Yq - Y) <= bound * (1 + 1e-9) + 1e-9)
    assert np.abs(Yq - Y).max() > 0          # it is a quantized product, not the exact one
    # per-output-channel steps: a row's codes do not depend on the other rows
    one = fo.weight_transform_quant(W[3:4], fo.inverse_transpose(P1), fo.inverse_transpose(P2), 1.0)
    assert np.array_equal(one["codes"][0], aw["codes"][3]) and one["scales"][0] == aw["scales"][3]


def test_query_side_transform_keeps_attention_scores():
    """Sec. 3.2: with keys stored as K P_h, queries through (P_h^-1)^T leave Q K^T unchanged (textbook identity,
    checked head by head against the untransformed scores); also pins kv_transform's head indexing."""
    r = rng(640)
    T, H, D = 5, 3, 8
    Q, K = rand_fp16(r, (T, H, D)), rand_fp16(r, (T, H, D))
    P = np.stack([_invertible(r, D) for _ in range(H)])
    Pq = np.stack([fo.inverse_transpose(P[h]) for h in range(H)])
    Kt, Qt = fo.kv_transform(K, P), fo.kv_transform(Q, Pq)
    for h in range(H):
        want = Q[:, h, :].astype(np.float64) @ K[:, h, :].astype(np.float64).T
        assert np.allclose(Qt[:, h, :] @ Kt[:, h, :].T, want, atol=1e-9)
    out = fo.head_transform_fp16(Q, Pq)
    assert out.dtype == np.float16 and np.all(np.abs(out.astype(np.float64) - Qt) <= 2.0 ** -11 * np.abs(Qt) + 2.0 ** -25)


def test_w4a4_gemm_is_the_product_of_the_dequantized_factors():
    """Integer dot products of codes times the two steps must equal deq(x) deq(w)^T (a different route through the
    oracle: de-quantize first, multiply in floating point), and a brute-force loop over a tiny case with hand-set
    codes pins nibble order and signedness."""
    r = rng(650)
    T, m, n = 7, 5, 64
    qx = r.integers(-8, 8, size=(T, n)).astype(np.int8)
    qw = r.integers(-8, 8, size=(m, n)).astype(np.int8)
    sx = (r.uniform(0.01, 3.0, size=T)).astype(np.float16)
    sw = (r.uniform(0.001, 0.1, size=m)).astype(np.float16)
    cx, cw = fo.pack_nibbles(qx), fo.pack_nibbles(qw)
    acc, y, y16 = fo.w4a4_gemm(cx, sx, cw, sw)
    for t in range(T):
        for o in range(m):
            want = sum(int(qx[t, k]) * int(qw[o, k]) for k in range(n))
            assert acc[t, o] == want
            assert y[t, o] == pytest.approx(want * float(sx[t]) * float(sw[o]), rel=1e-15)
    assert np.allclose(y, fo.quantized_linear(cx, sx, cw, sw), rtol=1e-12, atol=1e-300)
    assert y16.dtype == np.float16 and np.all(np.abs(y16.astype(np.float64) - y) <= 2.0 ** -11 * np.abs(y) + 2.0 ** -25)
    # hand-set bytes: 0x7F = codes (-1, 7), 0x80 = (0, -8)
    one = fo.w4a4_gemm(np.array([[0x7F, 0x80]], dtype=np.uint8), np.array([2.0], dtype=np.float16),
                       np.array([[0x21, 0x3F]], dtype=np.uint8), np.array([0.5], dtype=np.float16))
    assert one[0][0, 0] == (-1) * 1 + 7 * 2 + 0 * (-1) + (-8) * 3 and one[1][0, 0] == -11.0
