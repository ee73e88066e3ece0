"""Parity of the HIP path against the fp64 oracle, through the C ABI, on a real MI355X.

Bars (written here as the comparator enforces them, see oracle/parity.py):
steps within 1e-3 relative; codes bit-exact wherever the fp64 pre-round value is
more than 1e-3 away from a rounding boundary; de-quantized values within
1e-2 * step outside that band.
"""
import os

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from oracle import flatquant_oracle as fo  # noqa: E402
from oracle import parity  # noqa: E402
from paper_2410_09426_amd import binding as fq  # noqa: E402
from paper_2410_09426_amd import synth  # noqa: E402

from gpu_util import dev, run_dequant, run_tq  # noqa: E402


def check_case(c, rows=None, with_dequant=True, label=""):
    """Run the whole case on the GPU, compare `rows` (default: all) with the oracle."""
    print(f"[case] {c.name} T={c.T} n1={c.n1} n2={c.n2} {label}", flush=True)
    x, P1, P2, clip = dev(c.x), dev(c.P1), dev(c.P2), dev(c.clip)
    codes, scales, codes_d, scales_d = run_tq(x, P1, P2, clip, c.clip_mode, c.n1, c.n2)
    rows = np.arange(c.T) if rows is None else np.asarray(rows)
    P = fo.kron_dense(c.P1, c.P2)
    y = fo.affine_transform(c.x[rows], None, None, P=P)
    del P
    clipv = c.clip[rows] if c.clip_mode == 1 else float(c.clip[0])
    deq = None
    if with_dequant:
        deq = run_dequant(codes_d, scales_d, None, c.T, c.n)[rows]
    rep = parity.check_sym(y, clipv, codes[rows], scales[rows], deq_dev=deq, rows=rows)
    print(f"[parity] {c.name}: {rep}", flush=True)
    assert rep["band_flips"] <= parity.band_flip_allowance(rep["in_band"])
    return rep, codes, scales


def subset_rows(T, k, seed, must=(0,)):
    r = np.random.Generator(np.random.PCG64(seed))
    rows = set(int(t) for t in must if t < T)
    rows.update(int(v) for v in r.choice(T, size=min(k, T), replace=False))
    rows.add(T - 1)
    return np.array(sorted(rows))


def test_tiny():
    check_case(synth.tiny())


def test_prefill_7b_full():
    rep, _, _ = check_case(synth.prefill_7b())
    assert rep["rows"] == 2048


def test_prefill_7b_forced_persistent_loop(tuning):
    # one workgroup per CU: every workgroup walks 8 tokens through the prefetch / double barrier loop
    tuning("FLATQUANT_WG_PER_CU", "1")
    tuning("FLATQUANT_MODE", "2")
    c = synth.prefill_7b(2048 + 37)
    check_case(c, rows=subset_rows(c.T, 300, 5, must=(0, 255, 256, 257, 2047, 2048)), with_dequant=False, label="wg_per_cu=1")


def test_general_kernel_on_aligned_shapes(tuning):
    # the specialised kernels would take these shapes; force the general one so that it stays covered
    tuning("FLATQUANT_FORCE_GENERIC", "1")
    c = synth.prefill_7b(700)
    check_case(c, rows=subset_rows(c.T, 120, 6), with_dequant=False, label="general kernel")
    check_case(synth.decode_7b(64, wide=True), with_dequant=False, label="general kernel")


@pytest.mark.parametrize("mode", ["0", "1", "2", "3", "4"])
def test_every_kernel_flavour(tuning, mode):
    # 0: one slab per wave; 1: two slabs per wave; 2: software-pipelined loop; 3: one token per workgroup;
    # 4: one wave per token, several tokens per workgroup (the library picks one by shape and T)
    tuning("FLATQUANT_MODE", mode)
    c = synth.prefill_7b(1024 + 3)
    check_case(c, rows=subset_rows(c.T, 150, 11, must=(0, 1, 1023, 1024)), with_dequant=False, label=f"mode {mode}")
    c = synth.generic(90 + int(mode), 600, 64, 128)
    check_case(c, rows=subset_rows(c.T, 80, 12), with_dequant=False, label=f"mode {mode}")
    c = synth.generic(95 + int(mode), 40, 32, 64)
    check_case(c, with_dequant=False, label=f"mode {mode}")
    for T, n1 in ((1, 64), (6, 50), (9, 17)):   # fewer tokens than a workgroup holds, ragged n1
        check_case(synth.generic(195 + int(mode) + T, T, n1, 64), with_dequant=False, label=f"mode {mode}")


@pytest.mark.parametrize("mode", ["5", "6"])
@pytest.mark.parametrize("tpw", ["2", "4", "8"])
def test_wave_per_token_kernel(tuning, mode, tpw):
    # 5: one token per wave, no loop; 6: persistent loop.  tpw = waves (tokens in flight) per workgroup
    tuning("FLATQUANT_MODE", mode)
    tuning("FLATQUANT_WAVE_TPW", tpw)
    c = synth.prefill_7b(2048 + 37)
    check_case(c, rows=subset_rows(c.T, 260, 21, must=(0, 1, 7, 8, 2047, 2048, 2084)), with_dequant=False, label=f"wave kernel {mode}/{tpw}")
    c = synth.generic(300 + int(mode), 4099, 32, 64)
    check_case(c, rows=subset_rows(c.T, 200, 22, must=(0, 4095, 4096, 4098)), with_dequant=False, label=f"wave kernel {mode}/{tpw}")
    for T in (1, 3, 9, 17):   # fewer tokens than a workgroup has waves, and a ragged last workgroup
        check_case(synth.generic(310 + T, T, 64, 64), with_dequant=False, label=f"wave kernel {mode}/{tpw} T={T}")
    # a zero row, a small row, large magnitudes
    c = synth.generic(333, 40, 64, 64)
    c.x[3] = 0
    c.x[5] = (c.x[5].astype(np.float32) * 2.0 ** -4).astype(np.float16)
    c.x[7] = (np.sign(c.x[7].astype(np.float32)) * 900).astype(np.float16)
    check_case(c, with_dequant=False, label=f"wave kernel {mode}/{tpw} edge rows")


@pytest.mark.parametrize("mode", [None, "4"])
def test_mid_length_stream(tuning, mode):
    # more tokens than are resident at once; T % 4 = 3.  Default: the wave-per-token kernel, workgroups handed out by the
    # hardware; mode 4: four single-wave tokens per workgroup of the slab kernels
    if mode is not None:
        tuning("FLATQUANT_MODE", mode)
    c = synth.prefill_7b(4096 + 3)
    check_case(c, rows=subset_rows(c.T, 200, 14, must=(0, 3, 4, 4095, 4096, 4097, 4098)), with_dequant=False, label=f"2048 < T < 32768, mode {mode}")


@pytest.mark.parametrize("mode,T", [(None, 32768 + 5), ("1", 32768 + 5), ("5", 20480 + 5), ("6", 20480 + 7)])
def test_long_stream(tuning, mode, T):
    # default: persistent wave-per-token workgroups from T = 32768 on (5 / 6: one-shot / persistent forced); mode 1: two
    # slabs per wave in a persistent loop
    if mode is not None:
        tuning("FLATQUANT_MODE", mode)
    c = synth.prefill_7b(T)
    must = tuple(r for r in (0, 1, 2047, 2048, 20479, 20480, 32767, 32768, T - 2) if r < T)
    check_case(c, rows=subset_rows(c.T, 200, 13, must=must), with_dequant=False, label=f"long stream, mode {mode}")


def test_decode_shapes():
    check_case(synth.decode_7b(64))
    check_case(synth.decode_7b(64, wide=True))


def test_prefill_70b_8192_sampled():
    c = synth.prefill_70b()
    check_case(c, rows=subset_rows(c.T, 192, 7, must=(0, 2048, 4096, 16383)), with_dequant=False)


def test_prefill_70b_28672_sampled():
    c = synth.prefill_70b(wide=True)
    check_case(c, rows=subset_rows(c.T, 40, 9, must=(0, 2048)), with_dequant=False)


@pytest.mark.parametrize("n1,n2,T", [(64, 172, 33), (128, 224, 19), (1, 2, 5), (2, 2, 7), (3, 6, 70), (33, 34, 11),
                                      (16, 256, 9), (128, 32, 13), (96, 64, 300), (32, 96, 1), (50, 20, 64),
                                      (1, 128, 3000), (2, 64, 2500), (3, 128, 40), (87, 128, 600), (45, 64, 77)])
def test_shape_sweep(n1, n2, T):
    check_case(synth.generic(n1 * 1000 + n2, T, n1, n2, sigma=0.05 if n1 * n2 > 64 else 0.3))


def test_scalar_clip_and_clip_one():
    c = synth.generic(77, 130, 64, 64, clip_mode=0)
    check_case(c)
    c.clip[:] = 1.0
    rep, codes, _ = check_case(c, label="clip=1")
    q = fo.unpack_nibbles(codes, signed=True)
    assert q.min() >= -7 and np.all(np.abs(q).max(axis=1) == 7)


def test_hadamard_factors_and_identity():
    from test_oracle_pins import sylvester
    c = synth.generic(78, 65, 64, 64)
    c.P1 = (sylvester(64) / 8).astype(np.float16)
    c.P2 = (sylvester(64) / 8).astype(np.float16)
    check_case(c, label="hadamard")
    c.P1 = np.eye(64, dtype=np.float16)
    c.P2 = np.eye(64, dtype=np.float16)
    rep, codes, scales = check_case(c, label="identity")
    # identity transform is exact in fp32 as well: plain per-token INT4 of x, bit for bit
    q, s, _ = fo.quantize_sym_int4(c.x.astype(np.float64), c.clip, scale_fp16=scales)
    assert rep["band_flips"] == 0 and np.array_equal(fo.pack_nibbles(q), codes)


def test_degenerate_rows_and_small_magnitudes():
    c = synth.generic(79, 40, 64, 64, massive_tokens=())
    c.x[3] = 0                                   # all-zero token: step 0, codes 0
    c.x[5] = 0
    c.x[5, 4095] = -1.0                          # single non-zero in the last channel
    c.x[7] = (c.x[7].astype(np.float32) * 2.0 ** -12).astype(np.float16)   # fp16 subnormal-heavy row
    c.x[9] = (c.x[9].astype(np.float32) * 2.0 ** -6).astype(np.float16)
    rep, codes, scales = check_case(c)
    assert not codes[3].any() and float(scales[3]) == 0.0


def test_large_magnitudes_near_the_fp16_range():
    """The result is defined while x, the intermediate X~ P2 (kept as fp16 hi + lo) and Y stay finite in fp16 range.
    Rows built to come close to that edge (|x| = 30000 everywhere, signs chosen so that the sums against the
    near-identity P2 stay below 65504) must still match the oracle."""
    for n1, n2 in ((64, 64), (86, 128)):
        c = synth.generic(81 + n1, 24, n1, n2, massive_tokens=())
        r = np.random.Generator(np.random.PCG64(4))
        sign = r.choice(np.array([-1.0, 1.0], dtype=np.float32), size=(6, c.n))
        unit = np.einsum("tij,jk->tik", sign.astype(np.float64).reshape(6, n1, n2), c.P2.astype(np.float64))
        amp = 60000.0 / np.abs(unit).reshape(6, -1).max(axis=1)             # per row: the largest |X~ P2| entry becomes ~60000
        c.x[:6] = (amp[:, None] * sign).astype(np.float16)
        z = np.einsum("tij,jk->tik", c.x[:6].astype(np.float64).reshape(6, n1, n2), c.P2.astype(np.float64))
        assert 55000 < np.abs(z).max() < 65504                              # inside the contract, and near its edge
        rep, codes, scales = check_case(c, with_dequant=False, label="near the fp16 range")
        assert np.all(np.isfinite(scales.astype(np.float32)))


def test_power_of_two_scaling_keeps_codes():
    c = synth.generic(80, 48, 64, 64, massive_tokens=())
    _, codes, scales = check_case(c)
    c2 = synth.generic(80, 48, 64, 64, massive_tokens=())
    c2.x = (c.x.astype(np.float32) * 0.125).astype(np.float16)
    _, codes2, scales2 = check_case(c2, label="x/8")
    same = scales2.astype(np.float64) * 8 == scales.astype(np.float64)
    assert same.mean() > 0.9 and np.array_equal(codes[same], codes2[same])


def test_strided_and_unaligned_buffers():
    c = synth.generic(81, 21, 64, 64)
    n = c.n
    ref_codes, ref_scales, _, _ = run_tq(dev(c.x), dev(c.P1), dev(c.P2), dev(c.clip), c.clip_mode, c.n1, c.n2)
    # (a) row stride larger than n
    xs = torch.zeros((c.T, n + 72), dtype=torch.float16, device="cuda")
    xs[:, :n] = dev(c.x)
    a_codes, a_scales, _, _ = run_tq(xs, dev(c.P1), dev(c.P2), dev(c.clip), c.clip_mode, c.n1, c.n2, x_stride=n + 72)
    assert np.array_equal(a_codes, ref_codes) and np.array_equal(a_scales.view(np.uint16), ref_scales.view(np.uint16))
    # (b) x only 4-byte aligned (slow loader), odd guard so codes land on an odd address (byte stores)
    flat = torch.zeros((c.T * n + 8,), dtype=torch.float16, device="cuda")
    flat[2:2 + c.T * n] = dev(c.x).reshape(-1)
    xu = flat[2:2 + c.T * n].view(c.T, n)
    b_codes, b_scales, _, _ = run_tq(xu, dev(c.P1), dev(c.P2), dev(c.clip), c.clip_mode, c.n1, c.n2, guard=63)
    assert np.array_equal(b_codes, ref_codes) and np.array_equal(b_scales.view(np.uint16), ref_scales.view(np.uint16))


@pytest.mark.parametrize("n1,n2,T", [(64, 64, 70), (86, 128, 19), (32, 96, 300), (3, 6, 50), (64, 128, 2100), (33, 34, 40)])
@pytest.mark.parametrize("pad,xoff,poff,guard", [(2, 0, 0, 64), (8, 0, 0, 64), (10, 2, 0, 63), (0, 4, 1, 64), (24, 6, 1, 61), (0, 0, 1, 64)])
def test_alignment_and_stride_grid(n1, n2, T, pad, xoff, poff, guard):
    """Row strides that are not multiples of 8 elements, inputs that start 4, 8 or 12 bytes into a 16-byte unit, factors
    that start 2 bytes in, codes on odd addresses: whichever kernel the library falls back to, against the oracle."""
    n = n1 * n2
    c = synth.generic(60 + n1 + n2 + pad + xoff, T, n1, n2, sigma=0.05 if n > 64 else 0.3)
    stride = n + pad
    flat = torch.zeros((xoff + T * stride + 8,), dtype=torch.float16, device="cuda")
    xv = flat[xoff:xoff + T * stride].view(T, stride)
    xv[:, :n] = dev(c.x)
    xv[:, n:] = 777.0                                    # the gap between rows must not leak into any row
    def shifted(a):
        t = torch.zeros((a.size + 8,), dtype=torch.float16, device="cuda")
        t[poff:poff + a.size] = dev(a).reshape(-1)
        return t[poff:poff + a.size].view(*a.shape)
    print(f"[case] alignment grid {n1}x{n2} T={T} stride n+{pad} x+{xoff} P+{poff} guard {guard}", flush=True)
    codes, scales, _, _ = run_tq(xv, shifted(c.P1), shifted(c.P2), dev(c.clip), c.clip_mode, n1, n2, x_stride=stride, guard=guard)
    rows = subset_rows(T, 100, 33, must=(0, 1, T - 2))
    y = fo.affine_transform_factored(c.x[rows], c.P1, c.P2)
    rep = parity.check_sym(y, c.clip[rows], codes[rows], scales[rows], rows=rows)
    assert rep["band_flips"] <= parity.band_flip_allowance(rep["in_band"])


def test_determinism_and_empty_input():
    c = synth.prefill_7b(512)
    x, P1, P2, clip = dev(c.x), dev(c.P1), dev(c.P2), dev(c.clip)
    first = None
    for _ in range(5):
        codes, scales, _, _ = run_tq(x, P1, P2, clip, c.clip_mode, c.n1, c.n2)
        if first is None:
            first = (codes.copy(), scales.copy())
        assert np.array_equal(first[0], codes) and np.array_equal(first[1].view(np.uint16), scales.view(np.uint16))
    assert fq.flatquant_transform_quant(x, P1, P2, clip, 1, 0, 64, 64, 4096, None, None) == fq.FQ_OK


# ---- MXFP4 output ------------------------------------------------------------------------
def run_mx(c, rows=None):
    x, P1, P2, clip = dev(c.x), dev(c.P1), dev(c.P2), dev(c.clip)
    T, n = c.T, c.n
    cbuf = torch.full((T * (n // 2) + 256,), 0xCD, dtype=torch.uint8, device="cuda")
    sbuf = torch.full((T * (n // 32) + 256,), 0xCD, dtype=torch.uint8, device="cuda")
    fq.flatquant_transform_mxfp4(x, P1, P2, clip, c.clip_mode, T, c.n1, c.n2, n, cbuf, sbuf, stream=torch.cuda.current_stream())
    torch.cuda.synchronize()
    assert bool((cbuf[T * (n // 2):] == 0xCD).all()) and bool((sbuf[T * (n // 32):] == 0xCD).all()), "guard band overwritten"
    codes = cbuf[:T * (n // 2)].cpu().numpy().reshape(T, n // 2)
    exps = sbuf[:T * (n // 32)].cpu().numpy().reshape(T, n // 32)
    if T <= 600:   # the de-quantization helper returns exactly value * 2^(e - 127)
        deq = torch.full((T, n), float("nan"), dtype=torch.float32, device="cuda")
        fq.flatquant_dequant_mxfp4(cbuf, sbuf, T, n, deq, stream=torch.cuda.current_stream())
        torch.cuda.synchronize()
        assert np.array_equal(deq.cpu().numpy().astype(np.float64), fo.dequantize_mxfp4(codes, exps))
    sel = np.arange(T) if rows is None else np.asarray(rows)
    y = fo.affine_transform_factored(c.x[sel], c.P1, c.P2)
    clip_h = c.clip[sel] if c.clip_mode else float(c.clip[0])
    rep = parity.check_mx(y, clip_h, codes[sel], exps[sel])
    print(f"[parity] mxfp4 {c.name} T={T} {c.n1}x{c.n2}: {rep}", flush=True)
    return codes, exps


def _mx_grid():
    r = np.random.Generator(np.random.PCG64(3141))
    cases = set()
    for n1 in [1, 2, 3, 31, 32, 33, 63, 64, 65, 96, 100, 127, 128]:
        for n2 in (32, 64, 96, 128, 160, 192, 224, 256):
            if (n1 * n2) % 128 == 0 and r.random() < (0.75 if n2 in (64, 128, 256) else 0.4):
                T = int(r.choice([1, 2, 63, 300, 2049, 2600]))
                cases.add((n1, n2, min(T, max(600, 20_000_000 // (n1 * n2)))))
    return sorted(cases)


@pytest.mark.parametrize("n1,n2,T", _mx_grid())
def test_mxfp4_output_shape_grid(n1, n2, T):
    c = synth.generic(17 * n1 + n2 + T, T, n1, n2, clip_mode=(n1 + T) % 2)
    print(f"[case] mxfp4 grid {n1}x{n2} T={T}", flush=True)
    run_mx(c, rows=None if T <= 300 else subset_rows(T, 100, n1, must=(0, 1, 2047, 2048, T - 2)))


@pytest.mark.parametrize("mode", ["-1", "0", "3"])
def test_mxfp4_output(tuning, mode):
    if mode != "-1":
        tuning("FLATQUANT_MODE", mode)
    c = synth.prefill_7b(2048 if mode == "-1" else 515)
    run_mx(c, rows=subset_rows(c.T, 160, 21, must=(0, 1, c.T - 1)))
    c = synth.generic(400 + int(mode), 70, 64, 128)
    run_mx(c)
    if mode == "-1":
        for seed, T, n1, n2 in ((411, 33, 86, 128), (412, 9, 112, 256), (413, 1, 32, 64), (414, 300, 2, 64), (415, 40, 50, 256),
                                (416, 2600, 64, 64), (418, 77, 128, 224), (419, 40, 64, 32), (420, 130, 96, 160), (421, 300, 12, 96)):
            c = synth.generic(seed, T, n1, n2, clip_mode=seed % 2)
            run_mx(c, rows=None if T <= 300 else subset_rows(T, 120, 22, must=(0, T - 1)))
        # zero rows: exponent 0, all codes +0
        c = synth.generic(417, 6, 64, 64)
        c.x[2] = 0
        codes, exps = run_mx(c)
        assert not codes[2].any() and not exps[2].any()


@pytest.mark.parametrize("mode", ["5", "6"])
@pytest.mark.parametrize("tpw", ["2", "4", "8"])
def test_mxfp4_wave_per_token_kernel(tuning, mode, tpw):
    # 64-wide rows take the wave-per-token kernel with the MXFP4 quantizer (5: one token per wave, 6: persistent loop);
    # row-major exponents against the oracle, the tile order against the row-major output
    tuning("FLATQUANT_MODE", mode)
    tuning("FLATQUANT_WAVE_TPW", tpw)
    c = synth.prefill_7b(2048 + 37)
    run_mx(c, rows=subset_rows(c.T, 200, 21, must=(0, 1, 7, 8, 2047, 2048, 2084)))
    c = synth.generic(500 + int(mode), 4099, 32, 64, clip_mode=1)
    run_mx(c, rows=subset_rows(c.T, 160, 22, must=(0, 4095, 4096, 4098)))
    for T in (1, 3, 9, 130):
        run_mx(synth.generic(510 + T, T, 64, 64))
    c = synth.generic(533, 40, 64, 64)
    c.x[3] = 0
    codes, exps = run_mx(c)
    assert not codes[3].any() and not exps[3].any()
    for n1, T in ((64, 300), (32, 1029), (64, 2600)):
        test_mxfp4_tiled_exponents_equal_row_major(n1, 64, T)


@pytest.mark.parametrize("n1,n2,T", [(64, 172, 70), (64, 172, 2049), (10, 48, 33), (3, 32, 7), (64, 34, 300), (86, 16, 129), (128, 130, 40), (1, 32, 5)])
def test_mxfp4_output_general_kernel(n1, n2, T):
    """Right factors that are not a multiple of 32 (a block of 32 channels then straddles rows of X~; 64 x 172 is the
    paper's other factorization of 11008), and rows of fewer than 128 channels: the general kernel stages Y in LDS and
    quantizes block by block.  Row-major exponents against the oracle; the tile order, where the row has whole groups of
    256 channels, against the row-major output."""
    c = synth.generic(1700 + n1 + n2 + T, T, n1, n2, clip_mode=T % 2)
    print(f"[case] mxfp4 general kernel {n1}x{n2} T={T}", flush=True)
    run_mx(c, rows=None if T <= 300 else subset_rows(T, 100, 5, must=(0, 1, 2047, 2048, T - 1)))
    if (n1 * n2) % 256 == 0:
        test_mxfp4_tiled_exponents_equal_row_major(n1, n2, T)


def test_mxfp4_bottom_of_the_exponent_range():
    """Blocks whose clipped maximum lies below 2^-124 store exponent 0 (scale 2^-127, the smallest the format has) and
    their elements are converted with that scale; just above, exponents 1, 2, ...  Reached here through a tiny
    clipping threshold (it multiplies the block maximum before the exponent is taken)."""
    c = synth.generic(431, 24, 64, 64, clip_mode=1)
    c.clip[:] = np.float32(2.0) ** -np.arange(100, 124).astype(np.float32)   # alpha * max from about 2^-97 down to 2^-121
    c.x[:] = (c.x.astype(np.float32) * 2.0 ** -6).astype(np.float16)          # block maxima around 2^-6 .. 2^2
    codes, exps = run_mx(c)
    assert exps.min() <= 2 and exps.max() >= 20, (exps.min(), exps.max())    # the case does reach the bottom


def _grid_cases():
    """Left factors around every row-tile edge x right factors of every slab count x token counts below, at and above
    what is resident at once (a seeded selection of the full grid: every value of each axis appears several times)."""
    n1s = [1, 2, 3, 4, 31, 32, 33, 48, 63, 64, 65, 95, 96, 97, 127, 128]
    n2s = [32, 64, 96, 128, 160, 192, 224, 256, 2, 34, 130]
    Ts = [1, 2, 63, 300, 2049, 2600, 5000]
    r = np.random.Generator(np.random.PCG64(20241009))
    cases = set()
    for n1 in n1s:
        for n2 in r.choice(n2s, size=4, replace=False):
            cases.add((int(n1), int(n2), int(r.choice(Ts))))
    for n2 in n2s:
        for n1 in r.choice(n1s, size=3, replace=False):
            cases.add((int(n1), int(n2), int(r.choice(Ts))))
    # wide rows: fewer tokens (host-side generation time), still more than the workgroups resident for those shapes
    cases = {(n1, n2, min(T, max(600, 20_000_000 // (n1 * n2)))) for n1, n2, T in cases}
    return sorted(c for c in cases if (c[0] * c[1]) % 2 == 0)


@pytest.mark.parametrize("n1,n2,T", _grid_cases())
def test_shape_grid(n1, n2, T):
    """Codes and steps against the oracle's factored form of Eq. (2) (pinned to the dense Kronecker form on the CPU) on a
    subset of rows: the first and last tokens of the launch and of the first workgroups' second round."""
    c = synth.generic(7 * n1 + 13 * n2 + T, T, n1, n2, sigma=0.05 if n1 * n2 > 64 else 0.3)
    print(f"[case] grid {n1}x{n2} T={T}", flush=True)
    codes, scales, _, _ = run_tq(dev(c.x), dev(c.P1), dev(c.P2), dev(c.clip), c.clip_mode, n1, n2)
    rows = subset_rows(T, 96, n1 + n2, must=(0, 1, 2047, 2048, 2049, T - 2))
    y = fo.affine_transform_factored(c.x[rows], c.P1, c.P2)
    rep = parity.check_sym(y, c.clip[rows], codes[rows], scales[rows], rows=rows)
    print(f"[parity] {rep}", flush=True)
    assert rep["band_flips"] <= parity.band_flip_allowance(rep["in_band"])


# ---- KV-cache variant --------------------------------------------------------------------
def run_kv(kv, P, Hp, clip, bits=None):
    T, H, D = kv.shape
    G = T * H
    nb = G * D * (bits or 4) // 8
    kvd, Pd = dev(kv), dev(P)
    codes = torch.full((nb + 128,), 0xCD, dtype=torch.uint8, device="cuda")
    sc = torch.full((G + 64,), -1.0, dtype=torch.float16, device="cuda")
    zr = torch.full((G + 64,), -1.0, dtype=torch.float16, device="cuda")
    if bits is None:
        fq.flatquant_kv_transform_quant(kvd, Pd, Hp, clip, T, H, D, codes, sc, zr, stream=torch.cuda.current_stream())
    else:
        fq.flatquant_kv_transform_quant_bits(kvd, Pd, Hp, clip, bits, T, H, D, codes, sc, zr, stream=torch.cuda.current_stream())
    torch.cuda.synchronize()
    assert bool((codes[nb:] == 0xCD).all()) and bool((sc[G:] == -1).all()) and bool((zr[G:] == -1).all())
    deq = run_dequant(codes, sc, zr, G, D, bits)
    from gpu_util import host_f16
    return codes[:nb].cpu().numpy().reshape(G, nb // G), host_f16(sc[:G]), host_f16(zr[:G]), deq


@pytest.mark.parametrize("T,H,shared", [(32768, 8, False), (1, 8, False), (77, 3, False), (200, 8, True), (33, 1, True)])
def test_kv_cache(T, H, shared):
    kv = synth.kv_cache(T=T, H=H)
    P = kv.P[:1] if shared else kv.P
    for name, tensor in (("K", kv.k), ("V", kv.v)):
        print(f"[case] kv {name} T={T} H={H} shared={shared}", flush=True)
        codes, sc, zr, deq = run_kv(tensor, P, P.shape[0], kv.clip)
        y = fo.kv_transform(tensor, P).reshape(T * H, kv.D)
        rep = parity.check_kv(y, kv.clip, codes, sc, zr, deq_dev=deq)
        print(f"[parity] kv {name}: {rep}", flush=True)


def test_kv_ties_round_to_even_before_the_zero_point():
    """q = clamp(rne(y / s) + z): the rounding acts on y / s alone.  With P = I and clip = 1 a group whose range is
    [-3, 12] has step 1 and zero point 3 (odd): the exact ties k + 0.5 must go to the even neighbour of k + 0.5 and then
    be shifted, not to the even neighbour of k + 3.5.  Bit-exact against the oracle (no band)."""
    D, H = 128, 2
    vals = np.array([-3.0, 12.0] + [k + 0.5 for k in range(-3, 12)] + [0.0, 1.0, -1.0, 2.25, 7.75], dtype=np.float64)
    kv = np.zeros((5, H, D), dtype=np.float16)
    for t in range(5):
        for hh in range(H):
            row = np.zeros(D)
            row[:len(vals)] = vals
            row = np.roll(row, 7 * t + 3 * hh)
            if hh == 1:
                row[row == -3.0] = -5.0      # head 1: range [-5, 12] -> step 17/15 is no power of two: no exact ties, z = rne(5 / s)
            kv[t, hh] = row
    P = np.broadcast_to(np.eye(D, dtype=np.float16), (H, D, D)).copy()
    for bits in (None, 3):
        codes, sc, zr, _ = run_kv(kv, P, H, 1.0, bits)
        res = fo.kv_transform_quant(kv, P, 1.0, bits or 4)
        G = 5 * H
        if bits is None:
            assert np.all(sc.reshape(5, H)[:, 0] == 1.0) and np.all(zr.reshape(5, H)[:, 0] == 3.0)
        assert np.array_equal(sc, res["scales"].reshape(G)) and np.array_equal(zr.astype(np.float64), res["zeros"].reshape(G).astype(np.float64))
        assert np.array_equal(codes, res["codes"].reshape(G, -1)), "tie handling differs from rne(y / s) + z"


@pytest.mark.parametrize("bits", [4, 3])
@pytest.mark.parametrize("T,H", [(31, 2), (32, 5), (33, 16), (64, 40), (127, 1), (129, 2), (1000, 5), (3, 33), (4097, 3)])
def test_kv_cache_token_and_head_counts(bits, T, H):
    """Token counts around the 32-token step of a wave and head counts that are not powers of two."""
    kv = synth.kv_cache(T=T, H=H)
    shared = (T + H) % 2 == 0
    P = kv.P[:1] if shared else kv.P
    print(f"[case] kv bits={bits} T={T} H={H} shared={shared}", flush=True)
    codes, sc, zr, deq = run_kv(kv.k, P, P.shape[0], kv.clip, bits)
    y = fo.kv_transform(kv.k, P).reshape(T * H, kv.D)
    rep = parity.check_kv(y, kv.clip, codes, sc, zr, deq_dev=deq, bits=bits)
    print(f"[parity] {rep}", flush=True)


@pytest.mark.parametrize("bits,T,H", [(4, 1000, 8), (3, 33, 5), (2, 4097, 3), (4, 31, 40), (None, 700, 8)])
def test_shared_head_matrix_folded_or_not(tuning, bits, T, H):
    """One P_h for all heads: the library treats the groups as T * H rows of a single head; head by head (forced) must
    give the same bits.  bits = None: the fp16-out transform."""
    kv = synth.kv_cache(T=T, H=H)
    P = kv.P[:1]
    res = []
    for fold in (1, 0):
        tuning("FLATQUANT_KV_FOLD_HEADS", fold)
        if bits is None:
            out = torch.full((T * H * kv.D,), float("nan"), dtype=torch.float16, device="cuda")
            fq.flatquant_head_transform(dev(kv.k), dev(P), 1, T, H, kv.D, out, stream=torch.cuda.current_stream())
            torch.cuda.synchronize()
            res.append((out.cpu().view(torch.int16).numpy(),))
        else:
            codes, sc, zr, _ = run_kv(kv.k, P, 1, kv.clip, bits)
            res.append((codes, sc.view(np.uint16), zr.view(np.uint16)))
    for a, b in zip(*res):
        assert np.array_equal(a, b)


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("T,H,shared", [(4096 + 5, 8, False), (1, 8, False), (77, 3, False), (33, 1, True)])
def test_kv_cache_lower_bits(bits, T, H, shared):
    """Key / value caches at 2, 3 and 4 bits through the width-parametrised entry point (4 must equal the INT4 one)."""
    kv = synth.kv_cache(T=T, H=H)
    P = kv.P[:1] if shared else kv.P
    for name, tensor in (("K", kv.k), ("V", kv.v)):
        print(f"[case] kv {name} bits={bits} T={T} H={H} shared={shared}", flush=True)
        codes, sc, zr, deq = run_kv(tensor, P, P.shape[0], kv.clip, bits)
        assert codes.shape == (T * H, kv.D * bits // 8)
        y = fo.kv_transform(tensor, P).reshape(T * H, kv.D)
        rep = parity.check_kv(y, kv.clip, codes, sc, zr, deq_dev=deq, bits=bits)
        print(f"[parity] kv {name} {bits}-bit: {rep}", flush=True)
        if bits == 4:
            c4, s4, z4, _ = run_kv(tensor, P, P.shape[0], kv.clip)
            assert np.array_equal(c4, codes) and np.array_equal(s4.view(np.uint16), sc.view(np.uint16)) and np.array_equal(z4.view(np.uint16), zr.view(np.uint16))


def test_dequant_bits_helper():
    r = np.random.Generator(np.random.PCG64(4))
    for bits in (2, 3, 4):
        for rows, n in [(5, 8), (3, 128), (17, 256)]:
            q = r.integers(0, 1 << bits, size=(rows, n)).astype(np.uint8)
            codes = fo.pack_bits(q, bits)
            scales = (r.uniform(0.1, 4, rows)).astype(np.float16)
            zeros = r.integers(0, 1 << bits, rows).astype(np.float16)
            out = run_dequant(dev(codes), dev(scales), dev(zeros), rows, n, bits)
            assert np.array_equal(out.astype(np.float64), fo.dequantize(codes, scales, zeros, bits))


def test_dequant_helper_ragged():
    r = np.random.Generator(np.random.PCG64(3))
    for rows, n in [(5, 6), (3, 2), (17, 250), (4, 4096)]:
        codes = r.integers(0, 256, size=(rows, n // 2), dtype=np.uint8)
        scales = (r.uniform(0.1, 4, rows)).astype(np.float16)
        zeros = r.integers(0, 16, rows).astype(np.float16)
        out = run_dequant(dev(codes), dev(scales), None, rows, n)
        assert np.array_equal(out.astype(np.float64), fo.dequantize(codes, scales))
        out = run_dequant(dev(codes), dev(scales), dev(zeros), rows, n)
        assert np.array_equal(out.astype(np.float64), fo.dequantize(codes, scales, zeros))


@pytest.mark.gpu
@pytest.mark.parametrize("T,n,pad", [(2048, 4096, 0), (5000, 4096, 64), (7, 8192, 0), (3, 32, 32)])
def test_stream_probe_moves_every_byte_once(T, n, pad):
    """The measurement aid folds each row's four quarters with xor: every input byte reaches exactly one output byte."""
    rng = np.random.default_rng(77)
    x = rng.integers(0, 65536, size=(T, n + pad), dtype=np.uint16)
    xd = torch.from_numpy(x.view(np.int16)).cuda()
    out = torch.full((64 + T * (n // 2) + 64,), 0xCD, dtype=torch.uint8, device="cuda")
    fq.flatquant_stream_probe(xd, T, n, n + pad, out[64:], stream=torch.cuda.current_stream())
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert (got[:64] == 0xCD).all() and (got[-64:] == 0xCD).all()
    q = n // 4
    v = x[:, :n]
    want = v[:, :q] ^ v[:, q:2 * q] ^ v[:, 2 * q:3 * q] ^ v[:, 3 * q:]
    assert np.array_equal(got[64:-64].view(np.uint16).reshape(T, q), want)


# ---- weight side of Eq. (2) and the whole quantized layer ----------------------------------------------------------
def _layer_case(T, m, n1, n2, config_index, seed):
    c = synth.generic(seed, T, n1, n2, sigma=0.05, clip_mode=1)
    W = synth.weights(config_index, m, n1 * n2)
    cw = synth.weight_clip(config_index, m)
    A1, r1 = fq.fq_inverse_transpose(c.P1)
    A2, r2 = fq.fq_inverse_transpose(c.P2)
    print(f"[layer] T={T} m={m} {n1}x{n2}: inverse residuals {r1:.2e} {r2:.2e}", flush=True)
    return c, W, cw, A1, A2


@pytest.mark.parametrize("T,m,n1,n2", [(96, 300, 64, 64), (40, 130, 32, 64), (33, 70, 86, 128)])
def test_weight_side_parity_and_quantized_layer(T, m, n1, n2):
    """Right factor of Eq. (2) through the C ABI against the oracle (same fp16 inverse-transposed factors on both
    sides), then the product of the two de-quantized factors against X W^T."""
    n = n1 * n2
    c, W, cw, A1, A2 = _layer_case(T, m, n1, n2, 9, 700 + n1)
    Wd, A1d, A2d, cwd = dev(W), dev(A1), dev(A2), dev(cw)
    wcodes = torch.full((m, n // 2), 0xCD, dtype=torch.uint8, device="cuda")
    wsc = torch.full((m,), -1.0, dtype=torch.float16, device="cuda")
    fq.flatquant_weight_transform_quant(Wd, A1d, A2d, cwd, 1, m, n1, n2, n, wcodes, wsc, stream=torch.cuda.current_stream())
    torch.cuda.synchronize()
    yw = fo.weight_transform_factored(W, A1, A2)
    rep = parity.check_sym(yw, cw, wcodes.cpu().numpy(), wsc.cpu().numpy().view(np.float16))
    print(f"[parity] weight side {n1}x{n2}: {rep}", flush=True)
    assert rep["band_flips"] <= parity.band_flip_allowance(rep["in_band"])

    # activation side, then the layer: deq(Q(XP)) deq(Q(P^-1 W^T)) vs X W^T
    xcodes, xsc, xcodes_d, xsc_d = run_tq(dev(c.x), dev(c.P1), dev(c.P2), dev(c.clip), 1, n1, n2)
    xq = run_dequant(xcodes_d, xsc_d, None, T, n).astype(np.float64)
    wq = run_dequant(wcodes, wsc, None, m, n).astype(np.float64)
    Yq = xq @ wq.T
    Y = c.x.astype(np.float64) @ W.astype(np.float64).T
    # oracle's quantized layer from the oracle's own codes: the two must agree up to the in-band code differences
    ox = fo.transform_quant(c.x, c.P1, c.P2, c.clip)
    ow = fo.weight_transform_quant(W, A1, A2, cw)
    Yo = fo.quantized_linear(ox["codes"], ox["scales"], ow["codes"], ow["scales"])
    sx, sw = fo.as_f64(ox["scales"]), fo.as_f64(ow["scales"])
    flips_x = (fo.unpack_nibbles(xcodes, True) != ox["q"]).sum(1)
    flips_w = (fo.unpack_nibbles(wcodes.cpu().numpy(), True) != ow["q"]).sum(1)
    # a flipped code moves one factor by one step: |dY| <= flips_x s_x max|w^| + flips_w s_w max|x^| (+ product term)
    slack = (flips_x[:, None] * sx[:, None] * 8 * sw[None, :] + flips_w[None, :] * sw[None, :] * 8 * sx[:, None]) + 1e-6 * np.abs(Yo) + 1e-9
    assert np.all(np.abs(Yq - Yo) <= slack), float(np.abs(Yq - Yo).max())
    # how good W4A4 is with these untrained, random transforms is not a property of the kernels: reported only
    rel, rel_o = np.linalg.norm(Yq - Y) / np.linalg.norm(Y), np.linalg.norm(Yo - Y) / np.linalg.norm(Y)
    print(f"[layer] {n1}x{n2}: relative error of the W4A4 layer output {rel:.4f} (oracle's codes: {rel_o:.4f}); "
          f"code flips x {int(flips_x.sum())} w {int(flips_w.sum())}", flush=True)
    assert abs(rel - rel_o) <= 1e-3 * max(rel_o, 1e-6) + 1e-6 * (int(flips_x.sum()) + int(flips_w.sum()) + 1)


@pytest.mark.parametrize("n1,n2,T", [(64, 64, 1), (64, 64, 127), (64, 64, 128), (64, 64, 129), (86, 128, 300), (32, 256, 257), (4, 64, 640),
                                      (64, 64, 2600), (64, 128, 2100), (128, 256, 130)])
def test_mxfp4_tiled_exponents_equal_row_major(n1, n2, T):
    """Tile order of the exponents (what the MXFP4 product reads) against the row-major output of the same launch shape:
    same codes, same exponents after undoing the order, padding rows of the last tile untouched."""
    n = n1 * n2
    c = synth.generic(1300 + n1 + n2 + T, T, n1, n2)
    xd, P1, P2, cd = dev(c.x), dev(c.P1), dev(c.P2), dev(c.clip)
    c0 = torch.empty((T, n // 2), dtype=torch.uint8, device="cuda")
    e0 = torch.empty((T, n // 32), dtype=torch.uint8, device="cuda")
    c1 = torch.empty((T, n // 2), dtype=torch.uint8, device="cuda")
    e1 = torch.full((fq.fq_mxfp4_tiled_scale_bytes(T, n) + 64,), 0xFF, dtype=torch.uint8, device="cuda")
    st = torch.cuda.current_stream()
    print(f"[case] tiled exponents {n1}x{n2} T={T}", flush=True)
    fq.flatquant_transform_mxfp4(xd, P1, P2, cd, c.clip_mode, T, n1, n2, n, c0, e0, stream=st)
    fq.flatquant_transform_mxfp4_tiled(xd, P1, P2, cd, c.clip_mode, T, n1, n2, n, c1, e1, stream=st)
    torch.cuda.synchronize()
    assert torch.equal(c0, c1)
    e1h = e1.cpu().numpy()
    assert np.all(e1h[-64:] == 0xFF), "bytes past the tensor written"
    e1h = e1h[:-64]
    assert np.array_equal(fo.mx_untile_scales(e1h, T, n), e0.cpu().numpy())
    if T % 128:
        assert np.all(e1h.reshape(-1, n // 256, 128, 8)[-1, :, T % 128:, :] == 0xFF), "padding rows written"


def test_mxfp4_tiled_exponents_and_product_end_to_end():
    """The tile-ordered output equals the row-major one, and feeding it to the product reproduces the oracle's product of
    the same codes."""
    T, m, n1, n2 = 200, 136, 64, 64
    n = n1 * n2
    c, W, cw, A1, A2 = _layer_case(T, m, n1, n2, 9, 770)

    def both(xa, Pa, Pb, clip, rows):
        xd, Pad, Pbd, cd = dev(xa), dev(Pa), dev(Pb), dev(clip)
        c0 = torch.empty((rows, n // 2), dtype=torch.uint8, device="cuda")
        e0 = torch.empty((rows, n // 32), dtype=torch.uint8, device="cuda")
        c1 = torch.empty((rows, n // 2), dtype=torch.uint8, device="cuda")
        e1 = torch.full((fq.fq_mxfp4_tiled_scale_bytes(rows, n),), 0xFF, dtype=torch.uint8, device="cuda")
        st = torch.cuda.current_stream()
        fq.flatquant_transform_mxfp4(xd, Pad, Pbd, cd, 1, rows, n1, n2, n, c0, e0, stream=st)
        fq.flatquant_transform_mxfp4_tiled(xd, Pad, Pbd, cd, 1, rows, n1, n2, n, c1, e1, stream=st)
        torch.cuda.synchronize()
        assert torch.equal(c0, c1)
        e1h = e1.cpu().numpy()
        assert np.array_equal(fo.mx_untile_scales(e1h, rows, n), e0.cpu().numpy())
        pad = e1h.reshape(-1, n // 256, 128, 8)[-1, :, rows % 128 or 128:, :]
        assert np.all(pad == 0xFF), "padding rows written"
        return c1, e1, c0.cpu().numpy(), e0.cpu().numpy()

    xc, xe, xch, xeh = both(c.x, c.P1, c.P2, c.clip, T)
    wc, we, wch, weh = both(W, A1, A2, cw, m)
    out = torch.empty((T, m), dtype=torch.float16, device="cuda")
    fq.flatquant_mxfp4_gemm(xc, xe, wc, we, T, m, n, out, m, stream=torch.cuda.current_stream())
    torch.cuda.synchronize()
    got = out.cpu().view(torch.int16).numpy().view(np.float16).astype(np.float64)
    y, y16, ab = fo.mxfp4_gemm(xch, xeh, wch, weh)
    tol = 2.0 ** -11 * np.abs(y) * (1 + 2.0 ** -9) + n * 2.0 ** -24 * ab + 2.0 ** -25
    assert np.all(np.abs(got - y) <= tol)


def test_mxfp4_layer_both_factors():
    """The same two-factor layer with MXFP4 on both sides: the weight rows go through flatquant_transform_mxfp4 with
    the inverse-transposed factors; the product of the two de-quantized factors must agree with the oracle's."""
    T, m, n1, n2 = 96, 160, 64, 64
    n = n1 * n2
    c, W, cw, A1, A2 = _layer_case(T, m, n1, n2, 9, 760)

    def mx(xa, Pa, Pb, clip, rows):
        cbuf = torch.empty((rows, n // 2), dtype=torch.uint8, device="cuda")
        sbuf = torch.empty((rows, n // 32), dtype=torch.uint8, device="cuda")
        fq.flatquant_transform_mxfp4(dev(xa), dev(Pa), dev(Pb), dev(clip), 1, rows, n1, n2, n, cbuf, sbuf, stream=torch.cuda.current_stream())
        deq = torch.empty((rows, n), dtype=torch.float32, device="cuda")
        fq.flatquant_dequant_mxfp4(cbuf, sbuf, rows, n, deq, stream=torch.cuda.current_stream())
        torch.cuda.synchronize()
        return cbuf.cpu().numpy(), sbuf.cpu().numpy(), deq.cpu().numpy().astype(np.float64)

    xc, xe, xq = mx(c.x, c.P1, c.P2, c.clip, T)
    wc, we, wq = mx(W, A1, A2, cw, m)
    parity.check_mx(fo.affine_transform_factored(c.x, c.P1, c.P2), c.clip, xc, xe)
    parity.check_mx(fo.weight_transform_factored(W, A1, A2), cw, wc, we)
    ox = fo.transform_mxfp4(c.x, c.P1, c.P2, c.clip)
    qw, ew, _ = fo.mx_quantize(fo.weight_transform_factored(W, A1, A2), cw)
    xo = fo.dequantize_mxfp4(ox["codes"], ox["scales"])
    wo = fo.dequantize_mxfp4(fo.pack_nibbles(qw.astype(np.int8)), ew)
    Yq, Yo = xq @ wq.T, xo @ wo.T
    Y = c.x.astype(np.float64) @ W.astype(np.float64).T
    # elements that differ (rounding ties inside the comparator's band) move one factor by at most one grid step
    dx, dw = np.abs(xq - xo), np.abs(wq - wo)
    slack = dx.sum(1)[:, None] * np.abs(wo).max(1)[None, :] + dw.sum(1)[None, :] * np.abs(xo).max(1)[:, None] + dx.sum(1)[:, None] * dw.max(1)[None, :]
    assert np.all(np.abs(Yq - Yo) <= slack * (1 + 1e-9) + 1e-9 * np.abs(Yo) + 1e-12)
    rel, rel_o = np.linalg.norm(Yq - Y) / np.linalg.norm(Y), np.linalg.norm(Yo - Y) / np.linalg.norm(Y)
    print(f"[layer] MXFP4 x MXFP4 {n1}x{n2}: relative error of the layer output {rel:.4f} (oracle's codes: {rel_o:.4f}); "
          f"elements that differ x {int((dx > 0).sum())} w {int((dw > 0).sum())}", flush=True)
    assert abs(rel - rel_o) <= 1e-3 * rel_o + 1e-6 * (int((dx > 0).sum()) + int((dw > 0).sum()) + 1)


@pytest.mark.parametrize("T,m,n", [(128, 128, 256), (200, 300, 1280), (2048, 256, 4096), (1, 40, 768), (130, 129, 11008), (64, 4096, 1024), (300, 140, 512),
                                   (8, 200, 256), (16, 300, 2304), (17, 129, 11008), (33, 4099, 512), (50, 96, 4096), (64, 11008, 4096), (3, 8200, 1024),
                                   (65, 100, 2304), (128, 4100, 1024), (100, 40, 11008), (129, 70, 512), (70, 8300, 256)])
def test_mxfp4_gemm(T, m, n):
    _mxfp4_gemm_case(T, m, n)


@pytest.mark.parametrize("waves,depth,rows,T,m,n", [(16, 1, 32, 5, 100, 4096), (16, 2, 16, 64, 70, 2304), (4, 3, 32, 20, 330, 11008), (8, 8, 16, 40, 64, 4096),
                                                    (4, 1, 16, 1, 33, 256), (8, 2, 32, 9, 8200, 512), (8, 2, 16, 12, 8200, 512), (4, 2, 32, 64, 4096, 1024), (16, 3, 32, 120, 200, 2304), (4, 2, 16, 90, 100, 1024)])
@pytest.mark.parametrize("kind", ["int4", "mxfp4"])
def test_few_token_products_every_launch_shape(tuning, kind, waves, depth, rows, T, m, n):
    """The few-token kernels give a workgroup 16 or 32 output channels and split K over 4, 8 or 16 waves with rings of
    1 to 8 line slots; the library picks one shape per launch, the others are forced here (a depth the ring cannot hold
    is cut back by the launcher)."""
    tuning("FLATQUANT_GEMM_WAVES", waves)
    tuning("FLATQUANT_GEMM_DEPTH", depth)
    tuning("FLATQUANT_GEMM_ROWS", rows)
    if kind == "int4":
        _w4a4_case(T, m, n, 0)
    else:
        _mxfp4_gemm_case(T, m, n)


@pytest.mark.parametrize("kind", ["int4", "mxfp4"])
@pytest.mark.parametrize("T,m,n", [(129, 100, 512), (200, 4100, 1024), (333, 70, 2304), (512, 64, 11008)])
def test_ring_products_on_several_token_tiles(tuning, kind, T, m, n):
    """Past 128 tokens the ring kernels run on tiles of 64 tokens (second grid dimension); forced here for any T."""
    tuning("FLATQUANT_GEMM_RING_MAX_T", 1 << 20)
    if kind == "int4":
        _w4a4_case(T, m, n, 0)
    else:
        _mxfp4_gemm_case(T, m, n)


def _product_grid():
    Ts = [1, 7, 8, 9, 16, 17, 32, 33, 64, 65, 127, 128, 129, 191, 193, 256, 257, 500, 1100]
    ms = [1, 15, 16, 17, 31, 32, 33, 127, 128, 129, 255, 257, 1000, 4100]
    ns = [256, 512, 768, 1280, 4096, 11008]
    r = np.random.Generator(np.random.PCG64(9426))
    cases = set()
    for T in Ts:
        for _ in range(3):
            cases.add((T, int(r.choice(ms)), int(r.choice(ns))))
    for m in ms:
        for _ in range(2):
            cases.add((int(r.choice(Ts)), m, int(r.choice(ns))))
    return sorted(c for c in cases if c[0] * c[1] * c[2] <= 1_500_000_000)


@pytest.mark.parametrize("T,m,n", _product_grid())
@pytest.mark.parametrize("kind", ["int4", "mxfp4"])
def test_product_grid(kind, T, m, n):
    """Token and channel counts around every tile edge of the ring kernels (8, 16, 32, 64 tokens; 16, 32 channels) and
    of the tiled kernels (128, 256), in the launch shape the library picks by itself."""
    if kind == "int4":
        _w4a4_case(T, m, n, 0)
    else:
        _mxfp4_gemm_case(T, m, n)


@pytest.mark.parametrize("kind", ["int4", "mxfp4"])
@pytest.mark.parametrize("T,m", [(5, 33), (64, 100), (150, 40), (700, 130)])
def test_products_at_the_longest_rows(kind, T, m):
    """n = 65536: the longest row the INT4 product accepts (its int32 sums reach 2^30), 256 lines per row for the ring
    kernels and 256 iterations for the tiled ones."""
    if kind == "int4":
        _w4a4_case(T, m, 65536, 0)
    else:
        _mxfp4_gemm_case(T, m, 65536)


@pytest.mark.parametrize("knob,value", [("FLATQUANT_GEMM_WAVES", 5), ("FLATQUANT_GEMM_DEPTH", 0), ("FLATQUANT_GEMM_DEPTH", 9), ("FLATQUANT_GEMM_ROWS", 24)])
def test_ring_kernel_overrides_out_of_range_are_launch_errors(tuning, knob, value):
    """A tuning override the ring kernels cannot honour is reported (no launch, outputs untouched), not silently replaced."""
    tuning(knob, value)
    T, m, n = 8, 64, 512
    z = lambda *shape: torch.zeros(shape, dtype=torch.uint8, device="cuda")
    out = torch.full((T, m), float("nan"), dtype=torch.float16, device="cuda")
    sx = torch.ones((T,), dtype=torch.float16, device="cuda")
    sw = torch.ones((m,), dtype=torch.float16, device="cuda")
    assert fq.flatquant_w4a4_gemm(z(T, n // 2), sx, z(m, n // 2), sw, T, m, n, out, m, stream=torch.cuda.current_stream(), check=False) == fq.FQ_LAUNCH_FAILED
    assert fq.flatquant_mxfp4_gemm(z(T, n // 2), z(fq.fq_mxfp4_tiled_scale_bytes(T, n)), z(m, n // 2), z(fq.fq_mxfp4_tiled_scale_bytes(m, n)), T, m, n, out, m,
                                   stream=torch.cuda.current_stream(), check=False) == fq.FQ_LAUNCH_FAILED
    assert fq.last_hip_error() != 0
    torch.cuda.synchronize()
    assert bool(torch.isnan(out).all())


def test_int4_product_rows_do_not_depend_on_the_launch(tuning):
    """Integer sums and one fixed order of the two fp32 multiplications: a token's output row has the same bits whether it
    is computed alone, among 40 tokens (ring kernel), among 700 (tiled kernel) or by any forced form."""
    r = np.random.Generator(np.random.PCG64(77))
    T, m, n = 700, 200, 2304
    cx = dev(r.integers(0, 256, size=(T, n // 2), dtype=np.uint8))
    cw = dev(r.integers(0, 256, size=(m, n // 2), dtype=np.uint8))
    sx = dev(r.uniform(0.01, 2.0, size=T).astype(np.float16))
    sw = dev(r.uniform(0.001, 0.02, size=m).astype(np.float16))
    def run(Tn):
        out = torch.empty((Tn, m), dtype=torch.float16, device="cuda")
        fq.flatquant_w4a4_gemm(cx, sx, cw, sw, Tn, m, n, out, m, stream=torch.cuda.current_stream())
        torch.cuda.synchronize()
        return out.cpu().view(torch.int16).numpy()
    full = run(T)
    for Tn in (1, 8, 40, 64, 130, 300):
        assert np.array_equal(run(Tn), full[:Tn]), f"rows differ between T={Tn} and T={T}"
    tuning("FLATQUANT_GEMM_TILED", 1)
    assert np.array_equal(run(40), full[:40])
    tuning("FLATQUANT_GEMM_RING_MAX_T", 1 << 20)
    tuning("FLATQUANT_GEMM_TILED", 0)
    assert np.array_equal(run(T), full)


def test_mxfp4_product_is_reproducible():
    r = np.random.Generator(np.random.PCG64(78))
    for T, m, n in ((40, 200, 2304), (700, 200, 2304)):
        xc = dev(r.integers(0, 256, size=(T, n // 2), dtype=np.uint8))
        wc = dev(r.integers(0, 256, size=(m, n // 2), dtype=np.uint8))
        xe = dev(fo.mx_tile_scales(r.integers(118, 131, size=(T, n // 32), dtype=np.uint8), fill=0xFF))
        we = dev(fo.mx_tile_scales(r.integers(112, 126, size=(m, n // 32), dtype=np.uint8), fill=0xFF))
        outs = []
        for _ in range(3):
            out = torch.empty((T, m), dtype=torch.float16, device="cuda")
            fq.flatquant_mxfp4_gemm(xc, xe, wc, we, T, m, n, out, m, stream=torch.cuda.current_stream())
            torch.cuda.synchronize()
            outs.append(out.cpu().view(torch.int16).numpy())
        assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])


def test_few_token_mxfp4_product_tiled_form(tuning):
    tuning("FLATQUANT_GEMM_TILED", 1)
    _mxfp4_gemm_case(40, 200, 1024)


def _mxfp4_gemm_case(T, m, n):
    """Scaled-FP4 matrix product against the oracle's fp64 product of the de-quantized factors.  Products are exact; the
    fp32 accumulation may lose up to n * 2^-24 of sum |x^ w^|, and the result is rounded once to fp16."""
    r = np.random.Generator(np.random.PCG64(1000 + T + m + n))
    xc = r.integers(0, 256, size=(T, n // 2), dtype=np.uint8)
    wc = r.integers(0, 256, size=(m, n // 2), dtype=np.uint8)
    xe = r.integers(118, 131, size=(T, n // 32), dtype=np.uint8)
    we = r.integers(112, 126, size=(m, n // 32), dtype=np.uint8)
    print(f"[case] mxfp4 gemm T={T} m={m} n={n}", flush=True)
    stride = m + 8
    out = torch.full((T, stride), float("nan"), dtype=torch.float16, device="cuda")
    xet, wet = fo.mx_tile_scales(xe, fill=0xFF), fo.mx_tile_scales(we, fill=0xFF)   # padding rows: NaN scales, must not leak
    assert xet.size == fq.fq_mxfp4_tiled_scale_bytes(T, n) and wet.size == fq.fq_mxfp4_tiled_scale_bytes(m, n)
    fq.flatquant_mxfp4_gemm(dev(xc), dev(xet), dev(wc), dev(wet), T, m, n, out, stride, stream=torch.cuda.current_stream())
    torch.cuda.synchronize()
    got_all = out.cpu().view(torch.int16).numpy().view(np.float16)
    assert np.all(np.isnan(got_all[:, m:])), "padding columns overwritten"
    got = got_all[:, :m].astype(np.float64)
    y, y16, ab = fo.mxfp4_gemm(xc, xe, wc, we)
    assert np.all(np.isfinite(got))
    tol = 2.0 ** -11 * np.abs(y) * (1 + 2.0 ** -9) + n * 2.0 ** -24 * ab + 2.0 ** -25
    err = np.abs(got - y)
    assert np.all(err <= tol), f"max err/tol {float((err / tol).max()):.3f}"
    same = float(np.mean(got == y16.astype(np.float64)))
    print(f"[parity] mxfp4 gemm: identical to the once-rounded fp64 result in {same * 100:.2f} % of the outputs", flush=True)
    assert same > 0.9


# ---- one-sided transforms (a factor left out = identity) ------------------------------------------------------------
@pytest.mark.parametrize("n1,n2,T,which", [(32, 128, 200, "P1 only"), (32, 128, 3000, "P1 only"), (64, 64, 2048, "P1 only"),
                                           (64, 128, 2500, "P1 only"), (64, 128, 129, "P1 only"), (32, 128, 1, "P1 only"),
                                           (64, 64, 70, "P2 only"), (86, 128, 37, "P2 only"), (64, 64, 50, "none"),
                                           (33, 34, 21, "P1 only"), (6, 10, 9, "P2 only")])
def test_one_sided_transforms(n1, n2, T, which):
    """P_o's online part is the left factor alone (heads x heads, Sec. 3.2): a null factor must act as the identity."""
    c = synth.generic(800 + n1 + n2, T, n1, n2)
    use1, use2 = which in ("P1 only",), which in ("P2 only",)
    P1 = c.P1 if use1 else np.eye(n1, dtype=np.float16)
    P2 = c.P2 if use2 else np.eye(n2, dtype=np.float16)
    print(f"[case] one-sided {which} {n1}x{n2} T={T}", flush=True)
    codes, scales, _, _ = run_tq(dev(c.x), dev(c.P1) if use1 else None, dev(c.P2) if use2 else None, dev(c.clip), c.clip_mode, n1, n2)
    rows = subset_rows(T, 200, 31)
    y = fo.affine_transform(c.x[rows], P1, P2)
    rep = parity.check_sym(y, c.clip[rows], codes[rows], scales[rows], rows=rows)
    print(f"[parity] one-sided {which}: {rep}", flush=True)
    assert rep["band_flips"] <= parity.band_flip_allowance(rep["in_band"])


@pytest.mark.parametrize("mode", ["5", "0", "3"])
@pytest.mark.parametrize("n1,T", [(32, 2048 + 3), (32, 1), (32, 9), (64, 2500), (64, 130), (32, 9001)])
def test_left_factor_only_every_kernel(tuning, mode, n1, T):
    """128-wide rows with the left factor alone: the wave-per-token kernel (5) and the slab kernels' persistent loop (0)
    and loop-free launch (3), each forced (the default picks by token count); a zero row and large magnitudes included."""
    tuning("FLATQUANT_MODE", mode)
    c = synth.generic(860 + n1 + T, T, n1, 128)
    if T > 8:
        c.x[3] = 0
        c.x[5] = (np.sign(c.x[5].astype(np.float32)) * 700).astype(np.float16)
    print(f"[case] left factor only, mode {mode}, {n1}x128 T={T}", flush=True)
    codes, scales, _, _ = run_tq(dev(c.x), dev(c.P1), None, dev(c.clip), c.clip_mode, n1, 128)
    rows = subset_rows(T, 200, 33, must=(0, 3, 5, T - 1))
    y = fo.affine_transform_factored(c.x[rows], c.P1, np.eye(128, dtype=np.float16))
    rep = parity.check_sym(y, c.clip[rows], codes[rows], scales[rows], rows=rows)
    print(f"[parity] {rep}", flush=True)
    assert rep["band_flips"] <= parity.band_flip_allowance(rep["in_band"])


def _one_sided_grid():
    r = np.random.Generator(np.random.PCG64(2718))
    cases = set()
    for n1 in [1, 2, 31, 32, 33, 64, 65, 96, 128]:
        for n2 in [32, 64, 128, 160, 256, 34, 2]:
            if (n1 * n2) % 2 == 0 and r.random() < 0.55:
                T = int(r.choice([1, 2, 63, 300, 2049, 2600]))
                which = str(r.choice(["P1 only", "P2 only", "none"]))
                cases.add((n1, n2, min(T, max(600, 20_000_000 // (n1 * n2))), which))
    return sorted(cases)


@pytest.mark.parametrize("n1,n2,T,which", _one_sided_grid())
def test_one_sided_shape_grid(n1, n2, T, which):
    c = synth.generic(900 + 3 * n1 + n2 + T, T, n1, n2, sigma=0.05 if n1 * n2 > 64 else 0.3)
    use1, use2 = which == "P1 only", which == "P2 only"
    P1 = c.P1 if use1 else np.eye(n1, dtype=np.float16)
    P2 = c.P2 if use2 else np.eye(n2, dtype=np.float16)
    print(f"[case] one-sided grid {which} {n1}x{n2} T={T}", flush=True)
    codes, scales, _, _ = run_tq(dev(c.x), dev(c.P1) if use1 else None, dev(c.P2) if use2 else None, dev(c.clip), c.clip_mode, n1, n2)
    rows = subset_rows(T, 100, 32, must=(0, 1, 2047, 2048, T - 2))
    y = fo.affine_transform_factored(c.x[rows], P1, P2)
    rep = parity.check_sym(y, c.clip[rows], codes[rows], scales[rows], rows=rows)
    print(f"[parity] {rep}", flush=True)
    assert rep["band_flips"] <= parity.band_flip_allowance(rep["in_band"])


@pytest.mark.parametrize("T,H,shared", [(4096, 8, False), (1, 8, False), (77, 3, False), (200, 8, True), (31, 2, True), (32, 5, False), (33, 16, True),
                                        (127, 1, False), (129, 2, True), (1000, 5, False), (3, 33, False), (4097, 3, True), (64, 40, False)])
def test_head_transform_fp16_out(T, H, shared):
    """Query side of a transformed key cache: fp16(x P_h) against the oracle's single rounding of the fp64 product.
    Tolerance from the arithmetic: fp32 accumulation of 128 exact fp16 products (<= 128 * 2^-24 of the sum of their
    magnitudes) plus one fp16 rounding (2^-11 relative, + 2^-25 in the subnormal range)."""
    D = 128
    c = synth.kv_cache(T, H, D)
    Pq = np.stack([fq.fq_inverse_transpose(c.P[h])[0] for h in range(H)])
    if shared:
        Pq = Pq[:1]
    xd, Pd = dev(c.k), dev(Pq)
    out = torch.full((T * H * D + 64,), float("nan"), dtype=torch.float16, device="cuda")
    fq.flatquant_head_transform(xd, Pd, Pq.shape[0], T, H, D, out, stream=torch.cuda.current_stream())
    torch.cuda.synchronize()
    got = out.cpu().view(torch.int16).numpy().view(np.float16)
    assert np.all(np.isnan(got[T * H * D:]))
    got = got[:T * H * D].reshape(T, H, D).astype(np.float64)
    rows = subset_rows(T, 256, 41)
    y = fo.kv_transform(c.k[rows], Pq)
    mag = np.einsum("thd,hde->the", np.abs(c.k[rows].astype(np.float64)), np.abs(np.broadcast_to(Pq, (H, D, D)).astype(np.float64)))
    tol = 2.0 ** -11 * np.abs(y) * (1 + 2.0 ** -10) + 128 * 2.0 ** -24 * mag + 2.0 ** -25
    err = np.abs(got[rows] - y)
    assert np.all(err <= tol), float((err / tol).max())
    exact = (got[rows] == fo.head_transform_fp16(c.k[rows], Pq).astype(np.float64)).mean()
    print(f"[parity] head transform T={T} H={H}: max err/tol {float((err / tol).max()):.3f}, identical to the oracle's fp16 in {exact * 100:.2f} % of elements", flush=True)
    assert exact > 0.97


# ---- W4A4 matrix product ------------------------------------------------------------------------------------------------
def _w4a4_case(T, m, n, pad):
    """Integer accumulation is exact, so the only freedom is the final rounding: two fp32 multiplications and one fp16
    rounding against the oracle's single rounding of the fp64 value (2^-11 relative + two fp32 roundings)."""
    r = np.random.Generator(np.random.PCG64(900 + T + m + n))
    cx = r.integers(0, 256, size=(T, n // 2), dtype=np.uint8)
    cw = r.integers(0, 256, size=(m, n // 2), dtype=np.uint8)
    cx[0, :] = 0x88      # every code -8: the largest magnitude sums
    cw[0, :] = 0x88
    sx = r.uniform(0.01, 4.0, size=T).astype(np.float16)
    sw_hi = 0.2 * 256 / n                                                # keeps 64 n s_x s_w inside the fp16 range
    sw = r.uniform(min(0.001, sw_hi / 4), sw_hi, size=m).astype(np.float16)
    print(f"[case] w4a4 T={T} m={m} n={n}", flush=True)
    out = torch.full((64 + T * (m + pad) + 64,), float("nan"), dtype=torch.float16, device="cuda")
    fq.flatquant_w4a4_gemm(dev(cx), dev(sx), dev(cw), dev(sw), T, m, n, out[64:], m + pad, stream=torch.cuda.current_stream())
    torch.cuda.synchronize()
    got = out.cpu().view(torch.int16).numpy().view(np.float16)
    assert np.all(np.isnan(got[:64])) and np.all(np.isnan(got[64 + (T - 1) * (m + pad) + m:]))
    body = got[64:64 + T * (m + pad)].reshape(T, m + pad)
    if pad:
        assert np.all(np.isnan(body[:, m:]))
    dev_y = body[:, :m].astype(np.float64)
    acc, y, y16 = fo.w4a4_gemm(cx, sx, cw, sw)
    assert acc[0, 0] == 64 * n
    tol = 2.0 ** -11 * np.abs(y) * (1 + 2.0 ** -9) + 2.0 ** -25
    err = np.abs(dev_y - y)
    assert np.all(err <= tol), float((err / tol).max())
    same = float((body[:, :m] == y16).mean())
    print(f"[parity] w4a4 T={T} m={m} n={n}: max err/tol {float((err / tol).max()):.3f}, identical to the oracle's fp16 in {same * 100:.3f} %", flush=True)
    assert same > 0.99


@pytest.mark.parametrize("T,m,n,pad", [(300, 260, 512, 0), (128, 128, 256, 0), (1, 1, 256, 0), (2048, 384, 4096, 0), (77, 200, 11008, 24),
                                       (64, 4096, 4096, 0), (33, 100, 512, 0), (17, 4099, 11008, 5), (32, 64, 256, 0), (65, 96, 768, 0),
                                       (9, 40, 2304, 0), (64, 33, 11008, 0), (8, 64, 4096, 0), (65, 100, 2304, 0), (128, 4100, 1024, 3),
                                       (100, 40, 11008, 0), (129, 70, 512, 0)])
def test_w4a4_gemm(T, m, n, pad):
    _w4a4_case(T, m, n, pad)


@pytest.mark.parametrize("knob,value,T,m,n", [("FLATQUANT_GEMM_WIDE", 1, 300, 260, 768), ("FLATQUANT_GEMM_WIDE", 1, 513, 129, 256),
                                              ("FLATQUANT_GEMM_WIDE", 0, 2048, 4224, 512), ("FLATQUANT_GEMM_TILED", 1, 33, 96, 768),
                                              ("FLATQUANT_GEMM_TILED", 1, 100, 200, 1024)])
def test_w4a4_gemm_every_form(tuning, knob, value, T, m, n):
    """The forms the library would not pick by itself for these sizes: 256-token tiles on a small launch, 128-token
    tiles on a large one, the tiled product for few tokens."""
    tuning(knob, value)
    _w4a4_case(T, m, n, 0)
