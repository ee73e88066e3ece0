"""Maximum sizes: tensors past 2^31 elements and 2^32 bytes.  Every kernel forms its row addresses in 64 bits; these
cases put token rows, code rows and output rows on both sides of the 2^31- and 2^32-byte marks and compare sampled
rows (the first, the last, the ones around each mark, a random handful) with the oracle.  The inputs are seeded
normal deviates drawn on the device (several GB: too large to build on the host); the sampled rows are copied back and
the oracle gets exactly those bytes."""
import numpy as np
import pytest
import torch

from oracle import flatquant_oracle as fo
from oracle import parity
from paper_2410_09426_amd import binding as fq
from paper_2410_09426_amd import synth
from gpu_util import dev, host_f16

pytestmark = pytest.mark.gpu


def _rows_around(T, row_bytes_list, seed, extra=12):
    rows = {0, 1, T - 2, T - 1}
    for rb in row_bytes_list:
        for mark in (1 << 31, 1 << 32):
            t = mark // rb
            rows.update(r for r in (t - 1, t, t + 1) if 0 <= r < T)
    r = np.random.Generator(np.random.PCG64(seed))
    rows.update(int(v) for v in r.integers(0, T, size=extra))
    return np.array(sorted(rows))


def _device_normal(shape, seed, scale=1.0):
    g = torch.Generator(device="cuda").manual_seed(seed)
    out = torch.empty(shape, dtype=torch.float16, device="cuda")
    step = max(1, (1 << 28) // int(np.prod(shape[1:])))
    for r0 in range(0, shape[0], step):          # in pieces: the fp32 draw of the whole tensor would double the footprint
        r1 = min(shape[0], r0 + step)
        out[r0:r1] = (torch.randn((r1 - r0,) + tuple(shape[1:]), generator=g, device="cuda") * scale).half()
    return out


def test_activation_rows_past_4_gib():
    n1 = n2 = 64
    n = n1 * n2
    T = 1_100_000                                  # x: 9.0 GB, codes: 2.25 GB
    c = synth.generic(31, 8, n1, n2)               # the factors and a clip value; the rows come from the device
    x = _device_normal((T, n), 777)
    P1, P2 = dev(c.P1), dev(c.P2)
    clip = dev(np.array([0.9], dtype=np.float32))
    codes = torch.empty((T, n // 2), dtype=torch.uint8, device="cuda")
    scales = torch.empty((T,), dtype=torch.float16, device="cuda")
    print(f"[case] activation rows past 4 GiB: T={T} n={n}", flush=True)
    fq.flatquant_transform_quant(x, P1, P2, clip, 0, T, n1, n2, n, codes, scales, stream=torch.cuda.current_stream())
    torch.cuda.synchronize()
    rows = _rows_around(T, [2 * n, n // 2], 5)
    idx = torch.from_numpy(rows).cuda()
    xs = host_f16(x[idx])
    y = fo.affine_transform(xs, c.P1, c.P2)
    rep = parity.check_sym(y, 0.9, codes[idx].cpu().numpy(), host_f16(scales[idx]), rows=rows)
    print(f"[parity] rows {rows.tolist()}: {rep}", flush=True)
    assert rep["band_flips"] <= parity.band_flip_allowance(rep["in_band"])


def test_kv_cache_past_4_gib():
    T, H, D = 2_200_000, 8, 128                    # input: 4.5 GB, codes: 1.1 GB
    kvc = synth.kv_cache(T=4, H=H)
    kv = _device_normal((T, H, D), 778)
    P = dev(kvc.P)
    codes = torch.empty((T * H, D // 2), dtype=torch.uint8, device="cuda")
    sc = torch.empty((T * H,), dtype=torch.float16, device="cuda")
    zr = torch.empty((T * H,), dtype=torch.float16, device="cuda")
    print(f"[case] KV cache past 4 GiB: T={T} H={H}", flush=True)
    fq.flatquant_kv_transform_quant(kv, P, H, 0.95, T, H, D, codes, sc, zr, stream=torch.cuda.current_stream())
    torch.cuda.synchronize()
    rows = _rows_around(T, [2 * H * D, H * D // 2], 6)
    idx = torch.from_numpy(rows).cuda()
    ks = host_f16(kv[idx])                                            # [rows, H, D]
    y = fo.kv_transform(ks, kvc.P).reshape(len(rows) * H, D)
    take = lambda t, w: t.view(T, H, w)[idx].reshape(len(rows) * H, w)
    rep = parity.check_kv(y, 0.95, take(codes, D // 2).cpu().numpy(), host_f16(take(sc, 1).reshape(-1)), host_f16(take(zr, 1).reshape(-1)))
    print(f"[parity] tokens {rows.tolist()}: {rep}", flush=True)


@pytest.mark.parametrize("kind", ["int4", "mxfp4"])
def test_product_output_past_4_gib(kind):
    T, m, n = 600_000, 4096, 256                   # output: 4.9 GB
    r = np.random.Generator(np.random.PCG64(909))
    g = torch.Generator(device="cuda").manual_seed(779)
    xc = torch.randint(0, 256, (T, n // 2), generator=g, dtype=torch.uint8, device="cuda")
    wc_h = r.integers(0, 256, size=(m, n // 2), dtype=np.uint8)
    out = torch.empty((T, m), dtype=torch.float16, device="cuda")
    rows = _rows_around(T, [2 * m], 7)
    idx = torch.from_numpy(rows).cuda()
    print(f"[case] {kind} product with an output past 4 GiB: T={T} m={m} n={n}", flush=True)
    if kind == "int4":
        xs = (torch.rand((T,), generator=g, device="cuda") * 2 + 0.01).half()
        ws_h = r.uniform(0.001, 0.05, size=m).astype(np.float16)
        fq.flatquant_w4a4_gemm(xc, xs, dev(wc_h), dev(ws_h), T, m, n, out, m, stream=torch.cuda.current_stream())
        torch.cuda.synchronize()
        _, y, y16 = fo.w4a4_gemm(xc[idx].cpu().numpy(), host_f16(xs[idx]), wc_h, ws_h)
        got = host_f16(out[idx])
        assert np.array_equal(got.view(np.uint16), y16.view(np.uint16)) or float(np.mean(got == y16)) > 0.99
        tol = 2.0 ** -11 * np.abs(y) * (1 + 2.0 ** -9) + 2.0 ** -25
        assert np.all(np.abs(got.astype(np.float64) - y) <= tol)
    else:
        xe_h = r.integers(118, 131, size=(len(rows), n // 32), dtype=np.uint8)
        we_h = r.integers(112, 126, size=(m, n // 32), dtype=np.uint8)
        # token exponents: one byte value everywhere except the sampled rows, which get their own (tile order: 128-row
        # tiles, per tile and 256-code step the rows' 8 bytes contiguous)
        nk = n // 256
        xe = torch.full((fq.fq_mxfp4_tiled_scale_bytes(T, n),), 124, dtype=torch.uint8, device="cuda")
        xev = xe.view(-1, nk, 128, 8)
        for j, t in enumerate(rows.tolist()):
            xev[t >> 7, :, t & 127, :] = torch.from_numpy(xe_h[j].reshape(nk, 8)).cuda()
        fq.flatquant_mxfp4_gemm(xc, xe, dev(wc_h), dev(fo.mx_tile_scales(we_h, fill=0xFF)), T, m, n, out, m, stream=torch.cuda.current_stream())
        torch.cuda.synchronize()
        y, y16, ab = fo.mxfp4_gemm(xc[idx].cpu().numpy(), xe_h, wc_h, we_h)
        got = host_f16(out[idx]).astype(np.float64)
        tol = 2.0 ** -11 * np.abs(y) * (1 + 2.0 ** -9) + n * 2.0 ** -24 * ab + 2.0 ** -25
        assert np.all(np.isfinite(got)) and np.all(np.abs(got - y) <= tol)
    print(f"[parity] rows {rows.tolist()} agree with the oracle", flush=True)
