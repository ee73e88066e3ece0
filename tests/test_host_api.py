"""Host-side checks that need no GPU: the library loads, exports what the header
declares, and rejects bad arguments before touching a device."""
import ctypes
import os
import re

import pytest

from paper_2410_09426_amd import binding as fq

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "flatquant.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(flatquant_\w+|fq_\w+)\s*\(", hdr))
    declared -= {"fq_status"}
    assert declared == set(fq.EXPORTS)
    L = fq.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert fq.fq_abi_version() == 2


def test_header_is_plain_c_and_links_without_python(tmp_path):
    """The boundary is a C ABI: the header must compile as C99 (and C++), and a C program must link against the
    shared library and call the host-only entry points."""
    import shutil
    import subprocess
    cc = shutil.which("gcc")
    if cc is None:
        pytest.skip("no C compiler")
    src = tmp_path / "use.c"
    src.write_text(
        '#include "flatquant.h"\n#include <stdio.h>\n'
        "int main(void) {\n"
        "    int n1 = 0, n2 = 0;\n"
        "    if (fq_choose_factors(8192, &n1, &n2) != FQ_OK || n1 != 64 || n2 != 128) return 1;\n"
        "    if (!fq_supported(64, 64) || fq_supported(129, 64)) return 2;\n"
        "    if (flatquant_transform_quant(0, 0, 0, 0, 0, 0, 64, 64, 4096, 0, 0, 0) != FQ_OK) return 3;      /* T == 0 */\n"
        "    if (flatquant_transform_mxfp4(0, 0, 0, 0, 0, 4, 64, 96, 6144, 0, 0, 0) != FQ_UNSUPPORTED_SHAPE) return 4;\n"
        '    printf("%s %d\\n", fq_status_string(FQ_MISALIGNED), fq_abi_version());\n'
        "    return 0;\n}\n")
    inc = os.path.join(ROOT, "include")
    libdir = os.path.dirname(fq.LIB_PATH)
    exe = tmp_path / "use"
    subprocess.run([cc, "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", inc, str(src), "-o", str(exe),
                    "-L", libdir, "-lflatquant", f"-Wl,-rpath,{libdir}"], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    assert out[-1] == str(fq.fq_abi_version()) and len(out) >= 2
    cxx = shutil.which("g++")
    if cxx:
        subprocess.run([cxx, "-std=c++11", "-Wall", "-Werror", "-fsyntax-only", "-x", "c++", "-I", inc, str(src)], check=True)


def test_tuning_overrides():
    assert fq.lib().fq_set_tuning(b"FLATQUANT_NO_SUCH_KNOB", 1, 1) == fq.FQ_INVALID_ARG
    assert fq.lib().fq_set_tuning(None, 1, 1) == fq.FQ_INVALID_ARG
    fq.fq_set_tuning("FLATQUANT_MODE", 3)
    fq.fq_set_tuning("FLATQUANT_MODE", None)
    with pytest.raises(fq.FlatQuantError):
        fq.fq_set_tuning("flatquant_mode", 1)


def test_factor_rule_and_fit_conditions():
    # Sec. 3.1: argmin(n1 + n2), n1 <= n2; (64, 128) for 8192
    assert fq.fq_choose_factors(8192) == (64, 128)
    assert fq.fq_choose_factors(4096) == (64, 64)
    assert fq.fq_choose_factors(11008) == (86, 128)
    assert fq.fq_choose_factors(28672) == (128, 224)
    assert fq.fq_choose_factors(7) == (1, 7)
    assert fq.fq_choose_factors(1) == (1, 1)
    with pytest.raises(fq.FlatQuantError):
        fq.fq_choose_factors(0)
    # App. "Detailed Design of Kernel Fusion": default-design inequalities, with 160 KB of LDS
    m = 160 * 1024
    assert fq.fq_default_design_fits(64, 64, m) and fq.fq_default_design_fits(64, 128, m) and fq.fq_default_design_fits(86, 128, m)
    assert not fq.fq_default_design_fits(112, 256, m)            # (256^2 + 2*112*256)*2 = 245760 > m
    assert (64 * 64 + 2 * 64 * 64) * 2 == 24576 and fq.fq_default_design_fits(64, 64, 24577) and not fq.fq_default_design_fits(64, 64, 24576)
    # what this library actually keeps on chip stays under the 160 KB of a CU for every supported shape
    for n1, n2 in [(16, 16), (64, 64), (86, 128), (64, 128), (112, 256), (128, 256), (64, 172), (128, 224), (1, 2)]:
        assert fq.fq_supported(n1, n2)
        assert 0 < fq.fq_lds_bytes(n1, n2) <= 160 * 1024
    for n1, n2 in [(129, 64), (64, 258), (64, 63), (0, 64), (64, 0), (3, 5)]:
        assert not fq.fq_supported(n1, n2) and fq.fq_lds_bytes(n1, n2) == 0


def test_status_strings():
    assert fq.status_string(fq.FQ_OK) == "ok"
    seen = {fq.status_string(s) for s in range(5)}
    assert len(seen) == 5 and fq.status_string(99) == "unknown status"


def test_argument_validation_without_a_device():
    A = 0x10000   # fake, suitably aligned "device" addresses; validation must reject before any launch
    tq = lambda **k: fq.flatquant_transform_quant(**{**dict(x=A, P1=A + 0x100000, P2=A + 0x200000, clip=A + 0x300000, clip_mode=0, T=4,
                                                          n1=64, n2=64, x_stride=4096, out_codes=A + 0x400000, out_scales=A + 0x500000,
                                                          check=False), **k})
    assert tq(T=0) == fq.FQ_OK                      # empty input: nothing launched
    assert tq(T=0, x=None, out_codes=None) == fq.FQ_OK
    assert tq(T=-1) == fq.FQ_INVALID_ARG
    assert tq(x=None) == fq.FQ_INVALID_ARG
    assert tq(out_scales=None) == fq.FQ_INVALID_ARG
    assert tq(clip_mode=2) == fq.FQ_INVALID_ARG
    assert tq(x_stride=4095) == fq.FQ_INVALID_ARG   # stride shorter than a row
    assert tq(n1=3, n2=5, x_stride=15) == fq.FQ_INVALID_ARG     # odd n
    assert tq(n1=129, n2=64, x_stride=129 * 64) == fq.FQ_UNSUPPORTED_SHAPE
    assert tq(n1=2, n2=63, x_stride=126) == fq.FQ_UNSUPPORTED_SHAPE
    assert tq(x=A + 2) == fq.FQ_MISALIGNED
    assert tq(x_stride=4097) == fq.FQ_MISALIGNED
    assert tq(out_codes=A + 64) == fq.FQ_INVALID_ARG            # output overlaps the input
    with pytest.raises(fq.FlatQuantError):
        fq.flatquant_transform_quant(None, A, A, A, 0, 4, 64, 64, 4096, A, A)

    mx = lambda **k: fq.flatquant_transform_mxfp4(**{**dict(x=A, P1=A + 0x100000, P2=A + 0x200000, clip=A + 0x300000, clip_mode=1, T=4, n1=64,
                                                         n2=64, x_stride=4096, out_codes=A + 0x400000, out_scales=A + 0x500000, check=False), **k})
    assert mx(T=0) == fq.FQ_OK
    assert mx(n2=96, x_stride=64 * 96) == fq.FQ_UNSUPPORTED_SHAPE and mx(n1=129, x_stride=129 * 64) == fq.FQ_UNSUPPORTED_SHAPE
    assert mx(n1=3, n2=64, x_stride=192) == fq.FQ_UNSUPPORTED_SHAPE      # n not a multiple of 128
    assert mx(P2=None) == fq.FQ_INVALID_ARG and mx(clip_mode=2) == fq.FQ_INVALID_ARG
    assert mx(x=A + 8) == fq.FQ_MISALIGNED and mx(out_scales=A + 0x500002) == fq.FQ_MISALIGNED and mx(x_stride=4100) == fq.FQ_MISALIGNED
    assert mx(out_scales=A + 0x400000) == fq.FQ_INVALID_ARG            # exponents inside the code buffer

    gx = lambda **k: fq.flatquant_mxfp4_gemm(**{**dict(x_codes=A, x_scales=A + 0x100000, w_codes=A + 0x200000, w_scales=A + 0x300000, T=4, m=8,
                                                     n=1024, out=A + 0x400000, out_stride=8, check=False), **k})
    assert gx(T=0) == fq.FQ_OK and gx(m=0, out_stride=0) == fq.FQ_OK
    assert gx(n=500) == fq.FQ_UNSUPPORTED_SHAPE and gx(out_stride=7) == fq.FQ_INVALID_ARG and gx(w_scales=None) == fq.FQ_INVALID_ARG
    assert gx(x_codes=A + 8) == fq.FQ_MISALIGNED and gx(x_scales=A + 0x100008) == fq.FQ_MISALIGNED
    assert fq.fq_mxfp4_tiled_scale_bytes(1, 256) == 128 * 8 and fq.fq_mxfp4_tiled_scale_bytes(129, 512) == 256 * 16
    assert fq.fq_mxfp4_tiled_scale_bytes(5, 300) == 0
    mxt = lambda **k: fq.flatquant_transform_mxfp4_tiled(**{**dict(x=A, P1=A + 0x100000, P2=A + 0x200000, clip=A + 0x300000, clip_mode=1, T=4,
                                                                n1=64, n2=64, x_stride=4096, out_codes=A + 0x400000, out_scales=A + 0x500000,
                                                                check=False), **k})
    assert mxt(T=0) == fq.FQ_OK and mxt(out_scales=A + 0x500004) == fq.FQ_MISALIGNED
    assert mxt(n1=2, n2=64, x_stride=128) == fq.FQ_UNSUPPORTED_SHAPE      # 128 channels: not a whole group of 8 exponents
    assert gx(out=A + 0x300000) == fq.FQ_INVALID_ARG          # output overlaps the weight exponents

    dmx = lambda **k: fq.flatquant_dequant_mxfp4(**{**dict(codes=A, scales=A + 0x100000, rows=4, n=64, out=A + 0x200000, check=False), **k})
    assert dmx(rows=0) == fq.FQ_OK and dmx(n=48) == fq.FQ_INVALID_ARG and dmx(scales=None) == fq.FQ_INVALID_ARG
    assert dmx(codes=A + 2) == fq.FQ_MISALIGNED

    kv = lambda **k: fq.flatquant_kv_transform_quant(**{**dict(kv=A, P=A + 0x100000, Hp=8, clip=0.95, T=4, H=8, D=128,
                                                            out_codes=A + 0x400000, out_scales=A + 0x500000, out_zeros=A + 0x600000,
                                                            check=False), **k})
    assert kv(T=0) == fq.FQ_OK
    assert kv(Hp=3) == fq.FQ_INVALID_ARG
    assert kv(clip=0.0) == fq.FQ_INVALID_ARG
    assert kv(D=64) == fq.FQ_UNSUPPORTED_SHAPE
    assert kv(kv=A + 8) == fq.FQ_MISALIGNED
    assert kv(out_zeros=None) == fq.FQ_INVALID_ARG
    assert kv(out_zeros=A + 0x500000) == fq.FQ_INVALID_ARG      # scales and zeros alias
    kvb = lambda **k: fq.flatquant_kv_transform_quant_bits(**{**dict(kv=A, P=A + 0x100000, Hp=8, clip=0.95, bits=3, T=4, H=8, D=128,
                                                                  out_codes=A + 0x400000, out_scales=A + 0x500000, out_zeros=A + 0x600000,
                                                                  check=False), **k})
    assert kvb(T=0) == fq.FQ_OK
    assert kvb(bits=1) == fq.FQ_INVALID_ARG and kvb(bits=5) == fq.FQ_INVALID_ARG and kvb(bits=8) == fq.FQ_INVALID_ARG
    assert kvb(D=64) == fq.FQ_UNSUPPORTED_SHAPE and kvb(out_codes=A + 8) == fq.FQ_MISALIGNED
    assert kvb(out_scales=A + 0x400000) == fq.FQ_INVALID_ARG     # steps inside the code buffer
    dqb = lambda **k: fq.flatquant_dequant_bits(**{**dict(codes=A, scales=A + 0x100000, zeros=A + 0x180000, rows=4, n=64, bits=3,
                                                       out=A + 0x200000, check=False), **k})
    assert dqb(rows=0) == fq.FQ_OK
    assert dqb(n=60) == fq.FQ_INVALID_ARG and dqb(bits=5) == fq.FQ_INVALID_ARG and dqb(zeros=None) == fq.FQ_INVALID_ARG
    assert dqb(out=A + 0x200002) == fq.FQ_MISALIGNED

    assert fq.flatquant_stream_probe(A, 0, 4096, 4096, A + 0x400000, check=False) == fq.FQ_OK
    assert fq.flatquant_stream_probe(A, 4, 4100, 4100, A + 0x400000, check=False) == fq.FQ_UNSUPPORTED_SHAPE
    assert fq.flatquant_stream_probe(A + 2, 4, 4096, 4096, A + 0x400000, check=False) == fq.FQ_MISALIGNED
    assert fq.flatquant_stream_probe(None, 4, 4096, 4096, A + 0x400000, check=False) == fq.FQ_INVALID_ARG

    gm = lambda **k: fq.flatquant_w4a4_gemm(**{**dict(x_codes=A, x_scales=A + 0x100000, w_codes=A + 0x200000, w_scales=A + 0x300000, T=4, m=8,
                                                     n=512, out=A + 0x400000, out_stride=8, check=False), **k})
    assert gm(T=0) == fq.FQ_OK and gm(m=0, out_stride=0) == fq.FQ_OK
    assert gm(n=500) == fq.FQ_UNSUPPORTED_SHAPE and gm(n=65536 + 256) == fq.FQ_UNSUPPORTED_SHAPE
    assert gm(out_stride=7) == fq.FQ_INVALID_ARG and gm(out=None) == fq.FQ_INVALID_ARG
    assert gm(x_codes=A + 8) == fq.FQ_MISALIGNED
    assert gm(out=A + 0x200000) == fq.FQ_INVALID_ARG          # output overlaps the weight codes
    ht = lambda **k: fq.flatquant_head_transform(**{**dict(x=A, P=A + 0x100000, Hp=8, T=4, H=8, D=128, out=A + 0x400000, check=False), **k})
    assert ht(T=0) == fq.FQ_OK and ht(D=64) == fq.FQ_UNSUPPORTED_SHAPE and ht(Hp=3) == fq.FQ_INVALID_ARG
    assert ht(out=A) == fq.FQ_INVALID_ARG and ht(x=A + 4) == fq.FQ_MISALIGNED

    dq = lambda **k: fq.flatquant_dequant(**{**dict(codes=A, scales=A + 0x100000, zeros=None, rows=4, n=64, out=A + 0x200000, check=False), **k})
    assert dq(rows=0) == fq.FQ_OK
    assert dq(n=63) == fq.FQ_INVALID_ARG
    assert dq(codes=None) == fq.FQ_INVALID_ARG
    assert dq(out=A + 0x200002) == fq.FQ_MISALIGNED


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(fq, "_lib", None)
    monkeypatch.setattr(fq, "LIB_PATH", os.path.join(ROOT, "no_such_dir", "libflatquant.so"))
    with pytest.raises(FileNotFoundError):
        fq.lib()


def test_inverse_transpose_helper_against_numpy():
    """Host Gauss-Jordan of the library against numpy's LU inverse (an independent routine) and the defining property."""
    import numpy as np
    r = np.random.Generator(np.random.PCG64(4242))
    for n in (1, 2, 7, 64, 128, 256):
        P = (np.eye(n) + 0.05 * r.standard_normal((n, n))).astype(np.float16)
        out, res = fq.fq_inverse_transpose(P)
        want = np.linalg.inv(P.astype(np.float64)).T
        assert out.dtype == np.float16 and out.shape == (n, n)
        assert np.array_equal(out, want.astype(np.float16)) or np.abs(out.astype(np.float64) - want).max() <= 2.0 ** -11 * np.abs(want).max()
        assert res <= 2.0 ** -10 * n * np.abs(want).max() * np.abs(P.astype(np.float64)).max()
        assert abs(res - np.abs(P.astype(np.float64).T @ out.astype(np.float64) - np.eye(n)).max()) < 1e-12
    # a matrix that needs row exchanges
    P = np.array([[0, 1, 0], [0, 0, 2], [4, 0, 0]], dtype=np.float16)
    out, res = fq.fq_inverse_transpose(P)
    assert np.array_equal(out, np.linalg.inv(P.astype(np.float64)).T.astype(np.float16)) and res == 0.0
    with pytest.raises(fq.FlatQuantError):
        fq.fq_inverse_transpose(np.ones((4, 4), dtype=np.float16))       # singular
    with pytest.raises(fq.FlatQuantError):
        fq.fq_inverse_transpose(np.zeros((3, 3), dtype=np.float16))
    assert fq.lib().fq_inverse_transpose(None, 4, None, None) == fq.FQ_INVALID_ARG
    assert fq.flatquant_weight_transform_quant(None, None, None, None, 0, 0, 64, 64, 4096, None, None, check=False) == fq.FQ_OK
    assert fq.flatquant_weight_transform_quant(None, None, None, None, 0, 5, 64, 64, 4096, None, None, check=False) == fq.FQ_INVALID_ARG
