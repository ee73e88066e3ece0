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
        "    if (flatquant_transform_mxfp4(0, 0, 0, 0, 0, 4, 3, 34, 102, 0, 0, 0) != FQ_UNSUPPORTED_SHAPE) return 4;\n"
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
    assert mx(n1=3, n2=34, x_stride=3 * 34) == fq.FQ_UNSUPPORTED_SHAPE      # 102 channels: no whole blocks of 32
    assert mx(n1=129, x_stride=129 * 64) == fq.FQ_UNSUPPORTED_SHAPE
    assert mx(n1=3, n2=33, x_stride=99) == fq.FQ_UNSUPPORTED_SHAPE          # odd right factor
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


def test_host_layer_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    """The host side of the API layer (argument checks, overlap arithmetic, fq_inverse_transpose, fq_choose_factors, the
    tuning table) compiled with -fsanitize=address,undefined (host pass only; the kernels' objects are the library's own)
    and driven by a C program through every host-only path and every rejection that returns before a device is touched."""
    import glob
    import shutil
    import subprocess
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    clang = "/opt/rocm/lib/llvm/bin/clang"
    csrc = os.path.join(ROOT, "paper_2410_09426_amd", "csrc")
    objs = [o for o in glob.glob(os.path.join(csrc, "*.o")) if os.path.basename(o) != "fq_api.o"]
    if not (os.path.exists(hipcc) and os.path.exists(clang)) or len(objs) < 5:
        pytest.skip("needs hipcc, its clang and the library's object files (python -m paper_2410_09426_amd.build)")
    api_o = tmp_path / "fq_api_san.o"
    subprocess.run([hipcc, "-O1", "-g", "--offload-arch=gfx950", "-fPIC", "-std=c++17", "-w",
                    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                    "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                    "-Xarch_host", "-fno-sanitize-recover=undefined",
                    "-c", os.path.join(csrc, "fq_api.hip"), "-o", str(api_o)], check=True, capture_output=True)
    lib = tmp_path / "libflatquant_san.so"
    subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-w", "-fno-gpu-sanitize", "-fsanitize=address", "-fsanitize=undefined",
                    str(api_o), *objs, "-o", str(lib)], check=True, capture_output=True)
    src = tmp_path / "drive.c"
    src.write_text(r"""
#include "flatquant.h"
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#define CHECK(cond) do { if (!(cond)) { printf("line %d: %s\n", __LINE__, #cond); return 1; } } while (0)
static unsigned short h(float v) { /* a few exact fp16 constants */
    if (v == 0.0f) return 0; if (v == 1.0f) return 0x3c00; if (v == 2.0f) return 0x4000; if (v == 0.5f) return 0x3800;
    if (v == -1.0f) return 0xbc00; if (v == 4.0f) return 0x4400; if (v == 0.25f) return 0x3400; return 0x7e00; }
int main(void) {
    int n1 = 0, n2 = 0;
    CHECK(fq_choose_factors(8192, &n1, &n2) == FQ_OK && n1 == 64 && n2 == 128);
    CHECK(fq_choose_factors(11008, &n1, &n2) == FQ_OK && n1 == 86 && n2 == 128);
    CHECK(fq_choose_factors(1, &n1, &n2) == FQ_OK && n1 == 1 && n2 == 1);
    CHECK(fq_choose_factors(2147483647, &n1, &n2) == FQ_OK && (long long)n1 * n2 == 2147483647LL);
    CHECK(fq_choose_factors(0, &n1, &n2) == FQ_INVALID_ARG && fq_choose_factors(-5, &n1, &n2) == FQ_INVALID_ARG);
    CHECK(fq_supported(64, 64) && fq_supported(1, 2) && !fq_supported(129, 64) && !fq_supported(64, 258) && !fq_supported(0, 4) && !fq_supported(-3, -3));
    CHECK(fq_lds_bytes(64, 64) > 0 && fq_lds_bytes(112, 256) > 0 && fq_lds_bytes(1000, 2) == 0);
    CHECK(fq_default_design_fits(64, 64, 160 * 1024) == 1 && fq_default_design_fits(112, 256, 160 * 1024) == 0);
    CHECK(strlen(fq_status_string(FQ_MISALIGNED)) > 0 && strlen(fq_status_string(12345)) > 0 && strlen(fq_status_string(-1)) > 0);
    /* rejections that return before any device call */
    char* buf = (char*)malloc(1 << 16);   /* host memory standing in for device pointers: never dereferenced on these paths */
    float clip = 1.0f;
    CHECK(flatquant_transform_quant(buf, buf, buf, &clip, 0, -1, 64, 64, 4096, (uint8_t*)buf, buf, 0) == FQ_INVALID_ARG);
    CHECK(flatquant_transform_quant(buf, buf, buf, &clip, 2, 4, 64, 64, 4096, (uint8_t*)buf, buf, 0) == FQ_INVALID_ARG);
    CHECK(flatquant_transform_quant(buf, buf, buf, &clip, 0, 4, 3, 5, 15, (uint8_t*)buf, buf, 0) == FQ_INVALID_ARG);      /* odd n */
    CHECK(flatquant_transform_quant(buf, buf, buf, &clip, 0, 4, 64, 64, 100, (uint8_t*)buf, buf, 0) == FQ_INVALID_ARG);   /* stride < n */
    CHECK(flatquant_transform_quant(buf, buf, buf, &clip, 0, 4, 200, 64, 12800, (uint8_t*)buf, buf, 0) == FQ_UNSUPPORTED_SHAPE);
    CHECK(flatquant_transform_quant(0, 0, 0, 0, 0, 0, 64, 64, 4096, 0, 0, 0) == FQ_OK);                                     /* T == 0 */
    CHECK(flatquant_transform_quant(0, buf, buf, &clip, 0, 4, 64, 64, 4096, (uint8_t*)buf, buf, 0) == FQ_INVALID_ARG);     /* null x */
    CHECK(flatquant_transform_quant(buf, buf, buf, &clip, 0, 1, 2, 2, 4, (uint8_t*)buf + 1, buf + 4096, 0) != FQ_OK);      /* output inside the input */
    CHECK(flatquant_kv_transform_quant(buf, buf, 3, 0.9f, 4, 8, 128, (uint8_t*)buf, buf, buf, 0) != FQ_OK);                /* Hp neither 1 nor H */
    CHECK(flatquant_kv_transform_quant(buf, buf, 1, 0.9f, 4, 8, 64, (uint8_t*)buf, buf, buf, 0) != FQ_OK);                 /* D != 128 */
    CHECK(flatquant_kv_transform_quant(0, 0, 1, 0.9f, 0, 8, 128, 0, 0, 0, 0) == FQ_OK);                                     /* T == 0 */
    CHECK(flatquant_dequant((const uint8_t*)buf, buf, 0, -1, 64, (float*)buf, 0) == FQ_INVALID_ARG);
    CHECK(flatquant_w4a4_gemm(0, 0, 0, 0, 4, 8, 256, 0, 8, 0) == FQ_INVALID_ARG && flatquant_w4a4_gemm(0, 0, 0, 0, 4, 8, 64, 0, 8, 0) == FQ_UNSUPPORTED_SHAPE);
    CHECK(fq_set_tuning("FLATQUANT_NO_SUCH_KNOB", 1, 1) == FQ_INVALID_ARG && fq_set_tuning(0, 1, 1) == FQ_INVALID_ARG);
    CHECK(fq_set_tuning("FLATQUANT_MODE", 3, 1) == FQ_OK && fq_set_tuning("FLATQUANT_MODE", 0, 0) == FQ_OK);
    /* fq_inverse_transpose: diag(1, 2, 0.5) -> diag(1, 0.5, 2); a permutation; a singular matrix; sizes 1 and 256; bad sizes */
    unsigned short P[9] = {0}, O[9];
    P[0] = h(1); P[4] = h(2); P[8] = h(0.5f);
    double res = -1;
    CHECK(fq_inverse_transpose(P, 3, O, &res) == FQ_OK && O[0] == h(1) && O[4] == h(0.5f) && O[8] == h(2) && O[1] == 0 && res == 0.0);
    unsigned short Q[4] = {0, 0x3c00, 0x3c00, 0}, R[4];
    CHECK(fq_inverse_transpose(Q, 2, R, 0) == FQ_OK && R[0] == 0 && R[1] == h(1) && R[2] == h(1) && R[3] == 0);
    unsigned short S[4] = {0x3c00, 0x4000, 0x4000, 0x4400};   /* [[1, 2], [2, 4]] */
    CHECK(fq_inverse_transpose(S, 2, R, &res) == FQ_INVALID_ARG);
    unsigned short one = h(4), inv1 = 0;
    CHECK(fq_inverse_transpose(&one, 1, &inv1, 0) == FQ_OK && inv1 == h(0.25f));
    CHECK(fq_inverse_transpose(P, 0, O, 0) == FQ_INVALID_ARG && fq_inverse_transpose(P, 257, O, 0) == FQ_INVALID_ARG);
    CHECK(fq_inverse_transpose(0, 3, O, 0) == FQ_INVALID_ARG && fq_inverse_transpose(P, 3, 0, 0) == FQ_INVALID_ARG);
    unsigned short* big = (unsigned short*)calloc(256 * 256, 2);
    unsigned short* bigo = (unsigned short*)malloc(256 * 256 * 2);
    for (int i = 0; i < 256; ++i) big[i * 256 + (i * 7 + 3) % 256] = (i & 1) ? h(2) : h(-1);   /* a scaled permutation, 256 x 256 */
    CHECK(fq_inverse_transpose(big, 256, bigo, &res) == FQ_OK && res == 0.0);
    for (int i = 0; i < 256; ++i) CHECK(bigo[i * 256 + (i * 7 + 3) % 256] == ((i & 1) ? h(0.5f) : h(-1)));
    free(big); free(bigo); free(buf);
    CHECK(fq_mxfp4_tiled_scale_bytes(130, 512) == 2 * 2 * 128 * 8 && fq_mxfp4_tiled_scale_bytes(0, 512) == 0);
    printf("sanitized host layer ok\n");
    return 0;
}
""")
    exe = tmp_path / "drive"
    subprocess.run([clang, "-std=c99", "-g", "-w", "-fno-gpu-sanitize", "-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined",
                    "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe), "-L", str(tmp_path), "-lflatquant_san",
                    f"-Wl,-rpath,{tmp_path}"], check=True, capture_output=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([str(exe)], capture_output=True, text=True, env=env)
    assert r.returncode == 0 and "sanitized host layer ok" in r.stdout, r.stdout[-2000:] + r.stderr[-4000:]
