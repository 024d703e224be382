"""CPU-only checks of the library's host side: the C-ABI shared library loads
and exports every symbol the header declares, argument validation returns
error codes without touching a GPU, and the private packed layout decodes the
way the GEMV kernels read it (re-derived here in NumPy from the layout's
description, independent of the library's packer)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2412_20185_amd as dd

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "decdec.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(decdec_[a-z0-9_]+)\s*\(", hdr))
    assert declared == set(dd.EXPORTED_SYMBOLS)
    L = dd.lib()
    for name in declared:
        assert hasattr(L, name), name


def test_strerror_and_buffer_size():
    assert dd.decdec_strerror(0) == "ok"
    assert "invalid" in dd.decdec_strerror(-1)
    # Section 4.3: 1433 channels need 1433 * (4 + 2) bytes
    assert dd.decdec_sc_buffer_bytes(1433) == 8598
    assert dd.decdec_sc_buffer_bytes(0) == 0
    # the partial rows of the optional separate accumulate kernel: (16 + 16) rows of maxN floats
    assert dd.decdec_partial_buffer_bytes(28672) == 32 * 28672 * 4
    assert dd.decdec_partial_buffer_bytes(0) == 0
    assert "static" in dd.decdec_strerror(-6)


def test_validation_without_gpu():
    L = dd.lib()
    P = 1 << 20          # stands for a device pointer: validation fails before anything is read
    bad = [dd.Desc(100, 64, 4), dd.Desc(128, 60, 4), dd.Desc(128, 64, 5), dd.Desc(128, 64, 4, wfmt=7),
           dd.Desc(128, 64, 4, rfmt=4), dd.Desc(0, 64, 4)]
    for d in bad:
        assert dd.decdec_packed_bytes(d) == 0
        assert L.decdec_gemv(C.byref(d), P, P, P, P, P, P, 0, P, P, None) == -1
    assert dd.decdec_packed_bytes(dd.Desc(128, 64, 4, wfmt=dd.W_LUT_COL8)) == 0     # LUT is 3-bit only
    assert L.decdec_gemv(C.byref(dd.Desc(128, 64, 4, wfmt=dd.W_LUT_COL8)), P, P, P, P, P, P, 0, P, P, None) == -2
    good = dd.Desc(256, 128, 3)
    assert dd.decdec_packed_bytes(good) == 256 * 128 * 3 // 8
    assert dd.decdec_packed_bytes(dd.Desc(256, 128, 4)) == 256 * 128 // 2
    assert L.decdec_gemv(C.byref(good), None, P, P, P, P, P, 0, P, P, None) == -1     # null x
    assert L.decdec_gemv(C.byref(good), P, P, P, P, P, P, 0, P, None, None) == -1     # null workspace
    # select: K not a multiple of 8, k out of range, null pointers
    assert L.decdec_select_topk(P, 1001, 3, P, None, None) == -1
    assert L.decdec_select_topk(P, 1024, 1025, P, None, None) == -1
    assert L.decdec_select_topk(P, 1024, -1, P, None, None) == -1
    assert L.decdec_select_topk(None, 1024, 3, P, None, None) == -1
    assert L.decdec_select_topk(P, 1024, 3, None, None, None) == -1
    assert L.decdec_select_topk(P, 131072, 3, P, None, None) == -1
    assert L.decdec_select_topk(P, 1024, 0, None, None, None) == 0                   # k = 0 enqueues nothing
    assert L.decdec_select_topk(P + 2, 1024, 0, None, None, None) == -1              # x must be 16-byte aligned
    assert L.decdec_select_topk(P, 1024, 3, P + 2, None, None) == -1                 # idx must be 4-byte aligned
    assert L.decdec_select_bucket(P + 8, 2048, 0, C.c_float(2.0), C.c_float(1.0), None, None, None) == -1
    # approximate selector: K not a multiple of 1024, k_chunk out of range, boundaries out of order or NaN
    assert L.decdec_select_bucket(P, 1000, 3, C.c_float(2.0), C.c_float(1.0), P, None, None) == -1
    assert L.decdec_select_bucket(P, 2048, 1025, C.c_float(2.0), C.c_float(1.0), P, None, None) == -1
    assert L.decdec_select_bucket(P, 2048, 3, C.c_float(1.0), C.c_float(2.0), P, None, None) == -1
    assert L.decdec_select_bucket(P, 2048, 3, C.c_float(float("nan")), C.c_float(1.0), P, None, None) == -1
    assert L.decdec_select_bucket(P, 2048, 3, C.c_float(1.0), C.c_float(-1.0), P, None, None) == -1
    assert L.decdec_select_bucket(None, 2048, 3, C.c_float(2.0), C.c_float(1.0), P, None, None) == -1
    assert L.decdec_select_bucket(P, 2048, 0, C.c_float(2.0), C.c_float(1.0), None, None, None) == 0
    # packers
    codes = np.zeros((256, 128), np.uint8)
    codes[3, 5] = 8
    with pytest.raises(dd.DecdecError):
        dd.decdec_pack_weights(good, codes)                                           # code >= 2^3
    with pytest.raises(dd.DecdecError):
        dd.decdec_pack_residual_int4(np.full((4, 64), -8, np.int8))
    assert L.decdec_ws_gemv_launch_shape(None, 4096, 4096, None, None, None) == -1
    h = C.c_void_p()
    assert L.decdec_ws_create(0, 64, 0, C.byref(h)) == -1
    assert L.decdec_ws_create(128, 64, 129, C.byref(h)) == -1
    assert L.decdec_ws_destroy(None) == 0


def _lane_words(packed: np.ndarray, kind_words: int, nt: int, g: int, G: int, lane: int) -> np.ndarray:
    """32-bit words of one lane of tile (nt, g): piece p of lane l is at p*1024 + l*16."""
    tile_bytes = kind_words * 4 * 64
    tile = packed[(nt * G + g) * tile_bytes:(nt * G + g + 1) * tile_bytes]
    words = []
    for w in range(kind_words):
        off = (w // 4) * 1024 + lane * 16 + (w % 4) * 4
        words.append(int.from_bytes(tile[off:off + 4].tobytes(), "little"))
    return np.array(words, dtype=np.uint64)


def _decode_u4(words):
    out = np.zeros(128, np.int64)
    for w in range(16):
        t = int(words[w])
        for i in range(4):
            j = 4 * w + i
            out[2 * j] = (t >> (4 * i)) & 0xF
            out[2 * j + 1] = (t >> (16 + 4 * i)) & 0xF
    return out


def _decode_u3(words):
    out = np.zeros(128, np.int64)
    pos = [0, 4, 7, 10, 13]
    for w in range(12):
        t = int(words[w])
        for f in range(5):
            j = 5 * w + f
            out[2 * j] = (t >> pos[f]) & 7
            out[2 * j + 1] = (t >> (16 + pos[f])) & 7
        b, e = w // 3, w % 3
        out[2 * (60 + b)] |= ((t >> 3) & 1) << e
        out[2 * (60 + b) + 1] |= ((t >> 19) & 1) << e
    return out


def _decode_lut3(words):
    out = np.zeros(128, np.int64)
    m = 0x07070707
    for b in range(4):
        w0, w1, w2 = (int(words[3 * b + i]) for i in range(3))
        sel = [w0 & m, (w0 >> 3) & m, w1 & m, (w1 >> 3) & m, w2 & m, (w2 >> 3) & m,
               ((w0 >> 6) & 0x03030303) | ((w2 >> 4) & 0x04040404),
               ((w1 >> 6) & 0x03030303) | ((w2 >> 5) & 0x04040404)]
        for s in range(8):
            by = [(sel[s] >> (8 * y)) & 0xFF for y in range(4)]
            j = 16 * b + 2 * s
            out[2 * j], out[2 * j + 1] = by[0], by[1]
            out[2 * (j + 1)], out[2 * (j + 1) + 1] = by[2], by[3]
    return out


@pytest.mark.parametrize("bits,wfmt,nwords,decode", [(4, 0, 16, _decode_u4), (3, 0, 12, _decode_u3),
                                                     (3, 1, 12, _decode_lut3)])
def test_packed_layout_decodes_as_the_kernels_read_it(bits, wfmt, nwords, decode):
    g = np.random.default_rng(bits * 10 + wfmt)
    K, N = 384, 192
    codes = g.integers(0, 2 ** bits, size=(K, N)).astype(np.uint8)
    d = dd.Desc(K, N, bits, wfmt)
    packed = dd.decdec_pack_weights(d, codes)
    assert packed.size == K * N * bits // 8
    assert np.array_equal(dd.decdec_unpack_weights(d, packed), codes)
    G = K // 128
    for nt, grp, lane in [(0, 0, 0), (2, 1, 63), (1, 2, 17), (0, 2, 40)]:
        got = decode(_lane_words(packed, nwords, nt, grp, G, lane))
        assert np.array_equal(got, codes[grp * 128:(grp + 1) * 128, nt * 64 + lane].astype(np.int64)), (nt, grp, lane)


def test_int4_residual_rows():
    q = np.array([[-7, 7, 0, -1] * 16, [1, 2, 3, 4] * 16], np.int8)
    out = dd.decdec_pack_residual_int4(q)
    assert out.shape == (2, 32)
    assert out[0, 0] == ((-7) & 0xF) | (7 << 4) and out[0, 1] == 0 | (((-1) & 0xF) << 4)
    assert out[1, 0] == 1 | (2 << 4) and out[1, 1] == 3 | (4 << 4)


def test_int2_int8_residual_rows():
    """2-bit: column 4j+i in bits 2i..2i+1 of byte j; 8-bit: one two's-complement byte per column."""
    q = np.array([[-1, 1, 0, -1] * 16, [1, 0, 0, 1] * 16], np.int8)
    out = dd.decdec_pack_residual_int(q, 2)
    assert out.shape == (2, 16)
    assert out[0, 0] == (3 | (1 << 2) | (0 << 4) | (3 << 6)) and out[1, 0] == (1 | (1 << 6))
    q8 = np.array([[-127, 127, 0, -1] * 4], np.int8)
    out = dd.decdec_pack_residual_int(q8, 8)
    assert out.shape == (1, 16) and np.array_equal(out.view(np.int8), q8)
    assert np.array_equal(dd.decdec_pack_residual_int(np.tile(q8, (1, 2)), 4 * 2)[:, :16].view(np.int8), q8)
    for bad, bits in ((np.full((1, 64), 2, np.int8), 2), (np.full((1, 16), -128, np.int8), 8),
                      (np.zeros((1, 8), np.int8), 8), (np.zeros((1, 64), np.int8), 3)):
        with pytest.raises(dd.DecdecError):
            dd.decdec_pack_residual_int(bad, bits)


def test_header_is_plain_c_and_links_against_the_library(tmp_path):
    """The boundary is a C ABI: the header compiles as C99 with warnings as errors, and a C program that
    calls host-only entry points links against the shared library and runs (no GPU needed)."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no C compiler")
    src = tmp_path / "use_decdec.c"
    src.write_text('#include <stdio.h>\n#include "decdec.h"\n'
                   "int main(void) {\n"
                   "    decdec_desc d = {256, 128, 3, DECDEC_W_UNIFORM_G128, DECDEC_R_FP16};\n"
                   '    printf("%lu %lu %s\\n", (unsigned long)decdec_packed_bytes(&d),\n'
                   "           (unsigned long)decdec_sc_buffer_bytes(1433), decdec_strerror(DECDEC_EINVAL));\n"
                   "    return decdec_ws_destroy(NULL);\n}\n")
    libdir = os.path.join(ROOT, "paper_2412_20185_amd")
    exe = tmp_path / "use_decdec"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                    str(src), "-o", str(exe), "-L", libdir, "-ldecdec", f"-Wl,-rpath,{libdir}"], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split(None, 2)
    assert out[0] == str(256 * 128 * 3 // 8) and out[1] == "8598" and "invalid" in out[2]
