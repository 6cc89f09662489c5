"""CPU-side tests of libams.so: it loads, exports every symbol include/ams.h declares,
and its host quantizer / packer agrees bit for bit with the independent CPU oracle.
No GPU call is made here."""

import ctypes
import os
import re

import numpy as np
import pytest

import paper_2510_16045_amd as ams
from oracle import ams_oracle as O
from paper_2510_16045_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PAPER_PAIRS = [(ams.FP533, O.FP533), (ams.FP425, O.FP425)]  # the two formats the paper builds kernels for
PAIRS = PAPER_PAIRS + [(ams.FP45, O.FP45), (ams.FP433, O.FP433), (ams.FP6, O.FP6_E2M3), (ams.FP5, O.FP5_E2M2), (ams.FP4, O.FP4_E2M1)]
REC = {ams.FP533: (96, 1024), ams.FP425: (128, 1088), ams.FP45: (128, 1152), ams.FP433: (96, 832), ams.FP6: (96, 1152), ams.FP5: (128, 1280), ams.FP4: (128, 1024)}
# records of a strip that share one block of side dwords (K is padded to whole groups of them)
SIDE_GROUP = {ams.FP533: 1, ams.FP425: 4, ams.FP45: 2, ams.FP433: 4, ams.FP6: 2, ams.FP5: 1, ams.FP4: 1}


def test_library_exports_every_declared_symbol():
    lib = ams.load_library()
    header = open(os.path.join(ROOT, "include", "ams.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = re.findall(r"\b(ams_[a-z0-9_]+)\s*\(", header)
    assert len(set(names)) >= 11
    for n in set(names):
        assert hasattr(lib, n), n
    assert lib.ams_version() >= 100
    assert lib.ams_strerror(0) == b"ok"
    assert [lib.ams_group_size(f) for f in range(9)] == [3, 4, 2, 3, 1, 1, 1, 0, 0]
    assert [lib.ams_code_bits(f) for f in range(9)] == [6, 5, 5, 5, 6, 5, 4, 0, 0]


@pytest.mark.parametrize("fmt,ofmt", PAIRS)
@pytest.mark.parametrize("N,K", [(1, 1), (16, 96), (17, 100), (5, 13), (256, 768), (33, 1000), (32, 1536), (4096, 4096)])
def test_sizes(fmt, ofmt, N, K):
    if (fmt, ofmt) in PAPER_PAIRS:
        assert ams.ams_canonical_bytes(fmt, N, K) == O.canonical_packed_bytes(ofmt, N, K)
    rec_k, rec_b = REC[fmt]
    sg = SIDE_GROUP[fmt]
    want = (-(-N // 16)) * (-(-(-(-K // rec_k)) // sg) * sg) * rec_b
    assert ams.ams_packed_bytes(fmt, N, K) == want
    # a record holds exactly bits-per-weight * 16 * rec_k bits
    assert rec_b * 8 == round(ofmt.bits_per_weight * 16 * rec_k)
    # without padding the gfx950 layout takes exactly the bytes of the densest packing
    if N % 16 == 0 and K % (rec_k * sg) == 0:
        assert ams.ams_packed_bytes(fmt, N, K) == ams.ams_canonical_bytes(fmt, N, K)
        assert ams.ams_packed_bytes(fmt, N, K) * 8 == round(ofmt.bits_per_weight * N * K)


@pytest.mark.parametrize("fmt,ofmt", PAIRS)
@pytest.mark.parametrize(
    "maker,N,K",
    [
        (synth.gaussian_weights, 256, 768),
        (synth.gaussian_weights, 37, 1000),
        (synth.gaussian_weights, 3, 5),
        (synth.heavy_tail_weights, 64, 2050),
    ],
)
def test_quantizer_matches_oracle_bit_for_bit(fmt, ofmt, maker, N, K):
    W = maker(N, K, 21)
    packed, scales, codes = ams.ams_pack(fmt, W, return_codes=True)
    o_codes, o_scales, _ = O.ams_quantize(W, ofmt)
    assert np.array_equal(scales.view(np.uint16), o_scales.view(np.uint16))
    assert np.array_equal(codes, o_codes.astype(np.uint8))
    assert np.array_equal(ams.ams_unpack_host(fmt, packed, N, K), codes)


@pytest.mark.parametrize("fmt,ofmt", PAIRS)
def test_quantizer_on_every_fp16_value(fmt, ofmt):
    # every finite fp16 value as a weight, under several row scales (ties, saturation, subnormals)
    bits = np.arange(1 << 16, dtype=np.uint16)
    v = bits.view(np.float16)
    v = v[np.isfinite(v)]
    for top in (7.5, 7.0, 1.0, 0.0137, 60000.0):
        row = v[np.abs(v.astype(np.float64)) <= top]
        W = row[: (len(row) // 12) * 12].reshape(1, -1).copy()
        W[0, 0] = np.float16(top)
        _, scales, codes = ams.ams_pack(fmt, W, return_codes=True)
        o_codes, o_scales, _ = O.ams_quantize(W, ofmt)
        assert np.array_equal(scales, o_scales)
        assert np.array_equal(codes, o_codes.astype(np.uint8))


@pytest.mark.parametrize("fmt,ofmt", PAIRS)
@pytest.mark.parametrize("maker,N,K", [(synth.gaussian_weights, 64, 770), (synth.heavy_tail_weights, 33, 2050), (synth.gaussian_weights, 2, 4)])
def test_reround_search_matches_oracle_bit_for_bit(fmt, ofmt, maker, N, K):
    W = maker(N, K, 23)
    packed, scales, codes = ams.ams_pack_ex(fmt, ams.SEARCH_REROUND, W, return_codes=True)
    o_codes, o_scales, _ = O.ams_quantize(W, ofmt, search="reround")
    assert np.array_equal(scales.view(np.uint16), o_scales.view(np.uint16))
    assert np.array_equal(codes, o_codes.astype(np.uint8))
    assert np.array_equal(ams.ams_unpack_host(fmt, packed, N, K), codes)
    # the literal search through the same entry point is ams_pack
    p2, s2, c2 = ams.ams_pack_ex(fmt, ams.SEARCH_SET_BIT, W, return_codes=True)
    p1, s1, c1 = ams.ams_pack(fmt, W, return_codes=True)
    assert np.array_equal(p1, p2) and np.array_equal(s1, s2) and np.array_equal(c1, c2)
    with pytest.raises(ams.AmsError):
        ams.ams_pack_ex(fmt, 7, W)


@pytest.mark.parametrize("fmt,ofmt", PAIRS)
def test_reround_search_on_every_fp16_value(fmt, ofmt):
    v = np.arange(1 << 16, dtype=np.uint16).view(np.float16)
    v = v[np.isfinite(v)]
    for top in (7.5, 1.0, 0.0137):
        row = v[np.abs(v.astype(np.float64)) <= top]
        W = row[: (len(row) // 12) * 12].reshape(1, -1).copy()
        W[0, 0] = np.float16(top)
        _, scales, codes = ams.ams_pack_ex(fmt, ams.SEARCH_REROUND, W, return_codes=True)
        o_codes, o_scales, _ = O.ams_quantize(W, ofmt, search="reround")
        assert np.array_equal(scales, o_scales)
        assert np.array_equal(codes, o_codes.astype(np.uint8))


def rowmajor_scales(scales_dev: np.ndarray, N: int) -> np.ndarray:
    """[strip, run, row in strip] -> [N, runs]"""
    return scales_dev.transpose(0, 2, 1).reshape(-1, scales_dev.shape[1])[:N]


@pytest.mark.parametrize("fmt,ofmt", PAIRS)
@pytest.mark.parametrize("N,K,mult,search", [(40, 1000, 1, "set"), (16, 768, 2, "reround"), (3, 100, 4, "set")])
def test_grouped_scales_match_oracle_bit_for_bit(fmt, ofmt, N, K, mult, search):
    sg = REC[fmt][0] * mult
    W = synth.heavy_tail_weights(N, K, 27)
    packed, scales, codes = ams.ams_pack_grouped(fmt, W, sg, search=ams.SEARCH_REROUND if search == "reround" else ams.SEARCH_SET_BIT, return_codes=True)
    o_codes, o_scales = O.ams_quantize_grouped(W, ofmt, sg, search=search)
    assert scales.shape == (-(-N // 16), -(-K // sg), 16)
    assert np.array_equal(rowmajor_scales(scales, N).view(np.uint16), o_scales.view(np.uint16))
    pad = scales.transpose(0, 2, 1).reshape(-1, scales.shape[1])[N:]
    assert np.all(pad == np.float16(1.0))
    assert np.array_equal(codes, o_codes.astype(np.uint8))
    assert np.array_equal(ams.ams_unpack_host(fmt, packed, N, K), codes)
    for bad in (sg + 1, sg * 3, REC[fmt][0] // 2, 0, -96):
        with pytest.raises(ams.AmsError):
            ams.ams_group_scales_count(fmt, N, K, bad)


@pytest.mark.parametrize("fmt,ofmt", PAIRS)
def test_per_tensor_scale_matches_oracle_bit_for_bit(fmt, ofmt):
    W = synth.heavy_tail_weights(37, 500, 29)
    packed, scales, codes = ams.ams_pack_per_tensor(fmt, W, return_codes=True)
    o_codes, o_scales, _ = O.ams_quantize(W, ofmt, per_tensor=True)
    assert np.array_equal(scales.view(np.uint16), o_scales.view(np.uint16)) and len(set(scales.tolist())) == 1
    assert np.array_equal(codes, o_codes.astype(np.uint8))
    assert np.array_equal(ams.ams_unpack_host(fmt, packed, 37, 500), codes)
    Z = np.zeros((3, 8), dtype=np.float16)
    assert np.all(ams.ams_pack_per_tensor(fmt, Z)[1] == np.float16(1.0))
    Z[1, 2] = np.float16(np.nan)
    with pytest.raises(ams.AmsError, match="inf or NaN"):
        ams.ams_pack_per_tensor(fmt, Z)


@pytest.mark.parametrize("fmt,ofmt", PAIRS)
def test_degenerate_rows_and_errors(fmt, ofmt):
    W = np.zeros((3, 24), dtype=np.float16)
    W[1, 5] = np.float16(6e-8)
    W[2, :] = np.float16(-3.0)
    _, scales, codes = ams.ams_pack(fmt, W, return_codes=True)
    o_codes, o_scales, _ = O.ams_quantize(W, ofmt)
    assert np.array_equal(scales, o_scales) and np.array_equal(codes, o_codes)
    W[0, 3] = np.float16(np.inf)
    with pytest.raises(ams.AmsError, match="inf or NaN"):
        ams.ams_pack(fmt, W)
    with pytest.raises(ams.AmsError, match="unknown format"):
        ams.ams_packed_bytes(9, 4, 4)
    with pytest.raises(ams.AmsError, match="out of range"):
        ams.ams_packed_bytes(fmt, 0, 4)
    lib = ams.load_library()
    assert lib.ams_pack(fmt, None, 4, 4, 4, None, None, None) == -3


@pytest.mark.parametrize("fmt,ofmt", PAIRS)
@pytest.mark.parametrize("N,K", [(16, 96), (16, 128), (16, 192), (16, 256), (16, 384), (16, 512), (19, 131), (1, 1), (48, 777)])
def test_layout_roundtrip_random_codes(fmt, ofmt, N, K):
    rng = np.random.default_rng(N * 1000 + K)
    g = ofmt.group
    rem = rng.integers(0, 1 << (ofmt.code_bits - 1), size=(N, K))
    sh = rng.integers(0, 2, size=(N, -(-K // g)))
    codes = ((rem << 1) | np.repeat(sh, g, axis=1)[:, :K]).astype(np.uint8)
    packed = ams.ams_pack_codes(fmt, codes)
    assert np.array_equal(ams.ams_unpack_host(fmt, packed, N, K), codes)
    # every stored bit matters: flipping any bit of a record that holds no padding changes a code
    if N % 16 == 0 and K % (REC[fmt][0] * SIDE_GROUP[fmt]) == 0 and N * K <= 16 * 512:
        for byte in range(0, packed.size, 7):
            for bit in range(8):
                p2 = packed.copy()
                p2[byte] ^= 1 << bit
                assert not np.array_equal(ams.ams_unpack_host(fmt, p2, N, K), codes), (byte, bit)
    if (fmt, ofmt) in PAPER_PAIRS:
        # codes that went through the paper's own packing come back the same
        via_paper = O.unpack_canonical(O.pack_canonical(codes, ofmt), ofmt, K).astype(np.uint8)
        assert np.array_equal(ams.ams_unpack_host(fmt, ams.ams_pack_codes(fmt, via_paper), N, K), codes)
    bad = codes.copy()
    if K >= 2 and g > 1:
        bad[0, 0] ^= 1  # group 0 no longer agrees in its last bit
        with pytest.raises(ams.AmsError):
            ams.ams_pack_codes(fmt, bad)


@pytest.mark.parametrize("fmt,ofmt", PAIRS)
def test_layout_is_k_major_in_units_of_side_groups(fmt, ofmt):
    # record r of strip s lives in unit (r // sg, s) at ((r // sg) * n_strips + s) * unit_bytes: its lane chunks in
    # chunk block r % sg of the unit, its last bits (if the format keeps them beside the chunks) in the unit's side dwords
    rec_k, rec_b = REC[fmt]
    sg = SIDE_GROUP[fmt]
    n_strips, n_rec = 3, 2 * sg + 1
    N, K = 16 * n_strips - 5, rec_k * n_rec - 7
    unit = rec_b * sg
    chunk_block = 64 * {ams.FP433: 12}.get(fmt, 16)
    side_bytes = (rec_b - chunk_block) // 64
    assert ams.ams_packed_bytes(fmt, N, K) == (-(-n_rec // sg)) * n_strips * unit
    full = (1 << ofmt.code_bits) - 1  # all bits set: sign, largest magnitude, last bit 1
    for strip in range(n_strips):
        for rec in range(n_rec):
            codes = np.zeros((N, K), dtype=np.uint8)
            k0 = rec * rec_k
            codes[16 * strip + 2, k0 : min(K, k0 + rec_k)] = full  # one whole row of one record
            packed = ams.ams_pack_codes(fmt, codes)
            nz = np.flatnonzero(packed)
            base = ((rec // sg) * n_strips + strip) * unit
            lo, hi = base + (rec % sg) * chunk_block, base + (rec % sg + 1) * chunk_block
            in_chunks = (nz >= lo) & (nz < hi)
            in_side = (nz >= base + sg * chunk_block) & (nz < base + unit)
            assert np.all(in_chunks | in_side), (strip, rec)
            assert in_chunks.any()
            if side_bytes:
                # the record's own byte(s) of the lanes' side dwords, nothing else
                side_at = nz[in_side] - (base + sg * chunk_block)
                assert side_at.size and np.all((side_at % 4) // side_bytes == rec % sg), (strip, rec)
            else:
                assert not in_side.any()


def test_padding_is_zero_and_layout_is_deterministic():
    W = synth.gaussian_weights(5, 50, 3)
    for fmt, _ in PAIRS:
        a, _ = ams.ams_pack(fmt, W)
        b, _ = ams.ams_pack(fmt, W)
        assert np.array_equal(a, b)
        # rows 5..15 and k >= 50 are padding: a matrix of zero codes packs to all-zero bytes
        z = ams.ams_pack_codes(fmt, np.zeros((5, 50), dtype=np.uint8))
        assert not z.any()


def test_launch_plans_cover_the_kernels_and_the_split():
    # host logic only: which kernel and launch shape a problem gets (the GPU tests run these very shapes)
    plan = lambda *a, **k: dict(kv.split("=") for kv in ams.ams_linear_plan(*a, **k).split()[1:])
    kind = lambda *a, **k: ams.ams_linear_plan(*a, **k).split()[0]
    assert kind(ams.FP533, 1, 28672, 4096) == "column"
    p = plan(ams.FP533, 1, 28672, 4096)  # seven strips per workgroup: eight wavefronts, one alone on each strip, three records ahead
    assert (p["grid"], p["strips_per_wg"], p["k_slices"], p["waves"], p["waves_per_strip"], p["phases"], p["ahead"]) == ("256", "7", "1", "8", "1", "1", "3")
    p = plan(ams.FP425, 1, 28672, 4096)  # the same with the side groups dealt whole
    assert (p["grid"], p["strips_per_wg"], p["waves"], p["waves_per_strip"], p["ahead"], p["side_groups"]) == ("256", "7", "8", "1", "3", "1")
    p = plan(ams.FP433, 1, 28672, 4096)  # the other formats with side groups keep sixteen wavefronts, two on each strip
    assert (p["waves"], p["waves_per_strip"], p["ahead"]) == ("16", "2", "2")
    assert plan(ams.FP533, 32, 28672, 4096)["waves"] == "16" and plan(ams.FP533, 8, 28672, 4096)["waves"] == "8"
    assert plan(ams.FP425, 1, 4096, 14336)["waves"] == "16"  # one strip per workgroup: sixteen wavefronts share it
    assert plan(ams.FP533, 1, 4096, 14336)["waves"] == "8" and plan(ams.FP533, 4, 4096, 14336)["waves"] == "16"
    assert plan(ams.FP533, 1, 4096, 4096)["waves"] == "16"  # 43 records for 8 wavefronts: too short a stream
    assert plan(ams.FP533, 1, 6144, 4096)["waves"] == "16"  # 192 workgroups do not fill the chip
    p = plan(ams.FP425, 1, 4096, 14336)  # one strip per workgroup: all 16 wavefronts on it
    assert (p["grid"], p["strips_per_wg"], p["waves_per_strip"], p["phases"]) == ("256", "1", "16", "1")
    p = plan(ams.FP533, 1, 57344, 8192)  # fourteen strips per workgroup: eight wavefronts (seven busy) with two strips each
    assert (p["grid"], p["strips_per_wg"], p["waves"], p["waves_per_strip"], p["strips_per_wave"], p["ahead"]) == ("256", "14", "8", "1", "2", "3")
    p = plan(ams.FP425, 1, 57344, 8192)  # with side groups: sixteen wavefronts, fourteen of them alone on a strip
    assert (p["grid"], p["strips_per_wg"], p["waves"], p["waves_per_strip"], p["strips_per_wave"]) == ("256", "14", "16", "1", "1")
    assert plan(ams.FP533, 16, 57344, 8192)["strips_per_wave"] == "1"
    assert plan(ams.FP533, 1, 128256, 4096)["strips_per_wg"] == "16"  # more strips than 16 x 256: more workgroups
    assert int(plan(ams.FP533, 1, 128256, 4096)["grid"]) == -(-(-(-128256 // 16)) // 16)
    assert kind(ams.FP533, 32, 57344, 8192) == "column" and int(plan(ams.FP533, 32, 57344, 8192)["phases"]) > 1
    assert int(plan(ams.FP425, 8, 4096, 14336)["phases"]) > 1
    assert plan(ams.FP425, 8, 4096, 14336, with_workspace=True)["k_slices"] == "4"
    assert plan(ams.FP425, 1, 4096, 14336, with_workspace=True)["k_slices"] == "1"
    assert kind(-1, 1, 4096, 4096) == "gemv" and kind(-1, 4, 28672, 4096) == "gemv"  # small batches: rows dealt to wavefronts
    assert kind(-1, 4, 8192, 28672) == "sweep"  # four rows of 28672 activations do not fit in LDS
    assert kind(-1, 8, 4096, 4096) == "sweep"
    assert kind(-1, 32, 57344, 8192) == "stream"  # the baseline with many parked tiles and more than two phases
    for fmt, _ in PAIRS:
        for M in (1, 7, 16, 17, 32):
            for N, K in [(1, 1), (16, 5), (37, 1000), (100000, 64), (64, 100000), (1 << 20, 96)]:
                assert int(plan(fmt, M, N, K)["lds"]) <= 160 * 1024
                assert int(plan(fmt, M, N, K, with_workspace=True)["lds"]) <= 160 * 1024
    with pytest.raises(ams.AmsError):
        ams.ams_linear_plan(ams.FP533, 33, 16, 96)


def test_header_is_plain_c_and_links_from_a_c_program(tmp_path):
    # the boundary is a C ABI: the header must compile as C99 and the host entry points must be
    # callable from a program that has never heard of Python (no device call here)
    import os
    import shutil
    import subprocess

    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    libdir = os.path.join(root, "paper_2510_16045_amd")
    src = tmp_path / "abi.c"
    src.write_text(
        """
#include "ams.h"
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
int main(void) {
  size_t bytes = 0, canon = 0;
  const int64_t N = 20, K = 100;
  uint16_t W[20 * 100];
  uint16_t scales[20];
  uint8_t codes[20 * 100], back[20 * 100];
  void* packed;
  int i;
  for (i = 0; i < 20 * 100; i++) W[i] = (uint16_t)(0x2000 + 37 * i % 0x1400 + ((i & 1) << 15)); /* small fp16 values of both signs */
  if (ams_packed_bytes(AMS_FMT_FP425_E2M2, N, K, &bytes) != AMS_OK || ams_canonical_bytes(AMS_FMT_FP425_E2M2, N, K, &canon) != AMS_OK) return 1;
  packed = malloc(bytes);
  if (ams_pack(AMS_FMT_FP425_E2M2, W, N, K, K, packed, scales, codes) != AMS_OK) return 2;
  if (ams_unpack_host(AMS_FMT_FP425_E2M2, packed, N, K, back) != AMS_OK) return 3;
  if (memcmp(codes, back, sizeof codes) != 0) return 4;
  if (ams_pack(99, W, N, K, K, packed, scales, codes) == AMS_OK) return 5;
  printf("%d %lu %lu %s\\n", ams_version(), (unsigned long)bytes, (unsigned long)canon, ams_strerror(AMS_OK));
  free(packed);
  return 0;
}
"""
    )
    exe = tmp_path / "abi"
    cc = subprocess.run([gcc, "-std=c99", "-pedantic", "-Wall", "-Werror", "-I", os.path.join(root, "include"), str(src), "-o", str(exe),
                         "-L", libdir, "-lams", f"-Wl,-rpath,{libdir}"], capture_output=True, text=True)
    assert cc.returncode == 0, cc.stderr
    r = subprocess.run([str(exe)], capture_output=True, text=True, timeout=60)
    assert r.returncode == 0, (r.returncode, r.stdout, r.stderr)
    version, bytes_, canon, _ = r.stdout.split(None, 3)
    assert int(bytes_) == ams.ams_packed_bytes(ams.FP425, 20, 100) and int(canon) == 34 * 2 * 20


def test_launch_plans_random_shapes_stay_inside_the_machine():
    # seeded random shapes, every format and the baseline, with and without a workspace: the plan
    # must exist, fit the 160 KiB of LDS, use at most 16 wavefronts and a grid the kernel can index
    rng = np.random.default_rng(7)
    fmts = [f for f, _ in PAIRS] + [-1]
    for _ in range(1500):
        fmt = fmts[int(rng.integers(len(fmts)))]
        M = int(rng.integers(1, 33))
        N = int(2 ** rng.uniform(0, 20))
        K = int(2 ** rng.uniform(0, 17))
        if fmt == -1:
            K = max(8, K // 8 * 8)
        for ws in (False, True):
            text = ams.ams_linear_plan(fmt, M, N, K, with_workspace=ws)
            kind, kv = text.split()[0], dict(x.split("=") for x in text.split()[1:])
            assert kind == ("column" if fmt >= 0 else kind) and kind in ("column", "gemv", "sweep", "stream"), text
            assert 0 < int(kv["lds"]) <= 160 * 1024, text
            assert 1 <= int(kv["waves"]) <= 16 and int(kv["phases"]) >= 1 and int(kv["grid"]) >= 1, text
            n_strips = -(-N // 16)
            if kind == "gemv":
                assert M <= 4 and int(kv["rows_per_wave"]) * int(kv["grid"]) * 16 >= N and int(kv["lds"]) >= 2 * M * K, text
                continue
            assert int(kv["strips_per_wg"]) * int(kv["grid"]) >= n_strips * int(kv["k_slices"]) or kind == "stream", text
            if kind == "sweep":
                assert 16 % int(kv["waves_per_strip"]) == 0 or int(kv["waves_per_strip"]) == int(kv["waves"]), text
            if kind == "column":
                if kv["strips_per_wave"] == "1":
                    assert int(kv["strips_per_wg"]) <= 16 and int(kv["waves_per_strip"]) == int(kv["waves"]) // int(kv["strips_per_wg"]) >= 1, text
                else:  # wavefronts that own two strips each
                    assert (kv["strips_per_wave"], kv["waves"], kv["waves_per_strip"], kv["k_slices"]) == ("2", "8", "1", "1") and 9 <= int(kv["strips_per_wg"]) <= 16, text
                assert (kv["waves"], kv["ahead"]) in (("16", "2"), ("8", "3")), text
            if not ws:
                assert kv["k_slices"] == "1", text
            need = ams.ams_linear_workspace_bytes(fmt, M, N, K)
            assert (need > 0) == (ws and int(kv["k_slices"]) > 1) or not ws, text


def test_bench_refuses_more_than_one_gpu():
    import os
    import subprocess
    import sys

    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_device_entry_points_refuse_a_machine_without_the_gpu():
    # Argument checks come first, then the device check, then the launch: with valid-looking arguments and no
    # gfx950 current every device entry point returns AMS_ERR_DEVICE and never touches the pointers.
    torch = pytest.importorskip("torch")
    if torch.cuda.is_available():
        pytest.skip("a GPU is present: the device entry points would run")
    lib = ams.load_library()
    AMS_ERR_DEVICE = -7
    assert lib.ams_init() == AMS_ERR_DEVICE
    assert b"gfx950" in lib.ams_strerror(AMS_ERR_DEVICE)
    p = ctypes.c_void_p(1 << 20)  # aligned, never dereferenced
    M, N, K = 1, 256, 768
    assert lib.ams_linear(p, p, p, p, M, N, K, ams.FP425, None) == AMS_ERR_DEVICE
    assert lib.ams_linear_ws(p, p, p, p, M, N, K, ams.FP533, p, 1 << 20, None) == AMS_ERR_DEVICE
    assert lib.ams_linear_static_ws(p, p, p, p, M, N, K, ams.FP533, None) == AMS_ERR_DEVICE
    assert lib.ams_fp16_linear(p, p, p, M, N, K, None) == AMS_ERR_DEVICE
    assert lib.ams_dequant(ams.FP425, p, p, p, N, K, 1, None) == AMS_ERR_DEVICE
    assert lib.ams_read_probe(p, 4096, None, None) == AMS_ERR_DEVICE
    # argument errors still win over the device error
    assert lib.ams_linear(None, p, p, p, M, N, K, ams.FP425, None) == -3  # AMS_ERR_NULL
    assert lib.ams_linear(p, p, p, p, 33, N, K, ams.FP425, None) == -2  # AMS_ERR_SHAPE
    with pytest.raises(ams.AmsError):
        ams.ams_init()
