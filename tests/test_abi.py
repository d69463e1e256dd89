"""Host logic of the C ABI: exported symbols, argument checking, handle life-cycle.  No GPU."""
from __future__ import annotations

import ctypes as C
import os
import re

import numpy as np
import pytest

import gqsa_inputs as gi
import paper_2412_17560_amd as gq
from paper_2412_17560_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    """Every function declared in include/*.h (gqsa.h: the product; gqsa_bench.h: the measuring instruments)."""
    names = set()
    inc = os.path.join(ROOT, "include")
    for header in sorted(os.listdir(inc)):
        if not header.endswith(".h"):
            continue
        text = open(os.path.join(inc, header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names.update(re.findall(r"\b(gqsa_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    lib = C.CDLL(gq.library_path())
    names = declared_functions()
    assert "gqsa_pack" in names and "gqsa_gemv" in names and "gqsa_gemv_static" in names
    assert "gqsa_stream_read" in names and len(names) >= 25
    for name in names:
        assert hasattr(lib, name), f"libgqsa.so does not export {name}"


def test_status_strings():
    assert gq.gqsa_status_string(0) == "ok"
    assert len({gq.gqsa_status_string(s) for s in range(10)}) == 10


def status_of(fn, *args, **kw):
    with pytest.raises(gq.GqsaError) as e:
        fn(*args, **kw)
    return e.value.status


def test_pack_argument_errors():
    W = gi.dense_weight(8, 64, seed=1)
    assert status_of(gq.gqsa_pack, W, 16, 3, 0.5) == 3          # bits
    assert status_of(gq.gqsa_pack, W, 4, 4, 0.5) == 3           # G
    assert status_of(gq.gqsa_pack, W, 24, 4, 0.5) == 3
    assert status_of(gq.gqsa_pack, W[:, :40], 16, 4, 0.5) == 2  # K % G
    assert status_of(gq.gqsa_pack, W[:, :40], 8, 4, 0.5) == 2   # G = 8: K still a multiple of 16
    assert status_of(gq.gqsa_pack, W, 16, 4, 1.5) == 4
    assert status_of(gq.gqsa_pack, W, 16, 4, -0.1) == 4
    assert status_of(gq.gqsa_pack, W, 16, 4, float("nan")) == 4
    Wn = W.copy()
    Wn[2, 5] = np.nan
    assert status_of(gq.gqsa_pack, Wn, 16, 4, 0.5) == 4
    keep = np.full(8, 5, dtype=np.int32)
    assert status_of(gq.gqsa_pack_rows, W, keep, 16, 4) == 4    # 5 > K/G = 4
    keep[:] = -1
    assert status_of(gq.gqsa_pack_rows, W, keep, 16, 4) == 4
    lib = binding._lib()
    out = C.c_void_p(123)
    assert lib.gqsa_pack(None, 8, 64, 16, 4, 0.5, C.byref(out)) == 1
    assert out.value is None                                    # handle cleared on failure
    assert lib.gqsa_pack(C.c_void_p(W.ctypes.data), 8, 64, 16, 4, 0.5, None) == 1
    assert lib.gqsa_pack(C.c_void_p(W.ctypes.data), 0, 64, 16, 4, 0.5, C.byref(out)) == 2


def test_import_validation():
    ri = np.array([0, 2, 3], dtype=np.int32)
    va = np.zeros(3 * 8, dtype=np.uint8)
    sc = np.full(3, 0x3C00, dtype=np.uint16)
    ze = np.zeros(3, dtype=np.uint16)
    ok = gq.gqsa_import(ri, [0, 3, 1], va, sc, ze, 2, 64)
    assert gq.gqsa_info(ok)["nnz_groups"] == 3
    assert status_of(gq.gqsa_import, ri, [3, 0, 1], va, sc, ze, 2, 64) == 2   # not ascending in row
    assert status_of(gq.gqsa_import, ri, [0, 4, 1], va, sc, ze, 2, 64) == 2   # column out of range
    bad = np.array([0, 3, 2], dtype=np.int32)
    with pytest.raises((gq.GqsaError, ValueError)):
        gq.gqsa_import(bad, [0, 1], va[:16], sc[:2], ze[:2], 2, 64)
    bad0 = np.array([1, 2, 3], dtype=np.int32)
    assert status_of(gq.gqsa_import, bad0, [0, 3, 1], va, sc, ze, 2, 64) == 2


def test_partition_and_blob_buffer_errors():
    W = gi.dense_weight(8, 64, seed=1)
    h = gq.gqsa_pack(W, 16, 4, 0.5)
    assert status_of(gq.gqsa_set_partition, h, 0, 16) == 4
    assert status_of(gq.gqsa_set_partition, h, 5000, 16) == 4
    assert status_of(gq.gqsa_set_partition, h, 4, 0) == 4
    assert status_of(gq.gqsa_set_partition, h, 4, 17) == 4
    lib = binding._lib()
    buf = np.zeros(16, dtype=np.uint8)
    assert lib.gqsa_export_device_blob(h.ptr, C.c_void_p(buf.ctypes.data), 16) == 7
    info = binding._Info()
    assert lib.gqsa_info(None, C.byref(info)) == 1
    assert lib.gqsa_gemv(None, None, None, 1, None) == 1
    gq.gqsa_free(h)
    gq.gqsa_free(h)           # idempotent through the binding
    lib.gqsa_free(None)       # and NULL-safe in C


def test_gemv_host_side_checks_need_no_gpu():
    """Argument checks that fail before any HIP call (so they can run here)."""
    W = gi.dense_weight(8, 64, seed=1)
    h = gq.gqsa_pack(W, 16, 4, 0.5)
    lib = binding._lib()
    fake = C.c_void_p(0x1000)
    assert lib.gqsa_gemv(h.ptr, fake, fake, 0, None) == 3
    assert lib.gqsa_gemv(h.ptr, fake, fake, 17, None) == 3
    assert lib.gqsa_gemv(h.ptr, C.c_void_p(0x1008), fake, 1, None) == 8


def test_gemv_static_host_side_checks_need_no_gpu():
    """The entry point that allocates nothing never uploads: a handle that is not on the device is refused."""
    W = gi.dense_weight(8, 64, seed=1)
    h = gq.gqsa_pack(W, 16, 4, 0.5)
    lib = binding._lib()
    fake = C.c_void_p(0x1000)
    assert lib.gqsa_gemv_static(None, fake, fake, 1, None) == 1
    assert lib.gqsa_gemv_static(h.ptr, fake, fake, 0, None) == 3
    assert lib.gqsa_gemv_static(h.ptr, fake, fake, 17, None) == 3
    assert lib.gqsa_gemv_static(h.ptr, C.c_void_p(0x1008), fake, 1, None) == 8
    assert lib.gqsa_gemv_static(h.ptr, fake, fake, 1, None) == 3       # not uploaded
    assert gq.gqsa_info(h)["on_device"] == 0


@pytest.mark.skipif(bool(os.environ.get("GQSA_LIBRARY")),
                    reason="a sanitizer's operator new ends the process on an impossible request instead of throwing")
def test_allocation_failure_is_a_status_not_an_exception():
    """A device image far beyond the address space (2^31 tiles per span x 4096 spans): the failed
    allocation inside the library comes back as GQSA_ERR_ALLOC and the handle stays usable."""
    W = gi.dense_weight(8, 64, seed=1)
    h = gq.gqsa_pack(W, 16, 4, 0.5)
    before = gq.gqsa_export_device_blob(h)
    assert status_of(gq.gqsa_set_partition_aligned, h, 2**31 - 1, 4096, 16) == 5
    assert gq.gqsa_export_device_blob(h) == before
    assert gq.gqsa_info(h)["span_tiles"] != 2**31 - 1


def test_default_partition_entry_checks_its_arguments():
    lib = binding._lib()
    ri = np.array([0, 2, 3], dtype=np.int32)
    out = (C.c_int32 * 6)()
    assert lib.gqsa_default_partition(None, 2, 64, 16, 4, C.byref(out)) == 1
    assert lib.gqsa_default_partition(C.c_void_p(ri.ctypes.data), 2, 64, 16, 4, None) == 1
    assert lib.gqsa_default_partition(C.c_void_p(ri.ctypes.data), 2, 64, 16, 5, C.byref(out)) == 3
    assert lib.gqsa_default_partition(C.c_void_p(ri.ctypes.data), 2, 24, 16, 4, C.byref(out)) == 2
    bad = np.array([0, 9, 3], dtype=np.int32)                      # 9 groups in a row of 4 columns
    assert lib.gqsa_default_partition(C.c_void_p(bad.ctypes.data), 2, 64, 16, 4, C.byref(out)) == 2
    assert gq.gqsa_default_partition(ri, 64) == (1, 1, 0, 4, 64, 0)      # three groups fill no tile: one worker, one padded tile


def test_gemv_multi_host_side_checks_need_no_gpu():
    W = gi.dense_weight(8, 64, seed=1)
    W2 = gi.dense_weight(8, 128, seed=1)
    h, hk = gq.gqsa_pack(W, 16, 4, 0.5), gq.gqsa_pack(W2, 16, 4, 0.5)
    lib = binding._lib()
    fake = C.c_void_p(0x1000)
    hs = (C.c_void_p * 2)(h.ptr.value, hk.ptr.value)
    ys = (C.c_void_p * 2)(0x2000, 0x3000)
    assert lib.gqsa_gemv_multi(None, 1, fake, ys, 1, None) == 1
    assert lib.gqsa_gemv_multi(hs, 0, fake, ys, 1, None) == 3
    assert lib.gqsa_gemv_multi(hs, 5, fake, ys, 1, None) == 3
    assert lib.gqsa_gemv_multi(hs, 2, fake, ys, 17, None) == 3
    assert lib.gqsa_gemv_multi(hs, 2, C.c_void_p(0x1004), ys, 1, None) == 8
    assert lib.gqsa_gemv_multi(hs, 2, fake, ys, 1, None) == 2          # K differs
    same = (C.c_void_p * 2)(h.ptr.value, h.ptr.value)
    assert lib.gqsa_gemv_multi(same, 2, fake, ys, 1, None) == 2        # the same handle twice


def test_info_fields():
    W = gi.dense_weight(100, 512, seed=5)
    keep = gi.imbalanced_keep_counts(100, 32, seed=5)
    h = gq.gqsa_pack_rows(W, keep, 16, 8)
    info = gq.gqsa_info(h)
    nnz = int(keep.sum())
    assert info["N"] == 100 and info["K"] == 512 and info["G"] == 16 and info["bits"] == 8
    assert info["nnz_groups"] == nnz and info["values_bytes"] == nnz * 16
    # short rows (at most 32 groups) fill tiles of any shape well: by default whole rows per worker, one tile each
    assert info["span_tiles"] == 1 and info["span_per_worker"] == 1 and info["needs_fixup"] == 0
    assert info["n_blocks"] == info["tile_blocks"] * info["n_workgroups"] * info["waves_per_workgroup"]
    assert info["n_blocks"] * info["tile_lanes"] <= nnz + nnz // 8 + info["tile_blocks"] * info["tile_lanes"] * 4 * 3
    gq.gqsa_set_partition(h, 3, 2)
    info = gq.gqsa_info(h)
    assert info["span_tiles"] == 0 and info["n_blocks"] == 4 * ((nnz + 255) // 256) and info["tile_lanes"] == 64
    assert info["n_empty_rows"] == int((keep == 0).sum())
    assert info["on_device"] == 0
    assert info["algorithmic_bytes"] == nnz * 22 + 101 * 4 + (512 + 100) * 2


def test_pack_hessian_argument_checks():
    W = np.ones((4, 64), dtype=np.float32)
    d = np.ones(64, dtype=np.float32)
    for bad in (0.0, -2.0, np.inf, np.nan):
        db = d.copy()
        db[5] = bad
        assert status_of(gq.gqsa_pack_hessian, W, db, 16, 4, 0.5) == 4
    assert status_of(gq.gqsa_pack_hessian, W, d, 16, 4, 1.5) == 4
    assert status_of(gq.gqsa_pack_hessian, W, d, 24, 4, 0.5) == 3
    lib = C.CDLL(gq.library_path())
    lib.gqsa_pack_hessian.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_int, C.c_int, C.c_double,
                                      C.c_void_p, C.c_void_p]
    out = C.c_void_p()
    assert lib.gqsa_pack_hessian(C.c_void_p(W.ctypes.data), 4, 64, 16, 4, 0.5, None, C.byref(out)) == 1


def test_save_and_load_round_trip_and_damaged_files(tmp_path):
    W = gi.dense_weight(50, 512, seed=3)
    keep = gi.imbalanced_keep_counts(50, 512 // 32, seed=3)
    h = gq.gqsa_pack_rows(W, keep, 32, 4)
    path = str(tmp_path / "m.gqsa")
    gq.gqsa_save(h, path)
    e = gq.gqsa_export(h)
    assert os.path.getsize(path) == 48 + 51 * 4 + e["groups"].size * 4 + e["values"].size + e["groups"].size * 4
    h2 = gq.gqsa_load(path)
    e2 = gq.gqsa_export(h2)
    for k in e:
        assert np.array_equal(e[k], e2[k]), k
    i1, i2 = gq.gqsa_info(h), gq.gqsa_info(h2)
    assert {k: i1[k] for k in ("N", "K", "G", "bits", "nnz_groups")} == {k: i2[k] for k in ("N", "K", "G", "bits", "nnz_groups")}
    assert gq.gqsa_export_device_blob(h) == gq.gqsa_export_device_blob(h2)
    # an empty matrix goes through too
    h0 = gq.gqsa_pack(W, 16, 8, 1.0)
    gq.gqsa_save(h0, path)
    assert gq.gqsa_info(gq.gqsa_load(path))["nnz_groups"] == 0
    # damaged files are refused with a status, never read past their end
    gq.gqsa_save(h, path)
    raw = open(path, "rb").read()
    cases = {"truncated": (raw[:len(raw) - 7], 9), "header only": (raw[:48], 9), "short header": (raw[:20], 9),
             "foreign": (b"NOTGQSA!" + raw[8:], 2), "trailing": (raw + b"x", 2),
             "bad group size": (raw[:24] + (17).to_bytes(4, "little") + raw[28:], 3),
             "count too large": (raw[:32] + (1 << 40).to_bytes(8, "little") + raw[40:], 2)}
    descending = bytearray(raw)
    off = 48 + 51 * 4                       # first two group-columns of row 0 swapped
    descending[off:off + 4], descending[off + 4:off + 8] = raw[off + 4:off + 8], raw[off:off + 4]
    if keep[0] >= 2:
        cases["descending columns"] = (bytes(descending), 2)
    for name, (data, status) in cases.items():
        open(path, "wb").write(data)
        assert status_of(gq.gqsa_load, path) == status, name
    assert status_of(gq.gqsa_load, str(tmp_path / "missing.gqsa")) == 9
    assert status_of(gq.gqsa_save, h, str(tmp_path / "no_such_dir" / "m.gqsa")) == 9


def _balanced(n_rows, per_row):
    return np.arange(n_rows + 1, dtype=np.int64) * per_row


def test_default_partition_hand_table():
    """The partition the library chooses by itself, against values worked out by hand from its
    documented rule (include/gqsa.h, gqsa_set_partition): (workgroups, wavefronts per workgroup,
    tiles per span, blocks per tile, lanes in use, span per worker)."""
    dp = gq.gqsa_default_partition
    assert dp(_balanced(1, 0), 4096) == (1, 1, 0, 4, 64, 0)                # nothing stored: the plain deal of no tiles
    # K <= 4096, rows that fill tiles of the format's own shape: whole rows per worker, one tile each
    assert dp(_balanced(3, 256), 4096) == (1, 4, 1, 4, 64, 1)              # 3 tiles of 256 groups, a row each
    assert dp(_balanced(16, 128), 4096) == (2, 4, 1, 4, 64, 1)             # 8 tiles; two rows per tile
    assert dp(_balanced(17, 256), 4096) == (8, 4, 1, 4, 64, 1)             # 17 workers -> 5 workgroups -> a multiple of 4
    assert dp(_balanced(4096, 128), 4096) == (512, 4, 1, 4, 64, 1)         # 4096x4096 at S = 50 %: 2048 tiles
    assert dp(_balanced(11008, 128), 4096) == (1376, 4, 1, 4, 64, 1)       # 11008x4096: 5504 tiles
    assert dp(_balanced(8193, 256), 4096) == (2052, 4, 1, 4, 64, 1)
    assert dp(_balanced(16384, 256), 4096) == (4096, 4, 1, 4, 64, 1)       # the most workers
    assert dp(_balanced(16385, 256), 4096) == (2052, 4, 1, 8, 64, 1)       # beyond: two rows per tile of 8 x 64, 8193 workers
    assert dp(_balanced(128256, 128), 4096) == (4008, 4, 4, 4, 64, 1)      # 64128 tiles: four per worker
    assert dp(_balanced(2048, 32), 4096, G=128) == (256, 4, 1, 1, 64, 1)   # 64 code bytes: a tile is one block, two rows in it
    assert dp(_balanced(2048, 128), 4096, G=16, bits=8) == (256, 4, 1, 4, 64, 1)   # 16 code bytes: tiles of 4 blocks
    assert dp(_balanced(4096, 100), 4096, G=32) == (208, 4, 2, 4, 64, 1)   # no other shape for G = 32: 2 rows in 256 leave 28 % empty, 5 rows in two tiles 2.4 %
    # rows that do not fill such tiles: a shape that they do fill
    assert dp(_balanced(4096, 179), 4096) == (1024, 4, 1, 3, 60, 1)        # S = 30 %: 179 of 3 x 60 = 180 positions, a row per worker
    assert dp(_balanced(14336, 179), 4096) == (3584, 4, 1, 3, 60, 1)
    assert dp(_balanced(4096, 179), 4096, bits=8) == (1024, 4, 1, 3, 60, 1)
    assert dp(_balanced(4096, 205), 4096) == (1024, 4, 1, 4, 52, 1)        # 205 of 4 x 52 = 208 (three blocks hold 192 at most)
    assert dp(_balanced(4096, 77), 4096) == (512, 4, 1, 3, 52, 1)          # S = 70 %: two rows (154) of 3 x 52 = 156
    alternating = np.concatenate(([0], np.cumsum(np.tile([256, 8], 500))))
    assert dp(alternating, 4096) == (128, 4, 1, 5, 56, 1)                   # a long and a short row (264) of 5 x 56 = 280: 6 % empty
    alternating = np.concatenate(([0], np.cumsum(np.tile([256, 100], 500))))
    assert dp(alternating, 4096) == (128, 4, 1, 6, 60, 1)                   # a pair (356) of 6 x 60 = 360
    uneven = np.concatenate(([0], np.cumsum(np.tile([250, 30, 3, 140], 250))))
    assert dp(uneven, 4096) == (64, 4, 1, 8, 56, 1)                         # the four rows (423) of 8 x 56 = 448; 8 x 60 would leave 13.5 % empty, no smaller tile holds them
    # K > 4096, rows that fill a tile shape and at least a workgroup of 8 workers per compute unit: whole rows per
    # worker, the shape with the fewest workers (then the most lanes in use)
    assert dp(_balanced(4096, 344), 11008) == (512, 8, 1, 6, 60, 1)        # 4096x11008 at S = 50 %: a row of 344 in 6 x 60 = 360
    assert dp(_balanced(4096, 448), 14336) == (512, 8, 1, 8, 56, 1)        # 4096x14336: 448 = 8 x 56
    assert dp(_balanced(4096, 269), 14336) == (512, 8, 1, 5, 56, 1)        # at S = 70 %: 269 of 280
    assert dp(_balanced(4096, 256), 8192) == (256, 8, 1, 8, 64, 1)         # 4096x8192 at S = 50 %: two rows in 8 x 64, 2048 workers
    assert dp(_balanced(8191, 256), 8192) == (512, 8, 1, 8, 64, 1)         # 4096 workers
    assert dp(_balanced(4096, 206), 11008) == (256, 8, 1, 8, 52, 1)        # two rows of 206 in 8 x 52 = 416: 2048 workers (4 x 52 would take 4096)
    # K > 4096 otherwise: by size
    assert dp(_balanced(4096, 344), 11008, bits=8) == (256, 8, 22, 4, 64, 0)   # 8-bit codes have no tile of 6 blocks: 448 T / K = 224 -> one workgroup per compute unit; 16 rows (21.5 tiles) per span of 22
    assert dp(_balanced(4096, 688), 11008) == (256, 8, 43, 4, 64, 0)       # a row of 688 fits no tile: 448 T / K = 448 = 1.75 x 256, rounded down beyond K = 8192; 16 rows = 43 tiles per span
    assert dp(_balanced(3000, 256), 8192) == (376, 8, 1, 4, 64, 1)         # two rows per tile of 8 x 64 would be 1500 workers, fewer than 8 per compute unit: a row per 4 x 64
    assert dp(_balanced(2000, 256), 8192) == (500, 4, 4, 4, 64, 0)         # 2000 workers at most: too few; and fewer than 2048 tiles: the small shapes' deal
    assert dp(_balanced(100, 256), 32768) == (28, 4, 4, 4, 64, 0)          # few tiles: one per wavefront, whatever K (25 workgroups -> a multiple of 4)
    # too many null groups (a row of 600 per span of 1024: 424 of 1024 positions empty): the plain deal
    assert dp(_balanced(12000, 600), 16384) == (512, 8, 0, 4, 64, 0)
