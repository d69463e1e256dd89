"""The library's host packer and device-image builder against the oracle, bit for bit.

Runs without a GPU: gqsa_pack / gqsa_export / gqsa_export_device_blob never touch HIP.
"""
from __future__ import annotations

import numpy as np
import pytest

import gqsa_inputs as gi
import oracle
import paper_2412_17560_amd as gq


def assert_same_canonical(h, c):
    e = gq.gqsa_export(h)
    assert np.array_equal(e["rowIndex"], c.rowIndex)
    assert np.array_equal(e["groups"], c.groups)
    assert np.array_equal(e["values"], c.values)
    assert np.array_equal(e["scales"], c.scales)
    assert np.array_equal(e["zeros"], c.zeros)


def assert_same_blob(h, c):
    info = gq.gqsa_info(h)
    blob = gq.gqsa_export_device_blob(h)
    ref = oracle.device_blob_for(c, info)
    assert len(blob) == len(ref) == info["device_bytes"]
    assert blob == ref


@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("sparsity", [0.0, 0.3, 0.5, 0.7, 1.0])
def test_tiny_config_balanced(bits, sparsity):
    W, _ = gi.tiny_config()
    h = gq.gqsa_pack(W, 16, bits, sparsity)
    c = oracle.pack(W, 16, bits, sparsity=sparsity)
    assert_same_canonical(h, c)
    assert_same_blob(h, c)
    info = gq.gqsa_info(h)
    assert info["nnz_groups"] == c.nnzg
    assert gq.gqsa_partition(h) == gq.gqsa_default_partition(c.rowIndex, 256, 16, bits)
    assert info["algorithmic_bytes"] == oracle.algorithmic_bytes(256, 256, 16, bits, c.nnzg, 1)


@pytest.mark.parametrize("bits,G", [(4, 16), (8, 16), (4, 64), (4, 128)])
def test_rows_kept_inside_workgroup_spans(bits, G):
    """The aligned form of the stream: spans, null groups between them, worker records."""
    N, K = 301, 2048
    W = gi.dense_weight(N, K, seed=78)
    keep = gi.imbalanced_keep_counts(N, K // G, seed=78)
    keep[[0, 5, 6, 7, 300]] = 0                         # empty rows at the ends and in a run
    keep[100] = K // G                                  # a full row
    h = gq.gqsa_pack_rows(W, keep, G, bits)
    c = oracle.pack(W, G, bits, keep_per_row=keep)
    U = 4 if G * bits // 8 <= 16 else (2 if G * bits // 8 <= 32 else 1)
    for span, wgs, wpw in ((1, 0, 1), (1, 0, 4), (2, 0, 3), (4, 0, 4), (3, 0, 16), (16, 0, 8), (4, 64, 4), (1000, 0, 2), (1000, 3, 16)):
        _, L = oracle.row_positions(c.rowIndex, span * 64 * U)
        need = max(1, -(-L // (span * 64 * U)))
        if need > 4096:
            continue
        gq.gqsa_set_partition_aligned(h, span, wgs, wpw)
        info = gq.gqsa_info(h)
        assert info["span_tiles"] == span and info["waves_per_workgroup"] == wpw
        assert info["n_workgroups"] == (wgs if wgs else need)
        assert info["n_blocks"] == U * span * info["n_workgroups"]
        assert_same_blob(h, c)
    # fewer workgroups than the rows need spans; bad arguments
    _, L = oracle.row_positions(c.rowIndex, 64 * U)
    need = -(-L // (64 * U))
    if 1 < need <= 4096:
        with pytest.raises(gq.GqsaError) as e:
            gq.gqsa_set_partition_aligned(h, 1, need - 1, 4)
        assert e.value.status == 4
    for bad in ((0, 0, 4), (-1, 4, 4), (1, 4097, 4), (1, 0, 0), (1, 0, 17), (1, -1, 4)):
        with pytest.raises(gq.GqsaError) as e:
            gq.gqsa_set_partition_aligned(h, *bad)
        assert e.value.status == 4
    gq.gqsa_set_partition(h, 5, 3)                       # and back to the plain form
    assert gq.gqsa_info(h)["span_tiles"] == 0
    assert_same_blob(h, c)


def test_aligned_stream_keeps_rows_inside_spans():
    """Read back from the image: no row of at most a span's length has groups in two spans."""
    N, K, G, bits = 500, 4096, 16, 4
    W = gi.dense_weight(N, K, seed=79)
    keep = np.full(N, 179, dtype=np.int32)               # S = 30 %: 5 rows per span of 1024, 129 null groups after them
    h = gq.gqsa_pack_rows(W, keep, G, bits)
    gq.gqsa_set_partition_aligned(h, 4, 0, 4)
    info = gq.gqsa_info(h)
    assert gq.gqsa_partition(h) == (100, 4, 4, 4, 64, 0)
    blob = np.frombuffer(gq.gqsa_export_device_blob(h), dtype=np.uint8)
    nblocks = info["n_blocks"]
    blk = blob[:nblocks * 896].reshape(nblocks, 896)
    ix = blk[:, 768:].copy().view("<u2").reshape(nblocks // 4, 4, 64)      # [tile][block][lane]
    sz = blk[:, 512:768].copy().view("<u4").reshape(nblocks // 4, 4, 64)
    heads = (ix & 1).transpose(0, 2, 1).reshape(-1)      # stream order: position = tile*256 + lane*4 + block
    scale = (sz & 0xFFFF).transpose(0, 2, 1).reshape(-1)
    head_pos = np.nonzero(heads)[0]
    assert len(head_pos) == N
    assert np.all(head_pos // 1024 == (head_pos + 178) // 1024)
    assert np.array_equal(head_pos[:6], [0, 179, 358, 537, 716, 1024])
    assert np.all(scale[895:1024] == 0) and np.all(ix.transpose(0, 2, 1).reshape(-1)[895:1024] == 0)   # the null groups


@pytest.mark.parametrize("bits", [4, 8])
def test_rows_kept_inside_workers_tiles(bits):
    """The form with one span per worker and tiles of a chosen shape (blocks per tile, lanes in
    use): the image against the oracle's for uniform and ragged rows, the sizes that follow from
    the shape, and what the library refuses."""
    N, K = 301, 2048
    W = gi.dense_weight(N, K, seed=78)
    keep = gi.imbalanced_keep_counts(N, K // 16, seed=78)
    keep[[0, 5, 6, 7, 300]] = 0
    keep[100] = K // 16                                  # the longest row: 128 groups
    h = gq.gqsa_pack_rows(W, keep, 16, bits)
    c = oracle.pack(W, 16, bits, keep_per_row=keep)
    for (u, lanes, wgs, wpw) in ((3, 60, 0, 4), (3, 44, 0, 1), (4, 32, 0, 4), (4, 64, 0, 16), (5, 36, 0, 3), (5, 64, 40, 8)):
        gq.gqsa_set_partition_rows(h, u, lanes, 1, wgs, wpw)
        info = gq.gqsa_info(h)
        _, L = oracle.row_positions(c.rowIndex, u * lanes)
        spans = -(-L // (u * lanes))
        assert (info["tile_blocks"], info["tile_lanes"], info["span_tiles"], info["span_per_worker"]) == (u, lanes, 1, 1)
        assert info["n_workgroups"] == (wgs if wgs else -(-spans // wpw)) and info["waves_per_workgroup"] == wpw
        assert info["n_blocks"] == u * info["n_workgroups"] * wpw
        assert info["needs_fixup"] == 0                 # every row fits a tile of these shapes
        assert_same_blob(h, c)
    # rows longer than a tile are shared by workers as in the other forms
    gq.gqsa_set_partition_rows(h, 3, 32, 1, 0, 4)
    assert gq.gqsa_info(h)["needs_fixup"] == 1
    assert_same_blob(h, c)
    # several tiles per worker: of the format's own shape only
    gq.gqsa_set_partition_rows(h, 4, 64, 3, 0, 2)
    assert gq.gqsa_partition(h)[2:] == (3, 4, 64, 1)
    assert_same_blob(h, c)
    for (args, status) in (((3, 60, 2, 0, 4), 3), ((2, 64, 1, 0, 4), 3), ((7, 64, 1, 0, 4), 3), ((9, 64, 1, 0, 4), 3), ((3, 62, 1, 0, 4), 3),
                           ((3, 28, 1, 0, 4), 3), ((3, 68, 1, 0, 4), 3), ((0, 64, 1, 0, 4), 4), ((3, 0, 1, 0, 4), 4),
                           ((3, 60, 0, 0, 4), 4), ((3, 60, 1, 1, 4), 4), ((3, 60, 1, 0, 17), 4), ((3, 60, 1, 4097, 4), 4)):
        with pytest.raises(gq.GqsaError) as e:
            gq.gqsa_set_partition_rows(h, *args)
        assert e.value.status == status, args
    # tiles of 6 and 8 blocks: 4-bit codes only
    for u in (6, 8):
        if bits == 4:
            gq.gqsa_set_partition_rows(h, u, 48, 1, 0, 8)
            assert gq.gqsa_partition(h)[2:] == (1, u, 48, 1) and gq.gqsa_info(h)["needs_fixup"] == 0
            assert_same_blob(h, c)
        else:
            with pytest.raises(gq.GqsaError) as e:
                gq.gqsa_set_partition_rows(h, u, 48, 1, 0, 8)
            assert e.value.status == 3
    # other group sizes have their own shape only
    h64 = gq.gqsa_pack(W, 64, 4, 0.5)
    with pytest.raises(gq.GqsaError) as e:
        gq.gqsa_set_partition_rows(h64, 3, 60, 1, 0, 4)
    assert e.value.status == 3
    gq.gqsa_set_partition_rows(h64, 2, 64, 1, 0, 4)
    assert_same_blob(h64, oracle.pack(W, 64, 4, sparsity=0.5))


def test_default_keeps_uniform_rows_inside_workers_tiles():
    """Read back from the image: at S = 30 % (179 groups per row) every worker's tile of 3 x 60
    positions holds one row -- its head in lane 0 of block 0, one null group at the end."""
    N, K = 500, 4096
    W = gi.dense_weight(N, K, seed=79)
    h = gq.gqsa_pack(W, 16, 4, 0.3)
    assert gq.gqsa_partition(h) == (128, 4, 1, 3, 60, 1)       # 500 workers -> 125 workgroups -> a multiple of 4
    info = gq.gqsa_info(h)
    assert info["n_blocks"] == 3 * 512 and info["device_bytes"] >= 3 * 512 * 60 * 14
    blob = np.frombuffer(gq.gqsa_export_device_blob(h), dtype=np.uint8)
    blk = blob[:info["n_blocks"] * 840].reshape(-1, 3, 840)     # [tile][block][60 x (8 + 4 + 2) bytes]
    ix = blk[:, :, 720:].copy().view("<u2")                      # [tile][block][lane]
    sz = blk[:, :, 480:720].copy().view("<u4")
    heads = (ix & 1).transpose(0, 2, 1).reshape(-1, 180)         # stream order inside a tile: position = 3 * lane + block
    scale = (sz & 0xFFFF).transpose(0, 2, 1).reshape(-1, 180)
    assert np.all(heads[:N, 0] == 1) and heads[:N, 1:].sum() == 0
    assert np.all(scale[:N, :179] != 0) and np.all(scale[:N, 179] == 0)
    assert not blk[N:].any()                                     # the workers beyond the rows hold null tiles
    cols = (ix >> 4).transpose(0, 2, 1).reshape(-1, 180)[:N, :179]
    assert np.array_equal(cols.reshape(-1), oracle.pack(W, 16, 4, sparsity=0.3).groups)


@pytest.mark.parametrize("bits,G", [(4, 16), (8, 16), (4, 32), (4, 64), (4, 128), (8, 32), (8, 64)])
@pytest.mark.parametrize("shape", [(301, 2048), (16, 512), (33, 128), (1, 4096), (100, 1152)])
def test_panel_image(bits, G, shape):
    """The second image (groups of 16 rows ordered by group-column) against its written layout."""
    N, K = shape
    W = gi.dense_weight(N, K, seed=80 + N)
    keep = gi.imbalanced_keep_counts(N, K // G, seed=80 + N)
    if N > 8:
        keep[[0, 5, N - 1]] = 0
        keep[3] = K // G
    h = gq.gqsa_pack_rows(W, keep, G, bits)
    c = oracle.pack(W, G, bits, keep_per_row=keep)
    assert gq.gqsa_info(h)["panel_bytes"] == 0
    with pytest.raises(gq.GqsaError) as e:
        gq.gqsa_export_panel_blob(h)
    assert e.value.status == 3
    gq.gqsa_build_panels(h)
    ref = oracle.panel_blob(c)
    assert gq.gqsa_info(h)["panel_bytes"] == len(ref)
    assert gq.gqsa_export_panel_blob(h) == ref
    assert_same_blob(h, c)                                  # the first image is untouched
    # every stored group appears exactly once: the blocks' counts add up
    P, S = -(-N // 16), -(-(K // G) // 32)
    hdr = np.frombuffer(ref, dtype="<u4", count=P * S * 36).reshape(P * S, 36)
    assert int(hdr[:, 33].sum()) == c.nnzg
    last = hdr[:, 31].astype(np.int64)
    assert np.array_equal((last >> 16) + np.array([bin(v & 0xFFFF).count("1") for v in last]), hdr[:, 33])


def test_panel_image_notes_whether_zeros_are_small_integers():
    """gqsa_info tells which form of Eq. 3 the matrix-core kernel will take: zero off the codes
    (exact in fp16 only for integer zeros up to 1024 in magnitude) or off the product's sum."""
    N, K = 40, 512
    c = oracle.pack(gi.dense_weight(N, K, seed=7), 16, 4, sparsity=0.5)

    def flag(zeros_f16):
        h = gq.gqsa_import(c.rowIndex, c.groups, c.values, c.scales, zeros_f16.view(np.uint16), N, K, 16, 4)
        assert gq.gqsa_info(h)["panel_integer_zeros"] == 0          # no second image yet
        gq.gqsa_build_panels(h)
        return gq.gqsa_info(h)["panel_integer_zeros"]

    z = c.zeros.view(np.float16).copy()
    assert flag(z) == 1                                             # what Eq. 1 gives
    for bad in (0.5, 1025.0, -1026.0, np.inf, np.nan, 6e-8):
        zz = z.copy()
        zz[c.nnzg // 2] = bad
        assert flag(zz) == 0, bad
    zz = z.copy()
    zz[0], zz[1], zz[2] = 1024.0, -1024.0, -0.0
    assert flag(zz) == 1


def test_panel_image_is_refused_for_groups_of_eight():
    W = gi.dense_weight(8, 256, seed=3)
    h = gq.gqsa_pack(W, 8, 4, 0.5)
    with pytest.raises(gq.GqsaError) as e:
        gq.gqsa_build_panels(h)
    assert e.value.status == 3


@pytest.mark.parametrize("bits", [4, 8])
def test_outliers_and_imbalanced_rows(bits):
    N, K = 333, 1024
    W = gi.dense_weight(N, K, seed=77)
    keep = gi.imbalanced_keep_counts(N, K // 16, seed=77)
    h = gq.gqsa_pack_rows(W, keep, 16, bits)
    c = oracle.pack(W, 16, bits, keep_per_row=keep)
    assert_same_canonical(h, c)
    for part in (None, (1, 1), (2, 1), (3, 1), (5, 3), (1, 16), (17, 2), (4, 16), (63, 16), (256, 16)):
        if part is not None:
            gq.gqsa_set_partition(h, *part)
            info = gq.gqsa_info(h)
            assert (info["n_workgroups"], info["waves_per_workgroup"]) == part
        assert_same_blob(h, c)


@pytest.mark.parametrize("bits,G", [(4, 8), (8, 8), (4, 32), (4, 64), (4, 128), (8, 32), (8, 64)])
def test_other_group_sizes(bits, G):
    """Group sizes 32, 64, 128: canonical arrays and the device image (code planes, smaller
    tiles, index word = first 16-element slot) against the oracle, several partitions."""
    N, K = 150, 2048
    W = gi.dense_weight(N, K, seed=91)
    keep = gi.imbalanced_keep_counts(N, K // G, seed=91)
    h = gq.gqsa_pack_rows(W, keep, G, bits)
    c = oracle.pack(W, G, bits, keep_per_row=keep)
    assert_same_canonical(h, c)
    info = gq.gqsa_info(h)
    assert info["algorithmic_bytes"] == oracle.algorithmic_bytes(N, K, G, bits, c.nnzg, 1)
    assert gq.gqsa_partition(h) == gq.gqsa_default_partition(c.rowIndex, K, G, bits)
    for part in (None, (1, 1), (3, 1), (5, 3), (1, 16), (17, 2), (40, 16)):
        if part is not None:
            gq.gqsa_set_partition(h, *part)
        assert_same_blob(h, c)
    hb = gq.gqsa_pack(W, G, bits, 0.5)
    cb = oracle.pack(W, G, bits, sparsity=0.5)
    assert_same_canonical(hb, cb)
    assert_same_blob(hb, cb)


@pytest.mark.parametrize("G,bits", [(16, 4), (64, 4), (32, 8)])
def test_pack_hessian_matches_the_oracle(G, bits):
    """Pruning by the Hessian metric of Eq. 4 with a positive diagonal spread over decades."""
    N, K = 200, 2048
    W = gi.dense_weight(N, K, seed=55)
    d = np.exp(np.random.default_rng(56).standard_normal(K) * 1.5).astype(np.float32)
    for sparsity in (0.3, 0.5):
        h = gq.gqsa_pack_hessian(W, d, G, bits, sparsity)
        c = oracle.pack(W, G, bits, sparsity=sparsity, hinv_diag=d)
        assert_same_canonical(h, c)
        assert_same_blob(h, c)
    # and it is not the magnitude selection
    assert not np.array_equal(gq.gqsa_export(h)["groups"], gq.gqsa_export(gq.gqsa_pack(W, G, bits, 0.5))["groups"])
    # d = 1 is gqsa_pack
    h1 = gq.gqsa_pack_hessian(W, np.ones(K, dtype=np.float32), G, bits, 0.5)
    assert gq.gqsa_export_device_blob(h1) == gq.gqsa_export_device_blob(gq.gqsa_pack(W, G, bits, 0.5))


def test_unsupported_group_sizes_are_refused():
    W = np.zeros((4, 256), dtype=np.float32)
    for G, bits in ((4, 4), (48, 4), (256, 4), (128, 8)):
        with pytest.raises(gq.GqsaError) as e:
            gq.gqsa_pack(W, G, bits, 0.5)
        assert e.value.status == 3


def test_planted_ties_and_constant_groups():
    rng = np.random.default_rng(8)
    W = rng.standard_normal((20, 160)).astype(np.float32)
    W[:, 16:32] = W[:, 0:16]            # duplicate groups: equal saliency
    W[:, 48:64] = 0.0                   # all-zero groups
    W[3] = 0.25                         # a constant row: every group degenerate, all tie
    W[4] = 0.0
    for s in (0.3, 0.5, 0.8):
        h = gq.gqsa_pack(W, 16, 4, s)
        c = oracle.pack(W, 16, 4, sparsity=s)
        assert_same_canonical(h, c)
        assert_same_blob(h, c)


def test_full_size_7b_shape_bit_exact():
    """One full decode shape (4096x4096, W4S50) of the LLaMA-7B layer set, default partition."""
    W = gi.dense_weight(4096, 4096, seed=gi.config_seed(2, 0))
    h = gq.gqsa_pack(W, 16, 4, 0.5)
    c = oracle.pack(W, 16, 4, sparsity=0.5)
    assert_same_canonical(h, c)
    assert_same_blob(h, c)
    info = gq.gqsa_info(h)
    assert info["nnz_groups"] == 524288 and info["n_workgroups"] == 512 and info["waves_per_workgroup"] == 4
    assert info["algorithmic_bytes"] == 7372804
    assert info["needs_fixup"] == 0      # 128 groups per row: every worker's run (a tile of 256 groups) ends on a row end


def test_full_size_down_proj_shape_needs_fixup():
    W = gi.dense_weight(1024, 11008, seed=gi.config_seed(2, 6))   # a 1024-row slice of down_proj
    h = gq.gqsa_pack(W, 16, 4, 0.5)
    c = oracle.pack(W, 16, 4, sparsity=0.5)
    assert_same_canonical(h, c)
    assert_same_blob(h, c)
    assert gq.gqsa_info(h)["needs_fixup"] == 1   # 344 groups per row do not align with 256-group tiles


def test_import_round_trip_and_free_parameters():
    W = gi.dense_weight(50, 256, seed=3)
    keep = gi.imbalanced_keep_counts(50, 16, seed=3)
    c = oracle.pack(W, 16, 4, keep_per_row=keep)
    # Sec. 3.4 fine-tunes s and z freely: perturb them to non-integer zeros and other scales
    rng = np.random.default_rng(1)
    c.scales = (c.scales.view(np.float16) * np.float16(1.37)).view(np.uint16)
    c.zeros = (c.zeros.view(np.float16) + rng.standard_normal(c.nnzg).astype(np.float16)).view(np.uint16)
    h = gq.gqsa_import(c.rowIndex, c.groups, c.values, c.scales, c.zeros, 50, 256, 16, 4)
    assert_same_canonical(h, c)
    assert_same_blob(h, c)


def test_group_range_beyond_an_fp16_scale_is_refused():
    """Eq. 1's scale is stored in fp16: a kept group whose range over 2^n - 1 rounds to infinity
    cannot be dequantised by Eq. 3; the library and the oracle both refuse the matrix, and accept
    the largest range that still fits."""
    W = gi.dense_weight(8, 64, seed=3)
    ok = W.copy()
    ok[2, 16] = 0.0
    ok[2, 17] = 15.0 * 65504.0                  # scale = 65504 exactly, the largest fp16 number
    ok[2, 18:32] = 1000.0
    h = gq.gqsa_pack(ok, 16, 4, 0.0)
    c = oracle.pack(ok, 16, 4, sparsity=0.0)
    assert_same_canonical(h, c)
    assert int(gq.gqsa_export(h)["scales"][2 * 4 + 1]) == 0x7BFF
    bad = ok.copy()
    bad[2, 17] = 15.0 * 65536.0                 # rounds to infinity in fp16
    with pytest.raises(gq.GqsaError) as e:
        gq.gqsa_pack(bad, 16, 4, 0.0)
    assert e.value.status == 4
    with pytest.raises(ValueError):
        oracle.pack(bad, 16, 4, sparsity=0.0)
    # pruned away, the group is no obstacle
    keep = np.full(8, 4, dtype=np.int32)
    small = bad.copy()
    small[2, 16:32] = 0.0
    small[2, 17] = 0.0
    assert_same_canonical(gq.gqsa_pack_rows(small, keep, 16, 4), oracle.pack(small, 16, 4, keep_per_row=keep))
