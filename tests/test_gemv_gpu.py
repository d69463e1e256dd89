"""Parity of the HIP GEMV (through the C ABI) against the float64 oracle on MI355X.

Tolerance (stated by the benchmark spec): max relative error <= 2e-3 with fp32 accumulation and
fp16 output, the denominator floored at 1% of the rms of the reference vector.
Packed buffers are compared bit for bit in tests/test_pack_bitexact.py (no GPU needed).
"""
from __future__ import annotations

import numpy as np
import pytest

import gqsa_inputs as gi
import oracle
import paper_2412_17560_amd as gq

pytestmark = pytest.mark.gpu

TOL = 2e-3


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a HIP device")
    return torch


def run_gemv(torch, h, x_np, panels=False):
    x = torch.from_numpy(np.ascontiguousarray(x_np)).cuda()
    n = gq.gqsa_info(h)["N"]
    y = torch.full((x.shape[0], n), float("nan"), dtype=torch.float16, device="cuda")
    gq.gqsa_gemv(h, x, y, panels=panels)
    torch.cuda.synchronize()
    return y.cpu().numpy()


def check(torch, h, c, x_np, tol=TOL, panels=False):
    y = run_gemv(torch, h, x_np, panels)
    ref = oracle.gemv(c, x_np, threads=8)
    assert np.isfinite(y).all()
    for b in range(x_np.shape[0]):
        err = oracle.rel_error(y[b], ref[b])
        assert err <= tol, f"batch row {b}: rel err {err:.3e}"
    # rows without stored groups are exactly +0
    empty = np.diff(c.rowIndex) == 0
    if empty.any():
        assert (y.view(np.uint16)[:, empty] == 0).all()
    return y, ref


def test_tiny_config(torch_cuda):
    W, x = gi.tiny_config()
    h = gq.gqsa_pack(W, 16, 4, 0.5)
    c = oracle.pack(W, 16, 4, sparsity=0.5)
    check(torch_cuda, h, c, x)


@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("sparsity", [0.0, 0.3, 0.5, 0.7, 1.0])
def test_balanced_ragged_shapes(torch_cuda, bits, sparsity):
    # 301 rows x 61 group-columns: nothing aligns with 64-group blocks or 256-group tiles
    N, K = 301, 976
    W = gi.dense_weight(N, K, seed=100 + bits)
    h = gq.gqsa_pack(W, 16, bits, sparsity)
    c = oracle.pack(W, 16, bits, sparsity=sparsity)
    check(torch_cuda, h, c, gi.activations(1, K, seed=5))


@pytest.mark.parametrize("part", [(1, 1), (2, 1), (3, 1), (7, 1), (1, 16), (2, 16), (3, 5), (33, 2),
                                  (13, 16), (200, 1), (256, 16)])
def test_partition_sweep_imbalanced(torch_cuda, part):
    """Rows shared by 2 and by many wavefronts, inside one workgroup and across workgroups,
    empty rows, dense rows: the carry fix-up through LDS and through device memory."""
    N, K = 257, 2048
    W = gi.dense_weight(N, K, seed=31)
    keep = gi.imbalanced_keep_counts(N, K // 16, seed=31)
    c = oracle.pack(W, 16, 4, keep_per_row=keep)
    h = gq.gqsa_pack_rows(W, keep, 16, 4)
    gq.gqsa_set_partition(h, *part)
    check(torch_cuda, h, c, gi.activations(1, K, seed=6))


@pytest.mark.parametrize("part", [(8, 4), (5, 7), (16, 2), (3, 16)])
@pytest.mark.parametrize("batch", [1, 2])
def test_rows_spanning_two_and_more_workgroups(torch_cuda, part, batch):
    """Long rows over few blocks per wavefront: a row's workers sit in one, two or three
    workgroups, several of them on either side of a workgroup boundary (partial sums through LDS
    on each side, then one meeting point; three or more workgroups through the arrival counter)."""
    N, K = 9, 5120                       # 320 group-columns per row
    W = gi.dense_weight(N, K, seed=77)
    keep = np.array([320, 200, 0, 320, 37, 320, 1, 320, 255], dtype=np.int32)
    c = oracle.pack(W, 16, 4, keep_per_row=keep)
    h = gq.gqsa_pack_rows(W, keep, 16, 4)
    gq.gqsa_set_partition(h, *part)
    check(torch_cuda, h, c, gi.activations(batch, K, seed=8))


@pytest.mark.parametrize("part", [(1, 0, 1), (1, 0, 4), (2, 0, 3), (4, 0, 4), (3, 0, 16), (16, 0, 8), (4, 64, 4),
                                  (1000, 3, 16)])
@pytest.mark.parametrize("batch", [1, 3])
def test_rows_kept_inside_workgroup_spans(torch_cuda, part, batch):
    """The aligned form of the stream: null groups before the span boundaries, workers whose whole
    run is null, rows longer than a span (shared by workgroups as in the plain form), empty rows."""
    N, K = 301, 2048
    W = gi.dense_weight(N, K, seed=78)
    keep = gi.imbalanced_keep_counts(N, K // 16, seed=78)
    keep[[0, 5, 6, 7, 300]] = 0
    keep[100] = K // 16
    c = oracle.pack(W, 16, 4, keep_per_row=keep)
    h = gq.gqsa_pack_rows(W, keep, 16, 4)
    gq.gqsa_set_partition_aligned(h, *part)
    assert gq.gqsa_info(h)["span_tiles"] == part[0]
    check(torch_cuda, h, c, gi.activations(batch, K, seed=9))


@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("shape", [(3, 60, 0, 4), (3, 44, 0, 1), (4, 32, 0, 4), (4, 64, 0, 16), (5, 36, 0, 3), (5, 64, 40, 8), (3, 32, 0, 4),
                                   (6, 60, 0, 8), (8, 44, 0, 4), (8, 64, 0, 16)])
def test_rows_kept_inside_workers_tiles(torch_cuda, shape, bits):
    """Tiles of a chosen shape (3, 4, 5, 6, 8 blocks; 32..64 lanes in use), one per worker, whole rows in
    them -- and, with 3 x 32, rows longer than a tile, shared by workers as in the other forms;
    ragged rows, empty rows, workers whose tile is null; every kernel for 1, 2, 4, 8 activation
    rows (3 and 7 rows run in the kernels for 4 and 8)."""
    N, K = 301, 2048
    W = gi.dense_weight(N, K, seed=78)
    keep = gi.imbalanced_keep_counts(N, K // 16, seed=78)
    keep[[0, 5, 6, 7, 300]] = 0
    keep[100] = K // 16
    c = oracle.pack(W, 16, bits, keep_per_row=keep)
    h = gq.gqsa_pack_rows(W, keep, 16, bits)
    u, lanes, wgs, wpw = shape
    if u > 5 and bits == 8:
        pytest.skip("tiles of 6 and 8 blocks exist for 4-bit codes only")
    gq.gqsa_set_partition_rows(h, u, lanes, 1, wgs, wpw)
    assert gq.gqsa_info(h)["needs_fixup"] == (1 if u * lanes < 128 else 0)
    for batch in (1, 2, 3, 4, 7, 8, 16):
        check(torch_cuda, h, c, gi.activations(batch, K, seed=9 + batch))


def test_rows_of_a_batch_are_the_single_row_results_with_chosen_tile_shapes(torch_cuda):
    """Tiles of 3 x 60 (179 groups per row): every batch size gives, row for row, the bits of the
    one-row call; q/k/v-like matrices of that shape share a launch and give the bits of separate
    calls; a matrix of another tile shape in the same call goes out in a launch of its own."""
    torch = torch_cuda
    K = 4096
    hs, cs = [], []
    for i, (N, keep_n) in enumerate(((512, 179), (128, 179), (130, 179), (256, 77))):
        W = gi.dense_weight(N, K, seed=300 + i)
        keep = np.full(N, keep_n, dtype=np.int32)
        hs.append(gq.gqsa_pack_rows(W, keep, 16, 4))
        cs.append(oracle.pack(W, 16, 4, keep_per_row=keep))
    assert [gq.gqsa_partition(h)[3:5] for h in hs] == [(3, 60), (3, 60), (3, 60), (3, 52)]
    x16 = gi.activations(16, K, seed=31)
    y16 = run_gemv(torch, hs[0], x16)
    for batch in (1, 2, 3, 4, 5, 7, 8, 11):
        y = run_gemv(torch, hs[0], x16[:batch])
        assert np.array_equal(y.view(np.uint16), y16[:batch].view(np.uint16)), batch
    for batch in (1, 4):
        x = torch.from_numpy(x16[:batch]).cuda()
        for group in (hs[:3], hs):
            ys = gq.gqsa_gemv_multi(group, x)
            torch.cuda.synchronize()
            for h, c, y in zip(group, cs, ys):
                got = y.cpu().numpy()
                assert np.array_equal(got.view(np.uint16), run_gemv(torch, h, x16[:batch]).view(np.uint16))
                ref = oracle.gemv(c, x16[:batch])
                for b in range(batch):
                    assert oracle.rel_error(got[b], ref[b]) <= TOL


@pytest.mark.parametrize("keep_n,expect,aligned", [(179, (1024, 4, 1, 3, 60, 1), (820, 4, 4)), (77, (512, 4, 1, 3, 52, 1), (316, 4, 4)),
                                                   (100, (512, 4, 1, 4, 52, 1), (412, 4, 4)), (205, (1024, 4, 1, 4, 52, 1), (456, 4, 8))])
def test_default_keeps_rows_inside_workers_full_size(torch_cuda, keep_n, expect, aligned):
    """4096x4096 with rows that do not divide the tiles of 4 x 64 (S = 30 %, 70 %, 61 %, 20 %): the default
    takes a tile shape that whole rows fill and no worker shares a row; every output checked, also
    of the form that keeps the rows inside the workgroups' spans and of the plain form with as
    many workers (rows shared by wavefronts and by workgroups)."""
    N, K = 4096, 4096
    W = gi.dense_weight_chunked(N, K, seed=41)
    keep = np.full(N, keep_n, dtype=np.int32)
    c = oracle.pack(W, 16, 4, keep_per_row=keep)
    h = gq.gqsa_pack_rows(W, keep, 16, 4)
    assert gq.gqsa_partition(h) == expect
    info = gq.gqsa_info(h)
    assert info["needs_fixup"] == 0
    assert gq.gqsa_export_device_blob(h) == oracle.device_blob_for(c, info)
    x = gi.activations(1, K, seed=10)
    check(torch_cuda, h, c, x)
    gq.gqsa_free(h)
    h1 = gq.gqsa_pack_rows(W, keep, 16, 4)
    gq.gqsa_set_partition_aligned(h1, aligned[2], aligned[0], aligned[1])
    assert gq.gqsa_partition(h1) == aligned + (4, 64, 0) and gq.gqsa_info(h1)["needs_fixup"] == 1
    check(torch_cuda, h1, c, x)
    gq.gqsa_free(h1)
    h2 = gq.gqsa_pack_rows(W, keep, 16, 4)     # the plain form with the same workers: rows shared by workgroups
    gq.gqsa_set_partition(h2, aligned[0], 4)
    check(torch_cuda, h2, c, x)


def adversarial_keeps(N, kg):
    one_row = np.zeros(N, dtype=np.int32); one_row[N // 2] = kg
    alternating = np.where(np.arange(N) % 2 == 0, 0, kg).astype(np.int32)
    singles = np.ones(N, dtype=np.int32)                      # many rows inside one lane
    singles_gaps = np.where(np.arange(N) % 3 == 0, 0, 1).astype(np.int32)
    ends_empty = np.full(N, kg // 2, dtype=np.int32); ends_empty[:3] = 0; ends_empty[-3:] = 0
    ramp = (np.arange(N) % (kg + 1)).astype(np.int32)
    exact64 = np.full(N, 64, dtype=np.int32)                  # rows end exactly on block boundaries
    return {"one_row": one_row, "alternating": alternating, "singles": singles,
            "singles_gaps": singles_gaps, "ends_empty": ends_empty, "ramp": ramp, "exact64": exact64}


@pytest.mark.parametrize("name", ["one_row", "alternating", "singles", "singles_gaps", "ends_empty",
                                  "ramp", "exact64"])
@pytest.mark.parametrize("part", [None, (5, 1), (2, 3)])
def test_adversarial_row_structures(torch_cuda, name, part):
    N, K = 96, 2048
    keep = adversarial_keeps(N, K // 16)[name]
    W = gi.dense_weight(N, K, seed=41)
    c = oracle.pack(W, 16, 4, keep_per_row=keep)
    h = gq.gqsa_pack_rows(W, keep, 16, 4)
    if part:
        gq.gqsa_set_partition(h, *part)
    check(torch_cuda, h, c, gi.activations(2, K, seed=7))


def test_single_row_matrix(torch_cuda):
    W = gi.dense_weight(1, 4096, seed=43)
    for s in (0.0, 0.5):
        c = oracle.pack(W, 16, 4, sparsity=s)
        h = gq.gqsa_pack(W, 16, 4, s)
        check(torch_cuda, h, c, gi.activations(1, 4096, seed=8))


@pytest.mark.parametrize("bits", [4, 8])
def test_unit_vectors_are_bit_exact(torch_cuda, bits):
    """x = e_k: y is column k of W^ and (q - z) s is exact in fp32, so the fp16 output must
    equal the correctly rounded oracle value bit for bit (pins gather + dequantisation)."""
    N, K = 128, 512
    W = gi.dense_weight(N, K, seed=47)
    c = oracle.pack(W, 16, bits, sparsity=0.5)
    h = gq.gqsa_pack(W, 16, bits, 0.5)
    ks = [0, 1, 15, 16, 17, 255, 256, 300, 511]
    x = np.concatenate([gi.unit_vector(K, k) for k in ks])
    y = run_gemv(torch_cuda, h, x)
    ref = oracle.gemv(c, x).astype(np.float16)
    assert np.array_equal(y.view(np.uint16), ref.view(np.uint16))


def test_ones_vector_row_sums(torch_cuda):
    N, K = 128, 512
    W = gi.dense_weight(N, K, seed=53)
    c = oracle.pack(W, 16, 4, sparsity=0.3)
    h = gq.gqsa_pack(W, 16, 4, 0.3)
    check(torch_cuda, h, c, gi.ones_vector(K))


def test_free_scale_and_zero_parameters(torch_cuda):
    """Sec. 3.4 trains s and z after the codes are frozen: the kernel must take any fp16 s, z."""
    N, K = 64, 1024
    W = gi.dense_weight(N, K, seed=59)
    c = oracle.pack(W, 16, 4, sparsity=0.5)
    rng = np.random.default_rng(2)
    c.scales = (c.scales.view(np.float16) * np.float16(0.83)).view(np.uint16)
    c.zeros = (c.zeros.view(np.float16) + rng.standard_normal(c.nnzg).astype(np.float16) * np.float16(3)).view(np.uint16)
    h = gq.gqsa_import(c.rowIndex, c.groups, c.values, c.scales, c.zeros, N, K, 16, 4)
    check(torch_cuda, h, c, gi.activations(1, K, seed=9))


@pytest.mark.parametrize("bits", [4, 8])
def test_small_batches(torch_cuda, bits):
    N, K = 512, 2048
    W = gi.dense_weight(N, K, seed=61)
    c = oracle.pack(W, 16, bits, sparsity=0.5)
    h = gq.gqsa_pack(W, 16, bits, 0.5)
    x = gi.activations(16, K, seed=10)
    y16, _ = check(torch_cuda, h, c, x)
    for b in range(1, 16):
        yb, _ = check(torch_cuda, h, c, x[:b])
        assert np.array_equal(yb.view(np.uint16), y16[:b].view(np.uint16))


@pytest.mark.parametrize("part", [None, (37, 3)])
def test_three_and_seven_rows_in_the_kernels_for_four_and_eight(torch_cuda, part):
    """3 rows run in the kernel for 4 and 7 in the kernel for 8 (also as the tail of 11 and 15):
    the rows that are not there must neither be read past the end of x nor reach y.  y sits in
    the middle of a larger buffer of a marker value; rows shared by wavefronts and workgroups,
    rows without groups (their zero fill), several matrices per launch."""
    torch = torch_cuda
    N, K = 300, 2048
    W = gi.dense_weight(N, K, seed=62)
    keep = gi.imbalanced_keep_counts(N, K // 16, seed=62)
    keep[[0, 7, 299]] = 0
    c = oracle.pack(W, 16, 4, keep_per_row=keep)
    h = gq.gqsa_pack_rows(W, keep, 16, 4)
    h2 = gq.gqsa_pack_rows(W, keep, 16, 4)
    if part:
        gq.gqsa_set_partition(h, *part)
        gq.gqsa_set_partition(h2, *part)
    x16 = gi.activations(16, K, seed=11)
    y16 = run_gemv(torch, h, x16)
    marker = np.float16(-777.0)
    for b in (3, 7, 11, 15):
        xt = torch.from_numpy(x16[:b].copy()).cuda()              # exactly b rows: nothing behind them is ours
        big = torch.full((b + 4, N), float(marker), dtype=torch.float16, device="cuda")
        big2 = torch.full((b + 4, N), float(marker), dtype=torch.float16, device="cuda")
        gq.gqsa_gemv(h, xt, big[2:2 + b])
        torch.cuda.synchronize()
        out = big.cpu().numpy()
        assert np.array_equal(out[2:2 + b].view(np.uint16), y16[:b].view(np.uint16))
        assert (out[:2] == marker).all() and (out[2 + b:] == marker).all()
        big.fill_(float(marker))
        gq.gqsa_gemv_multi([h, h2], xt, [big[2:2 + b], big2[2:2 + b]])
        torch.cuda.synchronize()
        for o in (big.cpu().numpy(), big2.cpu().numpy()):
            assert np.array_equal(o[2:2 + b].view(np.uint16), y16[:b].view(np.uint16))
            assert (o[:2] == marker).all() and (o[2 + b:] == marker).all()
    err = max(oracle.rel_error(y16[i], oracle.gemv(c, x16, threads=8)[i]) for i in range(16))
    assert err <= TOL


@pytest.mark.parametrize("part", [None, (37, 3)])
def test_run_to_run_determinism(torch_cuda, part):
    """Same input -> same bits, also when calls with other inputs run in between (a stale
    carry record or counter from an earlier call would show up here)."""
    N, K = 1000, 11008
    W = gi.dense_weight(N, K, seed=67)
    h = gq.gqsa_pack(W, 16, 4, 0.5)
    if part:
        gq.gqsa_set_partition(h, *part)     # rows shared across workgroups
    assert gq.gqsa_info(h)["needs_fixup"] == 1
    c = oracle.pack(W, 16, 4, sparsity=0.5)
    xa = gi.activations(1, K, seed=11)
    xb = gi.activations(1, K, seed=12)
    ya, _ = check(torch_cuda, h, c, xa)
    yb, _ = check(torch_cuda, h, c, xb)
    for _ in range(10):
        assert np.array_equal(run_gemv(torch_cuda, h, xa).view(np.uint16), ya.view(np.uint16))
        assert np.array_equal(run_gemv(torch_cuda, h, xb).view(np.uint16), yb.view(np.uint16))


def test_y_is_fully_overwritten_and_nothing_else(torch_cuda):
    torch = torch_cuda
    N, K = 300, 1024
    W = gi.dense_weight(N, K, seed=71)
    h = gq.gqsa_pack(W, 16, 4, 0.5)
    x = torch.from_numpy(gi.activations(1, K, seed=12)).cuda()
    buf = torch.full((N + 64,), 7.0, dtype=torch.float16, device="cuda")
    y = buf[32:32 + N].view(1, N)
    gq.gqsa_gemv(h, x, y)
    torch.cuda.synchronize()
    out = buf.cpu().numpy()
    assert (out[:32] == 7.0).all() and (out[32 + N:] == 7.0).all()
    c = oracle.pack(W, 16, 4, sparsity=0.5)
    assert oracle.rel_error(out[32:32 + N], oracle.gemv(c, x.cpu().numpy())[0]) <= TOL


def test_gemv_error_paths_on_device(torch_cuda):
    torch = torch_cuda
    W = gi.dense_weight(16, 64, seed=1)
    h = gq.gqsa_pack(W, 16, 4, 0.5)
    x = torch.zeros((17, 64), dtype=torch.float16, device="cuda")
    with pytest.raises(gq.GqsaError) as e:
        gq.gqsa_gemv(h, x)
    assert e.value.status == 3
    xm = torch.zeros((1, 64 + 4), dtype=torch.float16, device="cuda")[:, 4:]
    with pytest.raises(gq.GqsaError) as e:
        gq.gqsa_gemv(h, xm)           # 8 bytes past a 16-byte boundary
    assert e.value.status == 8
    xt = torch.zeros((64, 2), dtype=torch.float16, device="cuda").t()
    with pytest.raises(ValueError):
        gq.gqsa_gemv(h, xt)           # not contiguous: refused by the binding
    gq.gqsa_upload(h)
    with pytest.raises(gq.GqsaError) as e:
        gq.gqsa_set_partition(h, 8, 16)   # not after upload
    assert e.value.status == 3
    assert gq.gqsa_info(h)["on_device"] == 1


# ----------------------------------------------------------------------------- several matrices, one launch

@pytest.mark.parametrize("part", [None, "mixed", (3, 4), (1, 16), (40, 2), (512, 4), (1024, 4)])
@pytest.mark.parametrize("batch", [1, 3, 8])
def test_gemv_multi_equals_separate_calls(torch_cuda, part, batch):
    """q/k/v-style: matrices of different N sharing x; the fused launch must give the bits of the
    separate calls (and both must match the oracle).  Partitions: the defaults (wavefronts per
    workgroup differ with the size: separate launches behind the call), different worker counts
    with the same workgroup size (one launch, each matrix its own share of the grid), equal ones;
    with (512, 4) and (1024, 4) the launches of several rows take the workers 8 and 16 to a workgroup."""
    torch = torch_cuda
    K = 2048
    shapes = [(300, 0.5, None), (64, 0.0, None), (257, None, "imbalanced"), (128, 1.0, None)]
    hs, cs = [], []
    for i, (N, sp, kind) in enumerate(shapes):
        W = gi.dense_weight(N, K, seed=200 + i)
        if kind:
            keep = gi.imbalanced_keep_counts(N, K // 16, seed=200 + i)
            h = gq.gqsa_pack_rows(W, keep, 16, 4)
            c = oracle.pack(W, 16, 4, keep_per_row=keep)
        else:
            h = gq.gqsa_pack(W, 16, 4, sp)
            c = oracle.pack(W, 16, 4, sparsity=sp)
        if part == "mixed":
            gq.gqsa_set_partition(h, (5, 1, 9, 2)[i], 4)
        elif part:
            gq.gqsa_set_partition(h, *part)
        hs.append(h)
        cs.append(c)
    x_np = gi.activations(batch, K, seed=77)
    x = torch.from_numpy(x_np).cuda()
    ys = [torch.full((batch, c.N), float("nan"), dtype=torch.float16, device="cuda") for c in cs]
    gq.gqsa_gemv_multi(hs, x, ys)
    torch.cuda.synchronize()
    for h, c, y in zip(hs, cs, ys):
        single = run_gemv(torch, h, x_np)
        got = y.cpu().numpy()
        assert np.array_equal(got.view(np.uint16), single.view(np.uint16))
        ref = oracle.gemv(c, x_np)
        for b in range(batch):
            assert oracle.rel_error(got[b], ref[b]) <= TOL
    # two matrices only, and the fused call again (workspaces are reusable)
    ys2 = gq.gqsa_gemv_multi(hs[:2], x)
    torch.cuda.synchronize()
    for y2, y in zip(ys2, ys[:2]):
        assert torch.equal(y2, y)


def test_gemv_multi_error_paths(torch_cuda):
    torch = torch_cuda
    W = gi.dense_weight(32, 256, seed=1)
    W2 = gi.dense_weight(32, 512, seed=2)
    h1, h1b, h2 = gq.gqsa_pack(W, 16, 4, 0.5), gq.gqsa_pack(W, 16, 8, 0.5), gq.gqsa_pack(W2, 16, 4, 0.5)
    x = torch.zeros((1, 256), dtype=torch.float16, device="cuda")
    y = [torch.zeros((1, 32), dtype=torch.float16, device="cuda") for _ in range(5)]
    for hs, status in (([h1, h1], 2), ([h1, h1b], 2), ([h1] * 5, 3)):
        with pytest.raises(gq.GqsaError) as e:
            gq.gqsa_gemv_multi(hs, x, y[:len(hs)])
        assert e.value.status == status
    with pytest.raises(ValueError):
        gq.gqsa_gemv_multi([h1, h2], x, y[:2])      # K differs: refused by the binding
    h3 = gq.gqsa_pack(gi.dense_weight(32, 256, seed=3), 16, 4, 0.5)
    gq.gqsa_set_partition(h3, 2, 8)
    gq.gqsa_gemv_multi([h1, h3], x, y[:2])          # partitions may differ
    torch.cuda.synchronize()


@pytest.mark.parametrize("bits", [4, 8])
def test_largest_and_smallest_reduction_lengths(torch_cuda, bits):
    """K = 32768 is the most gqsa_gemv takes (x, its halves and group sums fill 96 KB of LDS; a
    batch of 2 goes out as two launches), K = 16 with one row the least; one more group-column
    than the limit packs but is refused by gqsa_gemv."""
    torch = torch_cuda
    N, K = 48, 32768
    W = gi.dense_weight(N, K, seed=200 + bits)
    keep = gi.imbalanced_keep_counts(N, K // 16, seed=200 + bits)
    h = gq.gqsa_pack_rows(W, keep, 16, bits)
    c = oracle.pack(W, 16, bits, keep_per_row=keep)
    check(torch, h, c, gi.activations(2, K, seed=13))
    W1 = gi.dense_weight(1, 16, seed=300 + bits)
    h1 = gq.gqsa_pack(W1, 16, bits, 0.0)
    check(torch, h1, oracle.pack(W1, 16, bits, sparsity=0.0), gi.activations(3, 16, seed=14))
    Wb = np.zeros((2, 32768 + 16), dtype=np.float32)
    hb = gq.gqsa_pack(Wb, 16, bits, 0.5)
    x = torch.zeros((1, 32768 + 16), dtype=torch.float16, device="cuda")
    y = torch.zeros((1, 2), dtype=torch.float16, device="cuda")
    with pytest.raises(gq.GqsaError) as e:
        gq.gqsa_gemv(hb, x, y)
    assert e.value.status == 3


# ----------------------------------------------------------------------------- other group sizes

@pytest.mark.parametrize("bits,G", [(4, 8), (8, 8), (4, 32), (4, 64), (4, 128), (8, 32), (8, 64)])
@pytest.mark.parametrize("part", [None, (5, 3), (2, 16)])
def test_other_group_sizes(torch_cuda, bits, G, part):
    """G = 32, 64, 128: several 16-element chunks per stored group, code planes, smaller
    tiles; rows of very different lengths, shared rows, empty rows; batch 1 and 3."""
    N, K = 150, 2048
    W = gi.dense_weight(N, K, seed=91)
    keep = gi.imbalanced_keep_counts(N, K // G, seed=91)
    h = gq.gqsa_pack_rows(W, keep, G, bits)
    c = oracle.pack(W, G, bits, keep_per_row=keep)
    if part is not None:
        gq.gqsa_set_partition(h, *part)
    check(torch_cuda, h, c, gi.activations(1, K, seed=9))
    check(torch_cuda, h, c, gi.activations(3, K, seed=10))


@pytest.mark.parametrize("G", [8, 32, 64, 128])
def test_other_group_sizes_full_size_and_sparsities(torch_cuda, G):
    """4096x4096 W4 at G = 32, 64, 128, S = 0 and 50 %, default partition."""
    W = gi.dense_weight(4096, 4096, seed=gi.config_seed(3, 0))
    for sparsity in (0.0, 0.5):
        h = gq.gqsa_pack(W, G, 4, sparsity)
        c = oracle.pack(W, G, 4, sparsity=sparsity)
        info = gq.gqsa_info(h)
        assert gq.gqsa_export_device_blob(h) == oracle.device_blob_for(c, info)
        check(torch_cuda, h, c, gi.activations(1, 4096, seed=11))


def test_gemv_multi_with_larger_groups(torch_cuda):
    """Two G = 32 matrices of different N in one launch: the oracle's values and the bits of the
    separate calls."""
    torch = torch_cuda
    K = 1024
    x_np = gi.activations(1, K, seed=12)
    x = torch.from_numpy(x_np).cuda()
    hs, cs = [], []
    for i, N in enumerate((96, 200)):
        W = gi.dense_weight(N, K, seed=100 + i)
        hs.append(gq.gqsa_pack(W, 32, 4, 0.5))
        cs.append(oracle.pack(W, 32, 4, sparsity=0.5))
    for h in hs:
        gq.gqsa_set_partition(h, 3, 4)
    ys = gq.gqsa_gemv_multi(hs, x)
    torch.cuda.synchronize()
    for h, y, c in zip(hs, ys, cs):
        assert oracle.rel_error(y.cpu().numpy()[0], oracle.gemv(c, x_np, threads=4)[0]) <= TOL
        assert np.array_equal(y.cpu().numpy().view(np.uint16), run_gemv(torch, h, x_np).view(np.uint16))


def test_hessian_pruned_and_reloaded_matrices_multiply(torch_cuda, tmp_path):
    """A matrix pruned by the Hessian metric (Eq. 4) against the oracle, and the same matrix after
    a trip through a file: identical output bits."""
    N, K = 300, 4096
    W = gi.dense_weight(N, K, seed=61)
    d = np.exp(np.random.default_rng(62).standard_normal(K)).astype(np.float32)
    h = gq.gqsa_pack_hessian(W, d, 16, 4, 0.5)
    c = oracle.pack(W, 16, 4, sparsity=0.5, hinv_diag=d)
    x_np = gi.activations(2, K, seed=63)
    check(torch_cuda, h, c, x_np)
    path = str(tmp_path / "layer.gqsa")
    gq.gqsa_save(h, path)
    h2 = gq.gqsa_load(path)
    y1, y2 = run_gemv(torch_cuda, h, x_np), run_gemv(torch_cuda, h2, x_np)
    assert np.array_equal(y1.view(np.uint16), y2.view(np.uint16))


# ----------------------------------------------------------------------------- full sizes

@pytest.mark.parametrize("idx", [0, 4, 6])
def test_llama7b_layer_shapes_full_size(torch_cuda, idx):
    """q_proj 4096x4096, gate_proj 11008x4096, down_proj 4096x11008 at W4S50 G=16, batch 1,
    default partition (the launch configuration the benchmark times); every output checked."""
    name, N, K = gi.LLAMA7B_LAYER[idx]
    W = gi.dense_weight(N, K, seed=gi.config_seed(2, idx))
    h = gq.gqsa_pack(W, 16, 4, 0.5)
    c = oracle.pack(W, 16, 4, sparsity=0.5)
    info = gq.gqsa_info(h)
    assert gq.gqsa_export_device_blob(h) == oracle.device_blob_for(c, info)
    check(torch_cuda, h, c, gi.activations(1, K, seed=gi.config_seed(2, idx)))


@pytest.mark.parametrize("sparsity", [0.0, 0.3, 0.5, 0.7])
@pytest.mark.parametrize("idx", [0, 1, 2, 3])
def test_llama3_8b_sparsity_sweep_full_size(torch_cuda, idx, sparsity):
    """Every shape of the LLaMA-3-8B-like set at every sparsity of the sweep, at full size, with the
    default partition (the launch configuration the benchmark times): the device image bit for
    bit and every output against the oracle."""
    name, N, K = gi.LLAMA3_8B_SHAPES[idx]
    W = gi.dense_weight(N, K, seed=gi.config_seed(3, idx))
    h = gq.gqsa_pack(W, 16, 4, sparsity)
    c = oracle.pack(W, 16, 4, sparsity=sparsity)
    info = gq.gqsa_info(h)
    assert gq.gqsa_partition(h) == gq.gqsa_default_partition(c.rowIndex, K)
    assert gq.gqsa_export_device_blob(h) == oracle.device_blob_for(c, info)
    check(torch_cuda, h, c, gi.activations(1, K, seed=gi.config_seed(3, idx)))
    gq.gqsa_free(h)


@pytest.mark.parametrize("idx", [0, 1])
def test_imbalanced_stress_full_size(torch_cuda, idx):
    name, N, K = gi.IMBALANCED_SHAPES[idx]
    seed = gi.config_seed(4, idx)
    W = gi.dense_weight(N, K, seed=seed)
    keep = gi.imbalanced_keep_counts(N, K // 16, seed=seed)
    h = gq.gqsa_pack_rows(W, keep, 16, 4)
    c = oracle.pack(W, 16, 4, keep_per_row=keep)
    assert gq.gqsa_info(h)["needs_fixup"] == 1
    check(torch_cuda, h, c, gi.activations(1, K, seed=seed))


def test_vocabulary_sized_matrix(torch_cuda):
    """128256x4096 (the output projection of a LLaMA-3-8B-like model), W4S50: 16.4 M stored groups,
    64 128 tiles, four (eight rows) per wavefront in 4008 workgroups -- the largest deal the default makes.
    Every output checked."""
    N, K = 128256, 4096
    W = gi.dense_weight_chunked(N, K, seed=51)
    h = gq.gqsa_pack(W, 16, 4, 0.5)
    c = oracle.pack(W, 16, 4, sparsity=0.5)
    del W
    info = gq.gqsa_info(h)
    assert info["nnz_groups"] == N * 128
    assert gq.gqsa_partition(h) == (4008, 4, 4, 4, 64, 1)
    check(torch_cuda, h, c, gi.activations(1, K, seed=52))
    gq.gqsa_free(h)


@pytest.mark.parametrize("bits,G", [(4, 16), (8, 16), (4, 32), (4, 64), (4, 128), (8, 32), (8, 64)])
@pytest.mark.parametrize("batch", [1, 2, 5, 8, 9, 13, 16])
def test_panel_kernel_ragged(torch_cuda, bits, G, batch):
    """1..16 activation rows on the matrix cores, from the panel image: 301 rows (the last panel
    has 13), 61 group-columns (the second slice has 29), imbalanced rows, empty rows."""
    N, K = 301, 61 * G
    W = gi.dense_weight(N, K, seed=90 + bits)
    keep = gi.imbalanced_keep_counts(N, K // G, seed=90 + bits)
    keep[[0, 5, 6, 300]] = 0
    keep[17] = K // G
    c = oracle.pack(W, G, bits, keep_per_row=keep)
    h = gq.gqsa_pack_rows(W, keep, G, bits)
    gq.gqsa_build_panels(h)
    check(torch_cuda, h, c, gi.activations(batch, K, seed=11 + batch), panels=True)


def test_panel_kernel_unit_vectors_are_bit_exact(torch_cuda):
    """x = e_k in 16 activation rows: y[b] is column k_b of W^, and (q - z) s is exact in fp32, so
    every output is fp16((q - z) s) to the bit -- operand layout of the products, decode, scale
    and zero with no tolerance."""
    N, K = 100, 1024
    W = gi.dense_weight(N, K, seed=95)
    c = oracle.pack(W, 16, 4, sparsity=0.5)
    h = gq.gqsa_pack(W, 16, 4, 0.5)
    gq.gqsa_build_panels(h)
    ks = [0, 1, 15, 16, 17, 255, 256, 511, 512, 513, 777, 1000, 1008, 1022, 1023, 300]
    x = np.zeros((16, K), dtype=np.float16)
    for b, k in enumerate(ks):
        x[b, k] = 1.0
    y = run_gemv(torch_cuda, h, x)        # 16 rows: gqsa_gemv itself takes the panel image
    Wd = oracle.densify(c)
    ref = Wd[:, ks].T.astype(np.float32).astype(np.float16)
    assert np.array_equal(y.view(np.uint16), ref.view(np.uint16))


def test_panel_kernel_only_from_five_rows(torch_cuda):
    """Below 5 activation rows a handle with a panel image runs the wavefront kernel in gqsa_gemv:
    same bits as a handle without one.  From 5 on it is gqsa_gemv_panels, whose results differ in
    rounding only."""
    N, K = 512, 2048
    W = gi.dense_weight(N, K, seed=96)
    c = oracle.pack(W, 16, 4, sparsity=0.3)
    h1 = gq.gqsa_pack(W, 16, 4, 0.3)
    h2 = gq.gqsa_pack(W, 16, 4, 0.3)
    gq.gqsa_build_panels(h2)
    assert gq.gqsa_info(h2)["panel_bytes"] > 0
    for batch in (1, 3, 4):
        x = gi.activations(batch, K, seed=12)
        assert np.array_equal(run_gemv(torch_cuda, h1, x).view(np.uint16), run_gemv(torch_cuda, h2, x).view(np.uint16))
    x = gi.activations(5, K, seed=13)
    y, _ = check(torch_cuda, h2, c, x)
    assert np.array_equal(y.view(np.uint16), run_gemv(torch_cuda, h2, x, panels=True).view(np.uint16))
    with pytest.raises(gq.GqsaError):
        gq.gqsa_build_panels(h1)         # not after the upload
    with pytest.raises(gq.GqsaError) as e:
        run_gemv(torch_cuda, h1, x, panels=True)     # no such image
    assert e.value.status == 3
    # K above 8192: from 3 rows on
    N, K = 48, 8208
    W = gi.dense_weight(N, K, seed=99)
    c = oracle.pack(W, 16, 4, sparsity=0.5)
    h1 = gq.gqsa_pack(W, 16, 4, 0.5)
    h2 = gq.gqsa_pack(W, 16, 4, 0.5)
    gq.gqsa_build_panels(h2)
    x = gi.activations(3, K, seed=18)
    assert np.array_equal(run_gemv(torch_cuda, h1, x[:2]).view(np.uint16), run_gemv(torch_cuda, h2, x[:2]).view(np.uint16))
    y, _ = check(torch_cuda, h2, c, x)
    assert np.array_equal(y.view(np.uint16), run_gemv(torch_cuda, h2, x, panels=True).view(np.uint16))


@pytest.mark.parametrize("bits,G", [(4, 16), (8, 16), (4, 32)])
def test_panel_kernel_several_matrices_share_a_launch(torch_cuda, bits, G):
    """q/k/v-like: three matrices of different N (4200 rows: 263 panels, more than one per
    workgroup; 130 and 70 rows: ragged last panels) and different sparsity on the same
    activations, 16 and 7 rows.  One launch gives the bits of three separate calls and stays
    within the bound against the oracle; a fourth matrix whose zeros are not integers (the other
    form of Eq. 3) makes the call fall back to one launch per matrix, same bits again."""
    torch = torch_cuda
    K = 24 * G
    shapes = [(4200, 0.5), (130, 0.3), (70, 0.0)]
    hs, cs = [], []
    for i, (N, sp) in enumerate(shapes):
        W = gi.dense_weight(N, K, seed=120 + i)
        cs.append(oracle.pack(W, G, bits, sparsity=sp))
        h = gq.gqsa_pack(W, G, bits, sp)
        gq.gqsa_build_panels(h)
        hs.append(h)
    c4 = oracle.pack(gi.dense_weight(50, K, seed=124), G, bits, sparsity=0.5)
    c4.zeros = (c4.zeros.view(np.float16) + np.float16(0.25)).view(np.uint16)
    h4 = gq.gqsa_import(c4.rowIndex, c4.groups, c4.values, c4.scales, c4.zeros, 50, K, G, bits)
    gq.gqsa_build_panels(h4)
    assert gq.gqsa_info(h4)["panel_integer_zeros"] == 0
    for batch in (16, 7):
        x = gi.activations(batch, K, seed=17 + batch)
        xt = torch.from_numpy(x).cuda()
        single = [check(torch, h, c, x, panels=True)[0] for h, c in zip(hs + [h4], cs + [c4])]
        for group in (hs, hs + [h4], [h4] + hs[:2]):
            ys = [torch.full((batch, gq.gqsa_info(h)["N"]), float("nan"), dtype=torch.float16, device="cuda") for h in group]
            gq.gqsa_gemv_multi(group, xt, ys)
            torch.cuda.synchronize()
            for h, yy in zip(group, ys):
                want = single[(hs + [h4]).index(h)]
                assert np.array_equal(yy.cpu().numpy().view(np.uint16), want.view(np.uint16))


@pytest.mark.parametrize("bits,G,sparsity", [(4, 16, 0.5), (8, 16, 0.3), (4, 64, 0.5), (4, 16, 0.0)])
def test_panel_kernel_more_workgroups_than_compute_units(torch_cuda, bits, G, sparsity):
    """More than 1024 panels (17 603 rows: 1101 panels, the last with 3 rows): 276 workgroups of
    8 wavefronts, two to a compute unit, each wavefront with several units of the panels."""
    N, K = 17603, 40 * G
    W = gi.dense_weight_chunked(N, K, seed=130)
    c = oracle.pack(W, G, bits, sparsity=sparsity)
    h = gq.gqsa_pack(W, G, bits, sparsity)
    gq.gqsa_build_panels(h)
    x = gi.activations(13, K, seed=19)
    y, _ = check(torch_cuda, h, c, x, panels=True)
    if (bits, G, sparsity) == (4, 16, 0.5):
        # two such matrices in one gqsa_gemv_multi call: too many panels for one launch, so one each
        torch = torch_cuda
        h2 = gq.gqsa_pack(W, G, bits, sparsity)
        gq.gqsa_build_panels(h2)
        ys = [torch.full((13, N), float("nan"), dtype=torch.float16, device="cuda") for _ in range(2)]
        gq.gqsa_gemv_multi([h, h2], torch.from_numpy(x).cuda(), ys)
        torch.cuda.synchronize()
        for yy in ys:
            assert np.array_equal(yy.cpu().numpy().view(np.uint16), y.view(np.uint16))


def test_panel_kernel_seeded_shapes(torch_cuda):
    """Forty seeded draws of (code width, group size, N, K, per-row keep counts, activation rows):
    row counts that leave the last panel ragged or give a workgroup one to four panels, K from one
    group-column to several slices with a short last one, rows from empty to full."""
    rng = np.random.default_rng(2024)
    formats = [(4, 16), (8, 16), (4, 32), (4, 64), (4, 128), (8, 32), (8, 64)]
    for case in range(40):
        bits, G = formats[case % len(formats)]
        N = int(rng.choice([1, 15, 16, 17, 100, 257, 1000, 4100, 4200, 8300]))
        cols = int(rng.choice([1, 2, 15, 16, 17, 31, 32, 33, 47, 64, 70]))
        if N > 1000:
            cols = min(cols, 33)
        K = cols * G
        batch = int(rng.integers(1, 17))
        style = case % 4
        if style == 0:
            keep = rng.integers(0, cols + 1, size=N)
        elif style == 1:
            keep = np.full(N, cols)
        elif style == 2:
            keep = np.where(rng.random(N) < 0.5, 0, rng.integers(0, cols + 1, size=N))
        else:
            keep = np.full(N, (cols + 1) // 2)
        keep = keep.astype(np.int32)
        W = gi.dense_weight(N, K, seed=500 + case)
        c = oracle.pack(W, G, bits, keep_per_row=keep)
        h = gq.gqsa_pack_rows(W, keep, G, bits)
        gq.gqsa_build_panels(h)
        try:
            check(torch_cuda, h, c, gi.activations(batch, K, seed=600 + case), panels=True)
        except AssertionError as e:
            raise AssertionError(f"case {case}: bits={bits} G={G} N={N} K={K} batch={batch} style={style}: {e}")
        gq.gqsa_free(h)


@pytest.mark.parametrize("bits,G,sparsity", [(4, 16, 0.0), (4, 16, 0.2), (8, 16, 0.0), (4, 64, 0.1), (8, 64, 0.0)])
def test_panel_kernel_dense_panels(torch_cuda, bits, G, sparsity):
    """Four panels per workgroup (769 panels on 256 workgroups) that are dense or nearly so: a
    wavefront's staging area in LDS then holds two panels' records at a time, not four (and the
    fullest records a unit can have, 16 rows x all its columns).  The last panel has 5 rows."""
    N, K = 16 * 768 + 5, 32 * G
    W = gi.dense_weight_chunked(N, K, seed=98)
    c = oracle.pack(W, G, bits, sparsity=sparsity)
    h = gq.gqsa_pack(W, G, bits, sparsity)
    gq.gqsa_build_panels(h)
    check(torch_cuda, h, c, gi.activations(16, K, seed=16), panels=True)


@pytest.mark.parametrize("bits,G", [(4, 16), (8, 16), (4, 64), (8, 32)])
@pytest.mark.parametrize("zeros", ["fractional", "large", "extreme_integers"])
def test_panel_kernel_any_zero(torch_cuda, bits, G, zeros):
    """The matrix-core kernel subtracts the zero from the codes only when every stored zero is an
    integer of at most 1024 in magnitude (then exactly); trained zeros (Sec. 3.4) may be any fp16
    number and take the other form of Eq. 3, s (sum q x - z sum x).  Fractional zeros, zeros
    beyond 1024, and integer zeros at +-1024 with the codes at both ends of their range."""
    N, K = 77, 40 * G
    W = gi.dense_weight(N, K, seed=97)
    c = oracle.pack(W, G, bits, sparsity=0.4)
    rng = np.random.default_rng(3)
    z = c.zeros.view(np.float16).astype(np.float32)
    if zeros == "fractional":
        z = z + rng.standard_normal(c.nnzg).astype(np.float32) * 3
    elif zeros == "large":
        z[::7] = 1025.0
        z[3::11] = -2048.0
    else:
        z[::2] = 1024.0
        z[1::2] = -1024.0
        c.values[: c.values.size // 2] = 0xFF
        c.values[c.values.size // 2:] = 0x00
    c.zeros = z.astype(np.float16).view(np.uint16)
    h = gq.gqsa_import(c.rowIndex, c.groups, c.values, c.scales, c.zeros, N, K, G, bits)
    gq.gqsa_build_panels(h)
    assert gq.gqsa_info(h)["panel_integer_zeros"] == (1 if zeros == "extreme_integers" else 0)
    check(torch_cuda, h, c, gi.activations(16, K, seed=15), panels=True)


@pytest.mark.parametrize("bits,shape_idx", [(4, 0), (8, 1)])
def test_panel_kernel_full_size(torch_cuda, bits, shape_idx):
    """4096x4096 (W4) and 14336x4096 (W8) at S = 50 %, 16 activation rows; every output checked.
    Also several matrices in one call."""
    name, N, K = gi.SMALL_BATCH_SHAPES[shape_idx]
    W = gi.dense_weight_chunked(N, K, seed=gi.config_seed(5, shape_idx))
    c = oracle.pack(W, 16, bits, sparsity=0.5)
    h = gq.gqsa_pack(W, 16, bits, 0.5)
    gq.gqsa_build_panels(h)
    x = gi.activations(16, K, seed=14)
    y, ref = check(torch_cuda, h, c, x)
    if shape_idx == 0:
        h2 = gq.gqsa_pack(W, 16, bits, 0.5)
        gq.gqsa_build_panels(h2)
        xt = torch_cuda.from_numpy(x).cuda()
        ys = [torch_cuda.full((16, N), float("nan"), dtype=torch_cuda.float16, device="cuda") for _ in range(2)]
        gq.gqsa_gemv_multi([h, h2], xt, ys)
        torch_cuda.cuda.synchronize()
        for yy in ys:
            assert np.array_equal(yy.cpu().numpy().view(np.uint16), y.view(np.uint16))


def test_graph_replays_match_eager(torch_cuda):
    """The calls captured in a HIP graph (as the benchmark and a decoder would issue them) and
    replayed several times, with eager work and synchronisation between the replays: every replay
    gives the bits of the eager calls.  Rows shared by wavefronts and by workgroups (the fix-up
    leaves its counters and meeting points ready for the next launch by itself), several
    matrices per launch, tiles of a chosen shape, and the matrix-core kernel."""
    torch = torch_cuda
    N, K = 257, 2048
    W = gi.dense_weight(N, K, seed=61)
    keep = gi.imbalanced_keep_counts(N, K // 16, seed=61)
    ha = gq.gqsa_pack_rows(W, keep, 16, 4)
    gq.gqsa_set_partition(ha, 37, 3)                         # chains across workgroups
    hb = gq.gqsa_pack_rows(W, keep, 16, 4)
    gq.gqsa_set_partition_aligned(hb, 4, 0, 4)               # rows kept inside the workgroups' spans
    hf = gq.gqsa_pack_rows(W, keep, 16, 4)
    gq.gqsa_set_partition_rows(hf, 5, 60, 1, 0, 4)            # tiles of a chosen shape, whole rows per worker
    hc = gq.gqsa_pack_rows(W, keep, 16, 4)
    gq.gqsa_set_partition(hc, 5, 4)
    hp = gq.gqsa_pack_rows(W, keep, 16, 8)
    gq.gqsa_build_panels(hp)
    hq = [gq.gqsa_pack_rows(W, keep, 16, 4) for _ in range(3)]   # three matrices in one launch of the matrix-core kernel
    for h in hq:
        gq.gqsa_build_panels(h)
    x7 = torch.from_numpy(gi.activations(7, K, seed=65)).cuda()
    x1 = torch.from_numpy(gi.activations(1, K, seed=62)).cuda()
    x3 = torch.from_numpy(gi.activations(3, K, seed=63)).cuda()
    x16 = torch.from_numpy(gi.activations(16, K, seed=64)).cuda()

    def outputs():
        return [torch.full((1, N), float("nan"), dtype=torch.float16, device="cuda"),
                torch.full((3, N), float("nan"), dtype=torch.float16, device="cuda"),
                torch.full((1, N), float("nan"), dtype=torch.float16, device="cuda"),
                torch.full((1, N), float("nan"), dtype=torch.float16, device="cuda"),
                torch.full((16, N), float("nan"), dtype=torch.float16, device="cuda"),
                torch.full((7, N), float("nan"), dtype=torch.float16, device="cuda"),
                torch.full((7, N), float("nan"), dtype=torch.float16, device="cuda"),
                torch.full((7, N), float("nan"), dtype=torch.float16, device="cuda"),
                torch.full((7, N), float("nan"), dtype=torch.float16, device="cuda"),
                torch.full((1, N), float("nan"), dtype=torch.float16, device="cuda"),
                torch.full((3, N), float("nan"), dtype=torch.float16, device="cuda")]

    def issue(ys):
        gq.gqsa_gemv(ha, x1, ys[0])
        gq.gqsa_gemv(ha, x3, ys[1])
        gq.gqsa_gemv_multi([hb, hc], x1, [ys[2], ys[3]])
        gq.gqsa_gemv(hp, x16, ys[4])
        gq.gqsa_gemv_multi(hq, x7, ys[5:8])
        gq.gqsa_gemv(hb, x7, ys[8])                         # 7 rows in the kernel for 8
        gq.gqsa_gemv(hf, x1, ys[9])
        gq.gqsa_gemv(hf, x3, ys[10])

    eager = outputs()
    issue(eager)
    torch.cuda.synchronize()
    want = [y.cpu().numpy().view(np.uint16).copy() for y in eager]
    assert all(np.isfinite(y.cpu().numpy()).all() for y in eager)

    ys = outputs()
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        issue(ys)                                           # (uploads and first-use set-up happen outside the capture)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=stream):
        issue(ys)
    torch.cuda.synchronize()
    for replay in range(4):
        for y in ys:
            y.fill_(float("nan"))                          # eager work between the replays
        issue(outputs())                                    # and the same kernels, eagerly, on the handles' workspaces
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for y, w in zip(ys, want):
            assert np.array_equal(y.cpu().numpy().view(np.uint16), w), f"replay {replay}"


def test_llama7b_qkv_and_gate_up_fused_full_size(torch_cuda):
    """The fused launches the benchmark times: q/k/v (3 x 4096x4096) and gate/up (2 x 11008x4096)."""
    torch = torch_cuda
    x_np = gi.activations(1, 4096, seed=gi.config_seed(2, 0))
    x = torch.from_numpy(x_np).cuda()
    for idxs in ((0, 1, 2), (4, 5)):
        hs, cs = [], []
        for idx in idxs:
            name, N, K = gi.LLAMA7B_LAYER[idx]
            W = gi.dense_weight(N, K, seed=gi.config_seed(2, idx))
            hs.append(gq.gqsa_pack(W, 16, 4, 0.5))
            cs.append(oracle.pack(W, 16, 4, sparsity=0.5))
        ys = gq.gqsa_gemv_multi(hs, x)
        torch.cuda.synchronize()
        for y, c in zip(ys, cs):
            assert oracle.rel_error(y.cpu().numpy()[0], oracle.gemv(c, x_np, threads=8)[0]) <= TOL


def test_w8_full_size(torch_cuda):
    W = gi.dense_weight(4096, 4096, seed=gi.config_seed(5, 0))
    h = gq.gqsa_pack(W, 16, 8, 0.5)
    c = oracle.pack(W, 16, 8, sparsity=0.5)
    check(torch_cuda, h, c, gi.activations(2, 4096, seed=gi.config_seed(5, 0)))


@pytest.mark.parametrize("bits", [4, 8])
def test_small_batch_4096x4096_wavefront_kernel_full_size(torch_cuda, bits):
    """4096x4096 S50 with 1, 2, 4, 8 and 16 activation rows on the wavefront kernel (a handle
    without the second image), default partition: every output of every row against the oracle,
    every row identical whatever the batch size it was part of."""
    torch = torch_cuda
    N, K = 4096, 4096
    seed = gi.config_seed(5, 0)
    W = gi.dense_weight(N, K, seed=seed)
    h = gq.gqsa_pack(W, 16, bits, 0.5)
    c = oracle.pack(W, 16, bits, sparsity=0.5)
    assert gq.gqsa_info(h)["panel_bytes"] == 0
    x_np = gi.activations(16, K, seed=seed)
    ref = oracle.gemv(c, x_np, threads=8)
    y16 = run_gemv(torch, h, x_np)
    for batch in (1, 2, 3, 4, 8, 16):
        y = run_gemv(torch, h, x_np[:batch])
        for b in range(batch):
            assert oracle.rel_error(y[b], ref[b]) <= TOL, (batch, b)
        assert np.array_equal(y.view(np.uint16), y16[:batch].view(np.uint16)), batch


@pytest.mark.parametrize("bits", [4, 8])
def test_small_batch_full_size(torch_cuda, bits):
    """14336x4096 S50 with 1, 2, 4, 8 and 16 activation rows (16 = two launches of 8): every
    output of every row against the oracle, and row 0 identical whatever the batch size."""
    torch = torch_cuda
    N, K = 14336, 4096
    seed = gi.config_seed(5, 1)
    W = gi.dense_weight(N, K, seed=seed)
    h = gq.gqsa_pack(W, 16, bits, 0.5)
    c = oracle.pack(W, 16, bits, sparsity=0.5)
    x_np = gi.activations(16, K, seed=seed)
    ref = oracle.gemv(c, x_np, threads=8)
    first = None
    for batch in (1, 2, 4, 8, 16):
        y = run_gemv(torch, h, x_np[:batch])
        for b in range(batch):
            assert oracle.rel_error(y[b], ref[b]) <= TOL, (batch, b)
        if first is None:
            first = y[0].copy()
        assert np.array_equal(y[0].view(np.uint16), first.view(np.uint16)), batch


# ----------------------------------------------------------------------------- side-by-side kernels

def test_dense_f16_gemv_baseline(torch_cuda):
    torch = torch_cuda
    N, K = 1000, 4096
    W = gi.dense_weight(N, K, seed=73).astype(np.float16)
    x = gi.activations(2, K, seed=13)
    y = gq.gqsa_dense_f16_gemv(torch.from_numpy(W).cuda(), torch.from_numpy(x).cuda())
    torch.cuda.synchronize()
    ref = x.astype(np.float64) @ W.astype(np.float64).T
    for b in range(2):
        assert oracle.rel_error(y[b].cpu().numpy(), ref[b]) <= TOL


def test_stream_read_kernel_runs(torch_cuda):
    torch = torch_cuda
    buf = torch.arange(1 << 20, dtype=torch.int32, device="cuda")
    sink = torch.zeros(gq.gqsa_stream_read_workgroups(), dtype=torch.int32, device="cuda")
    gq.gqsa_stream_read(buf, sink)
    torch.cuda.synchronize()
    x = 0
    for v in sink.cpu().numpy().view(np.uint32):
        x ^= int(v)
    ref = int(np.bitwise_xor.reduce(np.arange(1 << 20, dtype=np.uint32)))
    assert x == ref


def test_copy_kernel(torch_cuda):
    torch = torch_cuda
    src = torch.arange(1 << 18, dtype=torch.int32, device="cuda")
    dst = torch.zeros_like(src)
    gq.gqsa_copy(dst, src)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)
