"""Pins for the oracle's derivation of the device byte layout.

The layout is a permutation, so its pins are: hand-worked placements for small
block counts, and a decoder written here from the same specification (pure
Python loops) that must recover the canonical arrays from the blob.
"""
from __future__ import annotations

import numpy as np
import pytest

import gqsa_inputs as gi
import oracle
from oracle import layout


def test_row_positions():
    ri = np.array([0, 3, 3, 9, 10, 16, 17])         # rows of 3, 0, 6, 1, 6, 1 groups
    pos, L = oracle.row_positions(ri, 0)
    assert pos.tolist() == [0, 3, 3, 9, 10, 16] and L == 17
    pos, L = oracle.row_positions(ri, 8)             # 3 | skip to 8: 6, 1 | skip to 16: 6, 1
    assert pos.tolist() == [0, 3, 8, 14, 16, 22] and L == 23
    pos, L = oracle.row_positions(ri, 9)             # 3 + 6 fill the first span exactly
    assert pos.tolist() == [0, 3, 3, 9, 10, 16] and L == 17
    pos, L = oracle.row_positions(ri, 4)             # the rows of 6 are longer than a span: they start where the last one ended
    assert pos.tolist() == [0, 3, 3, 9, 10, 16] and L == 17
    pos, L = oracle.row_positions(np.array([0, 4, 8, 9]), 4)   # exact fits need nothing
    assert pos.tolist() == [0, 4, 8] and L == 9


def test_tile_deal_by_hand():
    # 23 tiles of 4 blocks over 12 workers: worker w starts at tile floor(23 w / 12) = 0 1 3 5 7 9 11 13 15 17 19 21
    assert list(layout.worker_block_counts(92, 12, 4)) == [4] + [8] * 11
    # 5 tiles of 2 blocks over 8 workers: starts 0 0 1 1 2 3 3 4 (5)
    assert list(layout.worker_block_counts(10, 8, 2)) == [0, 2, 0, 2, 2, 0, 2, 2]
    # LLaMA-7B down_proj at W4S50: 5504 tiles over 344 x 8 workers, two each
    c = layout.worker_block_counts(22016, 2752, 4)
    assert set(c) == {8} and c.sum() == 22016


def test_placement_single_worker_2_tiles_by_hand():
    block, lane, b_w, _ = layout.stream_placement(8, 1, 4)
    assert list(b_w) == [0]
    # tile of 4 blocks: position p -> block p mod 4, lane p div 4
    assert (block[0], lane[0]) == (0, 0)
    assert (block[1], lane[1]) == (1, 0)
    assert (block[5], lane[5]) == (1, 1)
    assert (block[255], lane[255]) == (3, 63)
    # second tile (blocks 4..7)
    assert (block[256], lane[256]) == (4, 0)
    assert (block[257], lane[257]) == (5, 0)
    assert (block[260], lane[260]) == (4, 1)
    assert (block[511], lane[511]) == (7, 63)


def test_placement_three_workers_by_hand():
    block, lane, b_w, n_w = layout.stream_placement(16, 3, 4)
    assert list(n_w) == [4, 4, 8] and list(b_w) == [0, 4, 8]      # 4 tiles: starts 0, 1, 2 (4)
    # the placement inside a tile does not depend on the worker
    assert (block[512], lane[512]) == (8, 0)
    assert (block[513], lane[513]) == (9, 0)
    assert (block[1023], lane[1023]) == (15, 63)


def test_placement_with_smaller_tiles_by_hand():
    # 32 code bytes per group: tiles of 2 blocks; 64: every block by itself
    assert layout.default_tile_blocks(8) == 4 and layout.default_tile_blocks(16) == 4
    assert layout.default_tile_blocks(32) == 2 and layout.default_tile_blocks(64) == 1
    block, lane, _, _ = layout.stream_placement(6, 1, 2)
    assert (block[0], lane[0]) == (0, 0)
    assert (block[1], lane[1]) == (1, 0)
    assert (block[127], lane[127]) == (1, 63)
    assert (block[128], lane[128]) == (2, 0)
    assert (block[129], lane[129]) == (3, 0)
    assert (block[383], lane[383]) == (5, 63)
    block, lane, _, _ = layout.stream_placement(7, 1, 1)
    assert np.array_equal(block, np.arange(448) // 64) and np.array_equal(lane, np.arange(448) % 64)


@pytest.mark.parametrize("U", [4, 2, 1])
@pytest.mark.parametrize("ntiles,n_waves", [(1, 1), (5, 16), (16, 16), (37, 16), (100, 21), (9, 4096)])
def test_placement_is_a_bijection(ntiles, n_waves, U):
    block, lane, _, _ = layout.stream_placement(ntiles * U, n_waves, U)
    slot = block * 64 + lane
    assert np.array_equal(np.sort(slot), np.arange(ntiles * U * 64))


def hand_tile(code_bytes):
    return 4 if code_bytes <= 16 else (2 if code_bytes <= 32 else 1)


def hand_counts(ntiles, n_waves):
    """Tiles per worker, written out with a plain loop."""
    return [(w + 1) * ntiles // n_waves - w * ntiles // n_waves for w in range(n_waves)]


def decode_blob(blob, N, K, bits, nnzg, n_wg, wpw, G=16):
    """Invert the layout with plain loops, walking workers / tiles / lanes."""
    cb = G * bits // 8
    plane = min(16, cb)
    blk_bytes = (cb + 6) * 64
    U = hand_tile(cb)
    ntiles = (nnzg + 64 * U - 1) // (64 * U)
    nblocks = ntiles * U
    raw = np.frombuffer(blob, dtype=np.uint8)
    codes = np.zeros((nblocks * 64, G), dtype=np.int64)
    scales = np.zeros(nblocks * 64, dtype=np.uint16)
    zeros = np.zeros(nblocks * 64, dtype=np.uint16)
    cols = np.zeros(nblocks * 64, dtype=np.int64)
    heads = np.zeros(nblocks * 64, dtype=bool)
    pos = 0
    b = 0
    counts = hand_counts(ntiles, n_wg * wpw)
    for w in range(n_wg * wpw):
        for _ in range(counts[w]):
            for p in range(64 * U):
                blk = b + p % U
                ln = p // U
                base = blk * blk_bytes
                # the lane's code string, plane by plane
                cbytes = bytearray()
                for k in range(cb // plane):
                    o = base + k * 64 * plane + ln * plane
                    cbytes += raw[o:o + plane].tobytes()
                if bits == 4:
                    for h in range(G // 8):
                        word = int.from_bytes(cbytes[4 * h:4 * h + 4], "little")
                        for m in range(4):
                            codes[pos, 8 * h + 2 * m] = (word >> (4 * m)) & 0xF
                            codes[pos, 8 * h + 2 * m + 1] = (word >> (16 + 4 * m)) & 0xF
                else:
                    codes[pos] = list(cbytes)
                o = base + 64 * cb + ln * 4
                sz = int.from_bytes(raw[o:o + 4].tobytes(), "little")
                scales[pos] = sz & 0xFFFF
                zeros[pos] = sz >> 16
                o = base + 64 * cb + 256 + ln * 2
                ix = int.from_bytes(raw[o:o + 2].tobytes(), "little")
                slot = ix >> 4
                per_group = max(1, G // 16)     # slots per group (G = 8: the index counts half-slots)
                assert slot % per_group == 0
                cols[pos] = slot // per_group
                heads[pos] = bool(ix & 1)
                assert ix & 0xE == 0
                pos += 1
            b += U
    assert b == nblocks
    return codes, scales, zeros, cols, heads


@pytest.mark.parametrize("bits,G", [(4, 8), (8, 8), (4, 16), (8, 16), (4, 32), (4, 64), (4, 128), (8, 32), (8, 64)])
@pytest.mark.parametrize("n_wg,wpw", [(1, 1), (3, 1), (1, 16), (3, 16), (5, 4), (2, 7)])
def test_blob_decodes_back_to_canonical(bits, G, n_wg, wpw):
    n_waves = n_wg * wpw
    N, K = 40, 512 * max(1, G // 16)
    W = gi.dense_weight(N, K, seed=41)
    keep = gi.imbalanced_keep_counts(N, K // G, seed=41)
    keep[5] = 0
    keep[N - 1] = 0
    c = oracle.pack(W, G=G, bits=bits, keep_per_row=keep)
    blob = oracle.device_blob(c, n_wg, wpw)
    assert len(blob) % 256 == 0
    codes, scales, zeros, cols, heads = decode_blob(blob, N, K, bits, c.nnzg, n_wg, wpw, G)
    nn = c.nnzg
    if bits == 4:
        v = np.asarray(c.values).reshape(nn, G // 2)
        ref = np.empty((nn, G), dtype=np.int64)
        ref[:, 0::2] = v & 0xF
        ref[:, 1::2] = v >> 4
    else:
        ref = np.asarray(c.values).reshape(nn, G).astype(np.int64)
    assert np.array_equal(codes[:nn], ref)
    assert np.array_equal(scales[:nn], c.scales) and np.array_equal(zeros[:nn], c.zeros)
    assert np.array_equal(cols[:nn], c.groups)
    # padding is null groups
    assert not codes[nn:].any() and not scales[nn:].any() and not cols[nn:].any() and not heads[nn:].any()
    # head flags: first stored group of every non-empty row
    exp_heads = np.zeros(nn, dtype=bool)
    for n in range(N):
        if c.rowIndex[n + 1] > c.rowIndex[n]:
            exp_heads[c.rowIndex[n]] = True
    assert np.array_equal(heads[:nn], exp_heads)
    # side tables
    cb = G * bits // 8
    U = hand_tile(cb)
    ntiles = (nn + 64 * U - 1) // (64 * U)
    nblocks = ntiles * U
    off = (nblocks * (cb + 6) * 64 + 255) // 256 * 256
    wave_info = np.frombuffer(blob, dtype="<i4", count=4 * n_waves, offset=off).reshape(n_waves, 4)
    # brute force: the row and the worker of every stored group
    row_of = np.repeat(np.arange(N), np.diff(c.rowIndex))
    worker_of = np.empty(nn, dtype=np.int64)
    counts = [U * t for t in hand_counts(ntiles, n_waves)]
    b = 0
    for w in range(n_waves):
        n_w = counts[w]
        worker_of[64 * b:min(64 * (b + n_w), nn)] = w
        b += n_w
    b = 0
    for w in range(n_waves):
        n_w = counts[w]
        first = 64 * b
        assert wave_info[w, 0] == int(exp_heads[:min(first, nn)].sum()) - 1
        b += n_w
        end = 64 * b
        closed = 1 if end >= nn or exp_heads[end] else 0
        lead_first, chain_len, lead_len = -1, 0, 0
        if first < nn and not exp_heads[first]:
            lead_first = worker_of[c.rowIndex[row_of[first]]]
            # workers from the one holding that row's head to the one holding its last group
            lead_len = worker_of[c.rowIndex[row_of[first] + 1] - 1] - lead_first + 1
        assert wave_info[w, 1] == closed + 2 * lead_len
        if n_w > 0 and not closed and exp_heads[first:end].any():
            last_row = row_of[end - 1]
            chain_len = worker_of[c.rowIndex[last_row + 1] - 1] - w + 1
        assert wave_info[w, 2] == lead_first
        assert wave_info[w, 3] == chain_len
    off = (off + 16 * n_waves + 255) // 256 * 256
    nonempty = [n for n in range(N) if keep[n] > 0]
    empty = [n for n in range(N) if keep[n] == 0]
    assert list(np.frombuffer(blob, dtype="<i4", count=len(nonempty), offset=off)) == nonempty
    off = (off + 4 * len(nonempty) + 255) // 256 * 256
    assert list(np.frombuffer(blob, dtype="<i4", count=len(empty), offset=off)) == empty
    assert len(blob) == (off + 4 * len(empty) + 255) // 256 * 256


@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("U,LN,n_wg,wpw", [(3, 60, 5, 4), (4, 36, 9, 2), (5, 64, 3, 4), (4, 64, 3, 7)])
def test_blob_with_a_span_per_worker_and_a_tile_shape_decodes_back(bits, U, LN, n_wg, wpw):
    """Spans per worker, tiles of U blocks with LN lanes in use (spec items 1, 3, 4), read back with
    plain loops: worker w's tile is blocks wU .. wU+U-1 of (cb + 6) * LN bytes, position p of the
    tile in block p mod U at entry p div U; the rows come back whole, in order, each inside one
    worker's tile, everything else is null, and no worker shares a row."""
    N, K, G = 40, 1024, 16
    cb = G * bits // 8
    W = gi.dense_weight(N, K, seed=43)
    keep = gi.imbalanced_keep_counts(N, K // G, seed=43)
    keep = np.minimum(keep, 40)
    keep[[5, N - 1]] = 0
    c = oracle.pack(W, G=G, bits=bits, keep_per_row=keep)
    n_waves = n_wg * wpw
    blob = oracle.device_blob(c, n_wg, wpw, 1, U, LN, True)
    raw = np.frombuffer(blob, dtype=np.uint8)
    bb = (cb + 6) * LN
    got_rows = []          # (worker, [columns], [scale bits], [zero bits], [[codes]])
    for w in range(n_waves):
        current = None
        for p in range(U * LN):
            base = (w * U + p % U) * bb
            e = p // U
            code = raw[base + e * cb:base + (e + 1) * cb]
            sz = int.from_bytes(raw[base + LN * cb + 4 * e:base + LN * cb + 4 * e + 4].tobytes(), "little")
            ix = int.from_bytes(raw[base + LN * (cb + 4) + 2 * e:base + LN * (cb + 4) + 2 * e + 2].tobytes(), "little")
            if ix & 1:
                current = (w, [], [], [], [])
                got_rows.append(current)
            if sz == 0 and ix == 0 and not code.any():
                continue                                 # a null group (no stored scale is 0: the floor is 2^-14)
            assert current is not None, "a stored group before the first row head of a tile"
            current[1].append(ix >> 4)
            current[2].append(sz & 0xFFFF)
            current[3].append(sz >> 16)
            if bits == 4:
                q = []
                for h in range(2):
                    word = int.from_bytes(code[4 * h:4 * h + 4].tobytes(), "little")
                    for m in range(4):
                        q += [(word >> (4 * m)) & 0xF, (word >> (16 + 4 * m)) & 0xF]
                current[4].append(q)
            else:
                current[4].append(list(code))
    rows = [n for n in range(N) if keep[n] > 0]
    assert len(got_rows) == len(rows)
    workers = []
    for (w, cols, sc, ze, q), n in zip(got_rows, rows):
        g0, g1 = c.rowIndex[n], c.rowIndex[n + 1]
        assert cols == list(c.groups[g0:g1]) and sc == list(c.scales[g0:g1]) and ze == list(c.zeros[g0:g1])
        v = np.asarray(c.values).reshape(c.nnzg, cb)[g0:g1]
        if bits == 4:
            ref = np.empty((g1 - g0, G), dtype=np.int64)
            ref[:, 0::2] = v & 0xF
            ref[:, 1::2] = v >> 4
        else:
            ref = v.astype(np.int64)
        assert np.array_equal(np.array(q), ref)
        workers.append(w)
    assert workers == sorted(workers)
    # greedy placement by hand: a row goes to the current worker's tile if it still fits
    w, used, expect = 0, 0, []
    for n in rows:
        if used + keep[n] > U * LN:
            w, used = w + 1, 0
        expect.append(w)
        used += keep[n]
    assert workers == expect
    # worker records: rank of the row open at the start = (rows before the worker) - 1; nothing shared
    off = (n_waves * U * bb + 255) // 256 * 256
    wave_info = np.frombuffer(blob, dtype="<i4", count=4 * n_waves, offset=off).reshape(n_waves, 4)
    for w in range(n_waves):
        assert list(wave_info[w]) == [sum(1 for x in expect if x < w) - 1, 1, -1, 0]
    with pytest.raises(ValueError):
        oracle.device_blob(c, 1, 1, 1, U, LN, True)      # more spans needed than workers


def test_blob_of_empty_matrix():
    W = gi.dense_weight(8, 64, seed=1)
    c = oracle.pack(W, sparsity=1.0)
    blob = oracle.device_blob(c, 1, 16)
    # no blocks; wave_info = {-1, 1, -1, 0} for every worker; no non-empty rows; 8 empty rows
    assert np.array_equal(np.frombuffer(blob, dtype="<i4", count=64).reshape(16, 4),
                          np.tile(np.array([-1, 1, -1, 0]), (16, 1)))
    assert list(np.frombuffer(blob, dtype="<i4", count=8, offset=256)) == list(range(8))
    assert len(blob) == 512


@pytest.mark.parametrize("bits,G", [(4, 16), (8, 16), (4, 32), (4, 64), (4, 128), (8, 32), (8, 64)])
def test_panel_blob_decodes_back_to_the_dequantised_matrix(bits, G):
    """The second image read as its consumer reads it -- header word of a column (row mask, groups
    before it), data offset, a group's record (codes by quarters and chunks, the 4-bit bytes
    regrouped, scale | zero in the middle; 8-bit codes with G = 16: the word stored twice) -- gives
    back W^ of Eq. 3 exactly, every stored group once.  Pins the written layout of that image to
    the canonical arrays, independently of the code that builds it."""
    N, K = 45, 70 * G            # 3 panels (the last with 13 rows), 3 slices (the last with 6 columns)
    W = gi.dense_weight(N, K, seed=31)
    keep = gi.imbalanced_keep_counts(N, K // G, seed=31)
    keep[[2, 44]] = 0
    keep[5] = K // G
    c = oracle.pack(W, G, bits, keep_per_row=keep)
    blob = np.frombuffer(layout.panel_blob(c), dtype=np.uint8)
    P, S, chunks = -(-N // 16), -(-(K // G) // 32), G // 16
    cb = G * bits // 8
    twice = bits == 8 and G == 16
    rb = cb + (8 if twice else 4)
    qb = bits // 2                                   # bytes of a quarter of a chunk
    header_bytes = -(-(P * S * 144) // 256) * 256
    headers = blob[: P * S * 144].view("<u4").reshape(P * S, 36)
    data = blob[header_bytes:]
    dense = np.zeros((N, K), dtype=np.float64)
    seen = 0
    for p in range(P):
        for s in range(S):
            h = headers[p * S + s]
            base = int(h[32]) * 16
            for j in range(32):
                mask, before = int(h[j]) & 0xFFFF, int(h[j]) >> 16
                rows = [r for r in range(16) if mask >> r & 1]
                for rank, r in enumerate(rows):
                    rec = data[base + (before + rank) * rb: base + (before + rank + 1) * rb]
                    q = np.zeros(G, dtype=np.int64)
                    for t in range(4):
                        for i in range(chunks):
                            at = (4 * t + (4 if t >= 1 else 0) + (4 if t >= 3 else 0)) if twice \
                                else (t * chunks + i) * qb + (4 if t >= 2 else 0)
                            b = rec[at: at + qb]
                            if bits == 4:
                                e = [b[0] & 15, b[1] & 15, b[0] >> 4, b[1] >> 4]
                            else:
                                e = list(b)
                            q[16 * i + 4 * t: 16 * i + 4 * t + 4] = e
                    words = [rec[4:8], rec[16:20]] if twice else [rec[cb // 2: cb // 2 + 4]]
                    assert all(bytes(w) == bytes(words[0]) for w in words)
                    sc, z = (float(v) for v in np.frombuffer(bytes(words[0]), dtype=np.float16))
                    n, col = 16 * p + r, 32 * s + j
                    assert n < N and col < K // G
                    dense[n, col * G: (col + 1) * G] = (q - z) * sc
                    seen += 1
            assert int(h[33]) == (int(h[31]) >> 16) + bin(int(h[31]) & 0xFFFF).count("1")
    assert seen == c.nnzg
    assert np.array_equal(dense, oracle.densify(c))
