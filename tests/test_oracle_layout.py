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


def test_default_partition():
    assert oracle.default_partition(0) == (1, 1)
    assert oracle.default_partition(2048) == (32, 1)            # 32 blocks -> one per workgroup
    assert oracle.default_partition(64 * 17) == (17, 1)
    assert oracle.default_partition(524288) == (256, 16)        # 8192 blocks: 32 per workgroup, 2 per wavefront
    assert oracle.default_partition(64 * 4096) == (256, 8)      # 16 per workgroup -> 8 wavefronts of 2
    assert oracle.default_partition(64 * 1000) == (256, 2)      # 4 (some 3) per workgroup
    assert oracle.default_partition(64 * 2048) == (256, 4)
    assert oracle.default_partition(64 * 1024, G=128) == (256, 4)   # heavy groups: one block per wavefront
    assert oracle.default_partition(64 * 2048, G=64) == (256, 8)
    assert oracle.default_partition(1409024) == (256, 16)       # 11008x4096 at S = 50 %


def test_two_level_block_deal_by_hand():
    # 23 blocks over 3 workgroups of 4 wavefronts: workgroups get 8, 8, 7; inside: 2,2,2,2 / 2,2,2,2 / 2,2,2,1
    assert list(layout.worker_block_counts(23, 3, 4)) == [2, 2, 2, 2, 2, 2, 2, 2, 2, 2, 2, 1]
    # 5 blocks over 2 workgroups of 4: 3 and 2 -> 1,1,1,0 / 1,1,0,0
    assert list(layout.worker_block_counts(5, 2, 4)) == [1, 1, 1, 0, 1, 1, 0, 0]
    # LLaMA-7B down_proj at W4S50: 22016 blocks over 256 x 16 -> 86 per workgroup = 6x6 + 10x5
    c = layout.worker_block_counts(22016, 256, 16)
    assert list(c[:16]) == [6] * 6 + [5] * 10 and c.sum() == 22016


def test_placement_single_worker_7_blocks_by_hand():
    block, lane, b_w, _ = layout.stream_placement(7, 1, 1)
    assert list(b_w) == [0]
    # superblock of 4 blocks: position p -> block p mod 4, lane p div 4
    assert (block[0], lane[0]) == (0, 0)
    assert (block[1], lane[1]) == (1, 0)
    assert (block[5], lane[5]) == (1, 1)
    assert (block[255], lane[255]) == (3, 63)
    # then a superblock of 2 blocks (blocks 4,5)
    assert (block[256], lane[256]) == (4, 0)
    assert (block[257], lane[257]) == (5, 0)
    assert (block[383], lane[383]) == (5, 63)
    # then a single block (block 6)
    assert (block[384], lane[384]) == (6, 0)
    assert (block[447], lane[447]) == (6, 63)


def test_placement_three_workers_7_blocks_by_hand():
    block, lane, b_w, _ = layout.stream_placement(7, 3, 1)
    assert list(b_w) == [0, 3, 5]                        # 3, 2, 2 blocks
    # worker 0: superblocks of 2 then 1
    assert (block[1], lane[1]) == (1, 0)
    assert (block[127], lane[127]) == (1, 63)
    assert (block[128], lane[128]) == (2, 0)
    assert (block[191], lane[191]) == (2, 63)
    # worker 1 starts at stream position 192, a superblock of 2
    assert (block[192], lane[192]) == (3, 0)
    assert (block[193], lane[193]) == (4, 0)
    # worker 2 starts at 320
    assert (block[320], lane[320]) == (5, 0)
    assert (block[447], lane[447]) == (6, 63)


def test_placement_with_capped_superblocks_by_hand():
    # 32 code bytes per group: superblocks of at most 2 blocks -> 7 blocks = 2 + 2 + 2 + 1
    assert layout.largest_superblock(8) == 4 and layout.largest_superblock(16) == 4
    assert layout.largest_superblock(32) == 2 and layout.largest_superblock(64) == 1
    block, lane, _, _ = layout.stream_placement(7, 1, 1, u_max=2)
    assert (block[0], lane[0]) == (0, 0)
    assert (block[1], lane[1]) == (1, 0)
    assert (block[127], lane[127]) == (1, 63)
    assert (block[128], lane[128]) == (2, 0)
    assert (block[129], lane[129]) == (3, 0)
    assert (block[383], lane[383]) == (5, 63)
    assert (block[384], lane[384]) == (6, 0)
    assert (block[447], lane[447]) == (6, 63)
    # 64 code bytes per group: every block by itself -> stream order
    block, lane, _, _ = layout.stream_placement(7, 1, 1, u_max=1)
    assert np.array_equal(block, np.arange(448) // 64) and np.array_equal(lane, np.arange(448) % 64)


@pytest.mark.parametrize("u_max", [4, 2, 1])
@pytest.mark.parametrize("nblocks,n_wg,wpw", [(1, 1, 1), (5, 1, 16), (16, 1, 16), (37, 2, 8), (100, 7, 3),
                                               (9, 256, 16)])
def test_placement_is_a_bijection(nblocks, n_wg, wpw, u_max):
    block, lane, _, _ = layout.stream_placement(nblocks, n_wg, wpw, u_max)
    slot = block * 64 + lane
    assert np.array_equal(np.sort(slot), np.arange(nblocks * 64))


def hand_counts(nblocks, n_wg, wpw):
    """Blocks per worker, written out with plain loops."""
    out = []
    for g in range(n_wg):
        m = nblocks // n_wg + (1 if g < nblocks % n_wg else 0)
        for l in range(wpw):
            out.append(m // wpw + (1 if l < m % wpw else 0))
    return out


def hand_superblocks(n_w, code_bytes):
    """Superblock sizes of a run of n_w blocks, written out (4s, then 2s, then 1s, capped)."""
    u_max = 4 if code_bytes <= 16 else (2 if code_bytes <= 32 else 1)
    sizes = []
    left = n_w
    for U in (4, 2, 1):
        while U <= u_max and left >= U:
            sizes.append(U)
            left -= U
    return sizes


def decode_blob(blob, N, K, bits, nnzg, n_wg, wpw, G=16):
    """Invert the layout with plain loops, walking workers / superblocks / lanes."""
    cb = G * bits // 8
    plane = min(16, cb)
    blk_bytes = (cb + 6) * 64
    nblocks = (nnzg + 63) // 64
    raw = np.frombuffer(blob, dtype=np.uint8)
    codes = np.zeros((nblocks * 64, G), dtype=np.int64)
    scales = np.zeros(nblocks * 64, dtype=np.uint16)
    zeros = np.zeros(nblocks * 64, dtype=np.uint16)
    cols = np.zeros(nblocks * 64, dtype=np.int64)
    heads = np.zeros(nblocks * 64, dtype=bool)
    pos = 0
    b = 0
    counts = hand_counts(nblocks, n_wg, wpw)
    for w in range(n_wg * wpw):
        for U in hand_superblocks(counts[w], cb):
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
                assert slot % (G // 16) == 0
                cols[pos] = slot // (G // 16)
                heads[pos] = bool(ix & 1)
                assert ix & 0xE == 0
                pos += 1
            b += U
    assert b == nblocks
    return codes, scales, zeros, cols, heads


@pytest.mark.parametrize("bits,G", [(4, 16), (8, 16), (4, 32), (4, 64), (4, 128), (8, 32), (8, 64)])
@pytest.mark.parametrize("n_wg,wpw", [(1, 1), (3, 1), (1, 16), (3, 16), (5, 4), (2, 7)])
def test_blob_decodes_back_to_canonical(bits, G, n_wg, wpw):
    n_waves = n_wg * wpw
    N, K = 40, 512 * (G // 16)
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
    nblocks = (nn + 63) // 64
    cb = G * bits // 8
    off = (nblocks * (cb + 6) * 64 + 255) // 256 * 256
    wave_info = np.frombuffer(blob, dtype="<i4", count=4 * n_waves, offset=off).reshape(n_waves, 4)
    # brute force: the row and the worker of every stored group
    row_of = np.repeat(np.arange(N), np.diff(c.rowIndex))
    worker_of = np.empty(nn, dtype=np.int64)
    counts = hand_counts(nblocks, n_wg, wpw)
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


def test_blob_of_empty_matrix():
    W = gi.dense_weight(8, 64, seed=1)
    c = oracle.pack(W, sparsity=1.0)
    blob = oracle.device_blob(c, 1, 16)
    # no blocks; wave_info = {-1, 1, -1, 0} for every worker; no non-empty rows; 8 empty rows
    assert np.array_equal(np.frombuffer(blob, dtype="<i4", count=64).reshape(16, 4),
                          np.tile(np.array([-1, 1, -1, 0]), (16, 1)))
    assert list(np.frombuffer(blob, dtype="<i4", count=8, offset=256)) == list(range(8))
    assert len(blob) == 512
