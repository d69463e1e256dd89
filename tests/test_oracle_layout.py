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


def test_default_worker_count():
    assert oracle.default_n_waves(0) == 16
    assert oracle.default_n_waves(2048) == 32            # 32 blocks -> 2 workgroups of 16
    assert oracle.default_n_waves(64 * 17) == 32
    assert oracle.default_n_waves(524288) == 4096        # 8192 blocks -> capped at 256 workgroups
    assert oracle.default_n_waves(64 * 4096) == 4096
    assert oracle.default_n_waves(64 * 1000) == 1008


def test_placement_single_worker_7_blocks_by_hand():
    block, lane, b_w = layout.stream_placement(7, 1)
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
    block, lane, b_w = layout.stream_placement(7, 3)
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


@pytest.mark.parametrize("nblocks,n_waves", [(1, 1), (5, 16), (16, 16), (37, 16), (100, 7), (9, 4096)])
def test_placement_is_a_bijection(nblocks, n_waves):
    block, lane, _ = layout.stream_placement(nblocks, n_waves)
    slot = block * 64 + lane
    assert np.array_equal(np.sort(slot), np.arange(nblocks * 64))


def decode_blob(blob, N, K, bits, nnzg, n_waves):
    """Invert the layout with plain loops, walking workers / superblocks / lanes."""
    G = 16
    cb = G * bits // 8
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
    for w in range(n_waves):
        n_w = nblocks // n_waves + (1 if w < nblocks % n_waves else 0)
        sizes = [4] * (n_w // 4)
        if n_w % 4 >= 2:
            sizes.append(2)
        if n_w % 2 == 1:
            sizes.append(1)
        for U in sizes:
            for p in range(64 * U):
                blk = b + p % U
                ln = p // U
                base = blk * blk_bytes
                cbytes = raw[base + ln * cb: base + (ln + 1) * cb]
                if bits == 4:
                    for h in range(2):
                        word = int.from_bytes(cbytes[4 * h:4 * h + 4].tobytes(), "little")
                        for m in range(4):
                            codes[pos, 8 * h + 2 * m] = (word >> (4 * m)) & 0xF
                            codes[pos, 8 * h + 2 * m + 1] = (word >> (16 + 4 * m)) & 0xF
                else:
                    codes[pos] = cbytes
                o = base + 64 * cb + ln * 4
                sz = int.from_bytes(raw[o:o + 4].tobytes(), "little")
                scales[pos] = sz & 0xFFFF
                zeros[pos] = sz >> 16
                o = base + 64 * cb + 256 + ln * 2
                ix = int.from_bytes(raw[o:o + 2].tobytes(), "little")
                cols[pos] = ix & 0x7FFF
                heads[pos] = bool(ix & 0x8000)
                pos += 1
            b += U
    assert b == nblocks
    return codes, scales, zeros, cols, heads


@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("n_waves", [1, 3, 16, 48])
def test_blob_decodes_back_to_canonical(bits, n_waves):
    N, K = 40, 512
    W = gi.dense_weight(N, K, seed=41)
    keep = gi.imbalanced_keep_counts(N, K // 16, seed=41)
    keep[5] = 0
    keep[N - 1] = 0
    c = oracle.pack(W, bits=bits, keep_per_row=keep)
    blob = oracle.device_blob(c, n_waves)
    assert len(blob) % 256 == 0
    codes, scales, zeros, cols, heads = decode_blob(blob, N, K, bits, c.nnzg, n_waves)
    nn = c.nnzg
    if bits == 4:
        v = np.asarray(c.values).reshape(nn, 8)
        ref = np.empty((nn, 16), dtype=np.int64)
        ref[:, 0::2] = v & 0xF
        ref[:, 1::2] = v >> 4
    else:
        ref = np.asarray(c.values).reshape(nn, 16).astype(np.int64)
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
    cb = 16 * bits // 8
    off = (nblocks * (cb + 6) * 64 + 255) // 256 * 256
    wave_info = np.frombuffer(blob, dtype="<i4", count=2 * n_waves, offset=off).reshape(n_waves, 2)
    b = 0
    for w in range(n_waves):
        n_w = nblocks // n_waves + (1 if w < nblocks % n_waves else 0)
        assert wave_info[w, 0] == int(exp_heads[:min(64 * b, nn)].sum()) - 1
        b += n_w
        end = 64 * b
        closed = 1 if end >= nn or exp_heads[end] else 0
        assert wave_info[w, 1] == closed
    off = (off + 8 * n_waves + 255) // 256 * 256
    nonempty = [n for n in range(N) if keep[n] > 0]
    empty = [n for n in range(N) if keep[n] == 0]
    assert list(np.frombuffer(blob, dtype="<i4", count=len(nonempty), offset=off)) == nonempty
    off = (off + 4 * len(nonempty) + 255) // 256 * 256
    assert list(np.frombuffer(blob, dtype="<i4", count=len(empty), offset=off)) == empty
    assert len(blob) == (off + 4 * len(empty) + 255) // 256 * 256


def test_blob_of_empty_matrix():
    W = gi.dense_weight(8, 64, seed=1)
    c = oracle.pack(W, sparsity=1.0)
    blob = oracle.device_blob(c, 16)
    # no blocks; {rank_base, tail_closed} = {-1, 1} for every worker; no non-empty rows; 8 empty rows
    assert np.array_equal(np.frombuffer(blob, dtype="<i4", count=32).reshape(16, 2),
                          np.tile(np.array([-1, 1]), (16, 1)))
    assert list(np.frombuffer(blob, dtype="<i4", count=8, offset=256)) == list(range(8))
    assert len(blob) == 512
