"""Device byte layout of a packed GQSA matrix, re-derived from its written
specification -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.

The layout is a pure permutation/padding of the canonical BSR arrays of the
paper's Sec. 3.2 listing (rowIndex / groups / values) and the per-group scale
and zero of Eq. 1; it adds no arithmetic.  The specification, restated:

 1. Stream.  The stored groups in canonical order g = 0..nnzg-1 form a stream;
    it is padded with null groups (all bytes zero) to nblocks*64 positions,
    nblocks = ceil(nnzg/64).
 2. Partition, two levels.  The blocks are dealt to n_workgroups workgroups in
    contiguous runs: workgroup g gets nblocks div n_workgroups blocks (+1 if
    g < nblocks mod n_workgroups).  A workgroup's run of m blocks is dealt the
    same way to its waves_per_workgroup wavefronts: wavefront l gets
    m div waves_per_workgroup (+1 if l < m mod waves_per_workgroup).  Worker
    w = g*waves_per_workgroup + l; n_waves = n_workgroups*waves_per_workgroup;
    b_w = first block of worker w = sum of the earlier workers' counts.
 3. Superblocks.  A worker's run is cut, from its start, into superblocks of 4
    blocks as long as 4 fit, then one of 2 blocks if at least 2 remain, then
    one of 1 block if one remains.  A superblock of U blocks starting at block
    b covers stream positions 64b .. 64(b+U)-1 of the stream; the position
    64b + p lives in block b + (p mod U), lane p div U.
 4. Block.  Each block is (G*bits/8 + 6)*64 bytes: 64 lanes x code bytes, then
    64 x uint32 (fp16 scale bits | fp16 zero bits << 16), then 64 x uint16
    (group-column << 4, plus 1 if the group is the first stored group of its
    row; group-columns are below 4096).
    4-bit codes, G = 16: a lane holds two little-endian uint32; word h holds
    elements 8h..8h+7 of the group, element 8h+2m in bits 4m..4m+3 and element
    8h+2m+1 in bits 16+4m..16+4m+3 (m = 0..3).  8-bit codes: byte j of the
    lane's 16 bytes is element j.
 5. Side tables (int32): wave_info[n_waves][4] = {rank_base, tail_closed +
    2 * lead_len, lead_first, chain_len} with
      rank_base   = (number of row-head groups at stream positions before
                    worker w's first position) - 1;
      tail_closed = 1 if the first position after the worker's run is at or
                    beyond nnzg or holds a row-head group, else 0;
      lead_len    = chain_len of worker lead_first (below), 0 if lead_first = -1;
      lead_first  = for a worker (with or without blocks) whose first position
                    b_w*64 holds a stored group that is not a row head: the
                    worker that owns the head group of that group's row; else -1;
      chain_len   = for a worker with blocks, tail_closed = 0 and at least one
                    row head inside its run: (worker owning the last stored
                    group of the row that is open at the end of its run) - w + 1;
                    else 0;
    row_of_rank[r] = index of the r-th non-empty row; empty_rows = indices of
    the empty rows.
 6. Blob = blocks, wave_info, row_of_rank, empty_rows, each region starting
    at a multiple of 256 bytes, zero padded, total a multiple of 256 (>= 256).
"""
from __future__ import annotations

import numpy as np

LANES = 64
ALIGN = 256
MAX_WAVES = 4096
WAVES_PER_WORKGROUP = 16


def default_partition(nnzg: int):
    """(n_workgroups, waves_per_workgroup) the library picks when not told otherwise:
    workgroups of 16 wavefronts, at most 256 of them, no more than the blocks can feed."""
    nblocks = (nnzg + LANES - 1) // LANES
    wgs = (nblocks + WAVES_PER_WORKGROUP - 1) // WAVES_PER_WORKGROUP
    wgs = max(1, min(MAX_WAVES // WAVES_PER_WORKGROUP, wgs))
    return wgs, WAVES_PER_WORKGROUP


def worker_block_counts(nblocks: int, n_workgroups: int, waves_per_workgroup: int) -> np.ndarray:
    """Blocks owned by every worker (spec item 2)."""
    base, extra = divmod(nblocks, n_workgroups)
    out = np.zeros(n_workgroups * waves_per_workgroup, dtype=np.int64)
    for g in range(n_workgroups):
        m = base + (1 if g < extra else 0)
        b2, e2 = divmod(m, waves_per_workgroup)
        row = np.full(waves_per_workgroup, b2, dtype=np.int64)
        row[:e2] += 1
        out[g * waves_per_workgroup:(g + 1) * waves_per_workgroup] = row
    return out


def _align(n: int) -> int:
    return (n + ALIGN - 1) // ALIGN * ALIGN


def stream_placement(nblocks: int, n_workgroups: int, waves_per_workgroup: int):
    """For every stream position: (block, lane) it is stored at (spec items 2-3)."""
    n_w = worker_block_counts(nblocks, n_workgroups, waves_per_workgroup)
    b_w = np.concatenate(([0], np.cumsum(n_w)[:-1]))
    pos = np.arange(nblocks * LANES, dtype=np.int64)
    blk_of_pos = pos // LANES
    # worker owning each block: block counts expanded
    w = np.repeat(np.arange(n_w.size), n_w)[blk_of_pos]
    q = pos - LANES * b_w[w]                    # position inside the worker's run
    nw = n_w[w]
    n4 = nw // 4
    rem = nw % 4
    in4 = q < 256 * n4
    qq = q - 256 * n4
    has2 = rem >= 2
    in2 = (~in4) & has2 & (qq < 128)
    in1 = (~in4) & (~in2)
    U = np.where(in4, 4, np.where(in2, 2, 1))
    sb_blk = np.where(in4, 4 * (q // 256), np.where(in2, 4 * n4, 4 * n4 + np.where(has2, 2, 0)))
    p = np.where(in4, q % 256, np.where(in2, qq, qq - np.where(has2, 128, 0)))
    assert (p[in1] < 64).all() and (p >= 0).all()
    block = b_w[w] + sb_blk + (p % U)
    lane = p // U
    return block, lane, b_w, n_w


def device_blob(c, n_workgroups: int, waves_per_workgroup: int) -> bytes:
    """Exact bytes the library must hold on the device for canonical arrays `c`."""
    if c.G != 16 or c.bits not in (4, 8):
        raise ValueError("device layout is specified for G=16, bits in {4,8}")
    nnzg = c.nnzg
    nblocks = (nnzg + LANES - 1) // LANES
    code_bytes = c.G * c.bits // 8
    blk_bytes = (code_bytes + 6) * LANES

    ri = np.asarray(c.rowIndex, dtype=np.int64)
    counts = ri[1:] - ri[:-1]
    nonempty = np.nonzero(counts > 0)[0].astype(np.int32)
    empty = np.nonzero(counts == 0)[0].astype(np.int32)
    head_pos = ri[:-1][counts > 0]                 # stream position of each row's first group

    n_waves = n_workgroups * waves_per_workgroup
    blocks = np.zeros((nblocks, blk_bytes), dtype=np.uint8)
    wave_info = np.zeros((n_waves, 4), dtype=np.int32)
    wave_info[:, 0] = -1
    wave_info[:, 1] = 1
    wave_info[:, 2] = -1
    if nblocks > 0:
        block, lane, b_w, n_w = stream_placement(nblocks, n_workgroups, waves_per_workgroup)
        block = block[:nnzg]
        lane = lane[:nnzg]
        # codes
        vals = np.asarray(c.values, dtype=np.uint8).reshape(nnzg, code_bytes)
        if c.bits == 4:
            elems = np.empty((nnzg, 16), dtype=np.uint32)
            elems[:, 0::2] = vals & 0xF
            elems[:, 1::2] = vals >> 4
            words = np.zeros((nnzg, 2), dtype=np.uint32)
            for h in range(2):
                for m in range(4):
                    words[:, h] |= elems[:, 8 * h + 2 * m] << np.uint32(4 * m)
                    words[:, h] |= elems[:, 8 * h + 2 * m + 1] << np.uint32(16 + 4 * m)
            lane_bytes = words.astype("<u4").view(np.uint8).reshape(nnzg, 8)
        else:
            lane_bytes = vals
        codes_view = blocks[:, :LANES * code_bytes].reshape(nblocks, LANES, code_bytes)
        codes_view[block, lane, :] = lane_bytes
        # scale | zero << 16
        sz = (np.asarray(c.scales, dtype=np.uint32) |
              (np.asarray(c.zeros, dtype=np.uint32) << np.uint32(16))).astype("<u4")
        sz_off = LANES * code_bytes
        sz_view = blocks[:, sz_off:sz_off + LANES * 4].reshape(nblocks, LANES, 4)
        sz_view[block, lane, :] = sz.view(np.uint8).reshape(nnzg, 4)
        # group-column | head flag
        is_head = np.zeros(nnzg, dtype=np.uint16)
        is_head[head_pos] = 1
        gcol = np.asarray(c.groups, dtype=np.int64)
        if gcol.size and gcol.max() >= 4096:
            raise ValueError("group-column does not fit 12 bits")
        idx = ((gcol << 4).astype(np.uint16) | is_head).astype("<u2")
        idx_off = sz_off + LANES * 4
        idx_view = blocks[:, idx_off:idx_off + LANES * 2].reshape(nblocks, LANES, 2)
        idx_view[block, lane, :] = idx.view(np.uint8).reshape(nnzg, 2)
        # rank_base: heads strictly before the worker's first stream position, minus one
        first_pos = LANES * b_w
        wave_info[:, 0] = np.searchsorted(head_pos, first_pos, side="left") - 1
        # tail_closed: does the row that is open at the end of the run stop there?
        end_pos = LANES * (b_w + n_w)
        head_set = np.zeros(nblocks * LANES + 1, dtype=bool)
        head_set[head_pos] = True
        wave_info[:, 1] = np.where(end_pos >= nnzg, 1, head_set[np.minimum(end_pos, nblocks * LANES)])
        # carry chains: which worker owns a given block
        owner = np.repeat(np.arange(n_waves), n_w)
        for w in range(n_waves):
            f = int(first_pos[w])
            e = int(end_pos[w])
            if f < nnzg and not head_set[f]:
                row_head = int(head_pos[np.searchsorted(head_pos, f, side="right") - 1])
                wave_info[w, 2] = owner[row_head // LANES]
            heads_inside = (np.searchsorted(head_pos, min(e, nnzg), side="left") -
                            np.searchsorted(head_pos, f, side="left"))
            if n_w[w] > 0 and wave_info[w, 1] == 0 and heads_inside > 0:
                nxt = int(np.searchsorted(head_pos, e, side="left"))
                row_last = (int(head_pos[nxt]) if nxt < len(head_pos) else nnzg) - 1
                wave_info[w, 3] = owner[row_last // LANES] - w + 1
        for w in range(n_waves):
            if wave_info[w, 2] >= 0:
                wave_info[w, 1] += 2 * wave_info[wave_info[w, 2], 3]

    parts = [blocks.tobytes(), wave_info.astype("<i4").tobytes(),
             nonempty.astype("<i4").tobytes(), empty.astype("<i4").tobytes()]
    out = bytearray()
    for part in parts:
        out += part
        out += b"\0" * (_align(len(out)) - len(out))
    if len(out) == 0:
        out += b"\0" * ALIGN
    return bytes(out)
