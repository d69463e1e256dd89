"""Device byte layout of a packed GQSA matrix, re-derived from its written
specification -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.

The layout is a pure permutation/padding of the canonical BSR arrays of the
paper's Sec. 3.2 listing (rowIndex / groups / values) and the per-group scale
and zero of Eq. 1; it adds no arithmetic.  The specification, restated:

 1. Stream.  The stored groups in canonical order g = 0..nnzg-1 form a stream.
    LN consecutive positions make a block, U consecutive blocks a tile.  By
    default LN = 64 (one position per lane of a wavefront) and U = 4 for up to
    16 code bytes per group (G*bits/8), 2 for 32, 1 for 64; a partition may name
    another tile shape (tile_blocks = U, tile_lanes = LN <= 64).
    Plain form (span_tiles = 0): group g sits at position g; the stream is
    padded with null groups (all bytes zero) to whole tiles:
    ntiles = ceil(nnzg / (LN U)), nblocks = U * ntiles.
    Aligned form (span_tiles = s > 0): spans of S = LN U s positions.  The rows
    are placed in order from position 0; a row with c groups, 0 < c <= S, that
    does not fit what is left of the current span ((pos mod S) + c > S) starts at
    the next multiple of S; every other row starts where the previous one ended.
    Positions without a stored group hold null groups.  There is one span per
    workgroup (nspans = n_workgroups) or, if span_per_worker, one per worker
    (nspans = n_workgroups * waves_per_workgroup); nspans must be at least the
    number of spans the rows reach into; ntiles = s * nspans.
    Below, "past the last group" means at or beyond L = one past the last stored
    group's position (L = nnzg in the plain form), and a null group before L
    counts as part of the row before it.
 2. Partition.  The tiles are dealt to the n_waves = n_workgroups *
    waves_per_workgroup workers in contiguous runs: worker w gets the tiles
    floor(w * ntiles / n_waves) .. floor((w+1) * ntiles / n_waves) - 1.
    b_w = first block of worker w = U * floor(w * ntiles / n_waves).  (The
    grouping of the workers into workgroups does not enter the layout.)
 3. Tiles.  A tile starting at block b covers stream positions
    LN b .. LN (b+U) - 1; the position LN b + p lives in block b + (p mod U),
    lane p div U.
 4. Block.  Each block is (G*bits/8 + 6)*LN bytes: the code planes, then
    LN x uint32 (fp16 scale bits | fp16 zero bits << 16), then LN x uint16
    index words.  G = 16*M with M in {1, 2, 4, 8}, or G = 8.  The index word is
    (group-column * M) << 4 -- sixteen times the number of the 16-element slot
    of K at which the group starts (slots are below 4096) -- plus 1 if the
    group is the first stored group of its row; for G = 8 it is group-column
    << 4 (the number of the 8-element half-slot, below 4096) plus that flag.
    Codes.  A lane's code string has G*bits/8 bytes.  4-bit codes: it is a
    sequence of little-endian uint32, word h holding elements 8h..8h+7 of the
    group, element 8h+2m in bits 4m..4m+3 and element 8h+2m+1 in bits
    16+4m..16+4m+3 (m = 0..3).  8-bit codes: byte j is element j.  The string
    is stored in planes: with P = min(16, G*bits/8) bytes per lane and plane,
    plane k (LN*P bytes, lanes in order) holds bytes k*P .. k*P+P-1 of every
    lane's string; the planes follow each other.
 5. Side tables (int32): wave_info[n_waves][4] = {rank_base, tail_closed +
    2 * lead_len, lead_first, chain_len} with
      rank_base   = (number of row-head groups at stream positions before
                    worker w's first position) - 1;
      tail_closed = 1 if the first position after the worker's run is at or
                    beyond L or holds a row-head group, else 0;
      lead_len    = chain_len of worker lead_first (below), 0 if lead_first = -1;
      lead_first  = for a worker (with or without blocks) whose first position
                    b_w*LN is before L and does not hold a row head: the
                    worker that owns the head group of that group's row; else -1;
      chain_len   = for a worker with blocks, tail_closed = 0 and at least one
                    row head inside its run: (worker owning the last position
                    before the next row head -- or before L -- after its run) - w + 1;
                    else 0;
    row_of_rank[r] = index of the r-th non-empty row; empty_rows = indices of
    the empty rows.
 6. Blob = blocks, wave_info, row_of_rank, empty_rows, each region starting
    at a multiple of 256 bytes, zero padded, total a multiple of 256 (>= 256).

Second image (panel_blob; G >= 16), for calls with many activation rows --
again a pure reordering of the canonical arrays:
 P1. Panels of 16 consecutive rows (P = ceil(N/16); rows >= N have no groups)
     and slices of 32 consecutive group-columns (S = ceil(K/G/32); columns
     >= K/G have no groups).  Block (p, s) holds the stored groups of panel p
     whose group-column lies in slice s, ordered by (group-column, row).
 P2. Header of block (p, s): 36 x uint32 at byte 144 (p S + s) of the image.
     Word j < 32, for group-column 32 s + j: bit r (r < 16) set if row 16 p + r
     stores a group in that column; bits 16..31 = number of groups of the block
     in the columns before it.  Word 32 = start of the block's data in 16-byte
     units from the start of the data region; word 33 = number of groups of the
     block; words 34, 35 = 0.  The header region is zero padded to a multiple
     of 256 bytes.
 P3. Data region: the blocks' data follow each other in header order without
     gaps.  A block's data: one record per group, zero padded as a whole to a
     multiple of 16 bytes.  Record = the code bytes of quarters 0 and 1, then
     uint32 fp16 scale bits | fp16 zero bits << 16, then the code bytes of
     quarters 2 and 3 (G*bits/8 + 4 bytes).  Code bytes: quarter t = 0..3 after
     quarter, and inside a quarter chunk i = 0..G/16-1 after chunk, the codes of
     elements 16 i + 4 t .. 16 i + 4 t + 3 (e0..e3): 8-bit codes as four bytes
     in element order; 4-bit codes as the two bytes (e0 | e2 << 4),
     (e1 | e3 << 4).  Exception, 8-bit codes with G = 16: the scale | zero
     word is stored twice, record = quarter 0, word, quarter 1, quarter 2, word,
     quarter 3 (24 bytes).  After the last block 256 zero bytes; the image is
     zero padded to a multiple of 256 bytes.
"""
from __future__ import annotations

import numpy as np

LANES = 64
ALIGN = 256


def default_tile_blocks(code_bytes: int) -> int:
    """U of spec item 1."""
    return 4 if code_bytes <= 16 else (2 if code_bytes <= 32 else 1)


def row_positions(rowIndex, span_groups: int):
    """(first stream position of every row, L) -- spec item 1."""
    ri = np.asarray(rowIndex, dtype=np.int64)
    counts = ri[1:] - ri[:-1]
    if span_groups <= 0:
        return ri[:-1].copy(), int(ri[-1])
    pos = 0
    out = np.zeros(len(counts), dtype=np.int64)
    for n, c in enumerate(counts.tolist()):
        if 0 < c <= span_groups and pos % span_groups + c > span_groups:
            pos = (pos // span_groups + 1) * span_groups
        out[n] = pos
        pos += c
    return out, pos


def worker_block_counts(nblocks: int, n_waves: int, U: int) -> np.ndarray:
    """Blocks owned by every worker (spec item 2)."""
    ntiles = nblocks // U
    first = np.arange(n_waves + 1, dtype=np.int64) * ntiles // n_waves
    return (first[1:] - first[:-1]) * U


def _align(n: int) -> int:
    return (n + ALIGN - 1) // ALIGN * ALIGN


def stream_placement(nblocks: int, n_waves: int, U: int, LN: int = LANES):
    """For every stream position: (block, lane) it is stored at (spec items 2-3)."""
    n_w = worker_block_counts(nblocks, n_waves, U)
    b_w = np.concatenate(([0], np.cumsum(n_w)[:-1]))
    pos = np.arange(nblocks * LN, dtype=np.int64)
    tile = pos // (LN * U)
    p = pos % (LN * U)
    block = tile * U + (p % U)
    lane = p // U
    return block, lane, b_w, n_w


def device_blob(c, n_workgroups: int, waves_per_workgroup: int, span_tiles: int = 0, tile_blocks: int = 0,
                tile_lanes: int = LANES, span_per_worker: bool = False) -> bytes:
    """Exact bytes the library must hold on the device for canonical arrays `c`."""
    if c.G not in (8, 16, 32, 64, 128) or c.bits not in (4, 8) or c.G * c.bits // 8 > 64:
        raise ValueError("device layout is specified for G in {8,16,32,64,128}, bits in {4,8}, at most 64 code bytes")
    nnzg = c.nnzg
    code_bytes = c.G * c.bits // 8
    U = tile_blocks or default_tile_blocks(code_bytes)
    LN = tile_lanes or LANES
    if not (1 <= LN <= LANES):
        raise ValueError("a block has 1..64 positions")
    blk_bytes = (code_bytes + 6) * LN
    slots_per_group = max(1, c.G // 16)

    ri = np.asarray(c.rowIndex, dtype=np.int64)
    counts = ri[1:] - ri[:-1]
    nonempty = np.nonzero(counts > 0)[0].astype(np.int32)
    empty = np.nonzero(counts == 0)[0].astype(np.int32)
    row_pos, L = row_positions(ri, span_tiles * LN * U)
    if span_tiles > 0:
        nspans = n_workgroups * (waves_per_workgroup if span_per_worker else 1)
        if -(-L // (span_tiles * LN * U)) > nspans:
            raise ValueError("the rows reach into more spans than there are")
        nblocks = U * span_tiles * nspans
    else:
        if span_per_worker:
            raise ValueError("spans per worker need span_tiles > 0")
        nblocks = U * (-(-L // (LN * U)))
    head_pos = row_pos[counts > 0]                 # stream position of each row's first group
    # stream position of every stored group
    group_pos = np.arange(nnzg, dtype=np.int64) + np.repeat(row_pos - ri[:-1], counts)

    n_waves = n_workgroups * waves_per_workgroup
    blocks = np.zeros((nblocks, blk_bytes), dtype=np.uint8)
    wave_info = np.zeros((n_waves, 4), dtype=np.int32)
    wave_info[:, 0] = -1
    wave_info[:, 1] = 1
    wave_info[:, 2] = -1
    if nblocks > 0:
        block, lane, b_w, n_w = stream_placement(nblocks, n_waves, U, LN)
        block = block[group_pos]
        lane = lane[group_pos]
        # codes
        vals = np.asarray(c.values, dtype=np.uint8).reshape(nnzg, code_bytes)
        if c.bits == 4:
            elems = np.empty((nnzg, c.G), dtype=np.uint32)
            elems[:, 0::2] = vals & 0xF
            elems[:, 1::2] = vals >> 4
            words = np.zeros((nnzg, code_bytes // 4), dtype=np.uint32)
            for h in range(code_bytes // 4):
                for m in range(4):
                    words[:, h] |= elems[:, 8 * h + 2 * m] << np.uint32(4 * m)
                    words[:, h] |= elems[:, 8 * h + 2 * m + 1] << np.uint32(16 + 4 * m)
            lane_bytes = words.astype("<u4").view(np.uint8).reshape(nnzg, code_bytes)
        else:
            lane_bytes = vals
        plane = min(16, code_bytes)
        for k in range(code_bytes // plane):
            plane_view = blocks[:, k * LN * plane:(k + 1) * LN * plane].reshape(nblocks, LN, plane)
            plane_view[block, lane, :] = lane_bytes[:, k * plane:(k + 1) * plane]
        # scale | zero << 16
        sz = (np.asarray(c.scales, dtype=np.uint32) |
              (np.asarray(c.zeros, dtype=np.uint32) << np.uint32(16))).astype("<u4")
        sz_off = LN * code_bytes
        sz_view = blocks[:, sz_off:sz_off + LN * 4].reshape(nblocks, LN, 4)
        sz_view[block, lane, :] = sz.view(np.uint8).reshape(nnzg, 4)
        # group-column | head flag
        is_head = np.zeros(nnzg, dtype=np.uint16)
        is_head[ri[:-1][counts > 0]] = 1
        gcol = np.asarray(c.groups, dtype=np.int64)
        if gcol.size and gcol.max() * slots_per_group + slots_per_group - 1 >= 4096:
            raise ValueError("slot number does not fit 12 bits")
        idx = (((gcol * slots_per_group) << 4).astype(np.uint16) | is_head).astype("<u2")
        idx_off = sz_off + LN * 4
        idx_view = blocks[:, idx_off:idx_off + LN * 2].reshape(nblocks, LN, 2)
        idx_view[block, lane, :] = idx.view(np.uint8).reshape(nnzg, 2)
        # rank_base: heads strictly before the worker's first stream position, minus one
        first_pos = LN * b_w
        wave_info[:, 0] = np.searchsorted(head_pos, first_pos, side="left") - 1
        # tail_closed: does the row that is open at the end of the run stop there?
        end_pos = LN * (b_w + n_w)
        head_set = np.zeros(max(nblocks * LN, L) + 1, dtype=bool)
        head_set[head_pos] = True
        wave_info[:, 1] = np.where(end_pos >= L, 1, head_set[np.minimum(end_pos, nblocks * LN)])
        # carry chains: which worker owns a given block
        owner = np.repeat(np.arange(n_waves), n_w)
        for w in range(n_waves):
            f = int(first_pos[w])
            e = int(end_pos[w])
            if f < L and not head_set[f]:
                row_head = int(head_pos[np.searchsorted(head_pos, f, side="right") - 1])
                wave_info[w, 2] = owner[row_head // LN]
            heads_inside = (np.searchsorted(head_pos, min(e, L), side="left") -
                            np.searchsorted(head_pos, f, side="left"))
            if n_w[w] > 0 and wave_info[w, 1] == 0 and heads_inside > 0:
                nxt = int(np.searchsorted(head_pos, e, side="left"))
                row_last = (int(head_pos[nxt]) if nxt < len(head_pos) else L) - 1
                wave_info[w, 3] = owner[row_last // LN] - w + 1
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


def device_blob_for(c, partition: dict) -> bytes:
    """device_blob for a partition given by name (the keys n_workgroups, waves_per_workgroup, span_tiles,
    tile_blocks, tile_lanes, span_per_worker; other keys are ignored)."""
    return device_blob(c, partition["n_workgroups"], partition["waves_per_workgroup"], partition["span_tiles"],
                       partition["tile_blocks"], partition["tile_lanes"], bool(partition["span_per_worker"]))


def panel_blob(c) -> bytes:
    """Exact bytes of the second (panel) image for canonical arrays `c` (spec items P1-P3)."""
    if c.G not in (16, 32, 64, 128) or c.bits not in (4, 8) or c.G * c.bits // 8 > 64:
        raise ValueError("the panel image is specified for G in {16,32,64,128}, bits in {4,8}, at most 64 code bytes")
    cb = c.G * c.bits // 8
    ri = np.asarray(c.rowIndex, dtype=np.int64)
    gcol = np.asarray(c.groups, dtype=np.int64)
    nnzg = c.nnzg
    P = -(-c.N // 16)
    S = -(-(c.K // c.G) // 32)
    row = np.repeat(np.arange(c.N, dtype=np.int64), ri[1:] - ri[:-1])
    blk = (row // 16) * S + gcol // 32
    # order inside the image: block, then group-column, then row
    order = np.lexsort((row, gcol, blk))
    counts = np.bincount(blk, minlength=P * S).astype(np.int64)
    pad16 = lambda v: (v + 15) // 16 * 16
    twice = c.bits == 8 and c.G == 16
    rb = cb + (8 if twice else 4)
    sizes = pad16(counts * rb)
    starts = np.concatenate(([0], np.cumsum(sizes)))
    header_bytes = _align(P * S * 144)
    total = _align(header_bytes + int(starts[-1]) + 256)
    img = np.zeros(total, dtype=np.uint8)
    # every group's codes as elements, then as the record's code bytes
    vals = np.asarray(c.values, dtype=np.uint8).reshape(nnzg, cb)
    if c.bits == 4:
        elems = np.empty((nnzg, c.G), dtype=np.uint8)
        elems[:, 0::2] = vals & 0xF
        elems[:, 1::2] = vals >> 4
    else:
        elems = vals
    chunks = c.G // 16
    e4 = elems.reshape(nnzg, chunks, 4, 4)                      # [group][chunk i][quarter t][e0..e3]
    e4 = e4.transpose(0, 2, 1, 3)                               # [group][quarter t][chunk i][e0..e3]
    if c.bits == 4:
        stored = np.empty((nnzg, 4, chunks, 2), dtype=np.uint8)
        stored[..., 0] = e4[..., 0] | (e4[..., 2] << 4)
        stored[..., 1] = e4[..., 1] | (e4[..., 3] << 4)
    else:
        stored = e4
    stored = np.ascontiguousarray(stored).reshape(nnzg, cb)
    sz = (np.asarray(c.scales, dtype=np.uint32) | (np.asarray(c.zeros, dtype=np.uint32) << np.uint32(16))).astype("<u4")
    szb = sz.view(np.uint8).reshape(nnzg, 4)
    if twice:
        records = np.concatenate([stored[:, 0:4], szb, stored[:, 4:8], stored[:, 8:12], szb, stored[:, 12:16]], axis=1)
    else:
        records = np.concatenate([stored[:, :cb // 2], szb, stored[:, cb // 2:]], axis=1)                 # [group][rb]
    first = np.concatenate(([0], np.cumsum(counts)))          # index into `order` of each block's first group
    for b in range(P * S):
        k = int(counts[b])
        g = order[first[b]:first[b] + k]
        header = np.zeros(36, dtype=np.uint32)
        cols = gcol[g] - (b % S) * 32
        rows = row[g] - (b // S) * 16
        before = 0
        for j in range(32):
            here = rows[cols == j]
            mask = 0
            for r in here.tolist():
                mask |= 1 << r
            header[j] = mask | (before << 16)
            before += len(here)
        header[32] = starts[b] // 16
        header[33] = k
        img[b * 144:(b + 1) * 144] = header.astype("<u4").view(np.uint8)
        if k:
            base = header_bytes + int(starts[b])
            img[base:base + k * rb] = records[g].reshape(-1)
    return img.tobytes()
