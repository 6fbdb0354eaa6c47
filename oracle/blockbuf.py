"""Block buffers and Blockwise Copy, written out as plain loops.
Test infrastructure (numpy only, nothing shared with the HIP path).

Definitions followed:
  * Sec. 5 "Block buffers": all data blocks of one type live in one contiguous buffer; a block is
    identified by its index (slot) in that buffer.  Here a slot holds `block_size` rows, a row
    being one token's [heads, D] slab; a block shorter than block_size (the last block of a
    sequence) uses the first rows of its slot.
  * Sec. 5 "Blockwise Copy": several data blocks are copied inside one device's memory in one
    operation.  An entry (src_row, dst_row, n_rows) moves n_rows consecutive rows.
  * Sec. 5 "Blockwise Attention" with block tables: attention over blocks addressed through the
    buffer (start address + per-block offset) gives what attention over the packed tensors
    gives; `gather_blocks` / `scatter_blocks` are that change of addressing and nothing else.
"""
import numpy as np


def blockwise_copy(src, dst, entries):
    """dst[dst_row + r] = src[src_row + r] for every entry (src_row, dst_row, n_rows), r < n_rows.
    src, dst: arrays whose first axis is the row.  Entries are applied in order; destination ranges
    are expected to be disjoint, so the order does not matter.  Returns dst (modified in place)."""
    for s, d, n in np.asarray(entries, dtype=np.int64).reshape(-1, 3):
        for r in range(int(n)):
            dst[d + r] = src[s + r]
    return dst


def copy_entries_for_blocks(blk_start, blk_len, slots, block_size, to_buffer=True):
    """Copy list that moves every block b between the packed layout (rows blk_start[b] ..) and
    slot slots[b] of a block buffer (rows slots[b] * block_size ..).  slots[b] < 0: block absent."""
    out = []
    for b in range(len(blk_start)):
        if slots[b] < 0:
            continue
        packed, buf = int(blk_start[b]), int(slots[b]) * int(block_size)
        out.append((packed, buf, int(blk_len[b])) if to_buffer else (buf, packed, int(blk_len[b])))
    return np.asarray(out, dtype=np.int32).reshape(-1, 3)


def gather_blocks(x, blk_start, blk_len, slots, n_slots, block_size, fill=0):
    """Packed [T, ...] -> block buffer [n_slots * block_size, ...]; rows no block uses hold `fill`."""
    buf = np.full((n_slots * block_size,) + x.shape[1:], fill, dtype=x.dtype)
    for b in range(len(blk_start)):
        if slots[b] < 0:
            continue
        for r in range(int(blk_len[b])):
            buf[slots[b] * block_size + r] = x[blk_start[b] + r]
    return buf


def scatter_blocks(buf, blk_start, blk_len, slots, block_size, total_tokens):
    """Block buffer -> packed [T, ...] (the inverse of gather_blocks on the rows blocks use)."""
    x = np.zeros((total_tokens,) + buf.shape[1:], dtype=buf.dtype)
    for b in range(len(blk_start)):
        if slots[b] < 0:
            continue
        for r in range(int(blk_len[b])):
            x[blk_start[b] + r] = buf[slots[b] * block_size + r]
    return x


def gather_rows_hT(x_hT, blk_start, blk_len, slots, n_slots, block_size, fill=0.0):
    """[H, T] per-token scalars (LSE, delta) -> [H, n_slots * block_size] in buffer row order."""
    return np.ascontiguousarray(gather_blocks(np.ascontiguousarray(x_hT.T), blk_start, blk_len, slots, n_slots, block_size, fill).T)


def scatter_rows_hT(buf_hR, blk_start, blk_len, slots, block_size, total_tokens):
    return np.ascontiguousarray(scatter_blocks(np.ascontiguousarray(buf_hR.T), blk_start, blk_len, slots, block_size, total_tokens).T)
