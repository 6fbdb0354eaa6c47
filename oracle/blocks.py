"""Integer reference for block generation and block-table handling (Sec. 4.1 "Block
Generation"; Sec. 5 "Blockwise Attention": a list of (query, key-value, output) tuples
addressed through block tables).  Test infrastructure, fp-free, numpy + plain loops.

Block numbering: sequence s of length L_s is cut into ceil(L_s / B) data blocks, the last
one possibly short; blocks never straddle sequences (the paper partitions "each sequence");
global block id = blocks of earlier sequences + index within the sequence.
"""
import numpy as np

MASK_NONE, MASK_CAUSAL, MASK_RANGES, MASK_SKIP, MASK_WINDOW = 0, 1, 2, 3, 4


def block_partition(cu_seqlens, B):
    """Returns dict with int64 arrays: seq_first_blk[n_seq+1], blk_seq[n_blk],
    blk_start[n_blk], blk_end[n_blk] (packed token range of each block)."""
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    first = [0]
    blk_seq, blk_start, blk_end = [], [], []
    for s in range(len(cu) - 1):
        L = int(cu[s + 1] - cu[s])
        nb = -(-L // B)
        for i in range(nb):
            blk_seq.append(s)
            blk_start.append(int(cu[s]) + i * B)
            blk_end.append(min(int(cu[s]) + (i + 1) * B, int(cu[s + 1])))
        first.append(first[-1] + nb)
    return dict(seq_first_blk=np.asarray(first, np.int64), blk_seq=np.asarray(blk_seq, np.int64),
                blk_start=np.asarray(blk_start, np.int64), blk_end=np.asarray(blk_end, np.int64))


def table_from_mask(mask_rows, cu_seqlens, B, other_kind=MASK_RANGES):
    """Block generation (Sec. 4.1): a computation block (Q_i, KV_j) exists iff the mask tile
    M[rows of Q_i, cols of KV_j] is not all zeros.  `mask_rows(s, L, r0, r1)` returns the dense
    bool rows of sequence s.  Classification of a tile: all ones -> NONE; equal to the causal
    predicate (col <= row) on the tile -> CAUSAL; otherwise `other_kind`: RANGES (the per-token
    range arrays describe the tile) or, for a table made from a window / sink specification,
    WINDOW.  Rows are emitted in ascending (q_blk, kv_blk) order.  int32[n, 3]."""
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    part = block_partition(cu, B)
    rows = []
    for s in range(len(cu) - 1):
        L = int(cu[s + 1] - cu[s])
        nb = -(-L // B)
        g0 = int(part["seq_first_blk"][s])
        for i in range(nb):
            r0, r1 = i * B, min((i + 1) * B, L)
            M = mask_rows(s, L, r0, r1)
            ii = np.arange(r0, r1)[:, None]
            for j in range(nb):
                c0, c1 = j * B, min((j + 1) * B, L)
                tile = M[:, c0:c1]
                if not tile.any():
                    continue
                if tile.all():
                    kind = MASK_NONE
                elif np.array_equal(tile, np.arange(c0, c1)[None, :] <= ii):
                    kind = MASK_CAUSAL
                else:
                    kind = other_kind
                rows.append((g0 + i, g0 + j, kind))
    return np.asarray(rows, dtype=np.int32).reshape(-1, 3)


def dense_causal_table(cu_seqlens, B):
    """Every same-sequence (q_blk, kv_blk) pair, all tagged CAUSAL (config 1's table)."""
    part = block_partition(cu_seqlens, B)
    f = part["seq_first_blk"]
    rows = [(i, j, MASK_CAUSAL) for s in range(len(f) - 1) for i in range(f[s], f[s + 1])
            for j in range(f[s], f[s + 1])]
    return np.asarray(rows, dtype=np.int32).reshape(-1, 3)


class Visibility:
    """The mask a block table *defines*: key j is visible to query i iff some listed entry
    (q_blk, kv_blk, kind) covers (i, j) and its predicate holds:
      NONE always; CAUSAL j <= i; RANGES packed index of j in [r0,r1) or [r2,r3) of row i;
      WINDOW (sliding window with attention sink, Sec. 2.4 "Lambda"; parameters window W and
      sink, one pair for the whole table) j <= i and (i - j < W or j is one of the first `sink`
      tokens of the sequence);
      SKIP never.  Unlisted pairs are invisible."""

    def __init__(self, cu_seqlens, B, table, ranges=None, select=None, window=None):
        self.cu = np.asarray(cu_seqlens, dtype=np.int64)
        self.B = int(B)
        self.part = block_partition(self.cu, B)
        t = np.asarray(table, dtype=np.int64).reshape(-1, 3)
        if select is not None:
            t = t[np.asarray(select)]
        self.table = t
        self.ranges = None if ranges is None else np.asarray(ranges, dtype=np.int64)
        self.window = None if window is None else (int(window[0]), int(window[1]))   # (W, sink)
        self.by_q = {}
        for e in range(len(t)):
            self.by_q.setdefault(int(t[e, 0]), []).append(e)

    def rows(self, s, r0, r1):
        """bool[r1 - r0, L_s]: visibility of in-sequence query rows [r0, r1) of sequence s."""
        cu, B, p = self.cu, self.B, self.part
        L = int(cu[s + 1] - cu[s])
        M = np.zeros((r1 - r0, L), dtype=bool)
        g0 = int(p["seq_first_blk"][s])
        base = int(cu[s])
        for bi in range(r0 // B, -(-r1 // B)):
            qb = g0 + bi
            a0, a1 = max(r0, bi * B), min(r1, (bi + 1) * B, L)
            if a1 <= a0:
                continue
            i_pack = base + np.arange(a0, a1, dtype=np.int64)[:, None]
            for e in self.by_q.get(qb, []):
                kb, kind = int(self.table[e, 1]), int(self.table[e, 2])
                if kind == MASK_SKIP:
                    continue
                assert int(p["blk_seq"][kb]) == s, "entry joins blocks of different sequences"
                c0, c1 = int(p["blk_start"][kb]), int(p["blk_end"][kb])
                j_pack = np.arange(c0, c1, dtype=np.int64)[None, :]
                if kind == MASK_NONE:
                    vis = np.ones((a1 - a0, c1 - c0), dtype=bool)
                elif kind == MASK_CAUSAL:
                    vis = j_pack <= i_pack
                elif kind == MASK_RANGES:
                    r = self.ranges[base + a0: base + a1]
                    vis = ((j_pack >= r[:, 0:1]) & (j_pack < r[:, 1:2])) | \
                          ((j_pack >= r[:, 2:3]) & (j_pack < r[:, 3:4]))
                elif kind == MASK_WINDOW:
                    W, sink = self.window
                    vis = (j_pack <= i_pack) & ((i_pack - j_pack < W) | (j_pack - base < sink))
                else:
                    raise ValueError(f"bad mask kind {kind}")
                M[a0 - r0: a1 - r0, c0 - base: c1 - base] |= vis
        return M

    def pair_counts(self):
        """Visible (query, key) pairs of each table entry taken alone, int64[n]."""
        p = self.part
        out = np.zeros(len(self.table), dtype=np.int64)
        for e in range(len(self.table)):
            qb, kb, kind = (int(x) for x in self.table[e])
            if kind == MASK_SKIP:
                continue
            q0, q1 = int(p["blk_start"][qb]), int(p["blk_end"][qb])
            c0, c1 = int(p["blk_start"][kb]), int(p["blk_end"][kb])
            i = np.arange(q0, q1, dtype=np.int64)
            if kind == MASK_NONE:
                out[e] = (q1 - q0) * (c1 - c0)
            elif kind == MASK_CAUSAL:
                out[e] = int(np.clip(i + 1 - c0, 0, c1 - c0).sum())
            elif kind == MASK_WINDOW:
                W, sink = self.window
                base = int(self.cu[int(p["blk_seq"][qb])])
                n = 0
                for q in range(q0, q1):                      # plain count, key by key
                    for k in range(c0, c1):
                        n += int(k <= q and (q - k < W or k - base < sink))
                out[e] = n
            else:
                r = self.ranges[q0:q1]
                j = np.arange(c0, c1, dtype=np.int64)[None, :]
                vis = ((j >= r[:, 0:1]) & (j < r[:, 1:2])) | ((j >= r[:, 2:3]) & (j < r[:, 3:4]))
                out[e] = int(vis.sum())
        return out


def group_entries(table, key_col, n_groups, group_of=None):
    """CSR grouping of the non-SKIP table rows: ptr int64[n_groups+1], idx int64[nnz] holding
    original row numbers, grouped by `group_of[row]` (default: table[row, key_col]) and, inside a
    group, ascending by the other block index, ties kept in table order (stable)."""
    t = np.asarray(table, dtype=np.int64).reshape(-1, 3)
    other = 1 - key_col
    keep = [e for e in range(len(t)) if t[e, 2] != MASK_SKIP]
    g = (lambda e: int(t[e, key_col])) if group_of is None else (lambda e: int(group_of[e]))
    keep.sort(key=lambda e: (g(e), int(t[e, other])))   # python sort is stable
    ptr = np.zeros(n_groups + 1, dtype=np.int64)
    for e in keep:
        ptr[g(e) + 1] += 1
    ptr = np.cumsum(ptr)
    return ptr, np.asarray(keep, dtype=np.int64)
