"""Seeded synthetic inputs for the block-attention hot path.

This module only *draws inputs*: sequence lengths, packed q/k/v/dO tensors, per-token
attention ranges for the paper's mask families (Sec. 7.1 "Attention Masks"), and the
seeded assignment of computation blocks to a device share / divisions (Sec. 4.3, T = 4).
It holds none of the attention arithmetic and none of the block-table logic, so both the
HIP path and the CPU oracle can consume its output without sharing method code.

The paper's datasets (LongDataCollections, LongAlign) are not reproduced; length
distributions below are synthetic stand-ins with the same long-tailed shape.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import numpy as np

# mask_kind codes of the block table (a row is q_blk, kv_blk, mask_kind)
MASK_NONE, MASK_CAUSAL, MASK_RANGES, MASK_SKIP, MASK_WINDOW = 0, 1, 2, 3, 4


@dataclass(frozen=True)
class MaskSpec:
    """A mask family and its parameters (Sec. 2.4 and Sec. 7.1 "Attention Masks").

    kind: "causal" | "window" | "lambda" | "causal_blockwise" | "shared_question"
    window: number of keys a query sees including itself (window / lambda), or the number
            of mask blocks (causal_blockwise)
    sink:   number of sink tokens (lambda) or sink mask blocks (causal_blockwise)
    mblock: token size of a mask block (causal_blockwise)
    n_answers / frac: shared_question layout: one question of (1 - n_answers*frac) of the
            sequence followed by n_answers answers of frac each
    """
    kind: str = "causal"
    window: int = 0
    sink: int = 0
    mblock: int = 256
    n_answers: int = 4
    frac: float = 0.2


def shared_question_bounds(L: int, n_answers: int, frac: float) -> List[int]:
    """Token boundaries [0, q_end, a1_end, ..., L] of a shared-question sequence."""
    a = int(math.floor(L * frac))
    q_end = L - n_answers * a
    return [0, q_end] + [q_end + (i + 1) * a for i in range(n_answers)]


def attn_ranges(spec: MaskSpec, cu_seqlens: np.ndarray) -> np.ndarray:
    """Per-token visible key ranges, int32[T, 4] = [lo1, hi1, lo2, hi2), half-open, in
    packed token coordinates (at most two ranges per token, Sec. 5 "Blockwise Attention").
    An empty range is [0, 0)."""
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    T = int(cu[-1])
    r = np.zeros((T, 4), dtype=np.int64)
    for s in range(len(cu) - 1):
        b, e = int(cu[s]), int(cu[s + 1])
        L = e - b
        i = np.arange(L, dtype=np.int64)
        if spec.kind == "causal":
            lo1, hi1 = np.zeros(L, np.int64), i + 1
            lo2 = hi2 = np.zeros(L, np.int64)
        elif spec.kind == "window":
            lo1, hi1 = np.maximum(i - spec.window + 1, 0), i + 1
            lo2 = hi2 = np.zeros(L, np.int64)
        elif spec.kind == "lambda":
            lo2, hi2 = np.maximum(i - spec.window + 1, 0), i + 1
            lo1, hi1 = np.zeros(L, np.int64), np.minimum(spec.sink, lo2)
        elif spec.kind == "causal_blockwise":
            mb = i // spec.mblock
            last = (L - 1) // spec.mblock
            lo2 = np.maximum(mb - spec.window + 1, 0) * spec.mblock
            lo2 = np.where(mb == last, 0, lo2)
            hi2 = i + 1
            lo1, hi1 = np.zeros(L, np.int64), np.minimum(spec.sink * spec.mblock, lo2)
        elif spec.kind == "shared_question":
            bd = shared_question_bounds(L, spec.n_answers, spec.frac)
            seg = np.searchsorted(np.asarray(bd[1:], dtype=np.int64), i, side="right")
            seg_start = np.asarray(bd, dtype=np.int64)[seg]
            lo2, hi2 = seg_start, i + 1
            lo1 = np.zeros(L, np.int64)
            hi1 = np.where(seg == 0, 0, bd[1])
        else:
            raise ValueError(f"unknown mask kind {spec.kind!r}")
        empty1 = hi1 <= lo1
        lo1 = np.where(empty1, -b, lo1)
        hi1 = np.where(empty1, -b, hi1)
        empty2 = hi2 <= lo2
        lo2 = np.where(empty2, -b, lo2)
        hi2 = np.where(empty2, -b, hi2)
        r[b:e, 0], r[b:e, 1], r[b:e, 2], r[b:e, 3] = lo1 + b, hi1 + b, lo2 + b, hi2 + b
    return r.astype(np.int32)


def draw_lengths(total: int, dist: str, lo: int, hi: int, seed: int, median: int = 0,
                 sigma: float = 1.0) -> np.ndarray:
    """Packed-batch sequence lengths: draw, round, clip to [lo, hi], append while the sum
    fits in `total`; the remainder becomes a final sequence if it is >= lo, else it is
    added to the shortest sequence.  Lengths are not rounded to the block size."""
    rng = np.random.default_rng(seed)
    lens: List[int] = []
    while True:
        if dist == "lognormal":
            x = rng.lognormal(mean=math.log(median), sigma=sigma)
        elif dist == "uniform":
            x = rng.integers(lo, hi + 1)
        else:
            raise ValueError(dist)
        n = int(min(max(int(round(float(x))), lo), hi))
        if sum(lens) + n > total:
            break
        lens.append(n)
    rem = total - sum(lens)
    if rem > 0:
        if rem >= lo or not lens:
            lens.append(rem)
        else:
            lens[int(np.argmin(lens))] += rem
    return np.asarray(lens, dtype=np.int32)


def cu_from_lengths(lens) -> np.ndarray:
    cu = np.zeros(len(lens) + 1, dtype=np.int32)
    cu[1:] = np.cumsum(np.asarray(lens, dtype=np.int64))
    return cu


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest even), returned as uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to fp64."""
    u = b.astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


@dataclass
class Workload:
    name: str
    cu_seqlens: np.ndarray          # int32[n_seq + 1]
    block_size: int
    hq: int
    hkv: int
    d: int
    dtype: str                      # "bf16" | "f32"
    mask: MaskSpec
    tensor_seed: int
    input_scale: float              # q/k/v are N(0,1) * input_scale; dO is N(0,1)
    dense_causal_table: bool = False  # config 1: list all same-sequence pairs, all CAUSAL
    share: Optional[Tuple[int, int, int, int]] = None  # (n_shares, share_seed, n_div, div_seed)
    softmax_scale: float = 0.0
    ranges: np.ndarray = field(default=None, repr=False)

    @property
    def total_tokens(self) -> int:
        return int(self.cu_seqlens[-1])


def make_workload(cfg: int, tokens: Optional[int] = None) -> Workload:
    """The five benchmark configurations, plus the two remaining mask families of the paper (6, 7) at the
    shapes of configs 3 / 4.  `tokens` shrinks the packed batch (same
    distribution, same seeds) for parity cases the CPU oracle can finish."""
    if cfg == 1:
        w = Workload("tiny_causal_f32", cu_from_lengths([128, 384]), 64, 1, 1, 64, "f32",
                     MaskSpec("causal"), 0, 1.0, dense_causal_table=True)
    elif cfg == 2:
        T = tokens or 65536
        lens = draw_lengths(T, "lognormal", 512, 32768, seed=2, median=2048)
        w = Workload("causal_varlen_bf16", cu_from_lengths(lens), 1024, 32, 8, 128, "bf16",
                     MaskSpec("causal"), 102, 1.0 / math.sqrt(128))
    elif cfg == 3:
        T = tokens or 131072
        lens = draw_lengths(T, "uniform", 8192, 65536, seed=3)
        w = Workload("sliding_window_bf16", cu_from_lengths(lens), 1024, 32, 8, 128, "bf16",
                     MaskSpec("window", window=4096), 103, 1.0 / math.sqrt(128))
    elif cfg == 4:
        T = tokens or 131072
        w = Workload("lambda_bf16", cu_from_lengths([T // 4] * 4), 512, 32, 8, 128, "bf16",
                     MaskSpec("lambda", window=8192, sink=64), 104, 1.0 / math.sqrt(128))
    elif cfg == 5:
        T = tokens or 262144
        lens = draw_lengths(T, "lognormal", 1024, 131072, seed=5, median=8192)
        w = Workload("dcp_share_bf16", cu_from_lengths(lens), 2048, 32, 8, 128, "bf16",
                     MaskSpec("causal"), 105, 1.0 / math.sqrt(128), share=(8, 205, 4, 305))
    elif cfg == 6:
        # Sec. 7.1 "Attention Masks", causal blockwise: 256-token mask blocks, a window of 2 blocks, one sink
        # block, the final (test) block attends to everything before it
        T = tokens or 131072
        lens = draw_lengths(T, "uniform", 8192, 65536, seed=6)
        w = Workload("causal_blockwise_bf16", cu_from_lengths(lens), 1024, 32, 8, 128, "bf16",
                     MaskSpec("causal_blockwise", window=2, sink=1, mblock=256), 106, 1.0 / math.sqrt(128))
    elif cfg == 7:
        # Sec. 7.1 "Attention Masks", shared question: one question and 4 answers of 20 % of the sequence each
        T = tokens or 131072
        lens = draw_lengths(T, "lognormal", 1024, 65536, seed=7, median=8192)
        w = Workload("shared_question_bf16", cu_from_lengths(lens), 1024, 32, 8, 128, "bf16",
                     MaskSpec("shared_question", n_answers=4, frac=0.2), 107, 1.0 / math.sqrt(128))
    elif cfg == 8:
        # the longest sequence of the paper's evaluation (maximum sequence length 131 072, Sec. 7.1) as one causal
        # sequence, with a five-token sequence beside it so that the long one ends in a ragged block
        T = tokens or 131072
        w = Workload("one_long_sequence_bf16", cu_from_lengths([T - 5, 5]), 1024, 32, 8, 128, "bf16",
                     MaskSpec("causal"), 108, 1.0 / math.sqrt(128))
    else:
        raise ValueError(f"config {cfg} not in 1..8")
    w.softmax_scale = 1.0 / math.sqrt(w.d)
    w.ranges = attn_ranges(w.mask, w.cu_seqlens)
    return w


def custom_workload(name: str, lens, block_size: int, hq: int, hkv: int, d: int, dtype: str,
                    mask: MaskSpec, seed: int, input_scale: float = 1.0) -> Workload:
    w = Workload(name, cu_from_lengths(lens), block_size, hq, hkv, d, dtype, mask, seed, input_scale)
    w.softmax_scale = 1.0 / math.sqrt(d)
    w.ranges = attn_ranges(mask, w.cu_seqlens)
    return w


def make_tensors(w: Workload, with_dout: bool = True) -> Dict[str, np.ndarray]:
    """q [T,Hq,D], k, v [T,Hkv,D] ~ N(0,1) * input_scale and dout [T,Hq,D] ~ N(0,1), drawn in fp32.
    Tensor number i (q, k, v, dout = 0..3) is cut into chunks of whole token rows (about 2^22
    elements); chunk c is filled from its own generator PCG64(SeedSequence([tensor_seed, i, c])),
    so the result does not depend on how many threads fill the chunks.  For bf16 workloads the
    arrays are uint16 bf16 bit patterns (rounded here, once, so every consumer sees the same bits);
    for f32 they are float32."""
    from concurrent.futures import ThreadPoolExecutor
    T = w.total_tokens
    out = {}
    shapes = [("q", (T, w.hq, w.d), w.input_scale), ("k", (T, w.hkv, w.d), w.input_scale),
              ("v", (T, w.hkv, w.d), w.input_scale)]
    if with_dout:
        shapes.append(("dout", (T, w.hq, w.d), 1.0))
    jobs = []
    for ti, (name, shp, sc) in enumerate(shapes):
        rows = max(1, (1 << 22) // (shp[1] * shp[2]))
        dst = np.empty(shp, dtype=np.uint16 if w.dtype == "bf16" else np.float32)
        out[name] = dst
        for ci, r0 in enumerate(range(0, T, rows)):
            jobs.append((dst, ti, ci, r0, min(T, r0 + rows), shp, sc))

    def fill(job):
        dst, ti, ci, r0, r1, shp, sc = job
        rng = np.random.default_rng([w.tensor_seed, ti, ci])
        x = rng.standard_normal((r1 - r0,) + shp[1:], dtype=np.float32)
        if sc != 1.0:
            x *= np.float32(sc)
        dst[r0:r1] = f32_to_bf16_bits(x) if w.dtype == "bf16" else x

    with ThreadPoolExecutor(max_workers=min(16, max(1, len(jobs)))) as ex:
        list(ex.map(fill, jobs))
    return out


def to_f64(w: Workload, a: np.ndarray) -> np.ndarray:
    return bf16_bits_to_f64(a) if a.dtype == np.uint16 else a.astype(np.float64)


def deal_share(n_entries: int, n_shares: int, share_seed: int, share: int = 0) -> np.ndarray:
    """Indices (ascending) of the table rows dealt to `share`: a seeded permutation of all
    rows dealt round-robin over n_shares devices."""
    perm = np.random.default_rng(share_seed).permutation(n_entries)
    return np.sort(perm[share::n_shares]).astype(np.int64)


def deal_divisions(q_blk_of_entry: np.ndarray, n_div: int, div_seed: int):
    """Split a device's rows into n_div divisions by a seeded permutation and give every
    (division, q_blk) pair that occurs its own output slot.
    Returns (out_slot int32[n], n_slots, slot_q_blk int32[n_slots])."""
    n = len(q_blk_of_entry)
    perm = np.random.default_rng(div_seed).permutation(n)
    div = np.empty(n, dtype=np.int64)
    div[perm] = np.arange(n) % n_div
    keys = div * (int(q_blk_of_entry.max()) + 1 if n else 1) + q_blk_of_entry.astype(np.int64)
    uniq, inv = np.unique(keys, return_inverse=True)
    slot_q = (uniq % (int(q_blk_of_entry.max()) + 1 if n else 1)).astype(np.int32)
    return inv.astype(np.int32), int(len(uniq)), slot_q
