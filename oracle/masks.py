"""Dense boolean attention masks M[L, L] written straight from the mask definitions
(Sec. 2.1: M is a boolean [B, L, L] mask; Sec. 2.4 and Sec. 7.1 "Attention Masks" for the
families).  Test infrastructure: this is the formula-side of the mask, independent of the
per-token range arrays the kernels consume.

Every function returns rows [r0, r1) of the mask of ONE sequence of length L, as
bool[r1 - r0, L], entry [i, j] true iff query i may attend to key j (positions in-sequence).
"""
import math

import numpy as np


def _ij(L, r0, r1):
    i = np.arange(r0, r1, dtype=np.int64)[:, None]
    j = np.arange(L, dtype=np.int64)[None, :]
    return i, j


def causal(L, r0=0, r1=None):
    """Key j visible to query i iff j <= i."""
    r1 = L if r1 is None else r1
    i, j = _ij(L, r0, r1)
    return j <= i


def window(L, W, r0=0, r1=None):
    """Sliding window of W keys including the query itself, causal: 0 <= i - j < W."""
    r1 = L if r1 is None else r1
    i, j = _ij(L, r0, r1)
    return (j <= i) & (i - j < W)


def lambda_mask(L, W, sink, r0=0, r1=None):
    """Lambda-shaped mask (Sec. 2.4): attention sink (first `sink` tokens visible to all
    later tokens) combined with a causal sliding window of W keys."""
    r1 = L if r1 is None else r1
    i, j = _ij(L, r0, r1)
    return (j <= i) & ((j < sink) | (i - j < W))


def causal_blockwise(L, mblock, n_window, n_sink, r0=0, r1=None):
    """Causal blockwise mask (Sec. 2.4, Sec. 7.1): tokens are grouped in mask blocks of
    `mblock`; a token sees, causally, the first `n_sink` mask blocks and the last
    `n_window` mask blocks up to its own; the final mask block (the test sample) sees
    every earlier token."""
    r1 = L if r1 is None else r1
    i, j = _ij(L, r0, r1)
    bi, bj = i // mblock, j // mblock
    last = (L - 1) // mblock
    return (j <= i) & ((bj < n_sink) | (bi - bj < n_window) | (bi == last))


def shared_question(L, n_answers, frac, r0=0, r1=None):
    """Shared question mask (Sec. 2.4, Sec. 7.1): one question followed by n_answers
    answers, each floor(frac * L) tokens; the question is causal in itself; each answer
    sees the whole question and, causally, itself, never another answer."""
    r1 = L if r1 is None else r1
    i, j = _ij(L, r0, r1)
    a = int(math.floor(L * frac))
    q_end = L - n_answers * a

    def seg(x):
        return np.where(x < q_end, 0, 1 + (x - q_end) // max(a, 1))

    si, sj = seg(i), seg(j)
    return (j <= i) & ((sj == 0) | (sj == si))


def dense_rows(spec, L, r0=0, r1=None):
    """Dispatch on a mask specification object with fields kind/window/sink/mblock/
    n_answers/frac."""
    k = spec.kind
    if k == "causal":
        return causal(L, r0, r1)
    if k == "window":
        return window(L, spec.window, r0, r1)
    if k == "lambda":
        return lambda_mask(L, spec.window, spec.sink, r0, r1)
    if k == "causal_blockwise":
        return causal_blockwise(L, spec.mblock, spec.window, spec.sink, r0, r1)
    if k == "shared_question":
        return shared_question(L, spec.n_answers, spec.frac, r0, r1)
    raise ValueError(k)
