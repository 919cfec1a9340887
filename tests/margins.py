"""Margin audit: how far the decisions of a float32 run (the canonical-order oracle, or the GPU) may
stray from the float64 definition, and the check that they stray no further.

Three kinds of decisions turn a score into an integer: the kept count k_t = floor(r_t f + 1/2), the
top-k_t set of a frame, and cos < M per visual token.  A float32 evaluation can decide differently
from the float64 definition only where the float64 value sits within the float32 evaluation error of
the decision's boundary ("fragile" decisions).  The functions below count the fragile decisions from
the float64 oracle's output and assert that every difference between a float32 run and the float64
oracle is one of them.

Bands (absolute, on float64 values).  The float32 inner products over d <= 4096 elements are summed
as trees, so their relative error is a few 2^-24; cosines and ratios come out within ~1e-6, Eq.1's
sqrt(2 - 2cos) within ~1e-5 for the dissimilarities that occur (> 0.05).  The bands are set an order
of magnitude wider:
    scores I          BAND_SCORE = 8e-5   two tokens can change places only if their float64 scores
                                          are closer than this
    r_t * f + 1/2     BAND_RATIO * f, BAND_RATIO = 2e-5   distance to the nearest integer
    cosines (Eq.7)    BAND_COS = 2e-5     distance of the float64 cosine from M
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from typing import Dict, List

import numpy as np

from oracle import sharpv_ref as ref

BAND_SCORE = 8e-5
BAND_RATIO = 2e-5
BAND_COS = 2e-5


def frame_sets(idx: np.ndarray, offsets: np.ndarray, f: int) -> List[set]:
    return [set((idx[offsets[t]:offsets[t + 1]] - t * f).tolist()) for t in range(len(offsets) - 1)]


def token_margins(a: Dict[str, np.ndarray], f: int) -> Dict[str, int]:
    """Fragile stage-1 decisions of the float64 result `a` (adaptive mode): frames whose r_t f + 1/2
    lies within the band of an integer, and frames whose k-th and (k+1)-th scores are closer than
    the score band."""
    k_fragile = topk_fragile = 0
    for t in range(len(a["counts"])):
        x = float(a["ratio"][t]) * f + 0.5
        if abs(x - round(x)) < BAND_RATIO * f:
            k_fragile += 1
        k = int(a["counts"][t])
        if 0 < k < f:
            s = np.sort(a["I"][t])[::-1]
            if s[k - 1] - s[k] < BAND_SCORE:
                topk_fragile += 1
    return {"frames": int(len(a["counts"])), "k_fragile": k_fragile, "topk_fragile": topk_fragile}


def audit_token_decisions(a: Dict[str, np.ndarray], counts: np.ndarray, idx: np.ndarray, offsets: np.ndarray,
                          f: int) -> Dict[str, int]:
    """Kept counts and kept sets of a float32 run against the float64 result `a`.  A frame whose count
    differs must have r_t f + 1/2 within the band of an integer; a frame with the same count and another
    set must differ only in tokens whose float64 scores lie within the score band of each other."""
    sets_a = frame_sets(a["idx"], a["offsets"], f)
    sets_b = frame_sets(np.asarray(idx), np.asarray(offsets), f)
    k_differs = sets_differ = 0
    for t in range(len(a["counts"])):
        if int(a["counts"][t]) != int(counts[t]):
            x = float(a["ratio"][t]) * f + 0.5
            assert abs(int(a["counts"][t]) - int(counts[t])) == 1 and abs(x - round(x)) < BAND_RATIO * f, \
                f"frame {t}: kept count {counts[t]} vs {a['counts'][t]} away from a rounding boundary (r f + 1/2 = {x})"
            k_differs += 1
        elif sets_a[t] != sets_b[t]:
            diff = sorted(sets_a[t] ^ sets_b[t])
            sc = a["I"][t, diff]
            assert sc.max() - sc.min() < BAND_SCORE, \
                f"frame {t}: kept sets differ in tokens {diff} whose scores are {sc.max() - sc.min()} apart"
            sets_differ += 1
    return {"k_differs": k_differs, "sets_differ": sets_differ}


def cos64_rows(hidden: np.ndarray, orig: np.ndarray, dtype: int, seq_offsets, vis_start, vis_offsets,
               threads: int = 8, rows: int = 1024) -> np.ndarray:
    """Float64 cosine of every visual token of a packed batch: the oracle's `cosine` (Eq.7's left side)
    called on chunks of rows, chunks spread over a few threads."""
    n_vis = int(vis_offsets[-1])
    out = np.empty(n_vis)
    jobs = []
    for b in range(len(vis_start)):
        lo, hi = int(vis_offsets[b]), int(vis_offsets[b + 1])
        p0 = int(seq_offsets[b]) + int(vis_start[b])
        for c in range(lo, hi, rows):
            jobs.append((c, min(hi, c + rows), p0 + (c - lo)))

    def work(job):
        lo, hi, p = job
        out[lo:hi] = ref.cosine(ref.widen(hidden[p:p + (hi - lo)], dtype), ref.widen(orig[lo:hi], dtype))

    with ThreadPoolExecutor(max_workers=max(1, threads)) as ex:
        list(ex.map(work, jobs))
    return out


def audit_kv_decisions(cos64: np.ndarray, M: float, kept_visual: np.ndarray) -> Dict[str, int]:
    """Eq.7 decisions of a float32 run (`kept_visual`: one bool per visual token) against the float64
    cosines: a token decided differently must have its float64 cosine within the band of M."""
    want = ~(cos64 < M)
    differs = np.nonzero(want != np.asarray(kept_visual, bool))[0]
    assert np.all(np.abs(cos64[differs] - M) < BAND_COS), \
        f"tokens {differs[:8].tolist()} decided against the definition away from M: cos = {cos64[differs[:8]].tolist()}"
    return {"tokens": int(len(cos64)), "near_M": int(np.sum(np.abs(cos64 - M) < BAND_COS)), "differs": int(len(differs))}


def kept_visual_mask(idx: np.ndarray, seq_offsets, vis_start, vis_offsets) -> np.ndarray:
    """Kept packed positions -> one bool per visual token (orig-row order)."""
    S = int(seq_offsets[-1])
    keep = np.zeros(S, bool)
    keep[np.asarray(idx)] = True
    parts = []
    for b in range(len(vis_start)):
        p0 = int(seq_offsets[b]) + int(vis_start[b])
        parts.append(keep[p0:p0 + int(vis_offsets[b + 1] - vis_offsets[b])])
    return np.concatenate(parts) if parts else np.zeros(0, bool)
