"""SharpV two-stage pruning, written out from the paper's definitions in float64 (NumPy).

TEST INFRASTRUCTURE ONLY.  This is the slow, plain checker that the GPU library is compared
against; nothing in the product path may import it.  It shares no code with the HIP
kernels and takes its inputs as plain NumPy arrays.

Every function follows one passage of the paper (Sec. 3.1 "Information-Aware Visual Space
Pruning", Sec. 3.2 "Information-Aware Memory Space Pruning"); equation numbers count the
displayed equations in order of appearance: Eq.1 Dissim, Eq.2 spatial importance S, Eq.3
temporal importance T, Eq.4 score I, Eq.5 threshold_t, Eq.6 threshold_1, Eq.7 Discard(l).

Readings taken where the paper is silent:
  * thresholds of Eq.5/6 are *retention* ratios; kept count k_t = floor(r_t*f + 1/2),
    clamped to [min_keep, f];
  * the first frame of a video uses T := S (the virtual preceding frame of Sec. 3.1 whose
    every token is the frame mean), so Eq.6 is Eq.5 applied to that T;
  * a zero-norm vector has cosine 0 to everything;
  * top-k ties go to the lowest token index, kept tokens stay in stream order;
  * the rescaled cosine 1 - cos that Sec. 3.1 allows in place of Eq.1 comes only together with
    the fixed threshold K (mode 1), as the paper pairs them; S, T and I keep their roles;
  * Eq.7 is applied per visual token (kv_mode 0) or to the mean over a sequence's visual
    tokens (kv_mode 1); non-visual positions are always kept; "< M" is strict;
  * pruning carried from layer to layer (Sec. 3.2: discarded features do not propagate further)
    is read as: a layer sees only the positions that survived the layers before it, each with
    a pointer to the row of the original visual features it started from;
  * the positional re-encoding of Sec. 4.1 (Implementation Details) is read as: every kept K
    row gets the rotary embedding of its new place in the compacted cache; the paper names no
    rotary convention, so frequencies (as cos/sin tables) and pairing come from the caller.

Pins: tests/test_oracle_pins.py (closed forms, invariants, brute force, library routines).
No function here is "parity unpinned".
"""
from __future__ import annotations

import math
from typing import Dict, Optional

import numpy as np


# ----------------------------------------------------------------------------- widening
def widen(a: np.ndarray, dtype: int) -> np.ndarray:
    """Storage array -> float64, exactly.  dtype 0: float32; dtype 1: bfloat16 bit patterns (uint16)."""
    if dtype == 0:
        return np.asarray(a, dtype=np.float32).astype(np.float64)
    bits = np.asarray(a, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return bits.view(np.float32).astype(np.float64)


# ----------------------------------------------------------------------------- Eq.1
def cosine(a: np.ndarray, b: np.ndarray) -> np.ndarray:
    """cos(theta) between corresponding rows of a and b (b may be a single broadcast row).
    A zero-norm row has cosine 0."""
    a = np.asarray(a, dtype=np.float64)
    b = np.broadcast_to(np.asarray(b, dtype=np.float64), a.shape)
    na = np.sqrt(np.sum(a * a, axis=-1))
    nb = np.sqrt(np.sum(b * b, axis=-1))
    dot = np.sum(a * b, axis=-1)
    den = na * nb
    out = np.zeros_like(den)
    np.divide(dot, den, out=out, where=den > 0)
    return np.clip(out, -1.0, 1.0)


def dissim(a: np.ndarray, b: np.ndarray) -> np.ndarray:
    """Eq.1, first form: Euclidean distance between the L2-normalised rows.
    (A zero-norm row is treated as having cosine 0, i.e. distance sqrt(2).)"""
    a = np.asarray(a, dtype=np.float64)
    b = np.broadcast_to(np.asarray(b, dtype=np.float64), a.shape)
    na = np.sqrt(np.sum(a * a, axis=-1, keepdims=True))
    nb = np.sqrt(np.sum(b * b, axis=-1, keepdims=True))
    ok = (na[..., 0] > 0) & (nb[..., 0] > 0)
    ua = np.divide(a, na, out=np.zeros_like(a), where=na > 0)
    ub = np.divide(b, nb, out=np.zeros_like(a), where=nb > 0)
    dist = np.sqrt(np.sum((ua - ub) ** 2, axis=-1))
    return np.where(ok, dist, math.sqrt(2.0))


def dissim_from_cos(c: np.ndarray) -> np.ndarray:
    """Eq.1, second form: sqrt(2 - 2 cos(theta))."""
    return np.sqrt(np.maximum(0.0, 2.0 - 2.0 * np.asarray(c, dtype=np.float64)))


def one_minus_cos(a: np.ndarray, b: np.ndarray) -> np.ndarray:
    """The rescaled cosine that Sec. 3.1 (Dissimilarity Computation Module) allows in place of
    Eq.1 together with a fixed threshold K: 1 - cos(theta), in [0, 2]."""
    return 1.0 - cosine(a, b)


def _measure(kind: int):
    if kind not in (0, 1):
        raise ValueError("measure must be 0 (Eq.1) or 1 (one minus cosine)")
    return dissim if kind == 0 else one_minus_cos


# ----------------------------------------------------------------------------- Eq.2 - Eq.6
def spatial_importance(frame: np.ndarray, measure: int = 0) -> np.ndarray:
    """Eq.2: S_i = Dissim(F_t[i], mean_j F_t[j]); the mean row is broadcast over tokens."""
    mean = np.mean(np.asarray(frame, dtype=np.float64), axis=0, keepdims=True)
    return _measure(measure)(frame, mean)


def temporal_importance(frame: np.ndarray, prev: np.ndarray, measure: int = 0) -> np.ndarray:
    """Eq.3: T_i = Dissim(F_t[i], F_{t-1}[i]) -- the same token slot in adjacent frames."""
    return _measure(measure)(frame, prev)


def importance(T: np.ndarray, S: np.ndarray, w: float) -> np.ndarray:
    """Eq.4: I = T + w*S."""
    return T + w * S


def keep_ratio(T_frame: np.ndarray) -> float:
    """Eq.5 (and Eq.6 with T := S): ||T_t||_2 / (2 sqrt(f)), in [0, 1]."""
    f = T_frame.shape[0]
    r = math.sqrt(float(np.sum(T_frame * T_frame))) / (2.0 * math.sqrt(f))
    return min(1.0, max(0.0, r))


def kept_count(r: float, f: int, min_keep: int = 0) -> int:
    """k_t = round-half-up(r_t * f), clamped to [min_keep, f]."""
    return int(min(f, max(min_keep, math.floor(r * f + 0.5))))


def select_topk(I: np.ndarray, k: int) -> np.ndarray:
    """Top-k of one frame by score (Sec. 3.1, last paragraph).  Token i is kept iff fewer
    than k tokens precede it in the order (score descending, index ascending).  Returns
    the kept token indices in ascending order."""
    I = np.asarray(I)
    idx = np.arange(I.shape[0])
    greater = (I[None, :] > I[:, None]).sum(axis=1)
    tie_before = ((I[None, :] == I[:, None]) & (idx[None, :] < idx[:, None])).sum(axis=1)
    return np.nonzero(greater + tie_before < k)[0]


def prune_tokens(feats: np.ndarray, dtype: int, frame_offsets: np.ndarray, w: float = 1.0,
                 mode: int = 0, K: float = 1.6, min_keep: int = 0, measure: int = 0) -> Dict[str, np.ndarray]:
    """Pre-LLM stage over a packed batch of videos.

    feats [n_total, f, d] storage array; frame_offsets [B+1] cumulative frames per video.
    mode 0: adaptive ratio (Eq.5/6) + per-frame top-k; mode 1: keep token iff I >= K.
    measure 0: S and T by Eq.1; measure 1: by one minus the cosine (only with mode 1, the
    pairing Sec. 3.1 names).
    Returns S, T, I [n_total, f]; ratio [n_total]; counts [n_total]; offsets [n_total+1];
    idx [sum k] global row indices t*f+i ascending; out_feats = the kept rows, bit-copied."""
    if measure == 1 and mode != 1:
        raise ValueError("one minus cosine goes with the fixed threshold K (mode 1)")
    n_total, f, d = feats.shape
    x = widen(feats, dtype)
    S = np.zeros((n_total, f))
    T = np.zeros((n_total, f))
    ratio = np.zeros(n_total)
    counts = np.zeros(n_total, dtype=np.int32)
    kept = []
    for b in range(len(frame_offsets) - 1):
        for t in range(int(frame_offsets[b]), int(frame_offsets[b + 1])):
            S[t] = spatial_importance(x[t], measure)
            T[t] = S[t] if t == int(frame_offsets[b]) else temporal_importance(x[t], x[t - 1], measure)
    I = importance(T, S, w)
    for t in range(n_total):
        ratio[t] = keep_ratio(T[t])
        if mode == 0:
            sel = select_topk(I[t], kept_count(ratio[t], f, min_keep))
        else:
            sel = np.nonzero(I[t] >= K)[0]
        counts[t] = len(sel)
        kept.append(t * f + sel)
    offsets = np.zeros(n_total + 1, dtype=np.int32)
    offsets[1:] = np.cumsum(counts)
    idx = np.concatenate(kept).astype(np.int32) if kept else np.zeros(0, np.int32)
    out_feats = np.asarray(feats).reshape(n_total * f, d)[idx]
    return {"S": S, "T": T, "I": I, "ratio": ratio, "counts": counts, "offsets": offsets,
            "idx": idx, "out_feats": out_feats}


# ----------------------------------------------------------------------------- Eq.7
def prune_kv(hidden: np.ndarray, orig: np.ndarray, Kc: np.ndarray, Vc: np.ndarray, dtype: int,
             seq_offsets: np.ndarray, vis_start: np.ndarray, vis_offsets: np.ndarray,
             M: float = 0.2, kv_mode: int = 0) -> Dict[str, np.ndarray]:
    """Intra-LLM stage for one layer over a packed batch of sequences (Sec. 3.2, Eq.7).

    hidden [S, d] layer-l hidden states; orig [n_vis, d] original visual embeddings; Kc, Vc
    [H, S, D].  Visual token p of sequence b sits at packed position
    seq_offsets[b] + vis_start[b] + (p - vis_offsets[b]).
    kv_mode 0: visual token discarded iff cos(hidden, orig) < M.
    kv_mode 1: all visual tokens of a sequence discarded iff their mean cosine < M.
    Returns cos [n_vis], mean_cos [B], idx (kept packed positions ascending), counts [B],
    K_out, V_out [H, S_kept, D] bit-copied."""
    S_total = hidden.shape[0]
    B = len(vis_start)
    h = widen(hidden, dtype)
    o = widen(orig, dtype)
    keep = np.ones(S_total, dtype=bool)
    cos = np.zeros(o.shape[0])
    mean_cos = np.zeros(B)
    counts = np.zeros(B, dtype=np.int32)
    for b in range(B):
        lo, hi = int(vis_offsets[b]), int(vis_offsets[b + 1])
        p0 = int(seq_offsets[b]) + int(vis_start[b])
        c = cosine(h[p0:p0 + (hi - lo)], o[lo:hi])
        cos[lo:hi] = c
        mean_cos[b] = float(np.mean(c)) if hi > lo else 0.0
        if kv_mode == 0:
            keep[p0:p0 + (hi - lo)] = ~(c < M)
        elif hi > lo and mean_cos[b] < M:
            keep[p0:p0 + (hi - lo)] = False
        counts[b] = int(keep[int(seq_offsets[b]):int(seq_offsets[b + 1])].sum())
    idx = np.nonzero(keep)[0].astype(np.int32)
    return {"cos": cos, "mean_cos": mean_cos, "idx": idx, "counts": counts,
            "K_out": np.asarray(Kc)[:, idx, :], "V_out": np.asarray(Vc)[:, idx, :]}


def prune_kv_mapped(hidden: np.ndarray, orig: np.ndarray, orig_row: np.ndarray, Kc: np.ndarray, Vc: np.ndarray,
                    dtype: int, seq_offsets: np.ndarray, M: float = 0.2) -> Dict[str, np.ndarray]:
    """Eq.7 on a sequence that earlier layers have already thinned out (Sec. 3.2, Degradation-Aware
    Pruning: a discarded token's degraded features do not propagate further, so the layers after it
    work on the survivors only).

    hidden [S, d], Kc / Vc [H, S, D] hold the positions still alive at this layer;
    orig_row[s] is the row of `orig` that position s started from, or -1 for a system /
    instruction position (anything outside [0, len(orig)) counts as -1).  A visual position is
    discarded iff cos(hidden[s], orig[orig_row[s]]) < M; the others are always kept.
    Returns cos [S] (NaN at non-visual positions), idx, counts [B], K_out, V_out and
    orig_row_out = orig_row[idx], the map the next layer starts from."""
    h = widen(hidden, dtype)
    o = widen(orig, dtype)
    rows = np.asarray(orig_row, dtype=np.int64).copy()
    rows[(rows < 0) | (rows >= o.shape[0])] = -1
    S_total = h.shape[0]
    cos = np.full(S_total, np.nan)
    keep = np.ones(S_total, dtype=bool)
    vis = np.nonzero(rows >= 0)[0]
    if len(vis):
        cos[vis] = cosine(h[vis], o[rows[vis]])
        keep[vis] = ~(cos[vis] < M)
    so = np.asarray(seq_offsets, dtype=np.int64)
    counts = np.array([int(keep[so[b]:so[b + 1]].sum()) for b in range(len(so) - 1)], dtype=np.int32)
    idx = np.nonzero(keep)[0].astype(np.int32)
    return {"cos": cos, "idx": idx, "counts": counts, "orig_row_out": rows[idx].astype(np.int32),
            "K_out": np.asarray(Kc)[:, idx, :], "V_out": np.asarray(Vc)[:, idx, :]}


# ----------------------------------------------------------------------------- rotary re-encoding
def rope_reencode(K_kept: np.ndarray, dtype: int, idx: np.ndarray, seq_offsets: np.ndarray,
                  cos_tab: np.ndarray, sin_tab: np.ndarray, layout: int = 0) -> np.ndarray:
    """Positional re-encoding of the compacted K cache (Sec. 4.1, Implementation Details: the
    positional embedding is re-encoded during intra-LLM pruning).

    K_kept [H, S_kept, D] holds the kept K rows in stream order, idx their packed positions.
    A row that sat at position p of its sequence and is now the j-th kept row of that sequence
    carries a rotary embedding for p and needs the one for j: every pair (x, y) of the row is
    turned back by delta = p - j steps of its frequency,
        x' = x cos(delta*theta_i) + y sin(delta*theta_i),   y' = y cos(delta*theta_i) - x sin(delta*theta_i).
    The caller's model fixes the frequencies and hands over cos_tab / sin_tab [L, D/2] with
    row delta = cos / sin of delta*theta_i (L > every delta).  layout 0 pairs element i with
    i + D/2 (the "rotate half" convention), layout 1 pairs 2i with 2i+1.
    Returns float64 [H, S_kept, D] (not rounded back to the storage type)."""
    K = widen(K_kept, dtype)
    H, n_kept, D = K.shape
    half = D // 2
    so = np.asarray(seq_offsets, dtype=np.int64)
    idx = np.asarray(idx, dtype=np.int64)
    out = np.empty_like(K)
    ia = np.arange(half) if layout == 0 else 2 * np.arange(half)
    ib = ia + half if layout == 0 else ia + 1
    rank_in_seq = 0
    seq = 0
    for j in range(n_kept):
        s = int(idx[j])
        while s >= so[seq + 1]:
            seq += 1
            rank_in_seq = 0
        delta = (s - int(so[seq])) - rank_in_seq
        c = np.asarray(cos_tab[delta], dtype=np.float64)
        sn = np.asarray(sin_tab[delta], dtype=np.float64)
        x, y = K[:, j, ia], K[:, j, ib]
        out[:, j, ia] = x * c + y * sn
        out[:, j, ib] = y * c - x * sn
        rank_in_seq += 1
    return out


# ----------------------------------------------------------------------------- retention figures
def retention(counts_tokens: np.ndarray, f: int, kept_kv: Optional[int] = None, S: Optional[int] = None) -> Dict[str, float]:
    """VR = kept visual tokens / all visual tokens; MR = kept KV positions / all positions;
    token budget = VR * MR (Sec. 4.1, Metrics)."""
    vr = float(np.sum(counts_tokens)) / float(len(counts_tokens) * f)
    out = {"VR": vr}
    if kept_kv is not None and S:
        out["MR"] = kept_kv / float(S)
        out["budget"] = vr * out["MR"]
    return out
