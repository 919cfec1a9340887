"""Seeded synthetic inputs shaped like the paper's video workloads.

This module only *draws inputs*: AR(1) frame sequences with scene cuts (stand-ins for
projected visual tokens of sampled video frames, Table 2 shapes: f=196 tokens per frame,
d=3584 for the 7B model), layer hidden states that drift away from the original visual
embedding with depth (the degradation trend of Sec. 3.2 / Fig. 3), and random K/V caches.
It contains none of the method's arithmetic (no dissimilarity, score, ratio, selection or
cosine) and is imported by the tests, the benchmark and the oracle-side scripts alike.

bf16 tensors are carried as numpy uint16 bit patterns; the rounding to bf16
(round-to-nearest-even) happens here, once, so every consumer sees identical bytes.
"""
from __future__ import annotations

import math
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

F32 = 0
BF16 = 1


# ----------------------------------------------------------------------------- dtype helpers
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to float32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_storage(a32: np.ndarray, dtype: int) -> np.ndarray:
    """float32 array -> storage array of the workload's element type."""
    if dtype == F32:
        return np.ascontiguousarray(a32, dtype=np.float32)
    return f32_to_bf16_bits(a32)


def storage_to_f32(a: np.ndarray, dtype: int) -> np.ndarray:
    return np.asarray(a, dtype=np.float32) if dtype == F32 else bf16_bits_to_f32(a)


def elem_bytes(dtype: int) -> int:
    return 4 if dtype == F32 else 2


def _pool_normal(seed_key: Sequence[int], shape: Tuple[int, ...], threads: int = 8,
                 rows_per_chunk: int = 2048) -> np.ndarray:
    """N(0,1) float32 array; rows are drawn in fixed-size chunks, each from its own
    SeedSequence child, so the values do not depend on the number of threads."""
    rows = shape[0]
    out = np.empty(shape, dtype=np.float32)
    n_chunks = (rows + rows_per_chunk - 1) // rows_per_chunk
    children = np.random.SeedSequence(list(seed_key)).spawn(max(n_chunks, 1))

    def work(c: int) -> None:
        lo = c * rows_per_chunk
        hi = min(rows, lo + rows_per_chunk)
        g = np.random.Generator(np.random.PCG64(children[c]))
        g.standard_normal(out=out[lo:hi], dtype=np.float32)

    if n_chunks <= 1 or threads <= 1:
        for c in range(n_chunks):
            work(c)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(work, range(n_chunks)))
    return out


# ----------------------------------------------------------------------------- stage-1 inputs
@dataclass
class VideoSpec:
    """One video of the pre-LLM stage: n frames, AR(1) in time.

    rho[t] (t>=1) is the correlation between frame t and frame t-1; frames listed in
    `cuts` are drawn fresh (scene cut). `slot_sigma` > 0 multiplies every token slot by a
    log-normal factor shared by all frames."""
    n: int
    rho: np.ndarray                     # [n] float64, rho[0] unused
    cuts: Tuple[int, ...] = ()
    slot_sigma: float = 0.0
    seed: int = 0


@dataclass
class TokenWorkload:
    """Packed batch of videos for the pre-LLM stage."""
    feats: np.ndarray                   # [n_total, f, d] float32 or uint16 (bf16 bits)
    dtype: int
    f: int
    d: int
    frame_offsets: np.ndarray           # [B+1] int32, cumulative frames per video
    slot_scale: np.ndarray              # [B, f] float32, per-video token-slot scale (1 if unused)
    videos: List[VideoSpec] = field(default_factory=list)

    @property
    def n_total(self) -> int:
        return int(self.frame_offsets[-1])

    @property
    def B(self) -> int:
        return len(self.frame_offsets) - 1


def ar1_video(spec: VideoSpec, f: int, d: int, threads: int = 8) -> Tuple[np.ndarray, np.ndarray]:
    """x_0 ~ N(0,1); x_t = rho_t x_{t-1} + sqrt(1-rho_t^2) eps_t; fresh N(0,1) at a cut.
    Returns ([n,f,d] float32, slot scale [f] float32)."""
    eps = _pool_normal((spec.seed, 11), (spec.n * f, d), threads).reshape(spec.n, f, d)
    x = np.empty((spec.n, f, d), dtype=np.float32)
    x[0] = eps[0]
    cuts = set(int(c) for c in spec.cuts)
    for t in range(1, spec.n):
        if t in cuts:
            x[t] = eps[t]
        else:
            r = np.float32(spec.rho[t])
            s = np.float32(math.sqrt(max(0.0, 1.0 - float(spec.rho[t]) ** 2)))
            np.multiply(x[t - 1], r, out=x[t])
            x[t] += s * eps[t]
    scale = np.ones(f, dtype=np.float32)
    if spec.slot_sigma > 0.0:
        g = np.random.default_rng([spec.seed, 13])
        scale = np.exp(spec.slot_sigma * g.standard_normal(f)).astype(np.float32)
        x *= scale[None, :, None]
    return x, scale


def make_tokens(videos: Sequence[VideoSpec], f: int, d: int, dtype: int, threads: int = 8) -> TokenWorkload:
    parts, scales, offs = [], [], [0]
    for v in videos:
        x, sc = ar1_video(v, f, d, threads)
        parts.append(to_storage(x, dtype))
        scales.append(sc)
        offs.append(offs[-1] + v.n)
        del x
    feats = parts[0] if len(parts) == 1 else np.concatenate(parts, axis=0)
    return TokenWorkload(feats=feats, dtype=dtype, f=f, d=d,
                         frame_offsets=np.asarray(offs, dtype=np.int32),
                         slot_scale=np.stack(scales), videos=list(videos))


# ----------------------------------------------------------------------------- stage-2 inputs
@dataclass
class KVLayout:
    """Packed batch of sequences for the intra-LLM stage. Sequence b occupies packed
    positions [seq_offsets[b], seq_offsets[b+1]); its visual block starts vis_start[b]
    positions into the sequence and has vis_offsets[b+1]-vis_offsets[b] tokens, whose
    original embeddings are rows [vis_offsets[b], vis_offsets[b+1]) of `orig`."""
    seq_offsets: np.ndarray             # [B+1] int32
    vis_start: np.ndarray               # [B] int32
    vis_offsets: np.ndarray             # [B+1] int32
    H: int
    D: int

    @property
    def S(self) -> int:
        return int(self.seq_offsets[-1])

    @property
    def n_vis(self) -> int:
        return int(self.vis_offsets[-1])

    @property
    def B(self) -> int:
        return len(self.vis_start)

    def visual_positions(self) -> np.ndarray:
        """Packed sequence position of every visual token, in orig-row order."""
        pos = []
        for b in range(self.B):
            nv = int(self.vis_offsets[b + 1] - self.vis_offsets[b])
            start = int(self.seq_offsets[b]) + int(self.vis_start[b])
            pos.append(np.arange(start, start + nv, dtype=np.int64))
        return np.concatenate(pos) if pos else np.zeros(0, dtype=np.int64)


def make_kv_layout(n_vis_per_seq: Sequence[int], text_before: int, text_after: int, H: int, D: int) -> KVLayout:
    seq, vo, vs = [0], [0], []
    for nv in n_vis_per_seq:
        seq.append(seq[-1] + text_before + int(nv) + text_after)
        vo.append(vo[-1] + int(nv))
        vs.append(text_before)
    return KVLayout(np.asarray(seq, np.int32), np.asarray(vs, np.int32), np.asarray(vo, np.int32), H, D)


def layer_mean_cos(layer: int) -> float:
    """Target mean cosine between layer-`layer` visual hidden states and the original
    embeddings: 1 at the decoder input, decaying quickly, below 0.2 from about layer 11
    (qualitative shape of the similarity curves in Fig. 3)."""
    return 1.0 if layer <= 0 else 0.12 + 0.83 * math.exp(-layer / 4.5)


def drift_sigma(layer: int, n_vis: int, mode: str, sigma_max: float = 8.0) -> np.ndarray:
    """Per-visual-token noise scale (relative to the token's own scale), float32 [n_vis].

    mode "ramp":  sigma_p = sigma_max * p/(n_vis-1)            (tiny config: rises linearly over tokens)
    mode "layer": sigma_p = sigma_l * (0.5 + p/n_vis), sigma_l = sqrt(1/c_l^2 - 1), zero at layer 0."""
    p = np.arange(n_vis, dtype=np.float64)
    if mode == "ramp":
        s = sigma_max * p / max(n_vis - 1, 1)
    else:
        c = layer_mean_cos(layer)
        s = np.zeros(n_vis) if c >= 1.0 else math.sqrt(1.0 / (c * c) - 1.0) * (0.5 + p / n_vis)
    return s.astype(np.float32)


def make_hidden(orig32: np.ndarray, row_scale: np.ndarray, layout: KVLayout, layer: int, mode: str,
                seed: int, dtype: int, threads: int = 8) -> np.ndarray:
    """hidden_l [S, d]: visual rows = orig + sigma_p * row_scale_p * z, text rows ~ N(0,1).
    With sigma_p == 0 the visual rows equal the original embeddings bit for bit."""
    S, d = layout.S, orig32.shape[1]
    h = _pool_normal((seed, 21, layer), (S, d), threads)
    sig = drift_sigma(layer, layout.n_vis, mode) * row_scale.astype(np.float32)
    pos = layout.visual_positions()
    for b in range(layout.B):
        lo, hi = int(layout.vis_offsets[b]), int(layout.vis_offsets[b + 1])
        p0 = int(pos[lo]) if hi > lo else 0
        blk = h[p0:p0 + (hi - lo)]
        blk *= sig[lo:hi, None]
        blk += orig32[lo:hi]
    return to_storage(h, dtype)


def make_kv_cache(layout: KVLayout, layer: int, seed: int, dtype: int, threads: int = 8) -> Tuple[np.ndarray, np.ndarray]:
    """K, V ~ N(0,1), each [H, S, D] contiguous."""
    kv = _pool_normal((seed, 31, layer), (2 * layout.H * layout.S, layout.D), threads)
    kv = to_storage(kv, dtype).reshape(2, layout.H, layout.S, layout.D)
    return kv[0], kv[1]


# ----------------------------------------------------------------------------- the five configurations
@dataclass
class Config:
    name: str
    dtype: int
    f: int
    d: int
    videos: List[VideoSpec]
    text_before: int
    text_after: int
    H: int
    D: int
    n_layers: int                      # depth of the KV cache the config describes
    kv_layers: Tuple[int, ...]         # layers at which the intra-LLM stage is evaluated
    drift: str                         # "ramp" or "layer"
    seed: int

    @property
    def n_frames(self) -> int:
        return sum(v.n for v in self.videos)

    @property
    def n_vis(self) -> int:
        return self.n_frames * self.f


def _const_rho(n: int, rho: float) -> np.ndarray:
    return np.full(n, rho, dtype=np.float64)


def config(index: int, frames_scale: float = 1.0) -> Config:
    """The five benchmark workloads (index 1..5), the two other model shapes of the paper's
    Table 2 (6, 7) and a tall-frame shape (8). `frames_scale` < 1 shrinks frame counts for quick checks; 1.0 gives the
    stated sizes."""
    def nf(n: int) -> int:
        return max(2, int(round(n * frames_scale)))

    seed = 1000 + index
    if index == 1:      # 8 x 196, d=1152 fp32, rho 0.9, one cut at frame 4
        n = nf(8)
        v = VideoSpec(n=n, rho=_const_rho(n, 0.9), cuts=(n // 2,), seed=seed)
        return Config("c1_8f_d1152_f32", F32, 196, 1152, [v], 16, 48, 4, 128, 1, (0,), "ramp", seed)
    if index == 2:      # 32 x 196, d=3584 bf16, rho 0.95, cuts every 8 frames, log-normal slot scale
        n = nf(32)
        v = VideoSpec(n=n, rho=_const_rho(n, 0.95), cuts=tuple(range(8, n, 8)), slot_sigma=0.5, seed=seed)
        return Config("c2_32f_d3584_bf16", BF16, 196, 3584, [v], 32, 96, 4, 128, 28, (14,), "layer", seed)
    if index == 3:      # 64 frames, static (0.99) / high-motion (0.5) segments of 16 frames
        n = nf(64)
        rho = np.where((np.arange(n) // 16) % 2 == 0, 0.99, 0.5).astype(np.float64)
        v = VideoSpec(n=n, rho=rho, seed=seed)
        return Config("c3_64f_mixed_bf16", BF16, 196, 3584, [v], 32, 96, 4, 128, 28, (4, 14, 24), "layer", seed)
    if index == 4:      # ragged batch of 8 videos
        g = np.random.default_rng([seed, 1])
        vids = []
        for b in range(8):
            n = nf(int(g.integers(16, 65)))
            rho = float(g.uniform(0.5, 0.99))
            n_cuts = int(g.integers(0, 4))
            cuts = tuple(sorted(set(int(c) for c in g.integers(1, n, size=n_cuts)))) if n > 1 else ()
            vids.append(VideoSpec(n=n, rho=_const_rho(n, rho), cuts=cuts, seed=1400 + b))
        return Config("c4_ragged8_bf16", BF16, 196, 3584, vids, 32, 96, 4, 128, 28, (14,), "layer", seed)
    if index == 5:      # 256 frames, rho 0.97, Poisson scene cuts (mean gap 20)
        n = nf(256)
        g = np.random.default_rng([seed, 1])
        cuts, t = [], 0
        while True:
            t += max(1, int(g.poisson(20)))
            if t >= n:
                break
            cuts.append(t)
        v = VideoSpec(n=n, rho=_const_rho(n, 0.97), cuts=tuple(cuts), seed=seed)
        return Config("c5_256f_long_bf16", BF16, 196, 3584, [v], 64, 192, 4, 128, 28, tuple(range(28)), "layer", seed)
    if index == 6:      # PLLaVA-7B shape (Table 2): 16 frames x 144 tokens, d=4096, 32 layers, 32 KV heads x 128
        n = nf(16)
        v = VideoSpec(n=n, rho=_const_rho(n, 0.95), cuts=tuple(range(8, n, 8)), slot_sigma=0.5, seed=seed)
        return Config("c6_pllava7b_16f_d4096_bf16", BF16, 144, 4096, [v], 32, 96, 32, 128, 32, (16,), "layer", seed)
    if index == 7:      # LLaVA-OneVision-0.5B shape (Table 2): 32 frames x 196 tokens, d=896, 24 layers, 2 KV heads x 64
        n = nf(32)
        v = VideoSpec(n=n, rho=_const_rho(n, 0.95), cuts=tuple(range(8, n, 8)), slot_sigma=0.5, seed=seed)
        return Config("c7_llavaov05b_32f_d896_bf16", BF16, 196, 896, [v], 32, 96, 2, 64, 24, (12,), "layer", seed)
    if index == 8:      # tall frames: 87 frames x 576 tokens (a 24 x 24 grid per frame), d=3584 bf16 -- the volume of
                        # workload 5 in frames too tall for the register-resident statistics kernel
        n = nf(87)
        v = VideoSpec(n=n, rho=_const_rho(n, 0.95), cuts=tuple(range(8, n, 8)), seed=seed)
        return Config("c8_tall_87f_576t_d3584_bf16", BF16, 576, 3584, [v], 64, 192, 4, 128, 28, (14,), "layer", seed)
    raise ValueError("config index must be 1..8")


def tokens_for(cfg: Config, threads: int = 8) -> TokenWorkload:
    return make_tokens(cfg.videos, cfg.f, cfg.d, cfg.dtype, threads)


def kv_layout_for(cfg: Config) -> KVLayout:
    return make_kv_layout([v.n * cfg.f for v in cfg.videos], cfg.text_before, cfg.text_after, cfg.H, cfg.D)


def kv_layer_for(cfg: Config, tok: TokenWorkload, layer: int, threads: int = 8,
                 orig32: Optional[np.ndarray] = None) -> Dict[str, np.ndarray]:
    """hidden_l, K, V of one layer for the sequences built from `tok` (original visual
    embeddings = the stage-1 features, row p <-> visual token p)."""
    layout = kv_layout_for(cfg)
    if orig32 is None:
        orig32 = storage_to_f32(tok.feats, tok.dtype).reshape(-1, cfg.d)
    row_scale = np.concatenate([np.tile(tok.slot_scale[b], v.n) for b, v in enumerate(cfg.videos)])
    hidden = make_hidden(orig32, row_scale, layout, layer, cfg.drift, cfg.seed, cfg.dtype, threads)
    K, V = make_kv_cache(layout, layer, cfg.seed, cfg.dtype, threads)
    return {"hidden": hidden, "K": K, "V": V}
