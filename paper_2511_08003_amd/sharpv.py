"""Python binding of libsharpv (include/sharpv.h): argument marshalling only.

Every step of both pruning stages runs in the library's HIP kernels; this module turns torch
tensors into device pointers, owns the output / workspace tensors (PyTorch is used for device
memory and streams, nothing else) and raises when the library or a GPU is missing -- there is no
CPU or eager fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsharpv.so")

F32, BF16 = 0, 1
OK = 0
KERNEL_NAMES = ("frame_slab", "frame_mean", "token_dots", "frame_select", "count_scan", "token_gather",
                "kv_cosine", "kv_mean", "kv_mask_scan", "kv_gather", "kv_gather_rope", "stream_copy", "stream_read",
                "stream_read_slabs", "stream_gather_rows")
ROPE_HALF, ROPE_INTERLEAVED = 0, 1
DISSIM_EQ1, ONE_MINUS_COS = 0, 1


class Params(C.Structure):
    """Mirror of `sharpv_params`."""
    _fields_ = [("struct_size", C.c_uint32), ("dtype", C.c_int32), ("w", C.c_float), ("M", C.c_float),
                ("mode", C.c_int32), ("K", C.c_float), ("min_keep", C.c_int32), ("kv_mode", C.c_int32),
                ("measure", C.c_int32)]


_lib: Optional[C.CDLL] = None


def load() -> C.CDLL:
    """Opens libsharpv.so (built in-tree by `python -m paper_2511_08003_amd.build`)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2511_08003_amd.build`")
    L = C.CDLL(LIB_PATH)
    vp, ip, fp = C.c_void_p, C.c_void_p, C.c_void_p
    pp = C.POINTER(Params)
    L.sharpv_params_default.restype = C.c_int
    L.sharpv_params_default.argtypes = [pp]
    L.sharpv_status_string.restype = C.c_char_p
    L.sharpv_status_string.argtypes = [C.c_int]
    L.sharpv_version.restype = C.c_int
    L.sharpv_version.argtypes = []
    L.sharpv_prune_tokens_workspace.restype = C.c_size_t
    L.sharpv_prune_tokens_workspace.argtypes = [C.c_int, C.c_int, C.c_int, pp]
    L.sharpv_prune_tokens.restype = C.c_int
    L.sharpv_prune_tokens.argtypes = [vp, ip, C.c_int, C.c_int, C.c_int, C.c_int, pp, ip, ip, ip, vp, fp, fp,
                                      vp, C.c_size_t, vp]
    L.sharpv_prune_kv_workspace.restype = C.c_size_t
    L.sharpv_prune_kv_workspace.argtypes = [C.c_int, C.c_int, C.c_int, pp]
    L.sharpv_prune_kv.restype = C.c_int
    L.sharpv_prune_kv.argtypes = [vp, vp, vp, vp, C.c_int64, C.c_int64, ip, ip, ip, C.c_int, C.c_int, C.c_int,
                                  C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, pp, ip, ip, vp, vp, C.c_int64,
                                  fp, fp, vp, C.c_size_t, vp]
    L.sharpv_prune_kv_static.restype = C.c_int
    L.sharpv_prune_kv_static.argtypes = [vp, vp, vp, vp, C.c_int64, C.c_int64, ip, ip, ip, C.c_int, C.c_int, C.c_int,
                                         C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, pp, ip, ip, vp, vp, C.c_int64,
                                         fp, fp, vp]
    L.sharpv_prune_kv_rope.restype = C.c_int
    L.sharpv_prune_kv_rope.argtypes = [vp, vp, vp, vp, C.c_int64, C.c_int64, ip, ip, ip, C.c_int, C.c_int, C.c_int,
                                       C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, pp, ip, ip, vp, vp, C.c_int64,
                                       fp, fp, fp, fp, C.c_int, C.c_int, vp, C.c_size_t, vp]
    L.sharpv_prune_kv_carried_workspace.restype = C.c_size_t
    L.sharpv_prune_kv_carried_workspace.argtypes = [C.c_int, C.c_int, pp]
    L.sharpv_prune_kv_carried.restype = C.c_int
    L.sharpv_prune_kv_carried.argtypes = [vp, vp, ip, vp, vp, C.c_int64, C.c_int64, ip, C.c_int, C.c_int, C.c_int,
                                          C.c_int, C.c_int, C.c_int, C.c_int, pp, ip, ip, vp, vp, C.c_int64, ip, fp,
                                          fp, fp, C.c_int, C.c_int, vp, C.c_size_t, vp]
    L.sharpv_stream_copy.restype = C.c_int
    L.sharpv_stream_copy.argtypes = [vp, vp, C.c_size_t, vp]
    L.sharpv_stream_read.restype = C.c_int
    L.sharpv_stream_read.argtypes = [vp, C.c_size_t, vp, vp]
    L.sharpv_stream_read_slabs.restype = C.c_int
    L.sharpv_stream_read_slabs.argtypes = [vp, C.c_int, C.c_int, C.c_int, C.c_int, vp, vp]
    L.sharpv_stream_gather_rows.restype = C.c_int
    L.sharpv_stream_gather_rows.argtypes = [vp, vp, C.c_int, ip, C.c_int, vp]
    L.sharpv_timing_enable.restype = C.c_int
    L.sharpv_timing_enable.argtypes = [C.c_int]
    L.sharpv_timing_disable.restype = C.c_int
    L.sharpv_timing_disable.argtypes = []
    L.sharpv_timing_read.restype = C.c_int
    L.sharpv_timing_read.argtypes = [C.c_char_p, C.POINTER(C.c_int), C.POINTER(C.c_double)]
    _lib = L
    return L


def status_string(rc: int) -> str:
    return load().sharpv_status_string(rc).decode()


def check(rc: int, what: str) -> None:
    if rc != OK:
        raise RuntimeError(f"{what} failed: status {rc} ({status_string(rc)})")


def default_params(dtype: int = BF16, **over) -> Params:
    p = Params()
    check(load().sharpv_params_default(C.byref(p)), "sharpv_params_default")
    p.dtype = dtype
    for k, v in over.items():
        setattr(p, k, v)
    return p


def dtype_of(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype == torch.float32:
        return F32
    raise TypeError(f"unsupported element type {t.dtype}")


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _require_gpu(*tensors: Optional[torch.Tensor]) -> None:
    if not torch.cuda.is_available():
        raise RuntimeError("sharpv needs a GPU: there is no CPU path")
    for t in tensors:
        if t is not None and (not t.is_cuda or not t.is_contiguous()):
            raise ValueError("tensors must be contiguous and live on the GPU")


def _same_dtype(params: "Params", **tensors: Optional[torch.Tensor]) -> None:
    """Every storage tensor of a call must have the element type the parameter block names: the library
    only sees pointers, so a tensor of another type would be reinterpreted silently."""
    for name, t in tensors.items():
        if t is not None and dtype_of(t) != params.dtype:
            raise TypeError(f"{name} is {t.dtype} but params.dtype says {'bfloat16' if params.dtype == BF16 else 'float32'}")


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


class TokensPlan:
    """Pre-allocated outputs and workspace for `sharpv_prune_tokens` on one shape; `run` only
    marshals pointers and enqueues on torch's current stream."""

    def __init__(self, n_frames: int, f: int, d: int, params: Params, device="cuda",
                 scores: bool = True, ratio: bool = True):
        L = load()
        self.n, self.f, self.d, self.params = n_frames, f, d, params
        tdt = torch.bfloat16 if params.dtype == BF16 else torch.float32
        self.out_idx = torch.empty(n_frames * f, dtype=torch.int32, device=device)
        self.out_counts = torch.empty(n_frames, dtype=torch.int32, device=device)
        self.out_offsets = torch.empty(n_frames + 1, dtype=torch.int32, device=device)
        self.out_feats = torch.empty((n_frames * f, d), dtype=tdt, device=device)
        self.out_scores = torch.empty(n_frames * f, dtype=torch.float32, device=device) if scores else None
        self.out_ratio = torch.empty(n_frames, dtype=torch.float32, device=device) if ratio else None
        nbytes = L.sharpv_prune_tokens_workspace(n_frames, f, d, C.byref(params))
        if nbytes == 0:
            raise ValueError("sharpv_prune_tokens_workspace rejected the shape or the parameters")
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=device)
        self.workspace_bytes = nbytes

    def run(self, feats: torch.Tensor, frame_offsets: Optional[torch.Tensor] = None) -> int:
        B = 1 if frame_offsets is None else frame_offsets.numel() - 1
        return load().sharpv_prune_tokens(feats.data_ptr(), _ptr(frame_offsets), B, self.n, self.f, self.d,
                                          C.byref(self.params), self.out_idx.data_ptr(), self.out_counts.data_ptr(),
                                          self.out_offsets.data_ptr(), self.out_feats.data_ptr(),
                                          _ptr(self.out_scores), _ptr(self.out_ratio), self.workspace.data_ptr(),
                                          self.workspace_bytes, _stream())

    def results(self) -> Dict[str, torch.Tensor]:
        """Synchronises (reads the total count) and returns the valid parts of the outputs."""
        total = int(self.out_offsets[-1].item())
        res = {"idx": self.out_idx[:total], "counts": self.out_counts, "offsets": self.out_offsets,
               "out_feats": self.out_feats[:total]}
        if self.out_scores is not None:
            res["I"] = self.out_scores.view(self.n, self.f)
        if self.out_ratio is not None:
            res["ratio"] = self.out_ratio
        return res


def prune_tokens(feats: torch.Tensor, frame_offsets: Optional[torch.Tensor] = None,
                 params: Optional[Params] = None, **over) -> Dict[str, torch.Tensor]:
    """Pre-LLM stage on feats [n_frames, f, d] (bf16 or float32, GPU)."""
    _require_gpu(feats, frame_offsets)
    if feats.dim() != 3:
        raise ValueError("feats must be [n_frames, f, d]")
    if params is None:
        params = default_params(dtype_of(feats), **over)
    _same_dtype(params, feats=feats)
    n, f, d = feats.shape
    plan = TokensPlan(n, f, d, params, device=feats.device)
    check(plan.run(feats, frame_offsets), "sharpv_prune_tokens")
    return plan.results()


class KvPlan:
    """Pre-allocated outputs and workspace for `sharpv_prune_kv` on one shape."""

    def __init__(self, B: int, S: int, n_vis: int, d: int, H: int, D: int, params: Params, device="cuda",
                 cos: bool = True, mean_cos: bool = False):
        L = load()
        self.B, self.S, self.n_vis, self.d, self.H, self.D, self.params = B, S, n_vis, d, H, D, params
        tdt = torch.bfloat16 if params.dtype == BF16 else torch.float32
        self.out_idx = torch.empty(S, dtype=torch.int32, device=device)
        self.out_count = torch.empty(B, dtype=torch.int32, device=device)
        self.K_out = torch.empty((H, S, D), dtype=tdt, device=device)
        self.V_out = torch.empty((H, S, D), dtype=tdt, device=device)
        self.out_cos = torch.empty(max(n_vis, 1), dtype=torch.float32, device=device) if cos else None
        self.out_mean_cos = torch.empty(B, dtype=torch.float32, device=device) if mean_cos else None
        nbytes = L.sharpv_prune_kv_workspace(B, S, n_vis, C.byref(params))
        if nbytes == 0:
            raise ValueError("sharpv_prune_kv_workspace rejected the shape or the parameters")
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=device)
        self.workspace_bytes = nbytes

    def run(self, hidden: torch.Tensor, orig: torch.Tensor, K: torch.Tensor, V: torch.Tensor,
            vis_start0: int = 0, seq_offsets: Optional[torch.Tensor] = None,
            vis_start: Optional[torch.Tensor] = None, vis_offsets: Optional[torch.Tensor] = None,
            layer: int = 0, rope_cos: Optional[torch.Tensor] = None, rope_sin: Optional[torch.Tensor] = None,
            rope_layout: int = ROPE_HALF) -> int:
        """Enqueues `sharpv_prune_kv`, or `sharpv_prune_kv_rope` when the rotary tables
        rope_cos / rope_sin ([rope_len, D/2] float32, GPU, contiguous) are given."""
        if rope_cos is not None or rope_sin is not None:
            return load().sharpv_prune_kv_rope(
                hidden.data_ptr(), orig.data_ptr(), K.data_ptr(), V.data_ptr(), K.stride(0), K.stride(1),
                _ptr(seq_offsets), _ptr(vis_start), _ptr(vis_offsets), self.B, self.S, vis_start0, self.n_vis,
                self.d, self.H, self.D, layer, C.byref(self.params), self.out_idx.data_ptr(),
                self.out_count.data_ptr(), self.K_out.data_ptr(), self.V_out.data_ptr(), self.K_out.stride(0),
                _ptr(self.out_cos), _ptr(self.out_mean_cos), _ptr(rope_cos), _ptr(rope_sin),
                0 if rope_cos is None else rope_cos.shape[0], rope_layout, self.workspace.data_ptr(),
                self.workspace_bytes, _stream())
        return load().sharpv_prune_kv(hidden.data_ptr(), orig.data_ptr(), K.data_ptr(), V.data_ptr(),
                                      K.stride(0), K.stride(1), _ptr(seq_offsets), _ptr(vis_start),
                                      _ptr(vis_offsets), self.B, self.S, vis_start0, self.n_vis, self.d, self.H,
                                      self.D, layer, C.byref(self.params), self.out_idx.data_ptr(),
                                      self.out_count.data_ptr(), self.K_out.data_ptr(), self.V_out.data_ptr(),
                                      self.K_out.stride(0), _ptr(self.out_cos), _ptr(self.out_mean_cos),
                                      self.workspace.data_ptr(), self.workspace_bytes, _stream())

    def run_static(self, hidden: torch.Tensor, orig: torch.Tensor, K: torch.Tensor, V: torch.Tensor,
                   vis_start0: int = 0, seq_offsets: Optional[torch.Tensor] = None,
                   vis_start: Optional[torch.Tensor] = None, vis_offsets: Optional[torch.Tensor] = None,
                   layer: int = 0) -> int:
        """Enqueues `sharpv_prune_kv_static`: the same call on the library's built-in scratch (the plan's
        workspace is not used)."""
        return load().sharpv_prune_kv_static(hidden.data_ptr(), orig.data_ptr(), K.data_ptr(), V.data_ptr(),
                                             K.stride(0), K.stride(1), _ptr(seq_offsets), _ptr(vis_start),
                                             _ptr(vis_offsets), self.B, self.S, vis_start0, self.n_vis, self.d,
                                             self.H, self.D, layer, C.byref(self.params), self.out_idx.data_ptr(),
                                             self.out_count.data_ptr(), self.K_out.data_ptr(), self.V_out.data_ptr(),
                                             self.K_out.stride(0), _ptr(self.out_cos), _ptr(self.out_mean_cos),
                                             _stream())

    def results(self) -> Dict[str, torch.Tensor]:
        total = int(self.out_count.sum().item())
        res = {"idx": self.out_idx[:total], "counts": self.out_count,
               "K_out": self.K_out[:, :total, :], "V_out": self.V_out[:, :total, :]}
        if self.out_cos is not None:
            res["cos"] = self.out_cos[:self.n_vis]
        if self.out_mean_cos is not None:
            res["mean_cos"] = self.out_mean_cos
        return res


def prune_kv(hidden: torch.Tensor, orig: torch.Tensor, K: torch.Tensor, V: torch.Tensor, vis_start0: int = 0,
             seq_offsets: Optional[torch.Tensor] = None, vis_start: Optional[torch.Tensor] = None,
             vis_offsets: Optional[torch.Tensor] = None, params: Optional[Params] = None, layer: int = 0,
             mean_cos: bool = False, n_vis: Optional[int] = None, rope_cos: Optional[torch.Tensor] = None,
             rope_sin: Optional[torch.Tensor] = None, rope_layout: int = ROPE_HALF,
             **over) -> Dict[str, torch.Tensor]:
    """Intra-LLM stage for one layer: hidden [S, d], orig [n_vis, d], K / V [H, S, D] (GPU).
    `n_vis` defaults to the number of rows of `orig`.  With rope_cos / rope_sin ([rope_len, D/2] float32)
    the kept K rows are re-encoded for their new positions (`sharpv_prune_kv_rope`)."""
    _require_gpu(hidden, orig, seq_offsets, vis_start, vis_offsets, rope_cos, rope_sin)
    for tab in (rope_cos, rope_sin):
        if tab is not None and (tab.dtype != torch.float32 or not tab.is_contiguous() or tab.dim() != 2
                                or tab.shape[1] * 2 != K.shape[2]):
            raise ValueError("rotary tables must be contiguous float32 [rope_len, D/2]")
    if not (K.is_cuda and V.is_cuda) or K.stride(2) != 1 or V.stride() != K.stride():
        raise ValueError("K and V must be GPU tensors [H, S, D] with equal strides and D contiguous")
    if params is None:
        params = default_params(dtype_of(hidden), **over)
    _same_dtype(params, hidden=hidden, orig=orig, K=K, V=V)
    S, d = hidden.shape
    H, _, D = K.shape
    B = 1 if seq_offsets is None else seq_offsets.numel() - 1
    n_vis = orig.shape[0] if n_vis is None else n_vis
    plan = KvPlan(B, S, n_vis, d, H, D, params, device=hidden.device, mean_cos=mean_cos)
    check(plan.run(hidden, orig, K, V, vis_start0, seq_offsets, vis_start, vis_offsets, layer, rope_cos, rope_sin,
                   rope_layout), "sharpv_prune_kv")
    return plan.results()


class KvCarriedPlan:
    """Pre-allocated outputs and workspace for `sharpv_prune_kv_carried` on one shape."""

    def __init__(self, B: int, S: int, n_orig: int, d: int, H: int, D: int, params: Params, device="cuda",
                 cos: bool = True):
        L = load()
        self.B, self.S, self.n_orig, self.d, self.H, self.D, self.params = B, S, n_orig, d, H, D, params
        tdt = torch.bfloat16 if params.dtype == BF16 else torch.float32
        self.out_idx = torch.empty(S, dtype=torch.int32, device=device)
        self.out_count = torch.empty(B, dtype=torch.int32, device=device)
        self.out_orig_row = torch.empty(S, dtype=torch.int32, device=device)
        self.K_out = torch.empty((H, S, D), dtype=tdt, device=device)
        self.V_out = torch.empty((H, S, D), dtype=tdt, device=device)
        self.out_cos = torch.full((S,), float("nan"), dtype=torch.float32, device=device) if cos else None
        nbytes = L.sharpv_prune_kv_carried_workspace(B, S, C.byref(params))
        if nbytes == 0:
            raise ValueError("sharpv_prune_kv_carried_workspace rejected the shape or the parameters")
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=device)
        self.workspace_bytes = nbytes

    def run(self, hidden: torch.Tensor, orig: torch.Tensor, orig_row: torch.Tensor, K: torch.Tensor,
            V: torch.Tensor, seq_offsets: Optional[torch.Tensor] = None, layer: int = 0,
            rope_cos: Optional[torch.Tensor] = None, rope_sin: Optional[torch.Tensor] = None,
            rope_layout: int = ROPE_HALF) -> int:
        return load().sharpv_prune_kv_carried(
            hidden.data_ptr(), orig.data_ptr(), orig_row.data_ptr(), K.data_ptr(), V.data_ptr(), K.stride(0),
            K.stride(1), _ptr(seq_offsets), self.B, self.S, self.n_orig, self.d, self.H, self.D, layer,
            C.byref(self.params), self.out_idx.data_ptr(), self.out_count.data_ptr(), self.K_out.data_ptr(),
            self.V_out.data_ptr(), self.K_out.stride(0), self.out_orig_row.data_ptr(), _ptr(self.out_cos),
            _ptr(rope_cos), _ptr(rope_sin), 0 if rope_cos is None else rope_cos.shape[0], rope_layout,
            self.workspace.data_ptr(), self.workspace_bytes, _stream())

    def results(self) -> Dict[str, torch.Tensor]:
        total = int(self.out_count.sum().item())
        res = {"idx": self.out_idx[:total], "counts": self.out_count, "orig_row_out": self.out_orig_row[:total],
               "K_out": self.K_out[:, :total, :], "V_out": self.V_out[:, :total, :]}
        if self.out_cos is not None:
            res["cos"] = self.out_cos
        return res


def prune_kv_carried(hidden: torch.Tensor, orig: torch.Tensor, orig_row: torch.Tensor, K: torch.Tensor,
                     V: torch.Tensor, seq_offsets: Optional[torch.Tensor] = None, params: Optional[Params] = None,
                     layer: int = 0, rope_cos: Optional[torch.Tensor] = None, rope_sin: Optional[torch.Tensor] = None,
                     rope_layout: int = ROPE_HALF, **over) -> Dict[str, torch.Tensor]:
    """Intra-LLM stage on a sequence already thinned out by earlier layers (`sharpv_prune_kv_carried`):
    hidden [S, d], K / V [H, S, D] of the positions still alive, orig [n_orig, d], orig_row [S] int32
    (row of orig behind each position, -1 for non-visual positions).  Returns idx, counts, K_out, V_out,
    cos (by position, NaN where nothing is written) and orig_row_out, the map for the next layer."""
    _require_gpu(hidden, orig, orig_row, seq_offsets, rope_cos, rope_sin)
    if not (K.is_cuda and V.is_cuda) or K.stride(2) != 1 or V.stride() != K.stride():
        raise ValueError("K and V must be GPU tensors [H, S, D] with equal strides and D contiguous")
    if orig_row.dtype != torch.int32 or orig_row.numel() != hidden.shape[0]:
        raise ValueError("orig_row must be int32 [S]")
    if params is None:
        params = default_params(dtype_of(hidden), **over)
    _same_dtype(params, hidden=hidden, orig=orig, K=K, V=V)
    S, d = hidden.shape
    H, _, D = K.shape
    B = 1 if seq_offsets is None else seq_offsets.numel() - 1
    plan = KvCarriedPlan(B, S, orig.shape[0], d, H, D, params, device=hidden.device)
    check(plan.run(hidden, orig, orig_row, K, V, seq_offsets, layer, rope_cos, rope_sin, rope_layout),
          "sharpv_prune_kv_carried")
    return plan.results()


# ----------------------------------------------------------------------------- measurement aids
def stream_copy(dst: torch.Tensor, src: torch.Tensor) -> None:
    """Plain streaming copy of src's bytes into dst (both contiguous GPU tensors of equal byte size)."""
    _require_gpu(dst, src)
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() < nbytes:
        raise ValueError("dst is smaller than src")
    check(load().sharpv_stream_copy(dst.data_ptr(), src.data_ptr(), nbytes, _stream()), "sharpv_stream_copy")


def stream_read(src: torch.Tensor, sink: torch.Tensor) -> None:
    """Plain streaming read of src's bytes; `sink` is a GPU int32 tensor with at least one element."""
    _require_gpu(src, sink)
    check(load().sharpv_stream_read(src.data_ptr(), src.numel() * src.element_size(), sink.data_ptr(), _stream()),
          "sharpv_stream_read")


def stream_read_slabs(feats: torch.Tensor, sink: torch.Tensor) -> None:
    """Reads feats [n, f, d] in the fused statistics kernel's access pattern (f <= 208), arithmetic left out."""
    _require_gpu(feats, sink)
    n, f, d = feats.shape
    check(load().sharpv_stream_read_slabs(feats.data_ptr(), n, f, d, feats.element_size(), sink.data_ptr(), _stream()),
          "sharpv_stream_read_slabs")


def stream_gather_rows(dst: torch.Tensor, src: torch.Tensor, idx: torch.Tensor) -> None:
    """dst[j] = src[idx[j]] for 2-D contiguous GPU tensors of equal row size and an int32 index tensor."""
    _require_gpu(dst, src, idx)
    if idx.dtype != torch.int32 or src.dim() != 2 or dst.dim() != 2 or dst.shape[1] != src.shape[1] \
            or dst.dtype != src.dtype or dst.shape[0] < idx.numel():
        raise ValueError("stream_gather_rows: dst [>= len(idx), d] and src [rows, d] of one dtype, idx int32")
    if idx.numel() and (int(idx.min()) < 0 or int(idx.max()) >= src.shape[0]):
        raise ValueError("stream_gather_rows: an index points outside src")
    check(load().sharpv_stream_gather_rows(dst.data_ptr(), src.data_ptr(), src.shape[1] * src.element_size(),
                                           idx.data_ptr(), idx.numel(), _stream()), "sharpv_stream_gather_rows")


# ----------------------------------------------------------------------------- event timing
def timing_enable(max_launches: int) -> None:
    check(load().sharpv_timing_enable(max_launches), "sharpv_timing_enable")


def timing_disable() -> None:
    check(load().sharpv_timing_disable(), "sharpv_timing_disable")


def timing_read(kernel: str):
    """(launches, total milliseconds) recorded for one kernel since `timing_enable`."""
    n, ms = C.c_int(0), C.c_double(0.0)
    check(load().sharpv_timing_read(kernel.encode(), C.byref(n), C.byref(ms)), "sharpv_timing_read")
    return n.value, ms.value
