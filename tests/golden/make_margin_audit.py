"""Writes tests/golden/margin_audit.json: for each of the five configurations (and the three other
shapes), how many decisions of the float64 definition sit within float32 error of their boundary
(kept count k_t, top-k set, cos < M per evaluated layer), how many of them the float32 canonical-order
oracle decides differently, and a digest of the float64 decisions.  Calls only oracle/ (through
tests/margins.py) and the input generator; asserts on the way that every difference between the two
oracles is a fragile decision.

    python tests/golden/make_margin_audit.py [config ...]      (default: 1 .. 8; a few minutes)
"""
import hashlib
import json
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.dirname(HERE))

import margins                                         # noqa: E402
from oracle import canon, sharpv_ref as ref            # noqa: E402
from paper_2511_08003_amd import workloads as wl       # noqa: E402

PATH = os.path.join(HERE, "margin_audit.json")
M = 0.2


def audit_config(index: int, threads: int = 8) -> dict:
    cfg = wl.config(index)
    tok = wl.tokens_for(cfg, threads=threads)
    f = cfg.f
    a = ref.prune_tokens(tok.feats, cfg.dtype, tok.frame_offsets)
    b = canon.prune_tokens(tok.feats, cfg.dtype, tok.frame_offsets)
    rec = {"config": cfg.name, "visual_tokens": int(tok.n_total * f)}
    rec["stage1"] = margins.token_margins(a, f)
    rec["stage1"].update(margins.audit_token_decisions(a, b["counts"], b["idx"], b["offsets"], f))
    rec["stage1"]["kept_float64"] = int(a["counts"].sum())
    rec["stage1"]["kept_float32"] = int(b["counts"].sum())
    rec["stage1"]["idx_sha256_float64"] = hashlib.sha256(a["idx"].astype(np.int32).tobytes()).hexdigest()
    lay = wl.kv_layout_for(cfg)
    orig = tok.feats.reshape(-1, cfg.d)
    orig32 = wl.storage_to_f32(tok.feats, tok.dtype).reshape(-1, cfg.d)
    rec["kv"] = {}
    for layer in cfg.kv_layers:
        kv = wl.kv_layer_for(cfg, tok, layer, threads=threads, orig32=orig32)
        c64 = margins.cos64_rows(kv["hidden"], orig, cfg.dtype, lay.seq_offsets, lay.vis_start, lay.vis_offsets,
                                 threads=threads)
        kb = canon.prune_kv(kv["hidden"], orig, None, None, cfg.dtype, lay.seq_offsets, lay.vis_start,
                            lay.vis_offsets, M=M)
        kept = margins.kept_visual_mask(kb["idx"], lay.seq_offsets, lay.vis_start, lay.vis_offsets)
        r = margins.audit_kv_decisions(c64, M, kept)
        r["kept_visual_float64"] = int(np.sum(~(c64 < M)))
        r["kept_mask_sha256_float64"] = hashlib.sha256(np.packbits(~(c64 < M)).tobytes()).hexdigest()
        r["max_abs_cos_error_float32"] = float(np.max(np.abs(kb["cos"].astype(np.float64) - c64)))
        rec["kv"][str(layer)] = r
        print(f"config {index} layer {layer}: {r}", flush=True)
    print(f"config {index} stage 1: {rec['stage1']}", flush=True)
    return rec


def main() -> None:
    which = [int(x) for x in sys.argv[1:]] or [1, 2, 3, 4, 5, 6, 7, 8]
    out = json.load(open(PATH)) if os.path.exists(PATH) else {}
    out["bands"] = {"score": margins.BAND_SCORE, "ratio_times_f": margins.BAND_RATIO, "cos": margins.BAND_COS, "M": M}
    for i in which:
        out[str(i)] = audit_config(i)
    with open(PATH, "w") as fh:
        json.dump(out, fh, indent=1, sort_keys=True)
        fh.write("\n")


if __name__ == "__main__":
    main()
