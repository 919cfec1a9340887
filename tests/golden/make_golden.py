"""Writes tests/golden/config1_expected.json: the decisions of the two CPU oracles on the tiny
configuration (8 frames x 196 tokens, d=1152 float32; one KV layer).  Calls only oracle/ and
the input generator; run it again only when the oracle's arithmetic changes for a stated reason.

    python tests/golden/make_golden.py
"""
import hashlib
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import canon, sharpv_ref as ref            # noqa: E402
from paper_2511_08003_amd import workloads as wl       # noqa: E402


def main() -> None:
    cfg = wl.config(1)
    tok = wl.tokens_for(cfg, threads=1)
    lay = wl.kv_layout_for(cfg)
    kv = wl.kv_layer_for(cfg, tok, 0, threads=1)
    orig = tok.feats.reshape(-1, cfg.d)
    a = ref.prune_tokens(tok.feats, cfg.dtype, tok.frame_offsets)
    b = canon.prune_tokens(tok.feats, cfg.dtype, tok.frame_offsets)
    kargs = (kv["hidden"], orig, kv["K"], kv["V"], cfg.dtype, lay.seq_offsets, lay.vis_start, lay.vis_offsets)
    ka = ref.prune_kv(*kargs, M=0.2)
    kb = canon.prune_kv(*kargs, M=0.2)
    out = {
        "config": cfg.name,
        "inputs_sha256": hashlib.sha256(tok.feats.tobytes()).hexdigest(),
        "counts_float64": a["counts"].tolist(),
        "counts_float32": b["counts"].tolist(),
        "ratio_float64": [round(float(r), 9) for r in a["ratio"]],
        "idx_sha256_float32": hashlib.sha256(b["idx"].tobytes()).hexdigest(),
        "idx_equal_between_oracles": bool(np.array_equal(a["idx"], b["idx"])),
        "kv_kept_float64": int(len(ka["idx"])),
        "kv_kept_float32": int(len(kb["idx"])),
        "kv_idx_sha256_float32": hashlib.sha256(kb["idx"].tobytes()).hexdigest(),
        "kv_idx_equal_between_oracles": bool(np.array_equal(ka["idx"], kb["idx"])),
    }
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "config1_expected.json")
    with open(path, "w") as fh:
        json.dump(out, fh, indent=1)
        fh.write("\n")
    print(json.dumps(out, indent=1))


if __name__ == "__main__":
    main()
