"""The stored decisions of the tiny configuration (tests/golden/config1_expected.json, written by
tests/golden/make_golden.py from the CPU oracles alone) still come out of the oracles, and they sit
where the closed forms of the AR(1) generator put them.  CPU only."""
import hashlib
import json
import math
import os

import numpy as np
import pytest

from oracle import canon, sharpv_ref as ref
from paper_2511_08003_amd import workloads as wl

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "config1_expected.json")))


@pytest.fixture(scope="module")
def c1():
    cfg = wl.config(1)
    tok = wl.tokens_for(cfg, threads=1)
    return cfg, tok


def test_inputs_are_reproducible(c1):
    cfg, tok = c1
    assert hashlib.sha256(tok.feats.tobytes()).hexdigest() == GOLD["inputs_sha256"]


def test_stage1_decisions_match_stored(c1):
    cfg, tok = c1
    b = canon.prune_tokens(tok.feats, cfg.dtype, tok.frame_offsets)
    assert b["counts"].tolist() == GOLD["counts_float32"]
    assert hashlib.sha256(b["idx"].tobytes()).hexdigest() == GOLD["idx_sha256_float32"]
    a = ref.prune_tokens(tok.feats, cfg.dtype, tok.frame_offsets)
    assert a["counts"].tolist() == GOLD["counts_float64"]
    assert np.array_equal(a["idx"], b["idx"]) == GOLD["idx_equal_between_oracles"]


def test_stored_ratios_sit_on_the_generator_closed_forms():
    """rho = 0.9 inside a scene -> sqrt((1-rho)/2); fresh frame at the cut -> sqrt(1/2);
    first frame of iid tokens -> sqrt(2 - 2/sqrt f)/2."""
    r = GOLD["ratio_float64"]
    f = 196
    assert r[0] == pytest.approx(math.sqrt(2 - 2 / math.sqrt(f)) / 2, rel=5e-3)
    assert r[4] == pytest.approx(math.sqrt(0.5), rel=5e-3)
    for t in (1, 2, 3, 5, 6, 7):
        assert r[t] == pytest.approx(math.sqrt(0.05), rel=5e-3)
    assert GOLD["counts_float64"] == [math.floor(x * f + 0.5) for x in r]


def test_stage2_decisions_match_stored(c1):
    cfg, tok = c1
    lay = wl.kv_layout_for(cfg)
    kv = wl.kv_layer_for(cfg, tok, 0, threads=1)
    kb = canon.prune_kv(kv["hidden"], tok.feats.reshape(-1, cfg.d), None, None, cfg.dtype,
                        lay.seq_offsets, lay.vis_start, lay.vis_offsets, M=0.2)
    assert len(kb["idx"]) == GOLD["kv_kept_float32"]
    assert hashlib.sha256(kb["idx"].tobytes()).hexdigest() == GOLD["kv_idx_sha256_float32"]
