"""Margin audit of the float32 canonical-order oracle against the float64 definition (CPU only).

tests/golden/margin_audit.json (written by tests/golden/make_margin_audit.py from the oracles alone)
records, for each configuration, the number of decisions the float64 definition takes within float32
error of their boundary and how many of them the float32 oracle takes the other way.  Here the small
configurations are recomputed and compared with the stored record, and the record itself is checked
for completeness: every configuration, every evaluated layer (all 28 of the 256-frame one)."""
import json
import os

import numpy as np
import pytest

import margins
from oracle import canon, sharpv_ref as ref
from paper_2511_08003_amd import workloads as wl

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "margin_audit.json")))


def test_record_covers_every_configuration_and_layer():
    assert GOLD["bands"] == {"score": margins.BAND_SCORE, "ratio_times_f": margins.BAND_RATIO,
                             "cos": margins.BAND_COS, "M": 0.2}
    for i in range(1, 9):
        cfg = wl.config(i)
        rec = GOLD[str(i)]
        assert rec["config"] == cfg.name
        assert rec["stage1"]["frames"] == cfg.n_frames and rec["visual_tokens"] == cfg.n_vis
        assert sorted(int(k) for k in rec["kv"]) == list(cfg.kv_layers)
        for r in rec["kv"].values():
            assert r["tokens"] == cfg.n_vis
            assert r["differs"] <= r["near_M"]                   # only fragile decisions may differ
            assert r["max_abs_cos_error_float32"] < margins.BAND_COS / 10
        s = rec["stage1"]
        assert s["k_differs"] <= s["k_fragile"] and s["sets_differ"] <= s["topk_fragile"] + s["k_fragile"]
    assert len(GOLD["5"]["kv"]) == 28


@pytest.mark.parametrize("index", [1, 2])
def test_small_configurations_reproduce_the_record(index):
    cfg = wl.config(index)
    tok = wl.tokens_for(cfg, threads=4)
    a = ref.prune_tokens(tok.feats, cfg.dtype, tok.frame_offsets)
    b = canon.prune_tokens(tok.feats, cfg.dtype, tok.frame_offsets)
    got = margins.token_margins(a, cfg.f)
    got.update(margins.audit_token_decisions(a, b["counts"], b["idx"], b["offsets"], cfg.f))
    want = GOLD[str(index)]["stage1"]
    for k in got:
        assert got[k] == want[k], k
    assert int(a["counts"].sum()) == want["kept_float64"] and int(b["counts"].sum()) == want["kept_float32"]
    lay = wl.kv_layout_for(cfg)
    orig = tok.feats.reshape(-1, cfg.d)
    for layer in cfg.kv_layers:
        kv = wl.kv_layer_for(cfg, tok, layer, threads=4)
        c64 = margins.cos64_rows(kv["hidden"], orig, cfg.dtype, lay.seq_offsets, lay.vis_start, lay.vis_offsets, threads=4)
        # the chunked call of the oracle's cosine is the same thing as its whole-layer function
        whole = ref.prune_kv(kv["hidden"], orig, kv["K"], kv["V"], cfg.dtype, lay.seq_offsets, lay.vis_start,
                             lay.vis_offsets, M=0.2)
        np.testing.assert_array_equal(c64, whole["cos"])
        kb = canon.prune_kv(kv["hidden"], orig, None, None, cfg.dtype, lay.seq_offsets, lay.vis_start, lay.vis_offsets, M=0.2)
        kept = margins.kept_visual_mask(kb["idx"], lay.seq_offsets, lay.vis_start, lay.vis_offsets)
        np.testing.assert_array_equal(
            margins.kept_visual_mask(whole["idx"], lay.seq_offsets, lay.vis_start, lay.vis_offsets), ~(c64 < 0.2))
        r = margins.audit_kv_decisions(c64, 0.2, kept)
        w = GOLD[str(index)]["kv"][str(layer)]
        assert (r["near_M"], r["differs"], int(np.sum(~(c64 < 0.2)))) == (w["near_M"], w["differs"], w["kept_visual_float64"])


def test_audit_catches_a_decision_taken_away_from_its_boundary():
    """The audit itself: a planted wrong decision (far from any boundary) must be refused, a swap of
    two tokens whose scores are within the band must pass."""
    cfg = wl.config(1)
    tok = wl.tokens_for(cfg, threads=2)
    a = ref.prune_tokens(tok.feats, cfg.dtype, tok.frame_offsets)
    f = cfg.f
    counts, idx, offs = a["counts"].copy(), a["idx"].copy(), a["offsets"].copy()
    assert margins.audit_token_decisions(a, counts, idx, offs, f) == {"k_differs": 0, "sets_differ": 0}
    # frame 1: replace the best kept token by the worst dropped one
    t = 1
    kept = idx[offs[t]:offs[t + 1]] - t * f
    best = kept[np.argmax(a["I"][t, kept])]
    dropped = np.setdiff1d(np.arange(f), kept)
    worst = dropped[np.argmin(a["I"][t, dropped])]
    bad = idx.copy()
    seg = np.sort(np.where(kept == best, worst, kept)) + t * f
    bad[offs[t]:offs[t + 1]] = seg
    with pytest.raises(AssertionError):
        margins.audit_token_decisions(a, counts, bad, offs, f)
    # a kept count that is off by one away from a rounding boundary
    c2 = counts.copy(); c2[2] += 1
    with pytest.raises(AssertionError):
        margins.audit_token_decisions(a, c2, idx, np.concatenate([[0], np.cumsum(c2)]).astype(np.int32), f)
    # Eq.7: a token flipped far from M is refused, one inside the band is counted
    c64 = np.array([0.5, 0.19, 0.2 + 1e-6, 0.2 - 1e-6, -0.3])
    ok = ~(c64 < 0.2)
    assert margins.audit_kv_decisions(c64, 0.2, ok) == {"tokens": 5, "near_M": 2, "differs": 0}
    flip = ok.copy(); flip[3] = True
    assert margins.audit_kv_decisions(c64, 0.2, flip)["differs"] == 1
    flip = ok.copy(); flip[1] = True
    with pytest.raises(AssertionError):
        margins.audit_kv_decisions(c64, 0.2, flip)
