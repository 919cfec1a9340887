"""The seeded input generators: same bytes whatever the thread count, the stated shapes, and the
statistical structure the workloads are meant to have (temporal correlation, scene cuts, drift of the
hidden states).  Uses only the generators and NumPy."""
import numpy as np
import pytest

from paper_2511_08003_amd import workloads as wl


def test_generators_do_not_depend_on_the_thread_count():
    cfg = wl.config(2, frames_scale=0.25)
    a = wl.tokens_for(cfg, threads=1)
    b = wl.tokens_for(cfg, threads=5)
    np.testing.assert_array_equal(a.feats, b.feats)
    ka = wl.kv_layer_for(cfg, a, 7, threads=1)
    kb = wl.kv_layer_for(cfg, b, 7, threads=3)
    for k in ("hidden", "K", "V"):
        np.testing.assert_array_equal(ka[k], kb[k])
    # and a different layer is a different draw
    kc = wl.kv_layer_for(cfg, a, 8, threads=1)
    assert not np.array_equal(ka["hidden"], kc["hidden"])


@pytest.mark.parametrize("index,frames,f,d,dtype,H,D,layers", [
    (1, 8, 196, 1152, wl.F32, 4, 128, 1),
    (2, 32, 196, 3584, wl.BF16, 4, 128, 28),
    (3, 64, 196, 3584, wl.BF16, 4, 128, 28),
    (5, 256, 196, 3584, wl.BF16, 4, 128, 28),
    (6, 16, 144, 4096, wl.BF16, 32, 128, 32),
    (7, 32, 196, 896, wl.BF16, 2, 64, 24),
])
def test_config_shapes(index, frames, f, d, dtype, H, D, layers):
    cfg = wl.config(index)
    assert sum(v.n for v in cfg.videos) == frames
    assert (cfg.f, cfg.d, cfg.dtype, cfg.H, cfg.D, cfg.n_layers) == (f, d, dtype, H, D, layers)
    lay = wl.kv_layout_for(cfg)
    assert lay.n_vis == frames * f and lay.S == lay.n_vis + cfg.text_before + cfg.text_after


def test_ragged_config_is_eight_videos_of_16_to_64_frames():
    cfg = wl.config(4)
    assert len(cfg.videos) == 8 and all(16 <= v.n <= 64 for v in cfg.videos)
    lay = wl.kv_layout_for(cfg)
    assert lay.B == 8 and lay.seq_offsets[-1] == lay.S


def test_frames_are_correlated_in_time_and_fresh_after_a_cut():
    cfg = wl.config(2, frames_scale=0.5)             # 16 frames, rho 0.95, a cut at frame 8
    tok = wl.tokens_for(cfg, threads=2)
    x = wl.storage_to_f32(tok.feats, tok.dtype).astype(np.float64)
    def corr(a, b):
        a, b = a.ravel(), b.ravel()
        return float(a @ b / np.sqrt((a @ a) * (b @ b)))
    assert corr(x[3], x[4]) == pytest.approx(0.95, abs=0.01)
    assert abs(corr(x[7], x[8])) < 0.02              # scene cut: an independent frame
    assert corr(x[8], x[10]) == pytest.approx(0.95 ** 2, abs=0.01)


def test_hidden_states_drift_with_depth():
    cfg = wl.config(2, frames_scale=0.25)
    tok = wl.tokens_for(cfg, threads=2)
    lay = wl.kv_layout_for(cfg)
    orig = wl.storage_to_f32(tok.feats, tok.dtype).reshape(-1, cfg.d).astype(np.float64)
    pos = lay.visual_positions()
    means = []
    for layer in (0, 4, 12, 24):
        h = wl.storage_to_f32(wl.kv_layer_for(cfg, tok, layer, threads=2)["hidden"], cfg.dtype).astype(np.float64)[pos]
        c = np.sum(h * orig, axis=1) / np.sqrt(np.sum(h * h, axis=1) * np.sum(orig * orig, axis=1))
        means.append(float(c.mean()))
    assert means[0] == pytest.approx(1.0, abs=1e-6)   # decoder input: the embeddings themselves
    assert means[0] > means[1] > means[2] > means[3]
    assert means[2] < 0.25 and means[3] < 0.2         # below the threshold region in the deep layers
