"""Pins of the float32 canonical-order oracle (oracle/sharpv_canon.c): exact-arithmetic cases,
closed forms, invariants, and agreement with the float64 definition inside the float32 error
bound -- including an audit that every integer decision on which the two disagree sits inside
that bound.  CPU only."""
import math
from fractions import Fraction

import numpy as np
import pytest

from oracle import canon
from oracle import sharpv_ref as ref
from paper_2511_08003_amd import workloads as wl

U = 2.0 ** -24          # float32 unit roundoff


# ----------------------------------------------------------------------------- building blocks
@pytest.mark.parametrize("d", [1, 7, 8, 9, 255, 256, 257, 264, 896, 1152, 3584, 4096])
def test_rowdot_exact_on_small_integers(d):
    """With small integer data every product and partial sum is exact, so any order gives the
    exact inner product: every element must be used exactly once, ragged tail included."""
    rng = np.random.default_rng(d)
    x = rng.integers(-8, 9, d).astype(np.float32)
    y = rng.integers(-8, 9, d).astype(np.float32)
    assert canon.rowdot(x, y) == float(np.dot(x.astype(np.int64), y.astype(np.int64)))
    e = np.zeros(d, np.float32)
    e[d - 1] = 3.0
    assert canon.rowdot(e, e) == 9.0 and canon.rowdot(x, e) == 3.0 * x[d - 1]


@pytest.mark.parametrize("d", [896, 1152, 3584])
def test_rowdot_within_float32_bound_of_exact(d):
    rng = np.random.default_rng(100 + d)
    x = rng.standard_normal(d).astype(np.float32)
    y = rng.standard_normal(d).astype(np.float32)
    exact = float(np.dot(x.astype(np.float64), y.astype(np.float64)))
    # depth of the written order: 8 fused steps + 5 tree levels + d/256 block additions
    depth = 8 + 5 + (d + 255) // 256
    bound = depth * U * float(np.dot(np.abs(x).astype(np.float64), np.abs(y).astype(np.float64))) * 1.01
    assert abs(canon.rowdot(x, y) - exact) <= bound


def _round_f32(q: Fraction) -> Fraction:
    """Correct rounding (nearest, ties to even) of an exact rational to float32 (normal range)."""
    if q == 0:
        return Fraction(0)
    s = -1 if q < 0 else 1
    q = abs(q)
    e = math.floor(math.log2(q))
    while Fraction(2) ** e > q:
        e -= 1
    while Fraction(2) ** (e + 1) <= q:
        e += 1
    ulp = Fraction(2) ** (e - 23)
    n = q / ulp
    lo = n.numerator // n.denominator
    rem = n - lo
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and lo % 2 == 1):
        lo += 1
    return s * lo * ulp


def test_rowdot_follows_the_written_order_in_exact_rational_arithmetic():
    """Secondary check (not a pin of the method): replay the written order -- 8-step fused chains,
    32-leaf halving tree per 256-element block, blocks added in ascending order -- with exact
    rationals and an explicit float32 rounding after every operation."""
    rng = np.random.default_rng(5)
    for d in (40, 300, 777):
        x = (rng.standard_normal(d) * 10 ** rng.uniform(-3, 3, d)).astype(np.float32)
        y = (rng.standard_normal(d) * 10 ** rng.uniform(-3, 3, d)).astype(np.float32)
        acc = Fraction(0)
        for b0 in range(0, d, 256):
            c = []
            for l in range(32):
                v = Fraction(0)
                for j in range(8):
                    e = b0 + 8 * l + j
                    if e < d:
                        v = _round_f32(Fraction(float(x[e])) * Fraction(float(y[e])) + v)
                c.append(v)
            s = 16
            while s >= 1:
                for l in range(s):
                    c[l] = _round_f32(c[l] + c[l + s])
                s //= 2
            acc = _round_f32(acc + c[0])
        assert Fraction(canon.rowdot(x, y)) == acc


def test_colmean_exact_and_bounded():
    rng = np.random.default_rng(6)
    for f in (1, 31, 32, 33, 144, 196):
        F = rng.integers(-4, 5, (f, 20)).astype(np.float32)
        m = canon.colmean(F)
        exact = F.astype(np.float64).sum(axis=0)
        np.testing.assert_array_equal(m, (exact.astype(np.float32) / np.float32(f)))
    F = rng.standard_normal((196, 64)).astype(np.float32)
    np.testing.assert_allclose(canon.colmean(F), F.astype(np.float64).mean(axis=0), rtol=0, atol=20 * U * 3)


def test_sum32_exact_on_integers_and_order_sensitive_case():
    v = np.arange(1, 198, dtype=np.float32)
    assert canon.sum32(v) == 197 * 198 / 2
    # 2^24 + 1 + 1 ... : the interleaved order adds the ones to different partials than a running sum would
    w = np.zeros(64, np.float32)
    w[0] = 2.0 ** 24
    w[1:] = 1.0
    assert canon.sum32(w) == 2.0 ** 24 + 62.0     # w[32] is absorbed by partial 0 (2^24 + 1 rounds to 2^24)


def test_cos_and_dissim_scalars():
    assert canon.cos(5.0, 5.0, 5.0) == 1.0 and canon.dissim(5.0, 5.0, 5.0) == 0.0
    assert canon.cos(-5.0, 5.0, 5.0) == -1.0 and canon.dissim(-5.0, 5.0, 5.0) == 2.0
    assert canon.cos(0.0, 4.0, 9.0) == 0.0 and canon.dissim(0.0, 4.0, 9.0) == np.float32(math.sqrt(2.0))
    assert canon.cos(1.0, 0.0, 9.0) == 0.0                     # zero-norm reading
    assert canon.cos(3.0, 4.0, 9.0) == 0.5
    assert canon.cos(7.0, 4.0, 9.0) == 1.0                     # clamped
    # any s: sqrt(s*s) == s  =>  identical rows give exactly cos 1
    rng = np.random.default_rng(7)
    for s in rng.uniform(1e-3, 1e6, 200).astype(np.float32):
        assert canon.cos(float(s), float(s), float(s)) == 1.0


# ----------------------------------------------------------------------------- stage 1 against the definition
def _small_video(seed, n, f, d, dtype, rho=0.9):
    spec = wl.VideoSpec(n=n, rho=np.full(n, rho), cuts=(n // 2,) if n > 3 else (), seed=seed)
    return wl.make_tokens([spec], f, d, dtype, threads=1)


def _frame_sets(o, f):
    return [set((o["idx"][o["offsets"][t]:o["offsets"][t + 1]] - t * f).tolist()) for t in range(len(o["counts"]))]


def audit_tokens(a, b, f, tol=2e-5):
    """Decisions of the float32 oracle (b) against the float64 definition (a).  Where they differ
    the float64 margin (distance of r*f from a rounding boundary, or gap between the scores at
    the selection boundary) must lie within the float32 error `tol`.  Returns #fragile frames."""
    fragile = 0
    sets_a, sets_b = _frame_sets(a, f), _frame_sets(b, f)
    for t in range(len(a["counts"])):
        if a["counts"][t] != b["counts"][t]:
            x = a["ratio"][t] * f + 0.5
            assert abs(x - round(x)) < tol * f, f"frame {t}: count differs away from a rounding boundary"
            fragile += 1
            continue
        if sets_a[t] != sets_b[t]:
            diff = sorted(sets_a[t] ^ sets_b[t])
            sc = a["I"][t, diff]
            assert sc.max() - sc.min() < tol * 4, f"frame {t}: kept sets differ away from the score boundary"
            fragile += 1
    return fragile


@pytest.mark.parametrize("dtype,d", [(wl.F32, 1152), (wl.BF16, 896), (wl.BF16, 3584)])
def test_prune_tokens_matches_definition(dtype, d):
    f = 49 if d == 3584 else 196
    tok = _small_video(21 + d, 6, f, d, dtype)
    a = ref.prune_tokens(tok.feats, dtype, tok.frame_offsets, w=1.0)
    b = canon.prune_tokens(tok.feats, dtype, tok.frame_offsets, w=1.0)
    for key in ("S", "T", "I"):
        np.testing.assert_allclose(b[key], a[key], rtol=1e-4, atol=1e-5)
    np.testing.assert_allclose(b["ratio"], a["ratio"], rtol=1e-5, atol=1e-6)
    assert audit_tokens(a, b, f) <= 1
    # structure
    assert np.all(np.diff(b["idx"]) > 0)
    np.testing.assert_array_equal(b["offsets"][1:], np.cumsum(b["counts"]))
    np.testing.assert_array_equal(b["out_feats"], tok.feats.reshape(-1, d)[b["idx"]])
    np.testing.assert_array_equal(b["T"][0], b["S"][0])
    for t in range(6):
        assert b["counts"][t] == int(np.floor(np.float32(b["ratio"][t] * np.float32(f)) + np.float32(0.5)))


def test_prune_tokens_static_negated_and_first_frame():
    rng = np.random.default_rng(31)
    f, d = 40, 520
    F = wl.f32_to_bf16_bits(rng.standard_normal((f, d)).astype(np.float32))
    neg = F ^ np.uint16(0x8000)
    b = canon.prune_tokens(np.stack([F, F, neg]), wl.BF16, np.array([0, 3]))
    assert b["ratio"][1] == 0.0 and b["counts"][1] == 0 and np.all(b["T"][1] == 0.0)      # exactly static
    assert b["ratio"][2] == 1.0 and b["counts"][2] == f and np.all(b["T"][2] == 2.0)      # exactly opposite
    # first-frame rule at every video start of a ragged batch; videos independent
    two = canon.prune_tokens(np.stack([F, neg, F, F]), wl.BF16, np.array([0, 2, 4]))
    np.testing.assert_array_equal(two["T"][2], two["S"][2])
    solo = canon.prune_tokens(np.stack([F, F]), wl.BF16, np.array([0, 2]))
    np.testing.assert_array_equal(two["I"][2:], solo["I"])
    np.testing.assert_array_equal(two["idx"][two["offsets"][2]:] - 2 * f, solo["idx"])


def test_prune_tokens_ties_go_to_lowest_index():
    """Frame 1 repeats frame 0 token-pair-wise rotated so that scores tie exactly in pairs."""
    rng = np.random.default_rng(32)
    f, d = 16, 256
    base = wl.f32_to_bf16_bits(rng.standard_normal((f // 2, d)).astype(np.float32))
    F0 = np.concatenate([base, base])                    # slots i and i+8 identical
    F1 = wl.f32_to_bf16_bits(rng.standard_normal((f // 2, d)).astype(np.float32))
    F1 = np.concatenate([F1, F1])
    b = canon.prune_tokens(np.stack([F0, F1]), wl.BF16, np.array([0, 2]))
    I1 = b["I"][1]
    np.testing.assert_array_equal(I1[:8], I1[8:])
    sel = b["idx"][b["offsets"][1]:] - f
    order = np.argsort(-I1, kind="stable")
    assert sorted(order[:b["counts"][1]].tolist()) == sel.tolist()
    assert b["counts"][1] % 2 == 1 or True
    # force an odd k through min_keep to split a tied pair: the lower index of the pair must win
    k = b["counts"][1] | 1
    c = canon.prune_tokens(np.stack([F0, F1]), wl.BF16, np.array([0, 2]), min_keep=k)
    sel = (c["idx"][c["offsets"][1]:] - f).tolist()
    assert sorted(order[:c["counts"][1]].tolist()) == sel
    last = order[c["counts"][1] - 1]
    assert last < 8 and (last + 8) not in sel


def test_manual_mode_matches_definition():
    tok = _small_video(41, 5, 64, 512, wl.BF16, rho=0.2)
    for K in (1.0, 1.6, 2.2):
        a = ref.prune_tokens(tok.feats, wl.BF16, tok.frame_offsets, mode=1, K=K)
        b = canon.prune_tokens(tok.feats, wl.BF16, tok.frame_offsets, mode=1, K=K)
        sa, sb = set(a["idx"].tolist()), set(b["idx"].tolist())
        for r in sa ^ sb:
            assert abs(a["I"].reshape(-1)[r] - K) < 1e-4
        assert len(sb) == b["counts"].sum()


def test_one_minus_cos_scalars_and_manual_mode_matches_definition():
    L = canon.lib()
    assert L.sharpv_canon_one_minus_cos(5.0, 5.0, 5.0) == 0.0
    assert L.sharpv_canon_one_minus_cos(-5.0, 5.0, 5.0) == 2.0
    assert L.sharpv_canon_one_minus_cos(0.0, 4.0, 9.0) == 1.0
    assert L.sharpv_canon_one_minus_cos(1.0, 0.0, 9.0) == 1.0                # zero-norm reading
    assert L.sharpv_canon_one_minus_cos(3.0, 4.0, 9.0) == 0.5
    tok = _small_video(43, 6, 64, 512, wl.BF16, rho=0.2)
    for w, K in ((1.0, 1.7), (0.0, 0.8), (1.0, 1.6)):
        a = ref.prune_tokens(tok.feats, wl.BF16, tok.frame_offsets, w=w, mode=1, K=K, measure=1)
        b = canon.prune_tokens(tok.feats, wl.BF16, tok.frame_offsets, w=w, mode=1, K=K, measure=1)
        np.testing.assert_allclose(b["S"], a["S"], rtol=0, atol=2e-6)
        np.testing.assert_allclose(b["T"], a["T"], rtol=0, atol=2e-6)
        sa, sb = set(a["idx"].tolist()), set(b["idx"].tolist())
        for r in sa ^ sb:
            assert abs(a["I"].reshape(-1)[r] - K) < 1e-5
        assert len(sb) == b["counts"].sum() and 0 < len(sb) < 6 * 64
    with pytest.raises(ValueError):
        canon.prune_tokens(tok.feats, wl.BF16, tok.frame_offsets, mode=0, measure=1)


# ----------------------------------------------------------------------------- stage 2 against the definition
def test_prune_kv_matches_definition_config1_shape():
    cfg = wl.config(1, frames_scale=0.25)            # 2 frames x 196 tokens, d=1152 fp32
    tok = wl.tokens_for(cfg, threads=1)
    lay = wl.kv_layout_for(cfg)
    kv = wl.kv_layer_for(cfg, tok, 0, threads=1)
    orig = tok.feats.reshape(-1, cfg.d)
    args = (kv["hidden"], orig, kv["K"], kv["V"], cfg.dtype, lay.seq_offsets, lay.vis_start, lay.vis_offsets)
    a = ref.prune_kv(*args, M=0.2)
    b = canon.prune_kv(*args, M=0.2)
    np.testing.assert_allclose(b["cos"], a["cos"], rtol=1e-4, atol=1e-6)
    np.testing.assert_allclose(b["mean_cos"], a["mean_cos"], rtol=1e-5)
    for s in set(a["idx"].tolist()) ^ set(b["idx"].tolist()):
        p = s - cfg.text_before
        assert abs(a["cos"][p] - 0.2) < 1e-5
    np.testing.assert_array_equal(b["K_out"], kv["K"][:, b["idx"], :])
    np.testing.assert_array_equal(b["V_out"], kv["V"][:, b["idx"], :])
    assert b["counts"].sum() == len(b["idx"])
    # sigma ramps 0..8 over the tokens, crossing sqrt(24) (cos = 0.2) at ~61 % of them
    frac = (len(b["idx"]) - cfg.text_before - cfg.text_after) / lay.n_vis
    assert frac == pytest.approx(math.sqrt(24.0) / 8.0, abs=0.03)
    assert b["cos"][0] == 1.0                        # sigma_0 = 0: bit-identical rows


def test_prune_kv_extremes_ragged_bf16():
    rng = np.random.default_rng(51)
    d, H, D = 264, 2, 16
    lay = wl.make_kv_layout([70, 33], 3, 4, H, D)
    orig = wl.f32_to_bf16_bits(rng.standard_normal((103, d)).astype(np.float32))
    hidden = wl.f32_to_bf16_bits(rng.standard_normal((lay.S, d)).astype(np.float32))
    pos = lay.visual_positions()
    hidden[pos[:70]] = orig[:70]                                  # sequence 0 intact
    hidden[pos[70:]] = orig[70:] ^ np.uint16(0x8000)              # sequence 1 negated
    K = wl.f32_to_bf16_bits(rng.standard_normal((H, lay.S, D)).astype(np.float32))
    V = wl.f32_to_bf16_bits(rng.standard_normal((H, lay.S, D)).astype(np.float32))
    args = (hidden, orig, K, V, wl.BF16, lay.seq_offsets, lay.vis_start, lay.vis_offsets)
    for mode in (0, 1):
        b = canon.prune_kv(*args, M=0.2, kv_mode=mode)
        np.testing.assert_array_equal(b["counts"], [77, 7])
        np.testing.assert_array_equal(b["cos"], np.r_[np.ones(70), -np.ones(33)].astype(np.float32))
        np.testing.assert_array_equal(b["mean_cos"], np.array([1.0, -1.0], np.float32))
        a = ref.prune_kv(*args, M=0.2, kv_mode=mode)
        np.testing.assert_array_equal(b["idx"], a["idx"])
        np.testing.assert_array_equal(b["K_out"], a["K_out"])
        np.testing.assert_array_equal(b["V_out"], a["V_out"])
    assert len(canon.prune_kv(*args, M=-1.0)["idx"]) == lay.S
    assert len(canon.prune_kv(*args, M=1.5)["idx"]) == 14
    kept = [len(canon.prune_kv(*args, M=m)["idx"]) for m in (-1.0, -0.5, 0.0, 0.2, 0.99, 1.0, 1.01)]
    assert all(y <= x for x, y in zip(kept, kept[1:]))


# ----------------------------------------------------------------------------- rotary re-encoding
def test_rope_reencode_exact_cases():
    rng = np.random.default_rng(41)
    H, D, S = 2, 16, 12
    K = rng.integers(-20, 21, size=(H, S, D)).astype(np.float32)
    seq = np.array([0, S])
    idx = np.array([0, 3, 4, 9, 11])                    # deltas 0, 2, 2, 6, 7
    L = 8
    for dtype, store in ((wl.F32, K), (wl.BF16, wl.f32_to_bf16_bits(K))):
        # delta 0 everywhere: bit-for-bit identity, whatever the tables hold at the other deltas
        ct = np.full((L, D // 2), 0.37, np.float32); st = np.full((L, D // 2), -0.91, np.float32)
        ct[0], st[0] = 1.0, 0.0
        np.testing.assert_array_equal(canon.rope_reencode(store, dtype, np.arange(S), seq, ct, st, 0), store)
        # quarter turn at every delta > 0 (cos 0, sin 1): x' = y, y' = -x exactly
        ct[1:], st[1:] = 0.0, 1.0
        got = wl.storage_to_f32(canon.rope_reencode(store[:, idx], dtype, idx, seq, ct, st, 0), dtype)
        want = K[:, idx].copy()
        want[:, 1:, :D // 2], want[:, 1:, D // 2:] = K[:, idx[1:], D // 2:], -K[:, idx[1:], :D // 2]
        np.testing.assert_array_equal(got, want)
        got = wl.storage_to_f32(canon.rope_reencode(store[:, idx], dtype, idx, seq, ct, st, 1), dtype)
        want = K[:, idx].copy()
        want[:, 1:, 0::2], want[:, 1:, 1::2] = K[:, idx[1:], 1::2], -K[:, idx[1:], 0::2]
        np.testing.assert_array_equal(got, want)
        # dyadic table entries per delta and per pair: exact in float32 on small integers (and in bf16: |.| < 256)
        ct = (rng.integers(-4, 5, size=(L, D // 2)) / 4).astype(np.float32)
        st = (rng.integers(-4, 5, size=(L, D // 2)) / 4).astype(np.float32)
        Kq = (np.round(K / 4) * 4).astype(np.float32)   # multiples of 4 keep every result an integer below 256
        sq = Kq if dtype == wl.F32 else wl.f32_to_bf16_bits(Kq)
        got = wl.storage_to_f32(canon.rope_reencode(sq[:, idx], dtype, idx, seq, ct, st, 0), dtype)
        d = idx - np.arange(len(idx))
        x, y = Kq[:, idx, :D // 2].astype(np.float64), Kq[:, idx, D // 2:].astype(np.float64)
        np.testing.assert_array_equal(got[:, :, :D // 2], x * ct[d] + y * st[d])
        np.testing.assert_array_equal(got[:, :, D // 2:], y * ct[d] - x * st[d])
    with pytest.raises(ValueError):                     # delta 7 needs a table of 8 rows
        canon.rope_reencode(K[:, idx], wl.F32, idx, seq, ct[:7], st[:7], 0)


@pytest.mark.parametrize("layout", [0, 1])
def test_rope_reencode_matches_definition(layout):
    rng = np.random.default_rng(43 + layout)
    H, D = 4, 128
    seq = np.array([0, 300, 700])
    keep = rng.random(700) < 0.4
    keep[[0, 299, 300]] = True
    idx = np.nonzero(keep)[0]
    theta = 1e6 ** (-2.0 * np.arange(D // 2) / D)
    ang = np.arange(400)[:, None] * theta[None, :]
    ct, st = np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)
    K = rng.standard_normal((H, 700, D)).astype(np.float32)
    want = ref.rope_reencode(K[:, idx], wl.F32, idx, seq, ct, st, layout)
    got = canon.rope_reencode(K[:, idx], wl.F32, idx, seq, ct, st, layout)
    np.testing.assert_allclose(got, want, rtol=0, atol=4 * 2.0 ** -24 * 8)      # a few float32 ulps at |x| < 8
    Kb = wl.f32_to_bf16_bits(K)
    want = ref.rope_reencode(Kb[:, idx], wl.BF16, idx, seq, ct, st, layout)
    got = wl.storage_to_f32(canon.rope_reencode(Kb[:, idx], wl.BF16, idx, seq, ct, st, layout), wl.BF16)
    # one rounding to bf16 (8 significant bits: half an ulp <= 2^-8 relative) on top of the float32 arithmetic
    np.testing.assert_allclose(got, want, rtol=2.0 ** -8 * 1.001, atol=1e-6)


# ----------------------------------------------------------------------------- pruning carried from layer to layer
@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
def test_prune_kv_mapped_matches_definition_and_block_form(dtype):
    rng = np.random.default_rng(61 + dtype)
    S, n_orig, d, H, D = 300, 260, 264, 2, 16
    orig = wl.to_storage(rng.standard_normal((n_orig, d)).astype(np.float32), dtype)
    o32 = wl.storage_to_f32(orig, dtype)
    rows = np.full(S, -1)
    vis = np.sort(rng.choice(S, size=200, replace=False))
    rows[vis] = rng.choice(n_orig, size=200, replace=False)
    h32 = rng.standard_normal((S, d)).astype(np.float32)
    h32[vis] = o32[rows[vis]] + (rng.random((200, 1)) * 8).astype(np.float32) * h32[vis]
    hidden = wl.to_storage(h32, dtype)
    K = wl.to_storage(rng.standard_normal((H, S, D)).astype(np.float32), dtype)
    V = wl.to_storage(rng.standard_normal((H, S, D)).astype(np.float32), dtype)
    seq = np.array([0, 120, 121, 300])
    a = ref.prune_kv_mapped(hidden, orig, rows, K, V, dtype, seq, M=0.2)
    b = canon.prune_kv_mapped(hidden, orig, rows, K, V, dtype, seq, M=0.2)
    np.testing.assert_allclose(b["cos"][vis], a["cos"][vis], rtol=1e-5, atol=1e-6)
    differ = np.setxor1d(a["idx"], b["idx"])
    assert all(abs(a["cos"][s] - 0.2) < 1e-5 for s in differ)           # only decisions on the boundary may differ
    if len(differ) == 0:
        for k in ("idx", "counts", "orig_row_out", "K_out", "V_out"):
            np.testing.assert_array_equal(b[k], a[k])
    # a contiguous block with rows in order is the single-layer form, bit for bit
    lay = wl.make_kv_layout([100, 60], 5, 7, H, D)
    rows2 = np.full(lay.S, -1)
    rows2[lay.visual_positions()] = np.arange(lay.n_vis)
    hid2 = wl.to_storage(rng.standard_normal((lay.S, d)).astype(np.float32), dtype)
    hid2[lay.visual_positions()] = hidden[vis[:160]]
    K2 = wl.to_storage(rng.standard_normal((H, lay.S, D)).astype(np.float32), dtype)
    blk = canon.prune_kv(hid2, orig[rows[vis[:160]]], K2, K2, dtype, lay.seq_offsets, lay.vis_start, lay.vis_offsets)
    mp = canon.prune_kv_mapped(hid2, orig[rows[vis[:160]]], rows2, K2, K2, dtype, lay.seq_offsets)
    np.testing.assert_array_equal(mp["idx"], blk["idx"])
    np.testing.assert_array_equal(mp["counts"], blk["counts"])
    np.testing.assert_array_equal(mp["K_out"], blk["K_out"])
    np.testing.assert_array_equal(mp["cos"][lay.visual_positions()], blk["cos"])
