"""Pins of the float64 definition-level oracle (oracle/sharpv_ref.py) to things other than itself:
closed forms, hand-computed cases, invariants, brute force and library routines.  CPU only."""
import itertools
import math
import os

import numpy as np
import pytest

from oracle import sharpv_ref as ref

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def paper_facts():
    facts = {}
    for line in open(os.path.join(GOLDEN, "paper_facts.txt")):
        line = line.split("#")[0].strip()
        if "=" in line:
            k, v = line.split("=")
            facts[k.strip()] = [float(t) for t in v.split()]
    return facts


def rot2(v, theta, i=0, j=1):
    """Rotate vector v by theta in the (i, j) coordinate plane."""
    out = np.array(v, dtype=np.float64)
    c, s = math.cos(theta), math.sin(theta)
    out[..., i] = c * v[..., i] - s * v[..., j]
    out[..., j] = s * v[..., i] + c * v[..., j]
    return out


def planar(rng, n, d):
    """Rows that live in coordinates (0,1) only, so a planar rotation turns them by exactly theta."""
    x = np.zeros((n, d))
    x[:, :2] = rng.standard_normal((n, 2))
    return x


# ----------------------------------------------------------------------------- Eq.1
def test_dissim_two_forms_agree():
    rng = np.random.default_rng(0)
    a = rng.standard_normal((200, 64))
    b = rng.standard_normal((200, 64))
    np.testing.assert_allclose(ref.dissim(a, b), ref.dissim_from_cos(ref.cosine(a, b)), rtol=1e-12, atol=1e-12)


def test_dissim_special_values_and_range():
    facts = paper_facts()
    v = np.array([[3.0, 4.0, 0.0]])
    assert ref.dissim(v, 2.5 * v)[0] == pytest.approx(facts["dissim_min"][0], abs=1e-15)
    assert ref.dissim(v, np.array([[0.0, 0.0, 7.0]]))[0] == pytest.approx(math.sqrt(2.0), rel=1e-15)
    assert ref.dissim(v, -v)[0] == pytest.approx(facts["dissim_max"][0], rel=1e-15)
    rng = np.random.default_rng(1)
    dd = ref.dissim(rng.standard_normal((1000, 8)), rng.standard_normal((1000, 8)))
    assert dd.min() >= facts["dissim_min"][0] and dd.max() <= facts["dissim_max"][0]


def test_dissim_hand_value_and_chord_formula():
    # cos([1,0],[1,1]) = 1/sqrt2  ->  sqrt(2 - sqrt2)
    assert ref.dissim(np.array([[1.0, 0.0]]), np.array([[1.0, 1.0]]))[0] == pytest.approx(math.sqrt(2 - math.sqrt(2)), rel=1e-14)
    # chord of the unit circle: vectors theta apart are 2 sin(theta/2) apart
    rng = np.random.default_rng(2)
    x = planar(rng, 50, 6)
    th = rng.uniform(0, math.pi, 50)
    y = np.stack([rot2(x[i], th[i]) * (0.3 + i) for i in range(50)])
    np.testing.assert_allclose(ref.dissim(x, y), 2 * np.sin(th / 2), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(ref.cosine(x, y), np.cos(th), rtol=1e-10, atol=1e-12)


def test_cosine_is_not_symmetric_garbage():
    # asymmetric operands: a wrong normalisation (dividing by only one norm) changes the value
    a = np.array([[2.0, 0.0]])
    b = np.array([[3.0, 4.0]])
    assert ref.cosine(a, b)[0] == pytest.approx(0.6, rel=1e-15)
    assert ref.cosine(np.zeros((1, 2)), b)[0] == 0.0          # zero-norm reading
    assert ref.dissim(np.zeros((1, 2)), b)[0] == pytest.approx(math.sqrt(2.0))


# ----------------------------------------------------------------------------- Eq.2
def test_spatial_importance_hand_case_uses_raw_mean_including_self():
    # tokens (2,0) and (0,1): raw mean (1, .5).  A mean of *normalised* tokens would be (.5,.5) -> cos .7071.
    S = ref.spatial_importance(np.array([[2.0, 0.0], [0.0, 1.0]]))
    c0 = 2.0 / (2.0 * math.sqrt(1.25))
    c1 = 0.5 / (1.0 * math.sqrt(1.25))
    np.testing.assert_allclose(S, [math.sqrt(2 - 2 * c0), math.sqrt(2 - 2 * c1)], rtol=1e-14)
    # leave-one-out mean would give cos 0 for both tokens here
    assert abs(S[0] - math.sqrt(2.0)) > 0.1


def test_spatial_importance_uniform_frame_is_zero_and_scale_free():
    rng = np.random.default_rng(3)
    row = rng.standard_normal(32)
    assert np.allclose(ref.spatial_importance(np.tile(row, (7, 1))), 0.0, atol=1e-7)
    F = rng.standard_normal((9, 32))
    np.testing.assert_allclose(ref.spatial_importance(F), ref.spatial_importance(5.5 * F), rtol=1e-12)


# ----------------------------------------------------------------------------- Eq.3
def test_temporal_importance_pairs_same_slot_of_adjacent_frames():
    rng = np.random.default_rng(4)
    f, d = 12, 10
    prev = planar(rng, f, d)
    th = np.linspace(0.05, 3.0, f)                       # a different, known angle for every slot
    cur = np.stack([rot2(prev[i], th[i]) for i in range(f)])
    np.testing.assert_allclose(ref.temporal_importance(cur, prev), 2 * np.sin(th / 2), rtol=1e-10)
    # positive per-token rescaling leaves T unchanged
    sc = rng.uniform(0.1, 9, f)[:, None]
    np.testing.assert_allclose(ref.temporal_importance(cur * sc, prev), 2 * np.sin(th / 2), rtol=1e-10)


# ----------------------------------------------------------------------------- Eq.4 - Eq.6
def test_importance_is_T_plus_w_S():
    T = np.array([0.5, 1.0])
    S = np.array([0.25, 2.0])
    np.testing.assert_allclose(ref.importance(T, S, 3.0), [1.25, 7.0])
    np.testing.assert_allclose(ref.importance(T, S, 0.0), T)


def test_keep_ratio_closed_forms():
    facts = paper_facts()
    f = 196
    assert ref.keep_ratio(np.zeros(f)) == facts["ratio_min"][0]
    assert ref.keep_ratio(np.full(f, 2.0)) == pytest.approx(facts["ratio_max"][0])
    # every token turned by the same angle theta: ||T|| = 2 sin(theta/2) sqrt(f)  ->  r = sin(theta/2)
    for th in (0.1, 1.0, 2.5):
        assert ref.keep_ratio(np.full(f, 2 * math.sin(th / 2))) == pytest.approx(math.sin(th / 2), rel=1e-14)
    # it is the L2 norm (not the mean, not the L1 norm): one token at 2, rest 0 -> 2/(2 sqrt f)
    T = np.zeros(f)
    T[17] = 2.0
    assert ref.keep_ratio(T) == pytest.approx(1 / math.sqrt(f), rel=1e-14)


def test_kept_count_rounding_and_clamps():
    assert ref.kept_count(0.0, 196) == 0
    assert ref.kept_count(1.0, 196) == 196
    assert ref.kept_count(2.5 / 10, 10) == 3           # half rounds up
    assert ref.kept_count(0.2499, 10) == 2
    assert ref.kept_count(0.0, 196, min_keep=4) == 4
    ks = [ref.kept_count(r, 196) for r in np.linspace(0, 1, 2001)]
    assert all(b >= a for a, b in zip(ks, ks[1:]))      # more variation never keeps fewer tokens


def test_first_frame_equals_virtual_mean_frame():
    """Eq.6 == Eq.5 applied with a preceding frame whose every token is the frame mean."""
    rng = np.random.default_rng(5)
    f, d = 20, 24
    F1 = rng.standard_normal((f, d)) + 0.7
    virt = np.tile(F1.mean(axis=0), (f, 1))
    alone = ref.prune_tokens(F1[None].astype(np.float32), 0, np.array([0, 1]))
    both = ref.prune_tokens(np.stack([virt, F1]).astype(np.float32), 0, np.array([0, 2]))
    assert alone["ratio"][0] == pytest.approx(both["ratio"][1], rel=1e-6)
    np.testing.assert_allclose(alone["T"][0], both["T"][1], rtol=1e-5, atol=1e-6)
    np.testing.assert_allclose(alone["T"][0], alone["S"][0])
    assert alone["counts"][0] == both["counts"][1]


def test_static_and_negated_frames():
    rng = np.random.default_rng(6)
    f, d = 16, 12
    F = rng.standard_normal((f, d)).astype(np.float32)
    out = ref.prune_tokens(np.stack([F, F, -F]), 0, np.array([0, 3]))
    assert out["ratio"][1] == pytest.approx(0.0, abs=1e-7) and out["counts"][1] == 0
    assert out["ratio"][2] == pytest.approx(1.0, rel=1e-12) and out["counts"][2] == f


def test_ar1_closed_form_ratio():
    """x_t = rho x_{t-1} + sqrt(1-rho^2) eps  =>  cos -> rho, T -> sqrt(2-2rho), r -> sqrt((1-rho)/2)."""
    rng = np.random.default_rng(7)
    f, d = 64, 4096
    for rho in (0.5, 0.9, 0.97):
        a = rng.standard_normal((f, d))
        b = rho * a + math.sqrt(1 - rho * rho) * rng.standard_normal((f, d))
        T = ref.temporal_importance(b, a)
        assert ref.keep_ratio(T) == pytest.approx(math.sqrt((1 - rho) / 2), rel=0.02)
        assert np.mean(T) == pytest.approx(math.sqrt(2 - 2 * rho), rel=0.02)
    # independent frames -> sqrt(2)/2 ; iid first frame -> sqrt(2 - 2/sqrt f)/2
    a, b = rng.standard_normal((f, d)), rng.standard_normal((f, d))
    assert ref.keep_ratio(ref.temporal_importance(b, a)) == pytest.approx(math.sqrt(0.5), rel=0.02)
    assert ref.keep_ratio(ref.spatial_importance(a)) == pytest.approx(math.sqrt(2 - 2 / math.sqrt(f)) / 2, rel=0.02)


# ----------------------------------------------------------------------------- top-k
def test_select_topk_brute_force_tiny():
    rng = np.random.default_rng(8)
    for trial in range(60):
        f = int(rng.integers(1, 9))
        I = rng.integers(0, 4, f).astype(np.float64) if trial % 2 else rng.standard_normal(f)
        for k in range(f + 1):
            # best subset of size k by total score; among equals the lexicographically smallest index tuple
            best = max(itertools.combinations(range(f), k), key=lambda c: (sum(I[list(c)]), [-i for i in c]))
            assert list(ref.select_topk(I, k)) == list(best)


def test_select_topk_matches_stable_sort():
    rng = np.random.default_rng(9)
    I = np.round(rng.standard_normal(196), 1)            # many ties
    order = np.argsort(-I, kind="stable")
    for k in (0, 1, 17, 100, 196):
        assert list(ref.select_topk(I, k)) == sorted(order[:k].tolist())


# ----------------------------------------------------------------------------- whole pre-LLM stage
def _video(rng, n, f, d, rho=0.8):
    x = [rng.standard_normal((f, d))]
    for _ in range(n - 1):
        x.append(rho * x[-1] + math.sqrt(1 - rho * rho) * rng.standard_normal((f, d)))
    return np.stack(x).astype(np.float32)


def test_prune_tokens_structure_and_compaction():
    rng = np.random.default_rng(10)
    n, f, d = 5, 24, 40
    x = _video(rng, n, f, d)
    o = ref.prune_tokens(x, 0, np.array([0, n]), w=1.0)
    for t in range(n):
        assert o["counts"][t] == math.floor(o["ratio"][t] * f + 0.5)
    assert np.all(np.diff(o["idx"]) > 0)
    assert o["offsets"][-1] == len(o["idx"]) == o["counts"].sum()
    np.testing.assert_array_equal(o["offsets"][1:], np.cumsum(o["counts"]))
    np.testing.assert_array_equal(o["out_feats"], np.take(x.reshape(n * f, d), o["idx"], axis=0))
    np.testing.assert_allclose(o["I"], o["T"] + o["S"])
    # kept tokens of a frame are exactly its highest-scoring ones
    for t in range(n):
        sel = o["idx"][o["offsets"][t]:o["offsets"][t + 1]] - t * f
        rest = np.setdiff1d(np.arange(f), sel)
        if len(sel) and len(rest):
            assert o["I"][t, sel].min() >= o["I"][t, rest].max()


def test_prune_tokens_permutation_and_scaling():
    rng = np.random.default_rng(11)
    n, f, d = 4, 18, 32
    x = _video(rng, n, f, d)
    base = ref.prune_tokens(x, 0, np.array([0, n]))
    perm = rng.permutation(f)
    p = ref.prune_tokens(x[:, perm], 0, np.array([0, n]))
    np.testing.assert_allclose(p["I"], base["I"][:, perm], rtol=1e-9)
    np.testing.assert_array_equal(p["counts"], base["counts"])
    for t in range(n):
        a = set((base["idx"][base["offsets"][t]:base["offsets"][t + 1]] - t * f).tolist())
        b = set(perm[p["idx"][p["offsets"][t]:p["offsets"][t + 1]] - t * f].tolist())
        assert a == b
    s = ref.prune_tokens(x * np.float32(4.0), 0, np.array([0, n]))     # exact power-of-two scaling
    np.testing.assert_allclose(s["I"], base["I"], rtol=1e-9)
    np.testing.assert_array_equal(s["idx"], base["idx"])


def test_prune_tokens_ragged_batch_is_per_video():
    rng = np.random.default_rng(12)
    f, d = 10, 16
    vids = [_video(rng, n, f, d) for n in (3, 1, 4)]
    offs = np.array([0, 3, 4, 8])
    packed = ref.prune_tokens(np.concatenate(vids), 0, offs)
    pos = 0
    for v, lo in zip(vids, offs[:-1]):
        solo = ref.prune_tokens(v, 0, np.array([0, len(v)]))
        np.testing.assert_allclose(packed["I"][lo:lo + len(v)], solo["I"])
        np.testing.assert_array_equal(packed["counts"][lo:lo + len(v)], solo["counts"])
        np.testing.assert_array_equal(packed["idx"][pos:pos + len(solo["idx"])], solo["idx"] + lo * f)
        pos += len(solo["idx"])
    assert pos == len(packed["idx"])


def test_manual_threshold_mode():
    facts = paper_facts()
    rng = np.random.default_rng(13)
    n, f, d = 4, 30, 64
    x = _video(rng, n, f, d, rho=0.3)
    last = None
    for K in (0.5, 1.0, facts["K_manual"][0], 2.5, 10.0):
        o = ref.prune_tokens(x, 0, np.array([0, n]), mode=1, K=K)
        kept = set(o["idx"].tolist())
        assert kept == set(np.nonzero(o["I"].reshape(-1) >= K)[0].tolist())
        if last is not None:
            assert kept <= last                      # larger K keeps a subset
        last = kept
    assert len(last) == 0                            # I <= 2 + w*2 = 4 < 10


def test_one_minus_cos_closed_forms_and_relation_to_eq1():
    # Sec. 3.1 (Dissimilarity Computation Module): 1 - cos as the stand-in for Eq.1
    v = np.array([[3.0, 4.0, 0.0]])
    assert ref.one_minus_cos(v, 2.5 * v)[0] == pytest.approx(0.0, abs=1e-15)
    assert ref.one_minus_cos(v, np.array([[0.0, 0.0, 7.0]]))[0] == pytest.approx(1.0, abs=1e-15)
    assert ref.one_minus_cos(v, -v)[0] == pytest.approx(2.0, rel=1e-15)
    assert ref.one_minus_cos(v, np.zeros((1, 3)))[0] == 1.0                 # zero-norm reading: cos 0
    # vectors theta apart: 1 - cos(theta) = 2 sin^2(theta/2) (versine), half the squared chord of Eq.1
    rng = np.random.default_rng(21)
    x = planar(rng, 60, 5)
    th = rng.uniform(0, math.pi, 60)
    y = np.stack([rot2(x[i], th[i]) * (0.2 + i) for i in range(60)])
    np.testing.assert_allclose(ref.one_minus_cos(x, y), 2 * np.sin(th / 2) ** 2, rtol=1e-10, atol=1e-12)
    a = rng.standard_normal((300, 48))
    b = rng.standard_normal((300, 48))
    np.testing.assert_allclose(ref.one_minus_cos(a, b), ref.dissim(a, b) ** 2 / 2, rtol=1e-12, atol=1e-12)
    # not symmetric in a dropped-sign sense: turning one vector round mirrors the value about 1
    np.testing.assert_allclose(ref.one_minus_cos(a, -b), 2.0 - ref.one_minus_cos(a, b), rtol=1e-12, atol=1e-12)


def test_manual_mode_with_one_minus_cos():
    rng = np.random.default_rng(22)
    n, f, d = 5, 24, 32
    x = _video(rng, n, f, d, rho=0.4)
    fo = np.array([0, 2, n])                         # two videos: frames 0 and 2 take T := S
    xs = x.astype(np.float64)
    # scores by hand from library cosines
    S = np.empty((n, f)); T = np.empty((n, f))
    for t in range(n):
        m = xs[t].mean(axis=0)
        for i in range(f):
            S[t, i] = 1 - xs[t, i] @ m / (np.linalg.norm(xs[t, i]) * np.linalg.norm(m))
            if t in (0, 2):
                T[t, i] = S[t, i]
            else:
                T[t, i] = 1 - xs[t, i] @ xs[t - 1, i] / (np.linalg.norm(xs[t, i]) * np.linalg.norm(xs[t - 1, i]))
    for w, K in ((1.0, 0.8), (0.0, 0.5), (2.0, 1.2)):
        o = ref.prune_tokens(x, 0, fo, w=w, mode=1, K=K, measure=1)
        np.testing.assert_allclose(o["S"], S, rtol=1e-11, atol=1e-12)
        np.testing.assert_allclose(o["T"], T, rtol=1e-11, atol=1e-12)
        I = T + w * S
        near = np.abs(I - K) < 1e-9
        assert not near.any()
        assert o["idx"].tolist() == np.nonzero((I >= K).reshape(-1))[0].tolist()
        assert o["counts"].tolist() == (I >= K).sum(axis=1).tolist()
        np.testing.assert_array_equal(o["out_feats"], x.reshape(n * f, d)[o["idx"]])
    # w = 0: 1 - cos = Dissim^2 / 2 is monotone in Dissim, so threshold K here keeps what sqrt(2K) keeps under Eq.1
    for K in (0.5, 0.7, 1.0):
        a = ref.prune_tokens(x, 0, fo, w=0.0, mode=1, K=K, measure=1)
        b = ref.prune_tokens(x, 0, fo, w=0.0, mode=1, K=math.sqrt(2 * K), measure=0)
        assert a["idx"].tolist() == b["idx"].tolist() and 0 < len(a["idx"]) < n * f
    # the pairing of Sec. 3.1: the rescaled cosine comes with the fixed threshold only
    with pytest.raises(ValueError):
        ref.prune_tokens(x, 0, fo, mode=0, measure=1)
    with pytest.raises(ValueError):
        ref.prune_tokens(x, 0, fo, mode=1, measure=2)


# ----------------------------------------------------------------------------- Eq.7
def _kv_case(rng, n_vis, tb, ta, d, H=2, D=8):
    S = tb + n_vis + ta
    orig = rng.standard_normal((n_vis, d)).astype(np.float32)
    hidden = rng.standard_normal((S, d)).astype(np.float32)
    K = rng.standard_normal((H, S, D)).astype(np.float32)
    V = rng.standard_normal((H, S, D)).astype(np.float32)
    lay = (np.array([0, S]), np.array([tb]), np.array([0, n_vis]))
    return orig, hidden, K, V, lay


def test_kv_identity_negation_and_threshold_extremes():
    facts = paper_facts()
    M = facts["M_default"][0]
    rng = np.random.default_rng(14)
    n_vis, tb, ta, d = 40, 3, 5, 32
    orig, hidden, K, V, lay = _kv_case(rng, n_vis, tb, ta, d)
    S = tb + n_vis + ta
    hidden[tb:tb + n_vis] = orig                                   # decoder input: nothing degraded
    o = ref.prune_kv(hidden, orig, K, V, 0, *lay, M=M)
    np.testing.assert_allclose(o["cos"], 1.0, rtol=1e-12)
    np.testing.assert_array_equal(o["idx"], np.arange(S))
    np.testing.assert_array_equal(o["K_out"], K)
    hidden[tb:tb + n_vis] = -orig                                  # fully degraded
    o = ref.prune_kv(hidden, orig, K, V, 0, *lay, M=M)
    np.testing.assert_array_equal(o["idx"], np.r_[np.arange(tb), np.arange(tb + n_vis, S)])
    assert o["counts"][0] == tb + ta
    hidden[tb:tb + n_vis] = rng.standard_normal((n_vis, d))
    assert len(ref.prune_kv(hidden, orig, K, V, 0, *lay, M=-1.0)["idx"]) == S      # cos >= -1 always
    o = ref.prune_kv(hidden, orig, K, V, 0, *lay, M=1.5)                            # cos <= 1 < M
    np.testing.assert_array_equal(o["idx"], np.r_[np.arange(tb), np.arange(tb + n_vis, S)])
    np.testing.assert_array_equal(o["V_out"], V[:, o["idx"], :])


def test_kv_known_angles_pick_exactly_the_tokens_below_threshold():
    rng = np.random.default_rng(15)
    n_vis, tb, ta, d = 64, 4, 2, 16
    orig, hidden, K, V, lay = _kv_case(rng, n_vis, tb, ta, d)
    orig = planar(rng, n_vis, d).astype(np.float32)
    th = rng.uniform(0, math.pi, n_vis)
    hidden[tb:tb + n_vis] = np.stack([3.0 * rot2(orig[p].astype(np.float64), th[p]) for p in range(n_vis)])
    # text rows point *away* from everything: they must still be kept
    hidden[:tb] = -1.0
    M = 0.2
    o = ref.prune_kv(hidden, orig, K, V, 0, *lay, M=M)
    np.testing.assert_allclose(o["cos"], np.cos(th), atol=1e-6)
    expect = np.r_[np.arange(tb), tb + np.nonzero(~(np.cos(th) < M))[0], np.arange(tb + n_vis, tb + n_vis + ta)]
    np.testing.assert_array_equal(o["idx"], expect)
    np.testing.assert_array_equal(o["K_out"], np.take(K, expect, axis=1))


def test_kv_additive_noise_closed_form_and_monotone_in_M():
    rng = np.random.default_rng(16)
    n_vis, tb, ta, d = 128, 2, 2, 4096
    orig, hidden, K, V, lay = _kv_case(rng, n_vis, tb, ta, d)
    sigma = np.linspace(0.0, 8.0, n_vis)
    hidden[tb:tb + n_vis] = orig + sigma[:, None] * rng.standard_normal((n_vis, d))
    o = ref.prune_kv(hidden, orig, K, V, 0, *lay, M=0.2)
    np.testing.assert_allclose(o["cos"], 1 / np.sqrt(1 + sigma ** 2), atol=0.05)
    kept = [len(ref.prune_kv(hidden, orig, K, V, 0, *lay, M=m)["idx"]) for m in (-1, 0, 0.1, 0.2, 0.5, 0.9, 1.1)]
    assert all(b <= a for a, b in zip(kept, kept[1:]))


def test_kv_ragged_and_layer_mean_mode():
    rng = np.random.default_rng(17)
    d, H, D = 24, 2, 4
    nvs, tb, ta = [5, 9], 2, 3
    seq = np.array([0, tb + 5 + ta, 2 * (tb + ta) + 14])
    vs = np.array([tb, tb])
    vo = np.array([0, 5, 14])
    orig = rng.standard_normal((14, d)).astype(np.float32)
    hidden = rng.standard_normal((seq[-1], d)).astype(np.float32)
    hidden[tb:tb + 5] = orig[:5]                                   # sequence 0: intact
    hidden[seq[1] + tb:seq[1] + tb + 9] = -orig[5:]                # sequence 1: degraded
    K = rng.standard_normal((H, seq[-1], D)).astype(np.float32)
    for mode in (0, 1):
        o = ref.prune_kv(hidden, orig, K, K, 0, seq, vs, vo, M=0.2, kv_mode=mode)
        np.testing.assert_array_equal(o["counts"], [tb + 5 + ta, tb + ta])
        np.testing.assert_allclose(o["mean_cos"], [1.0, -1.0], rtol=1e-9)
    # layer-mean mode is all-or-nothing per sequence: a half-degraded sequence with mean above M keeps all
    hidden[seq[1] + tb:seq[1] + tb + 9] = orig[5:]
    hidden[seq[1] + tb] = -orig[5]
    o = ref.prune_kv(hidden, orig, K, K, 0, seq, vs, vo, M=0.2, kv_mode=1)
    assert o["counts"][1] == tb + 9 + ta
    o = ref.prune_kv(hidden, orig, K, K, 0, seq, vs, vo, M=0.2, kv_mode=0)
    assert o["counts"][1] == tb + 8 + ta


def test_widen_bf16_is_exact():
    bits = np.array([0x3F80, 0xC000, 0x0000, 0x3EAB, 0x7F7F], dtype=np.uint16)
    np.testing.assert_array_equal(ref.widen(bits, 1), [1.0, -2.0, 0.0, 0.333984375, 3.3895313892515355e38])


def test_retention_figures():
    r = ref.retention(np.array([10, 30]), 100, kept_kv=50, S=200)
    assert r["VR"] == pytest.approx(0.2) and r["MR"] == pytest.approx(0.25) and r["budget"] == pytest.approx(0.05)


# ----------------------------------------------------------------------------- rotary re-encoding of the kept K rows
def _rope_tables(L, D, base=10000.0):
    theta = base ** (-2.0 * np.arange(D // 2) / D)
    ang = np.arange(L)[:, None] * theta[None, :]
    return theta, np.cos(ang), np.sin(ang)


def _rotate_complex(k0, pos, theta, layout):
    """Textbook rotary embedding via complex numbers: pair (x, y) -> (x + iy) * exp(i * pos * theta)."""
    D = k0.shape[-1]
    ia = np.arange(D // 2) if layout == 0 else 2 * np.arange(D // 2)
    ib = ia + D // 2 if layout == 0 else ia + 1
    z = (k0[..., ia] + 1j * k0[..., ib]) * np.exp(1j * np.asarray(pos)[..., None] * theta)
    out = np.empty_like(k0)
    out[..., ia], out[..., ib] = z.real, z.imag
    return out


@pytest.mark.parametrize("layout", [0, 1])
def test_rope_reencode_moves_a_row_to_its_new_position(layout):
    # rows embedded for their old positions come out embedded for their ranks among the kept rows, per sequence
    rng = np.random.default_rng(31 + layout)
    H, D = 3, 16
    seq = np.array([0, 11, 30])                        # two sequences of 11 and 19 positions
    idx = np.array([0, 1, 4, 9, 10, 11, 13, 14, 22, 29])
    pos_old = np.array([0, 1, 4, 9, 10, 0, 2, 3, 11, 18])
    pos_new = np.array([0, 1, 2, 3, 4, 0, 1, 2, 3, 4])
    theta, ct, st = _rope_tables(32, D)
    k0 = rng.standard_normal((H, len(idx), D))
    K_old = _rotate_complex(k0, np.broadcast_to(pos_old, (H, len(idx))), theta, layout)
    got = ref.rope_reencode(K_old.astype(np.float32), 0, idx, seq, ct, st, layout)
    want = _rotate_complex(k0, np.broadcast_to(pos_new, (H, len(idx))), theta, layout)
    np.testing.assert_allclose(got, want, atol=2e-6)
    # and it is not a no-op: the rows that moved differ from their input
    moved = pos_old != pos_new
    assert np.all(np.abs(got[:, moved] - K_old[:, moved]).max(axis=-1) > 1e-3)


def test_rope_reencode_identity_norms_batches_and_layouts():
    rng = np.random.default_rng(37)
    H, D, S = 2, 8, 20
    theta, ct, st = _rope_tables(S, D)
    K = rng.standard_normal((H, S, D)).astype(np.float32)
    seq = np.array([0, S])
    # nothing pruned: every delta is 0 and the rows come back unchanged
    np.testing.assert_array_equal(ref.rope_reencode(K, 0, np.arange(S), seq, ct, st, 0), K.astype(np.float64))
    # a rotation: the norm of every pair, hence of every row, is preserved
    idx = np.array([2, 3, 7, 8, 15, 19])
    out = ref.rope_reencode(K[:, idx], 0, idx, seq, ct, st, 0)
    np.testing.assert_allclose(np.linalg.norm(out, axis=-1), np.linalg.norm(K[:, idx].astype(np.float64), axis=-1),
                               rtol=1e-7)
    # attention logits between re-encoded keys depend on the new distance only: <R(a)q, R(b)k> = <R(a-b)q, k>
    q = rng.standard_normal(D)
    for a, b in ((0, 3), (2, 5)):
        ka = _rotate_complex(K[0, idx[a]].astype(np.float64), 0, theta, 0)       # un-embedded stand-in
        lhs = _rotate_complex(q, b, theta, 0) @ _rotate_complex(ka, a, theta, 0)
        rhs = _rotate_complex(q, b - a, theta, 0) @ ka
        assert lhs == pytest.approx(rhs, rel=1e-9)
    # a packed batch is the concatenation of its sequences (delta restarts at each sequence)
    seq2 = np.array([0, 9, S])
    idx2 = np.array([1, 4, 8, 9, 12, 19])
    both = ref.rope_reencode(K[:, idx2], 0, idx2, seq2, ct, st, 0)
    first = ref.rope_reencode(K[:, idx2[:3]], 0, idx2[:3], np.array([0, 9]), ct, st, 0)
    second = ref.rope_reencode(K[:, idx2[3:]], 0, idx2[3:] - 9, np.array([0, S - 9]), ct, st, 0)
    np.testing.assert_array_equal(both, np.concatenate([first, second], axis=1))
    # the two pairings are the same rotation up to a fixed shuffle of the head dimension
    perm = np.empty(D, dtype=int)
    perm[0::2], perm[1::2] = np.arange(D // 2), np.arange(D // 2) + D // 2    # interleaved slot <- half-split slot
    inter = ref.rope_reencode(K[:, idx][:, :, perm], 0, idx, seq, ct, st, 1)
    np.testing.assert_array_equal(inter, out[:, :, perm])


# ----------------------------------------------------------------------------- pruning carried from layer to layer
def _mapped_case(seed, S=60, n_orig=40, d=24, H=2, D=4):
    rng = np.random.default_rng(seed)
    orig = rng.standard_normal((n_orig, d)).astype(np.float32)
    rows = np.full(S, -1)
    vis = np.sort(rng.choice(S, size=n_orig, replace=False))
    rows[vis] = rng.permutation(n_orig)                      # tokens refer to shuffled rows of orig
    hidden = rng.standard_normal((S, d)).astype(np.float32)
    sig = rng.random(n_orig) * 8
    hidden[vis] = orig[rows[vis]] + sig[:, None] * hidden[vis]
    K = rng.standard_normal((H, S, D)).astype(np.float32)
    V = rng.standard_normal((H, S, D)).astype(np.float32)
    return hidden, orig, rows, vis, K, V


def test_mapped_kv_pruning_reduces_to_the_block_form_and_to_library_cosines():
    # a contiguous visual block with rows in order is exactly the single-layer form
    rng = np.random.default_rng(51)
    tb, nv, ta, d = 3, 30, 4, 16
    S = tb + nv + ta
    orig = rng.standard_normal((nv, d)).astype(np.float32)
    hidden = rng.standard_normal((S, d)).astype(np.float32)
    hidden[tb:tb + nv] = orig + rng.random((nv, 1)).astype(np.float32) * 8 * hidden[tb:tb + nv]
    K = rng.standard_normal((2, S, 4)).astype(np.float32)
    rows = np.full(S, -1); rows[tb:tb + nv] = np.arange(nv)
    a = ref.prune_kv(hidden, orig, K, K, 0, np.array([0, S]), np.array([tb]), np.array([0, nv]), M=0.2)
    b = ref.prune_kv_mapped(hidden, orig, rows, K, K, 0, np.array([0, S]), M=0.2)
    np.testing.assert_array_equal(a["idx"], b["idx"])
    np.testing.assert_array_equal(a["counts"], b["counts"])
    np.testing.assert_array_equal(a["K_out"], b["K_out"])
    np.testing.assert_allclose(b["cos"][tb:tb + nv], a["cos"], rtol=1e-12)
    assert np.all(np.isnan(b["cos"][:tb])) and np.all(np.isnan(b["cos"][tb + nv:]))
    # shuffled rows: the cosines are those of the rows gathered with numpy, via scipy's cosine distance
    from scipy.spatial.distance import cosine as cosine_distance
    hidden, orig, rows, vis, K, V = _mapped_case(52)
    o = ref.prune_kv_mapped(hidden, orig, rows, K, V, 0, np.array([0, 25, 60]), M=0.2)
    want = np.array([1.0 - cosine_distance(hidden[s].astype(np.float64), orig[rows[s]].astype(np.float64)) for s in vis])
    np.testing.assert_allclose(o["cos"][vis], want, rtol=1e-10)
    kept = np.ones(60, bool); kept[vis] = ~(want < 0.2)
    np.testing.assert_array_equal(o["idx"], np.nonzero(kept)[0])
    np.testing.assert_array_equal(o["counts"], [kept[:25].sum(), kept[25:].sum()])
    np.testing.assert_array_equal(o["orig_row_out"], rows[kept])
    np.testing.assert_array_equal(o["V_out"], V[:, kept])
    # entries outside [0, n_orig) are non-visual positions: always kept, no cosine
    bad = rows.copy(); bad[vis[:3]] = [40, 999, -7]
    o2 = ref.prune_kv_mapped(hidden, orig, bad, K, V, 0, np.array([0, 60]), M=2.0)
    np.testing.assert_array_equal(o2["idx"], np.sort(np.concatenate([np.nonzero(rows < 0)[0], vis[:3]])))
    assert np.all(o2["orig_row_out"] == -1)


def test_pruning_carried_over_layers_is_the_intersection_of_the_layer_masks():
    # three layers on shrinking sequences == per-layer Eq.7 masks on the full sequence, intersected
    rng = np.random.default_rng(53)
    hidden0, orig, rows, vis, K, V = _mapped_case(54, S=90, n_orig=70)
    S = 90
    seq = np.array([0, 40, 90])
    layers = [hidden0]
    for l in range(2):                                                   # later layers drift further
        h = layers[-1].copy()
        h[vis] += rng.standard_normal((len(vis), h.shape[1])).astype(np.float32) * rng.random((len(vis), 1)) * 6
        layers.append(h)
    alive = np.arange(S)
    cur_rows, cur_seq = rows.copy(), seq.copy()
    want_alive = np.ones(S, bool)
    for h_full in layers:
        o = ref.prune_kv_mapped(h_full[alive], orig, cur_rows, K[:, alive], V[:, alive], 0, cur_seq, M=0.2)
        c_full = np.array([ref.cosine(h_full[s].astype(np.float64)[None], orig[rows[s]].astype(np.float64)[None])[0]
                           for s in vis])
        m = np.ones(S, bool); m[vis] = ~(c_full < 0.2)
        want_alive &= m
        np.testing.assert_array_equal(alive[o["idx"]], np.nonzero(want_alive)[0])
        np.testing.assert_array_equal(o["K_out"], K[:, want_alive])
        alive = alive[o["idx"]]
        cur_rows = o["orig_row_out"]
        np.testing.assert_array_equal(cur_rows, rows[want_alive])
        cur_seq = np.concatenate([[0], np.cumsum(o["counts"])])
    assert 0 < want_alive.sum() < S
