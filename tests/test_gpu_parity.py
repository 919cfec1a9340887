"""GPU parity: the HIP library, called through its C ABI, against the CPU oracles on the same
seeded inputs.

Bars: kept counts, kept-index lists, compacted features / K / V, scores I, ratios and cosines are
compared BIT-EXACTLY with the float32 canonical-order oracle (same precision, same order of
roundings); scores and cosines are also compared with the float64 definition within 1e-3 relative
(absolute floor 1e-4 where 2 - 2cos cancels near zero)."""
import json
import os

import numpy as np
import pytest
import torch

import margins
from oracle import canon, sharpv_ref as ref
from paper_2511_08003_amd import sharpv, workloads as wl

pytestmark = pytest.mark.gpu

RTOL, ATOL = 1e-3, 1e-4
GOLD_MARGINS = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "margin_audit.json")))


def dev(a: np.ndarray, dtype: int) -> torch.Tensor:
    if dtype == wl.BF16:
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).view(torch.bfloat16).cuda()
    return torch.from_numpy(np.ascontiguousarray(a, np.float32)).cuda()


def host(t: torch.Tensor, dtype: int) -> np.ndarray:
    t = t.contiguous()
    if dtype == wl.BF16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def i32(a) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, np.int32)).cuda()


def run_tokens(feats: np.ndarray, dtype: int, frame_offsets, **over):
    n, f, d = feats.shape
    fo = None if frame_offsets is None or len(frame_offsets) == 2 else i32(frame_offsets)
    got = sharpv.prune_tokens(dev(feats, dtype), fo, **over)
    torch.cuda.synchronize()
    return got


def check_tokens(feats, dtype, frame_offsets, ref_frames=None, **over):
    """Runs the GPU path and both oracles; returns the canonical-oracle result."""
    n, f, d = feats.shape
    offs = np.asarray([0, n] if frame_offsets is None else frame_offsets, np.int32)
    kw = {k: over[k] for k in ("w", "mode", "K", "min_keep", "measure") if k in over}
    got = run_tokens(feats, dtype, offs, **kw)
    exp = canon.prune_tokens(feats, dtype, offs, **kw)
    np.testing.assert_array_equal(got["counts"].cpu().numpy(), exp["counts"])
    np.testing.assert_array_equal(got["offsets"].cpu().numpy(), exp["offsets"])
    np.testing.assert_array_equal(got["idx"].cpu().numpy(), exp["idx"])
    np.testing.assert_array_equal(host(got["out_feats"], dtype), exp["out_feats"])
    np.testing.assert_array_equal(got["I"].cpu().numpy(), exp["I"])
    np.testing.assert_array_equal(got["ratio"].cpu().numpy(), exp["ratio"])
    # float64 definition on (a prefix of) the frames
    m = n if ref_frames is None else min(n, ref_frames)
    cut = [o for o in offs if o < m] + [m]
    a = ref.prune_tokens(feats[:m], dtype, np.asarray(cut), **kw)
    np.testing.assert_allclose(got["I"].cpu().numpy()[:m], a["I"], rtol=RTOL, atol=ATOL)
    np.testing.assert_allclose(got["ratio"].cpu().numpy()[:m], a["ratio"], rtol=RTOL, atol=ATOL)
    if m == n and kw.get("mode", 0) == 0:
        # the GPU's kept counts and kept sets against the float64 definition: they may differ only where
        # the definition's own value sits within float32 error of the decision's boundary
        exp["audit"] = margins.audit_token_decisions(a, got["counts"].cpu().numpy(), got["idx"].cpu().numpy(),
                                                     got["offsets"].cpu().numpy(), f)
        exp["audit"].update(margins.token_margins(a, f))
    return exp


def run_kv(hidden, orig, K, V, dtype, lay: wl.KVLayout, ragged=None, mean_cos=False, **over):
    ragged = lay.B > 1 if ragged is None else ragged
    kw = dict(over)
    if ragged:
        kw.update(seq_offsets=i32(lay.seq_offsets), vis_start=i32(lay.vis_start), vis_offsets=i32(lay.vis_offsets))
    else:
        kw.update(vis_start0=int(lay.vis_start[0]))
    got = sharpv.prune_kv(dev(hidden, dtype), dev(orig, dtype), dev(K, dtype), dev(V, dtype), mean_cos=mean_cos,
                          n_vis=lay.n_vis, **kw)
    torch.cuda.synchronize()
    return got


def check_kv(hidden, orig, K, V, dtype, lay, ragged=None, cos64=None, **over):
    kw = {k: over[k] for k in ("M", "kv_mode") if k in over}
    got = run_kv(hidden, orig, K, V, dtype, lay, ragged=ragged, mean_cos=True, **kw)
    args = (hidden, orig, K, V, dtype, lay.seq_offsets, lay.vis_start, lay.vis_offsets)
    exp = canon.prune_kv(*args, **kw)
    np.testing.assert_array_equal(got["counts"].cpu().numpy(), exp["counts"])
    np.testing.assert_array_equal(got["idx"].cpu().numpy(), exp["idx"])
    np.testing.assert_array_equal(got["cos"].cpu().numpy(), exp["cos"][:lay.n_vis])
    np.testing.assert_array_equal(got["mean_cos"].cpu().numpy(), exp["mean_cos"])
    np.testing.assert_array_equal(host(got["K_out"], dtype), exp["K_out"])
    np.testing.assert_array_equal(host(got["V_out"], dtype), exp["V_out"])
    if cos64 is None:
        cos64 = ref.prune_kv(hidden, orig, K, V, dtype, lay.seq_offsets, lay.vis_start, lay.vis_offsets, **kw)["cos"]
    np.testing.assert_allclose(got["cos"].cpu().numpy(), cos64, rtol=RTOL, atol=ATOL)
    if kw.get("kv_mode", 0) == 0:
        # the GPU's Eq.7 decisions against the float64 cosines: only tokens within float32 error of M may differ
        kept = margins.kept_visual_mask(got["idx"].cpu().numpy(), lay.seq_offsets, lay.vis_start, lay.vis_offsets)
        exp["audit"] = margins.audit_kv_decisions(cos64, kw.get("M", 0.2), kept)
    return exp


# ----------------------------------------------------------------------------- the five configurations
@pytest.fixture(scope="module")
def workloads():
    cache = {}

    def get(i):
        if i not in cache:
            cfg = wl.config(i)
            cache.clear()                       # one big workload at a time
            cache[i] = (cfg, wl.tokens_for(cfg, threads=8))
        return cache[i]
    return get


@pytest.mark.parametrize("index", [1, 2, 3, 4, 5, 6, 7, 8])
def test_prune_tokens_on_config(workloads, index):
    cfg, tok = workloads(index)
    print(f"config {index}: {cfg.name} frames={tok.n_total} f={cfg.f} d={cfg.d}", flush=True)
    exp = check_tokens(tok.feats, cfg.dtype, tok.frame_offsets)          # float64 definition on every frame
    vr = exp["counts"].sum() / (tok.n_total * cfg.f)
    assert 0.02 < vr < 0.9
    # the margin audit of this configuration is the one on record (tests/golden/margin_audit.json)
    want = GOLD_MARGINS[str(index)]["stage1"]
    print(f"config {index} margin audit: {exp['audit']}", flush=True)
    assert {k: exp["audit"][k] for k in ("k_fragile", "topk_fragile", "k_differs", "sets_differ")} == \
        {k: want[k] for k in ("k_fragile", "topk_fragile", "k_differs", "sets_differ")}


@pytest.mark.parametrize("index", [1, 2, 3, 4, 5, 6, 7, 8])
def test_prune_kv_on_config(workloads, index):
    cfg, tok = workloads(index)
    lay = wl.kv_layout_for(cfg)
    orig = tok.feats.reshape(-1, cfg.d)
    orig32 = wl.storage_to_f32(tok.feats, tok.dtype).reshape(-1, cfg.d)
    for layer in cfg.kv_layers:                      # every evaluated layer (all 28 of the 256-frame video)
        kv = wl.kv_layer_for(cfg, tok, layer, threads=16, orig32=orig32)
        cos64 = margins.cos64_rows(kv["hidden"], orig, cfg.dtype, lay.seq_offsets, lay.vis_start, lay.vis_offsets,
                                   threads=16)
        exp = check_kv(kv["hidden"], orig, kv["K"], kv["V"], cfg.dtype, lay, cos64=cos64)
        print(f"config {index} layer {layer}: S={lay.S} n_vis={lay.n_vis} kept={len(exp['idx'])} "
              f"audit={exp['audit']}", flush=True)
        want = GOLD_MARGINS[str(index)]["kv"][str(layer)]
        assert (exp["audit"]["near_M"], exp["audit"]["differs"]) == (want["near_M"], want["differs"])
        if layer == 0 and cfg.drift == "layer":
            assert len(exp["idx"]) == lay.S          # decoder input: nothing degraded yet


# ----------------------------------------------------------------------------- shapes and edge cases, stage 1
def small_video(seed, n, f, d, dtype, rho=0.8, cuts=()):
    spec = wl.VideoSpec(n=n, rho=np.full(n, rho), cuts=tuple(cuts), seed=seed)
    return wl.make_tokens([spec], f, d, dtype, threads=2)


@pytest.mark.parametrize("n,f,d,dtype", [
    (1, 196, 3584, wl.BF16),      # a single frame: only the first-frame rule
    (3, 1, 64, wl.BF16),          # one token per frame
    (2, 1024, 64, wl.BF16),       # the largest frame
    (5, 144, 4096, wl.BF16),      # PLLaVA-7B shape (Table 2)
    (6, 196, 896, wl.BF16),       # LLaVA-OV-0.5B shape (Table 2): ragged last block
    (4, 33, 8, wl.F32),           # a single chunk per row
    (4, 65, 264, wl.F32),         # one block + one chunk
    (7, 100, 520, wl.BF16),
    (40, 50, 1024, wl.F32),
    (3, 208, 256, wl.BF16),       # the tallest frame the fused kernel takes, all rows of every thread inside
    (3, 209, 256, wl.BF16),       # one row more: the two-kernel path
    (4, 17, 512, wl.BF16),        # two rows per thread, the second almost empty
    (9, 48, 264, wl.BF16),        # three rows per thread (odd), a second slab of one chunk
    (5, 160, 2056, wl.BF16),      # ten rows per thread (two rows left over after the four-row trees)
    (11, 112, 768, wl.BF16),      # seven rows per thread (three left over)
    (4, 80, 256, wl.BF16),        # 5, 6, 11 and 12 rows per thread of the fused kernel
    (5, 90, 512, wl.BF16),
    (3, 176, 264, wl.BF16),
    (6, 192, 256, wl.BF16),
    (3, 40, 65536, wl.BF16),      # the widest row: 256 slabs
    (2, 300, 8200, wl.F32),       # two-kernel path, 33 blocks with a ragged last one
    (4100, 3, 16, wl.BF16),       # more frames than the compaction stages offsets for
    (5000, 4, 8, wl.F32),
    (4096, 4, 256, wl.BF16),      # fused kernel, 16 frames per workgroup on 256 compute units: exactly one window of shares
    (4352, 5, 256, wl.BF16),      # 17 per workgroup: a full window and one frame more
    (8448, 3, 256, wl.BF16),      # 33: two windows and one
    (2100, 6, 512, wl.BF16),      # two slabs, runs of 16-17 frames, one of them across the slab boundary
    # workgroups whose share crosses a slab boundary (runs of 8-9 pairs on 256 compute units): the part before the
    # boundary has an even or odd number of frames, the slab behind it is full or ragged
    (701, 20, 520, wl.BF16),      # 6 frames, then a full slab; 3 frames, then the ragged last slab (one chunk)
    (705, 20, 768, wl.BF16),      # three full slabs: 6 frames before the first boundary, 7 before the second
    (702, 20, 768, wl.BF16),      # 4 frames, then 2 frames before the last slab
    # the two-kernel path (frames taller than 208 tokens, float32): sweeps per row, ragged last sweeps, runs of frames
    (3, 300, 2056, wl.BF16),      # five sweeps, the last one ragged
    (2, 210, 4096, wl.BF16),      # eight full sweeps: the widest row that is unrolled
    (2, 250, 3080, wl.BF16),      # seven sweeps, ragged
    (2, 222, 4104, wl.BF16),      # one chunk past the unrolled sweeps: the looped row kernel
    (60, 300, 264, wl.BF16),      # runs of five frames per wavefront, twelve runs
    (101, 209, 64, wl.BF16),      # runs of six, the last run shorter; 209 slots = 52 workgroups and one wavefront more
    (3, 40, 2048, wl.F32),        # float32, four full sweeps
    (3, 40, 1800, wl.F32),        # float32, four sweeps, ragged
    (2, 30, 2056, wl.F32),        # float32 past the unrolled sweeps
    (90, 50, 520, wl.F32),        # float32, runs of two frames
])
def test_prune_tokens_shapes(n, f, d, dtype):
    tok = small_video(500 + n * 7 + f, n, f, d, dtype, cuts=(n // 2,) if n > 2 else ())
    check_tokens(tok.feats, dtype, None)


def test_prune_tokens_beyond_four_gib_of_features():
    """3100 frames of the model shape are 4.36e9 bytes: byte offsets pass 2^32 (and the frame count passes
    what the compaction scans by itself)."""
    n, f, d = 3100, 196, 3584
    spec = wl.VideoSpec(n=n, rho=np.full(n, 0.9), cuts=tuple(range(50, n, 97)), seed=4242)
    tok = wl.make_tokens([spec], f, d, wl.BF16, threads=16)
    assert tok.feats.nbytes > 2**32
    got = sharpv.prune_tokens(dev(tok.feats, wl.BF16))
    torch.cuda.synchronize()
    exp = canon.prune_tokens(tok.feats, wl.BF16, tok.frame_offsets)
    np.testing.assert_array_equal(got["counts"].cpu().numpy(), exp["counts"])
    np.testing.assert_array_equal(got["idx"].cpu().numpy(), exp["idx"])
    np.testing.assert_array_equal(got["I"].cpu().numpy(), exp["I"])
    np.testing.assert_array_equal(host(got["out_feats"], wl.BF16), exp["out_feats"])


def test_prune_tokens_hyper_parameters():
    tok = small_video(601, 6, 128, 768, wl.BF16, rho=0.6)
    for w in (0.0, 0.5, 3.0):
        check_tokens(tok.feats, wl.BF16, None, w=w)
    check_tokens(tok.feats, wl.BF16, None, min_keep=100)
    check_tokens(tok.feats, wl.BF16, None, min_keep=128)
    for K in (0.5, 1.2, 1.6, 9.0):
        check_tokens(tok.feats, wl.BF16, None, mode=1, K=K)


def test_prune_tokens_one_minus_cosine_with_fixed_threshold():
    """Sec. 3.1: the rescaled cosine in place of Eq.1, together with the fixed threshold K."""
    tok = small_video(604, 9, 196, 896, wl.BF16, rho=0.5)
    kept = []
    for w, K in ((1.0, 0.4), (1.0, 1.4), (1.0, 1.5), (0.0, 0.5), (2.5, 2.9)):
        exp = check_tokens(tok.feats, wl.BF16, [0, 4, 9], mode=1, K=K, w=w, measure=1)
        kept.append(int(exp["counts"].sum()))
    assert kept[0] == 9 * 196 and 0 < kept[1] < kept[0] and kept[2] <= kept[1]
    tok = small_video(605, 5, 144, 1152, wl.F32, rho=0.8)              # the two-pass kernels
    exp = check_tokens(tok.feats, wl.F32, None, mode=1, K=1.1, measure=1)
    assert 0 < exp["counts"].sum() < 5 * 144
    # static and negated frames: 1 - cos is exactly 0 and exactly 2
    rng = np.random.default_rng(606)
    F = wl.f32_to_bf16_bits(rng.standard_normal((64, 512)).astype(np.float32))
    exp = check_tokens(np.stack([F, F, F ^ np.uint16(0x8000)]), wl.BF16, None, mode=1, K=2.0, w=0.0, measure=1)
    assert exp["counts"].tolist() == [0, 0, 64]
    with pytest.raises(ValueError):
        sharpv.prune_tokens(dev(tok.feats, wl.F32), measure=1)         # adaptive mode: refused


def test_prune_tokens_static_negated_tied_and_ragged():
    rng = np.random.default_rng(602)
    f, d = 64, 512
    F = wl.f32_to_bf16_bits(rng.standard_normal((f, d)).astype(np.float32))
    G = wl.f32_to_bf16_bits(rng.standard_normal((f, d)).astype(np.float32))
    neg = F ^ np.uint16(0x8000)
    feats = np.stack([F, F, neg, neg, G, G, F])
    exp = check_tokens(feats, wl.BF16, None)
    assert exp["counts"][1] == 0 and exp["counts"][2] == f and exp["counts"][3] == 0
    # every video one frame; and a few ragged splits of the same frames
    check_tokens(feats, wl.BF16, np.arange(8))
    check_tokens(feats, wl.BF16, [0, 2, 3, 7])
    check_tokens(feats, wl.BF16, [0, 6, 7])
    # exact ties inside a frame: slots i and i+32 identical in every frame
    half = wl.f32_to_bf16_bits(rng.standard_normal((3, f // 2, d)).astype(np.float32))
    tied = np.concatenate([half, half], axis=1)
    exp = check_tokens(tied, wl.BF16, None, min_keep=21)
    np.testing.assert_array_equal(exp["I"][:, :32], exp["I"][:, 32:])
    # everything static: nothing survives, outputs stay empty
    exp = check_tokens(np.stack([F, F, F])[1:], wl.BF16, None, w=0.0, mode=1, K=0.5)
    assert exp["counts"][1] == 0


def test_prune_tokens_is_deterministic():
    tok = small_video(603, 12, 196, 1152, wl.F32)
    x = dev(tok.feats, wl.F32)
    runs = []
    for _ in range(3):
        g = sharpv.prune_tokens(x)
        torch.cuda.synchronize()
        runs.append((g["idx"].cpu().numpy().copy(), g["I"].cpu().numpy().copy(), host(g["out_feats"], wl.F32).copy()))
    for r in runs[1:]:
        for a, b in zip(runs[0], r):
            np.testing.assert_array_equal(a, b)


# ----------------------------------------------------------------------------- shapes and edge cases, stage 2
def kv_case(seed, n_vis_per_seq, tb, ta, d, H, D, dtype, sigma_max=8.0):
    rng = np.random.default_rng(seed)
    lay = wl.make_kv_layout(n_vis_per_seq, tb, ta, H, D)
    orig32 = rng.standard_normal((lay.n_vis, d)).astype(np.float32)
    orig = wl.to_storage(orig32, dtype)
    orig32 = wl.storage_to_f32(orig, dtype)
    hidden32 = rng.standard_normal((lay.S, d)).astype(np.float32)
    sig = (sigma_max * rng.random(lay.n_vis)).astype(np.float32)
    pos = lay.visual_positions()
    if lay.n_vis:
        hidden32[pos] = orig32 + sig[:, None] * hidden32[pos]
    hidden = wl.to_storage(hidden32, dtype)
    K = wl.to_storage(rng.standard_normal((H, lay.S, D)).astype(np.float32), dtype)
    V = wl.to_storage(rng.standard_normal((H, lay.S, D)).astype(np.float32), dtype)
    return lay, hidden, orig, K, V


@pytest.mark.parametrize("nvs,tb,ta,d,H,D,dtype", [
    ([100], 0, 0, 512, 2, 64, wl.BF16),          # only visual tokens
    ([1], 5, 3, 64, 1, 8, wl.BF16),              # one visual token, 16-byte K rows
    ([63], 1, 0, 264, 4, 128, wl.F32),           # exactly one group of 64 positions
    ([64], 1, 0, 896, 4, 128, wl.BF16),          # spills into a second group by one
    ([300, 5, 77], 7, 9, 1152, 2, 32, wl.F32),   # ragged batch
    ([130, 131], 0, 3, 4096, 8, 128, wl.BF16),
    ([90, 40], 2, 2, 8200, 2, 64, wl.BF16),      # wider than the unrolled sweeps: the looped row kernel
    ([70], 3, 3, 2056, 2, 64, wl.F32),           # float32 rows beyond four sweeps take the loop as well
    ([50], 1, 1, 65536, 1, 8, wl.BF16),          # the widest row
])
def test_prune_kv_shapes(nvs, tb, ta, d, H, D, dtype):
    lay, hidden, orig, K, V = kv_case(700 + len(nvs) + d, nvs, tb, ta, d, H, D, dtype)
    check_kv(hidden, orig, K, V, dtype, lay)
    if lay.B == 1:
        check_kv(hidden, orig, K, V, dtype, lay, ragged=True)      # the array form of a single sequence


def test_prune_kv_thresholds_and_layer_mean_mode():
    lay, hidden, orig, K, V = kv_case(710, [200, 90], 4, 6, 768, 2, 64, wl.BF16)
    kept = []
    for M in (-1.0, 0.0, 0.2, 0.5, 0.99, 1.5):
        kept.append(len(check_kv(hidden, orig, K, V, wl.BF16, lay, M=M)["idx"]))
    assert kept[0] == lay.S and kept[-1] == lay.S - lay.n_vis
    assert all(b <= a for a, b in zip(kept, kept[1:]))
    for M in (0.05, 0.3, 0.9):
        check_kv(hidden, orig, K, V, wl.BF16, lay, M=M, kv_mode=1)


def test_prune_kv_identity_negation_and_no_visual_tokens():
    lay, hidden, orig, K, V = kv_case(711, [128], 3, 5, 512, 2, 64, wl.BF16)
    pos = lay.visual_positions()
    hidden[pos] = orig
    exp = check_kv(hidden, orig, K, V, wl.BF16, lay)
    assert len(exp["idx"]) == lay.S and np.all(exp["cos"] == 1.0)
    hidden[pos] = orig ^ np.uint16(0x8000)
    exp = check_kv(hidden, orig, K, V, wl.BF16, lay)
    assert len(exp["idx"]) == 8 and np.all(exp["cos"] == -1.0)
    hidden[pos[:5]] = 0                                             # zero rows: cosine 0 by convention
    exp = check_kv(hidden, orig, K, V, wl.BF16, lay)
    assert np.all(exp["cos"][:5] == 0.0)
    lay0, h0, o0, K0, V0 = kv_case(712, [0], 6, 4, 64, 1, 8, wl.BF16)
    got = run_kv(h0, np.zeros((1, 64), np.uint16), K0, V0, wl.BF16, lay0)
    np.testing.assert_array_equal(got["idx"].cpu().numpy(), np.arange(10))
    np.testing.assert_array_equal(host(got["K_out"], wl.BF16), K0)


def test_prune_kv_strided_cache():
    """K/V stored [S, H, D] and passed as a permuted [H, S, D] view (head stride D, position stride H*D)."""
    lay, hidden, orig, K, V = kv_case(713, [150], 2, 2, 512, 4, 64, wl.BF16)
    Kd = dev(K, wl.BF16).permute(1, 0, 2).contiguous().permute(1, 0, 2)
    Vd = dev(V, wl.BF16).permute(1, 0, 2).contiguous().permute(1, 0, 2)
    assert Kd.stride() == (64, 256, 1)
    got = sharpv.prune_kv(dev(hidden, wl.BF16), dev(orig, wl.BF16), Kd, Vd, vis_start0=2)
    torch.cuda.synchronize()
    exp = canon.prune_kv(hidden, orig, K, V, wl.BF16, lay.seq_offsets, lay.vis_start, lay.vis_offsets)
    np.testing.assert_array_equal(got["idx"].cpu().numpy(), exp["idx"])
    np.testing.assert_array_equal(host(got["K_out"], wl.BF16), exp["K_out"])
    np.testing.assert_array_equal(host(got["V_out"], wl.BF16), exp["V_out"])


def test_prune_kv_is_deterministic():
    lay, hidden, orig, K, V = kv_case(714, [500], 8, 8, 3584, 4, 128, wl.BF16)
    args = [dev(hidden, wl.BF16), dev(orig, wl.BF16), dev(K, wl.BF16), dev(V, wl.BF16)]
    outs = []
    for _ in range(3):
        g = sharpv.prune_kv(*args, vis_start0=8)
        torch.cuda.synchronize()
        outs.append((g["idx"].cpu().numpy().copy(), g["cos"].cpu().numpy().copy(), host(g["K_out"], wl.BF16).copy()))
    for o in outs[1:]:
        for a, b in zip(outs[0], o):
            np.testing.assert_array_equal(a, b)


def test_error_codes_with_real_buffers():
    x = torch.zeros((2, 16, 64), dtype=torch.bfloat16, device="cuda")
    p = sharpv.default_params()
    plan = sharpv.TokensPlan(2, 16, 64, p)
    plan.workspace_bytes = 8
    assert plan.run(x) == 5
    p2 = sharpv.default_params(); p2.min_keep = 99
    plan2 = sharpv.TokensPlan(2, 16, 64, sharpv.default_params())
    plan2.params = p2
    assert plan2.run(x) == 4


def test_prune_kv_long_sequences_take_the_scanned_prefix():
    """More than 8192 mask words (131 072 positions): the gathers read their output offsets from a scan
    of the mask instead of adding up the words themselves."""
    lay, hidden, orig, K, V = kv_case(730, [139000], 500, 500, 64, 1, 8, wl.BF16)
    assert lay.S > 131072
    check_kv(hidden, orig, K, V, wl.BF16, lay)
    lay, hidden, orig, K, V = kv_case(731, [70000, 3, 65000], 7, 9, 64, 2, 16, wl.BF16)
    check_kv(hidden, orig, K, V, wl.BF16, lay)
    check_kv(hidden, orig, K, V, wl.BF16, lay, M=0.4, kv_mode=1)
    check_kv_rope(hidden, orig, K, V, wl.BF16, lay, 0)


# ----------------------------------------------------------------------------- rotary re-encoding in the K gather
def rope_tables(rope_len, D, base=1e6):
    """cos / sin of delta * theta_i for a rotary embedding of the given base (float32 tables, as a model caches them)."""
    theta = base ** (-2.0 * np.arange(D // 2) / D)
    ang = np.arange(rope_len)[:, None] * theta[None, :]
    return np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)


def check_kv_rope(hidden, orig, K, V, dtype, lay, layout, ragged=None, strided=False, **over):
    H, S, D = K.shape
    ct, st = rope_tables(S, D)
    kw = {k: over[k] for k in ("M", "kv_mode") if k in over}
    is_ragged = lay.B > 1 if ragged is None else ragged
    call = dict(kw)
    if is_ragged:
        call.update(seq_offsets=i32(lay.seq_offsets), vis_start=i32(lay.vis_start), vis_offsets=i32(lay.vis_offsets))
    else:
        call.update(vis_start0=int(lay.vis_start[0]))
    Kd, Vd = dev(K, dtype), dev(V, dtype)
    if strided:                                           # stored [S, H, D], passed as a permuted view
        Kd = Kd.permute(1, 0, 2).contiguous().permute(1, 0, 2)
        Vd = Vd.permute(1, 0, 2).contiguous().permute(1, 0, 2)
    got = sharpv.prune_kv(dev(hidden, dtype), dev(orig, dtype), Kd, Vd, n_vis=lay.n_vis,
                          rope_cos=torch.from_numpy(ct).cuda(), rope_sin=torch.from_numpy(st).cuda(),
                          rope_layout=layout, **call)
    torch.cuda.synchronize()
    exp = canon.prune_kv(hidden, orig, K, V, dtype, lay.seq_offsets, lay.vis_start, lay.vis_offsets, **kw)
    K_exp = canon.rope_reencode(exp["K_out"], dtype, exp["idx"], lay.seq_offsets, ct, st, layout)
    np.testing.assert_array_equal(got["counts"].cpu().numpy(), exp["counts"])
    np.testing.assert_array_equal(got["idx"].cpu().numpy(), exp["idx"])
    np.testing.assert_array_equal(host(got["V_out"], dtype), exp["V_out"])           # V rows are plain copies
    np.testing.assert_array_equal(host(got["K_out"], dtype), K_exp)                  # bit for bit
    # float64 definition: float32 arithmetic plus (bf16) one rounding to 8 significant bits
    K_def = ref.rope_reencode(exp["K_out"], dtype, exp["idx"], lay.seq_offsets, ct, st, layout)
    rtol = 2.0 ** -8 * 1.001 if dtype == wl.BF16 else 1e-5
    np.testing.assert_allclose(wl.storage_to_f32(host(got["K_out"], dtype), dtype), K_def, rtol=rtol, atol=1e-5)
    return exp, K_exp


@pytest.mark.parametrize("nvs,tb,ta,d,H,D,dtype,layout", [
    ([600], 9, 7, 512, 4, 128, wl.BF16, 0),        # the benchmark's cache shape (4 heads x 128), half-split pairs
    ([600], 9, 7, 512, 4, 128, wl.BF16, 1),        # interleaved pairs
    ([300, 5, 77], 7, 9, 264, 2, 32, wl.F32, 0),   # ragged batch, float32: sequences start inside mask words
    ([3, 1, 2, 40, 1], 1, 2, 64, 3, 16, wl.BF16, 0),   # many short sequences in one mask word; 3 heads (any-H path)
    ([130, 131], 0, 3, 512, 8, 64, wl.BF16, 1),
    ([90], 2, 2, 64, 1, 16, wl.F32, 1),            # one head (any-H path), 8-byte half rows are refused below
    ([257], 16, 16, 128, 2, 256, wl.BF16, 0),      # 512-byte rows
])
def test_prune_kv_rope_shapes(nvs, tb, ta, d, H, D, dtype, layout):
    lay, hidden, orig, K, V = kv_case(900 + len(nvs) + D + layout, nvs, tb, ta, d, H, D, dtype)
    exp, K_exp = check_kv_rope(hidden, orig, K, V, dtype, lay, layout)
    assert 0 < len(exp["idx"]) < lay.S
    assert not np.array_equal(K_exp, exp["K_out"])                 # rows did move
    if lay.B == 1:
        check_kv_rope(hidden, orig, K, V, dtype, lay, layout, ragged=True)
        check_kv_rope(hidden, orig, K, V, dtype, lay, layout, strided=True)


def test_prune_kv_rope_nothing_or_everything_dropped():
    lay, hidden, orig, K, V = kv_case(921, [200], 4, 4, 256, 4, 128, wl.BF16)
    # M below every cosine: all positions kept, every shift is zero, K leaves unchanged
    exp, K_exp = check_kv_rope(hidden, orig, K, V, wl.BF16, lay, 0, M=-2.0)
    assert len(exp["idx"]) == lay.S
    np.testing.assert_array_equal(K_exp, K)
    # M above every cosine: only the text positions remain; the trailing ones shift by the whole visual block
    exp, K_exp = check_kv_rope(hidden, orig, K, V, wl.BF16, lay, 0, M=2.0)
    assert len(exp["idx"]) == 8
    np.testing.assert_array_equal(K_exp[:, :4], K[:, :4])
    assert not np.array_equal(K_exp[:, 4:], K[:, 204:])
    # per-sequence mean decision with re-encoding
    lay2, h2, o2, K2, V2 = kv_case(922, [60, 70], 3, 3, 256, 2, 64, wl.BF16)
    check_kv_rope(h2, o2, K2, V2, wl.BF16, lay2, 0, M=0.3, kv_mode=1)


def test_prune_kv_rope_on_the_second_config(workloads):
    cfg, tok = workloads(2)
    lay = wl.kv_layout_for(cfg)
    kv = wl.kv_layer_for(cfg, tok, cfg.kv_layers[0], threads=8)
    check_kv_rope(kv["hidden"], tok.feats.reshape(-1, cfg.d), kv["K"], kv["V"], cfg.dtype, lay, 0)


# ----------------------------------------------------------------------------- pruning carried from layer to layer
def carried_case(seed, seq_lens, n_orig, d, H, D, dtype, vis_frac=0.8):
    """A packed batch whose visual positions are scattered (as after earlier pruning) and point to
    shuffled rows of orig."""
    rng = np.random.default_rng(seed)
    S = int(sum(seq_lens))
    seq = np.concatenate([[0], np.cumsum(seq_lens)]).astype(np.int32)
    n_vis = min(n_orig, int(S * vis_frac))
    rows = np.full(S, -1, np.int32)
    vis = np.sort(rng.choice(S, size=n_vis, replace=False))
    rows[vis] = rng.choice(n_orig, size=n_vis, replace=False)
    orig = wl.to_storage(rng.standard_normal((n_orig, d)).astype(np.float32), dtype)
    o32 = wl.storage_to_f32(orig, dtype)
    h32 = rng.standard_normal((S, d)).astype(np.float32)
    h32[vis] = o32[rows[vis]] + (rng.random((n_vis, 1)) * 8).astype(np.float32) * h32[vis]
    hidden = wl.to_storage(h32, dtype)
    K = wl.to_storage(rng.standard_normal((H, S, D)).astype(np.float32), dtype)
    V = wl.to_storage(rng.standard_normal((H, S, D)).astype(np.float32), dtype)
    return seq, rows, vis, hidden, orig, K, V


def check_kv_carried(seq, rows, hidden, orig, K, V, dtype, M=0.2, rope_layout=None):
    S = hidden.shape[0]
    kw = {}
    if rope_layout is not None:
        ct, st = rope_tables(S, K.shape[2])
        kw = dict(rope_cos=torch.from_numpy(ct).cuda(), rope_sin=torch.from_numpy(st).cuda(), rope_layout=rope_layout)
    so = i32(seq) if len(seq) > 2 else None
    got = sharpv.prune_kv_carried(dev(hidden, dtype), dev(orig, dtype), i32(rows), dev(K, dtype), dev(V, dtype),
                                  seq_offsets=so, M=M, **kw)
    torch.cuda.synchronize()
    exp = canon.prune_kv_mapped(hidden, orig, rows, K, V, dtype, seq, M=M)
    np.testing.assert_array_equal(got["counts"].cpu().numpy(), exp["counts"])
    np.testing.assert_array_equal(got["idx"].cpu().numpy(), exp["idx"])
    np.testing.assert_array_equal(got["orig_row_out"].cpu().numpy(), exp["orig_row_out"])
    np.testing.assert_array_equal(got["cos"].cpu().numpy(), exp["cos"])              # NaN where nothing is written
    K_exp = exp["K_out"]
    if rope_layout is not None:
        K_exp = canon.rope_reencode(K_exp, dtype, exp["idx"], seq, ct, st, rope_layout)
    np.testing.assert_array_equal(host(got["K_out"], dtype), K_exp)
    np.testing.assert_array_equal(host(got["V_out"], dtype), exp["V_out"])
    a = ref.prune_kv_mapped(hidden, orig, rows, K, V, dtype, seq, M=M)
    vis = (rows >= 0) & (rows < orig.shape[0])
    np.testing.assert_allclose(got["cos"].cpu().numpy()[vis], a["cos"][vis], rtol=RTOL, atol=ATOL)
    return exp


@pytest.mark.parametrize("seq_lens,n_orig,d,H,D,dtype", [
    ([700], 900, 512, 4, 128, wl.BF16),              # more rows in orig than positions left
    ([300, 1, 77, 200], 400, 264, 2, 32, wl.F32),    # ragged batch, a one-position sequence
    ([45], 30, 64, 3, 16, wl.BF16),
    ([1000, 1000], 1500, 3584, 4, 128, wl.BF16),     # model width of the benchmark
])
def test_prune_kv_carried_shapes(seq_lens, n_orig, d, H, D, dtype):
    seq, rows, vis, hidden, orig, K, V = carried_case(940 + len(seq_lens) + D, seq_lens, n_orig, d, H, D, dtype)
    exp = check_kv_carried(seq, rows, hidden, orig, K, V, dtype)
    assert 0 < len(exp["idx"]) < hidden.shape[0]
    check_kv_carried(seq, rows, hidden, orig, K, V, dtype, rope_layout=0)
    bad = rows.copy()
    bad[vis[:4]] = [n_orig, n_orig + 7, -3, 2**30]           # out-of-range rows count as non-visual positions
    check_kv_carried(seq, bad, hidden, orig, K, V, dtype, M=2.0)


def test_prune_kv_carried_on_a_long_sequence():
    """The carried form past 131 072 positions (scanned mask prefix) with re-encoding."""
    seq, rows, vis, hidden, orig, K, V = carried_case(955, [90000, 50001], 100000, 64, 2, 16, wl.BF16)
    check_kv_carried(seq, rows, hidden, orig, K, V, wl.BF16, rope_layout=0)


def test_prune_kv_carried_block_map_equals_plain_call():
    lay, hidden, orig, K, V = kv_case(950, [300, 120], 6, 10, 768, 4, 64, wl.BF16)
    rows = np.full(lay.S, -1, np.int32)
    rows[lay.visual_positions()] = np.arange(lay.n_vis)
    exp = check_kv_carried(lay.seq_offsets, rows, hidden, orig, K, V, wl.BF16)
    plain = check_kv(hidden, orig, K, V, wl.BF16, lay)
    np.testing.assert_array_equal(exp["idx"], plain["idx"])
    np.testing.assert_array_equal(exp["K_out"], plain["K_out"])


def test_prune_kv_carried_over_three_layers():
    """Each layer runs on what the previous one kept; the survivors are the intersection of the layers' masks."""
    rng = np.random.default_rng(960)
    dtype, d, H, D = wl.BF16, 512, 2, 64
    seq, rows, vis, hidden0, orig, K, V = carried_case(961, [400, 250], 600, d, H, D, dtype, vis_frac=0.9)
    S = hidden0.shape[0]
    o32 = wl.storage_to_f32(orig, dtype)
    alive = np.arange(S)
    cur_seq, cur_rows = seq, rows
    want_alive = np.ones(S, bool)
    for l in range(3):
        noise = rng.standard_normal((S, d)).astype(np.float32) * (1.5 * l + rng.random((S, 1)) * 3).astype(np.float32)
        h32 = noise.copy()
        h32[vis] += o32[rows[vis]]
        h_full = wl.to_storage(h32, dtype)
        Kl = wl.to_storage(rng.standard_normal((H, S, D)).astype(np.float32), dtype)
        full = canon.prune_kv_mapped(h_full, orig, rows, Kl, Kl, dtype, seq)
        m = np.zeros(S, bool); m[full["idx"]] = True
        want_alive &= m
        exp = check_kv_carried(cur_seq, cur_rows, h_full[alive], orig, Kl[:, alive], Kl[:, alive], dtype,
                               rope_layout=l % 2)
        np.testing.assert_array_equal(alive[exp["idx"]], np.nonzero(want_alive)[0])
        alive = alive[exp["idx"]]
        cur_rows = exp["orig_row_out"]
        cur_seq = np.concatenate([[0], np.cumsum(exp["counts"])]).astype(np.int32)
    assert 0 < len(alive) < S


# ----------------------------------------------------------------------------- measurement aids and event timing
@pytest.mark.parametrize("nbytes", [16, 48, 8192, 16 * 1000003, 64 << 20])
def test_stream_copy_and_read(nbytes):
    g = torch.Generator(device="cuda")
    g.manual_seed(nbytes)
    src = torch.randint(-2**31, 2**31 - 1, (nbytes // 4,), dtype=torch.int32, device="cuda", generator=g)
    dst = torch.full((nbytes // 4 + 4,), 7, dtype=torch.int32, device="cuda")
    sharpv.stream_copy(dst, src)
    sink = torch.full((1,), -5, dtype=torch.int32, device="cuda")
    sharpv.stream_read(src, sink)
    torch.cuda.synchronize()
    assert torch.equal(dst[: nbytes // 4], src)
    assert torch.all(dst[nbytes // 4:] == 7)         # nothing written past the end
    assert int(sink[0]) == -5                        # the read leaves no trace
    L = sharpv.load()
    assert L.sharpv_stream_copy(dst.data_ptr(), src.data_ptr(), 24, None) == 2       # not a multiple of 16
    assert L.sharpv_stream_copy(dst.data_ptr() + 4, src.data_ptr(), 16, None) == 2   # misaligned
    assert L.sharpv_stream_read(None, 16, sink.data_ptr(), None) == 1


def test_floor_aids_read_in_bounds_and_copy_the_indexed_rows():
    """The two floor aids of the pre-LLM stage: the slab-pattern read leaves no trace for any shape the fused
    kernel takes, the indexed row copy equals torch's index_select."""
    sink = torch.full((1,), -5, dtype=torch.int32, device="cuda")
    for n, f, d, dt in ((1, 196, 3584, torch.bfloat16), (7, 1, 64, torch.bfloat16), (40, 208, 520, torch.bfloat16),
                        (300, 17, 256, torch.bfloat16), (5, 144, 1152, torch.float32)):
        x = torch.randn((n, f, d), device="cuda").to(dt)
        sharpv.stream_read_slabs(x, sink)
    torch.cuda.synchronize()
    assert int(sink[0]) == -5
    L = sharpv.load()
    assert L.sharpv_stream_read_slabs(x.data_ptr(), 5, 209, 1152, 4, sink.data_ptr(), None) == 2    # taller than the pattern covers
    g = torch.Generator(device="cuda"); g.manual_seed(77)
    for rows, d, k in ((50176, 3584, 7633), (10, 8, 1), (999, 520, 999)):
        src = torch.randn((rows, d), device="cuda", generator=g).to(torch.bfloat16)
        idx = torch.sort(torch.randperm(rows, device="cuda", generator=g)[:k])[0].to(torch.int32)
        dst = torch.full((k + 1, d), 7.0, dtype=torch.bfloat16, device="cuda")
        sharpv.stream_gather_rows(dst, src, idx)
        torch.cuda.synchronize()
        assert torch.equal(dst[:k], src[idx.long()])
        assert torch.all(dst[k] == 7.0)
    with pytest.raises(ValueError):
        sharpv.stream_gather_rows(dst, src, torch.tensor([rows], dtype=torch.int32, device="cuda"))


def test_event_timing_counts_launches():
    tok = small_video(801, 4, 64, 512, wl.BF16)
    x = dev(tok.feats, wl.BF16)
    sharpv.timing_enable(64)
    try:
        for _ in range(3):
            sharpv.prune_tokens(x)
        torch.cuda.synchronize()
        for name in ("frame_slab", "frame_select", "token_gather"):
            n, ms = sharpv.timing_read(name)
            assert n == 3 and 0.0 < ms < 1000.0
        assert sharpv.timing_read("kv_cosine") == (0, 0.0)
        with pytest.raises(RuntimeError):
            sharpv.timing_read("no_such_kernel")
    finally:
        sharpv.timing_disable()
    # disabled again: launches are no longer recorded, results unchanged
    a = sharpv.prune_tokens(x)["idx"].cpu().numpy()
    sharpv.timing_enable(1)                          # a pool smaller than the launches of one call
    try:
        b = sharpv.prune_tokens(x)["idx"].cpu().numpy()
        torch.cuda.synchronize()
    finally:
        sharpv.timing_disable()
    np.testing.assert_array_equal(a, b)


# ----------------------------------------------------------------------------- capture into a HIP graph
def test_both_stages_replay_from_a_captured_graph():
    """The entry points only enqueue kernels on the caller's stream (no allocation, no memset, no
    synchronisation), so a step can be captured once and replayed; every replay must reproduce the
    eager results, with other work on the device between replays."""
    tok = small_video(990, 12, 196, 1152, wl.BF16, cuts=(5,))
    x = dev(tok.feats, wl.BF16)
    lay, hidden, orig, K, V = kv_case(991, [700], 10, 14, 1152, 4, 128, wl.BF16)
    hd, od, Kd, Vd = dev(hidden, wl.BF16), dev(orig, wl.BF16), dev(K, wl.BF16), dev(V, wl.BF16)
    ct, st = rope_tables(lay.S, 128)
    ctd, std = torch.from_numpy(ct).cuda(), torch.from_numpy(st).cuda()
    p = sharpv.default_params(wl.BF16)
    tplan = sharpv.TokensPlan(12, 196, 1152, p)
    kplan = sharpv.KvPlan(1, lay.S, lay.n_vis, 1152, 4, 128, p)
    rplan = sharpv.KvPlan(1, lay.S, lay.n_vis, 1152, 4, 128, p)

    def step():
        assert tplan.run(x) == 0
        assert kplan.run(hd, od, Kd, Vd, int(lay.vis_start[0])) == 0
        assert rplan.run(hd, od, Kd, Vd, int(lay.vis_start[0]), rope_cos=ctd, rope_sin=std) == 0

    def snapshot():
        torch.cuda.synchronize()
        t, k, r = tplan.results(), kplan.results(), rplan.results()
        return [v.clone() for v in (t["idx"], t["counts"], t["out_feats"], t["I"], k["idx"], k["K_out"], k["V_out"],
                                    k["cos"], r["idx"], r["K_out"])]

    def scribble():
        for plan in (tplan, kplan, rplan):
            for name in ("out_idx", "out_counts", "out_count", "out_feats", "K_out", "V_out", "out_cos", "out_scores"):
                t = getattr(plan, name, None)
                if t is not None:
                    t.fill_(-1 if t.dtype == torch.int32 else 7)
            plan.workspace.fill_(0xA5)           # the workspace carries nothing from call to call

    step()
    want = snapshot()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for _ in range(3):
        scribble()
        y = (x.float() * 1.5).sum()              # unrelated eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        got = snapshot()
        assert float(y) == float(y)
        for a, b in zip(want, got):
            assert a.shape == b.shape and torch.equal(a, b)


# ----------------------------------------------------------------------------- seeded sweep over small shapes
def test_sweep_of_small_shapes_stage_1():
    rng = np.random.default_rng(20251127)
    for case in range(36):
        dtype = wl.BF16 if case % 3 else wl.F32
        f = int(rng.choice([1, 2, 15, 16, 31, 33, 64, 97, 143, 196, 207, 208, 209, 256, 300, 577, 1024]))
        d = 8 * int(rng.integers(1, 130))
        B = int(rng.integers(1, 5))
        ns = [int(rng.integers(1, 7)) for _ in range(B)]
        specs = [wl.VideoSpec(n=n, rho=np.full(n, float(rng.uniform(0.3, 0.99))),
                              cuts=tuple(sorted(set(int(c) for c in rng.integers(1, n, size=int(rng.integers(0, 2)))))) if n > 1 else (),
                              seed=3000 + 10 * case + b) for b, n in enumerate(ns)]
        tok = wl.make_tokens(specs, f, d, dtype, threads=2)
        kw = {}
        if case % 4 == 1:
            kw["min_keep"] = int(rng.integers(0, f + 1))
        if case % 4 == 2:
            kw["w"] = float(rng.choice([0.0, 0.25, 2.0]))
        if case % 7 == 3:
            kw.update(mode=1, K=float(rng.uniform(0.2, 2.5)))
        if case % 7 == 5:                                            # the fixed threshold on 1 - cos (own stream of draws)
            kw = dict(mode=1, measure=1, K=float(np.random.default_rng(77 + case).uniform(0.1, 1.9)),
                      w=kw.get("w", 1.0))
        print(f"case {case}: frames {ns} f={f} d={d} dtype={dtype} {kw}", flush=True)
        check_tokens(tok.feats, dtype, tok.frame_offsets if B > 1 else None, **kw)


def test_sweep_of_small_shapes_stage_2():
    rng = np.random.default_rng(20251128)
    for case in range(36):
        dtype = wl.BF16 if case % 3 else wl.F32
        esz = 2 if dtype == wl.BF16 else 4
        B = int(rng.integers(1, 5))
        nvs = [int(rng.integers(0, 200)) for _ in range(B)]
        tb, ta = int(rng.integers(0, 20)), int(rng.integers(0, 20))
        if sum(nvs) + B * (tb + ta) == 0:
            ta = 1
        d = 8 * int(rng.integers(1, 140))
        H = int(rng.choice([1, 2, 3, 4, 5, 8, 12]))
        D = (32 // esz) * int(rng.integers(1, 9))            # half rows are whole 16-byte pieces (needed by the rope form)
        lay, hidden, orig, K, V = kv_case(5000 + case, nvs, tb, ta, d, H, D, dtype)
        M = float(rng.choice([0.2, 0.2, 0.05, 0.6]))
        print(f"case {case}: nvs {nvs} text {tb}+{ta} d={d} H={H} D={D} dtype={dtype} M={M}", flush=True)
        if lay.n_vis == 0:
            orig = np.zeros((1, d), hidden.dtype)
        kind = case % 4
        if kind == 0:
            check_kv(hidden, orig, K, V, dtype, lay, M=M)
        elif kind == 1:
            check_kv(hidden, orig, K, V, dtype, lay, M=M, kv_mode=1)
        elif kind == 2 and lay.n_vis > 0:
            check_kv_rope(hidden, orig, K, V, dtype, lay, int(rng.integers(0, 2)), M=M)
        elif lay.n_vis > 0:
            rows = np.full(lay.S, -1, np.int32)
            rows[lay.visual_positions()] = rng.permutation(lay.n_vis).astype(np.int32)
            vis = lay.visual_positions()
            hidden[vis] = wl.to_storage(wl.storage_to_f32(orig, dtype)[rows[vis]]
                                        + (rng.random((lay.n_vis, 1)) * 8).astype(np.float32)
                                        * rng.standard_normal((lay.n_vis, d)).astype(np.float32), dtype)
            check_kv_carried(lay.seq_offsets, rows, hidden, orig, K, V, dtype, M=M,
                             rope_layout=int(rng.integers(0, 2)) if case % 8 == 3 else None)


# ----------------------------------------------------------------------------- tiny magnitudes
def test_tiny_magnitudes_follow_the_float32_oracle():
    """Features scaled by 2^-30 behave like the unscaled ones (every quantity is a ratio).  At 2^-60 and
    2^-66 the products of two squared norms underflow float32: the float32 contract then gives cosine 0
    (all scores tie, everything in the KV stage is below M) where the float64 definition does not, so only
    the float32 oracle is the reference there."""
    tok = small_video(995, 6, 64, 512, wl.BF16, rho=0.7)
    base = wl.storage_to_f32(tok.feats, wl.BF16)
    lay, hidden, orig, K, V = kv_case(996, [120], 4, 4, 512, 2, 64, wl.BF16)
    h32, o32 = wl.storage_to_f32(hidden, wl.BF16), wl.storage_to_f32(orig, wl.BF16)
    ref_counts = check_tokens(tok.feats, wl.BF16, None)["counts"]
    for e in (-30, -60, -66):
        scale = np.float32(2.0 ** e)
        feats = wl.to_storage(base * scale, wl.BF16)
        np.testing.assert_array_equal(wl.storage_to_f32(feats, wl.BF16), base * scale)      # exact scaling
        hs, os_ = wl.to_storage(h32 * scale, wl.BF16), wl.to_storage(o32 * scale, wl.BF16)
        if e == -30:
            np.testing.assert_array_equal(check_tokens(feats, wl.BF16, None)["counts"], ref_counts)
            check_kv(hs, os_, K, V, wl.BF16, lay)
            continue
        got = run_tokens(feats, wl.BF16, np.asarray([0, 6], np.int32))
        exp = canon.prune_tokens(feats, wl.BF16, np.asarray([0, 6], np.int32))
        assert np.all(exp["I"] == exp["I"][0, 0])                                            # everything ties
        for k, name in (("counts", "counts"), ("idx", "idx"), ("I", "I"), ("ratio", "ratio")):
            np.testing.assert_array_equal(got[k].cpu().numpy(), exp[name])
        np.testing.assert_array_equal(host(got["out_feats"], wl.BF16), exp["out_feats"])
        gk = run_kv(hs, os_, K, V, wl.BF16, lay)
        ek = canon.prune_kv(hs, os_, K, V, wl.BF16, lay.seq_offsets, lay.vis_start, lay.vis_offsets)
        assert np.all(ek["cos"] == 0.0) and len(ek["idx"]) == 8
        np.testing.assert_array_equal(gk["idx"].cpu().numpy(), ek["idx"])
        np.testing.assert_array_equal(gk["cos"].cpu().numpy(), ek["cos"])
        np.testing.assert_array_equal(host(gk["K_out"], wl.BF16), ek["K_out"])
