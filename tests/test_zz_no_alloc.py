"""`sharpv_prune_kv_static` (the intra-LLM stage on the library's built-in scratch, for callers that
cannot allocate) against `sharpv_prune_kv` on a caller workspace: same outputs bit for bit, on two calls
in a row that share the scratch, the second on a smaller input; then against the CPU oracle."""
import numpy as np
import pytest
import torch

from oracle import canon
from paper_2511_08003_amd import sharpv, workloads as wl

pytestmark = pytest.mark.gpu


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).view(torch.bfloat16).cuda()


def _bits(t):
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def _case(seed, nvs, tb, ta, d, H, D):
    rng = np.random.default_rng(seed)
    lay = wl.make_kv_layout(nvs, tb, ta, H, D)
    o32 = rng.standard_normal((lay.n_vis, d)).astype(np.float32)
    orig = wl.to_storage(o32, wl.BF16)
    o32 = wl.storage_to_f32(orig, wl.BF16)
    h32 = rng.standard_normal((lay.S, d)).astype(np.float32)
    pos = lay.visual_positions()
    h32[pos] = o32 + (8.0 * rng.random((lay.n_vis, 1))).astype(np.float32) * h32[pos]
    hidden = wl.to_storage(h32, wl.BF16)
    K = wl.to_storage(rng.standard_normal((H, lay.S, D)).astype(np.float32), wl.BF16)
    V = wl.to_storage(rng.standard_normal((H, lay.S, D)).astype(np.float32), wl.BF16)
    return lay, hidden, orig, K, V


def _run(static, lay, hidden, orig, K, V, d, H, D, **par):
    p = sharpv.default_params(wl.BF16, **par)
    plan = sharpv.KvPlan(lay.B, lay.S, lay.n_vis, d, H, D, p, mean_cos=True)
    for t in (plan.out_idx, plan.out_count):
        t.fill_(-7)
    for t in (plan.K_out, plan.V_out, plan.out_cos, plan.out_mean_cos):
        t.fill_(3.0)
    args = [_dev(hidden), _dev(orig), _dev(K), _dev(V)]
    kw = {}
    if lay.B > 1:
        i32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, np.int32)).cuda()
        kw = dict(seq_offsets=i32(lay.seq_offsets), vis_start=i32(lay.vis_start), vis_offsets=i32(lay.vis_offsets))
    else:
        kw = dict(vis_start0=int(lay.vis_start[0]))
    rc = (plan.run_static if static else plan.run)(*args, **kw)
    assert rc == 0, sharpv.status_string(rc)
    torch.cuda.synchronize()
    r = plan.results()
    return {"idx": r["idx"].cpu().numpy(), "counts": r["counts"].cpu().numpy(), "cos": r["cos"].cpu().numpy(),
            "mean_cos": r["mean_cos"].cpu().numpy(), "K_out": _bits(r["K_out"]), "V_out": _bits(r["V_out"])}


def test_static_scratch_entry_point_matches_the_workspace_one():
    d, H, D = 896, 4, 128
    big = _case(1201, [9000, 700], 12, 20, d, H, D)          # ragged batch, 9764 positions: 611 mask words
    small = _case(1202, [333], 5, 3, d, H, D)                # then a much shorter single sequence
    for lay, hidden, orig, K, V in (big, small):
        for par in ({}, {"M": 0.35, "kv_mode": 1}):
            print(f"static scratch: S={lay.S} B={lay.B} {par}", flush=True)
            got = _run(True, lay, hidden, orig, K, V, d, H, D, **par)
            want = _run(False, lay, hidden, orig, K, V, d, H, D, **par)
            assert 0 < len(want["idx"]) <= lay.S
            for k in want:
                np.testing.assert_array_equal(got[k], want[k], err_msg=k)
            exp = canon.prune_kv(hidden, orig, K, V, wl.BF16, lay.seq_offsets, lay.vis_start, lay.vis_offsets,
                                 M=par.get("M", 0.2), kv_mode=par.get("kv_mode", 0))
            for k in ("idx", "counts", "cos", "mean_cos", "K_out", "V_out"):
                np.testing.assert_array_equal(got[k], exp[k][:lay.n_vis] if k == "cos" else exp[k], err_msg=k)


def test_static_scratch_entry_point_refuses_what_it_cannot_hold():
    L = sharpv.load()
    p = sharpv.default_params(wl.BF16)
    S = 262144 + 16
    x = torch.zeros((S, 8), dtype=torch.bfloat16, device="cuda")
    kv = torch.zeros((1, S, 8), dtype=torch.bfloat16, device="cuda")
    plan = sharpv.KvPlan(1, S, 0, 8, 1, 8, p)           # no visual tokens: every position is kept
    plan.out_idx.fill_(-7)
    rc = plan.run_static(x, x, kv, kv)
    torch.cuda.synchronize()
    assert rc == 7 and "scratch" in sharpv.status_string(rc)
    assert int(plan.out_idx[0]) == -7                        # nothing was launched
    assert plan.run(x, x, kv, kv) == 0                       # the workspace form takes the same call
    torch.cuda.synchronize()
    assert int(plan.out_count[0]) == S
    assert L.sharpv_prune_kv_static(None, x.data_ptr(), kv.data_ptr(), kv.data_ptr(), S * 8, 8, None, None, None, 1, S,
                                    0, 0, 8, 1, 8, 0, None, None, None, None, None, S * 8, None, None, None) != 0
