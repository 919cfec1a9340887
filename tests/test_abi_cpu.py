"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments on the host before any launch."""
import ctypes as C
import os
import re

import pytest

from paper_2511_08003_amd import sharpv

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADERS = [os.path.join(ROOT, "include", "sharpv.h"), os.path.join(ROOT, "include", "sharpv_bench.h")]


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(sharpv.LIB_PATH):
        from paper_2511_08003_amd import build
        build.build()
    return sharpv.load()


def declared_functions():
    text = "".join(open(h).read() for h in HEADERS)
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sharpv_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert {"sharpv_prune_tokens", "sharpv_prune_kv", "sharpv_params_default", "sharpv_prune_tokens_workspace",
            "sharpv_prune_kv_workspace", "sharpv_status_string", "sharpv_version", "sharpv_timing_enable",
            "sharpv_timing_disable", "sharpv_timing_read"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_defaults_are_the_papers(lib):
    p = sharpv.default_params()
    assert p.struct_size == C.sizeof(sharpv.Params) == 36
    assert (p.dtype, p.mode, p.min_keep, p.kv_mode, p.measure) == (sharpv.BF16, 0, 0, 0, sharpv.DISSIM_EQ1)
    assert p.w == 1.0 and abs(p.M - 0.2) < 1e-7 and abs(p.K - 1.6) < 1e-6
    assert lib.sharpv_version() >= 100
    assert sharpv.status_string(0) == "ok" and "workspace" in sharpv.status_string(5)


def test_workspace_queries(lib):
    p = sharpv.default_params()
    n, f, d = 256, 196, 3584
    need = lib.sharpv_prune_tokens_workspace(n, f, d, C.byref(p))
    assert need >= n * d * 4 + 4 * n * f * 4 and need % 256 == 0
    assert lib.sharpv_prune_tokens_workspace(n, 0, d, C.byref(p)) == 0
    assert lib.sharpv_prune_tokens_workspace(n, f, 12, C.byref(p)) == 0          # d not a multiple of 8
    assert lib.sharpv_prune_tokens_workspace(n, 2048, d, C.byref(p)) == 0        # f > 1024
    assert lib.sharpv_prune_kv_workspace(1, 50432, 50176, C.byref(p)) >= 50176 * 4
    assert lib.sharpv_prune_kv_workspace(0, 100, 10, C.byref(p)) == 0


def _no_gpu_here():
    """The calls below pass made-up device addresses; every one of them must be rejected on the host.
    With a GPU in the process a regression of a check would launch kernels on those addresses, so the
    fake-pointer cases only run where no device is visible."""
    import torch
    if torch.cuda.is_available():
        pytest.skip("fake device addresses are only passed where no GPU could be reached")


def _tok_call(lib, p, feats=0x1000, fo=None, B=1, n=4, f=16, d=64, idx=0x2000, cnt=0x3000, off=0x4000,
              out=0x5000, ws=0x10000, ws_bytes=1 << 30):
    # fake, well-aligned addresses: validation must return before anything is dereferenced
    return lib.sharpv_prune_tokens(feats, fo, B, n, f, d, C.byref(p), idx, cnt, off, out, None, None, ws, ws_bytes, None)


def test_prune_tokens_rejects_bad_arguments_on_the_host(lib):
    _no_gpu_here()
    p = sharpv.default_params()
    assert _tok_call(lib, p, feats=None) == 1
    assert _tok_call(lib, p, idx=None) == 1
    assert _tok_call(lib, p, B=2) == 1                       # ragged batch without offsets
    assert _tok_call(lib, p, f=0) == 2
    assert _tok_call(lib, p, f=1025) == 2
    assert _tok_call(lib, p, d=20) == 2
    assert _tok_call(lib, p, B=5, fo=0x6000) == 2            # more videos than frames
    assert _tok_call(lib, p, feats=0x1004) == 2              # misaligned
    assert _tok_call(lib, p, ws=None) == 5
    assert _tok_call(lib, p, ws=0x10010) == 5
    assert _tok_call(lib, p, ws_bytes=16) == 5
    q = sharpv.default_params(); q.dtype = 7
    assert _tok_call(lib, q) == 3
    q = sharpv.default_params(); q.struct_size = 8
    assert _tok_call(lib, q) == 4
    q = sharpv.default_params(); q.mode = 2
    assert _tok_call(lib, q) == 4
    q = sharpv.default_params(); q.min_keep = 17
    assert _tok_call(lib, q) == 4
    q = sharpv.default_params(); q.w = float("nan")
    assert _tok_call(lib, q) == 4
    q = sharpv.default_params(); q.measure = sharpv.ONE_MINUS_COS      # goes with the fixed threshold only
    assert _tok_call(lib, q) == 4
    q.mode = 1
    assert _tok_call(lib, q, feats=None) == 1                         # accepted as parameters: next check fires
    q.measure = 2
    assert _tok_call(lib, q) == 4
    assert lib.sharpv_prune_tokens(0x1000, None, 1, 4, 16, 64, None, 0x2000, 0x3000, 0x4000, 0x5000, None, None,
                                   0x10000, 1 << 30, None) == 1


def _kv_call(lib, p, hidden=0x1000, orig=0x2000, K=0x30000, V=0x40000, sh=64 * 32, ss=32, so=None, vs=None, vo=None,
             B=1, S=64, v0=4, nv=40, d=64, H=2, D=32, idx=0x5000, cnt=0x6000, Ko=0x70000, Vo=0x80000, osh=64 * 32,
             ws=0x10000, ws_bytes=1 << 30):
    return lib.sharpv_prune_kv(hidden, orig, K, V, sh, ss, so, vs, vo, B, S, v0, nv, d, H, D, 0, C.byref(p), idx,
                               cnt, Ko, Vo, osh, None, None, ws, ws_bytes, None)


def test_prune_kv_rejects_bad_arguments_on_the_host(lib):
    _no_gpu_here()
    p = sharpv.default_params()
    assert _kv_call(lib, p, hidden=None) == 1
    assert _kv_call(lib, p, Ko=None) == 1
    assert _kv_call(lib, p, so=0x9000) == 1                  # only one of the three batch arrays
    assert _kv_call(lib, p, B=2) == 1                        # B > 1 needs the arrays
    assert _kv_call(lib, p, nv=80) == 2                      # more visual tokens than positions
    assert _kv_call(lib, p, v0=40) == 2                      # visual block runs past the sequence
    assert _kv_call(lib, p, D=4) == 2                        # row not a multiple of 16 bytes
    assert _kv_call(lib, p, ss=20) == 2
    assert _kv_call(lib, p, d=12) == 2
    assert _kv_call(lib, p, Ko=0x30000) == 2                 # output aliases input
    # K spans 2 heads x 64 positions x 32 bf16 = 8192 bytes from 0x3000; outputs may not touch any of them
    assert _kv_call(lib, p, K=0x30000, V=0x40000, Ko=0x30000 + 64) == 2      # in-place compaction, one row on
    assert _kv_call(lib, p, K=0x30000, V=0x40000, Ko=0x30000 + 8192 - 16) == 2
    assert _kv_call(lib, p, K=0x30000, V=0x40000, Ko=0x30000 - 8192 + 16) == 2
    assert _kv_call(lib, p, K=0x30000, V=0x40000, Ko=0x50000, Vo=0x50000 + 4096) == 2    # the outputs overlap each other
    assert _kv_call(lib, p, K=0x30000, V=0x40000, Ko=0x40000 + 4096, Vo=0x60000) == 2    # K_out inside V
    assert _kv_call(lib, p, K=0x30000, V=0x40000, Ko=0x32000, Vo=0x42000, ws_bytes=8) == 5   # adjacent is fine
    assert _kv_call(lib, p, ws_bytes=8) == 5
    q = sharpv.default_params(); q.kv_mode = 3
    assert _kv_call(lib, q) == 4


def test_prune_kv_static_rejects_bad_arguments_and_sizes_on_the_host(lib):
    _no_gpu_here()
    p = sharpv.default_params()

    def call(hidden=0x1000, S=64, B=1, nv=40, so=None, vs=None, vo=None, Ko=0x7 << 32, params=p):
        return lib.sharpv_prune_kv_static(hidden, 0x2000, 0x3 << 32, 0x4 << 32, S * 32, 32, so, vs, vo, B, S, 4, nv, 64, 2, 32,
                                          0, C.byref(params), 0x5000, 0x6000, Ko, 0x8 << 32, S * 32, None, None, None)
    assert call(hidden=None) == 1                            # the checks of sharpv_prune_kv come first
    assert call(nv=80) == 2
    assert call(Ko=0x3 << 32) == 2
    q = sharpv.default_params(); q.kv_mode = 3
    assert call(params=q) == 4
    assert call(S=262144 + 1) == 7                           # beyond the built-in scratch
    assert call(S=1 << 20, nv=0) == 7
    assert call(S=4096, B=257, so=0x9000, vs=0xA000, vo=0xB000) == 7
    assert "scratch" in sharpv.status_string(7)
    # a call that passes every check needs the scratch's device address next: no device here
    assert call() == 6


def _kv_rope_call(lib, p, cos=0xA000, sin=0xB000, rope_len=64, layout=0, D=32, ws_bytes=1 << 30, hidden=0x1000):
    return lib.sharpv_prune_kv_rope(hidden, 0x2000, 0x30000, 0x40000, 64 * D, D, None, None, None, 1, 64, 4, 40, 64, 2,
                                    D, 0, C.byref(p), 0x5000, 0x6000, 0x70000, 0x80000, 64 * D, None, None, cos, sin,
                                    rope_len, layout, 0x10000, ws_bytes, None)


def test_prune_kv_rope_rejects_bad_arguments_on_the_host(lib):
    _no_gpu_here()
    p = sharpv.default_params()
    assert _kv_rope_call(lib, p, cos=None) == 1
    assert _kv_rope_call(lib, p, sin=None) == 1
    assert _kv_rope_call(lib, p, layout=2) == 4
    assert _kv_rope_call(lib, p, rope_len=63) == 2           # a shift of S-1 must have a table row
    assert _kv_rope_call(lib, p, D=8) == 2                   # half a bf16 row of 8 elements is not whole 16-byte pieces
    assert _kv_rope_call(lib, p, cos=0xA002) == 2            # misaligned table
    assert _kv_rope_call(lib, p, hidden=None) == 1           # the checks of sharpv_prune_kv still apply
    assert _kv_rope_call(lib, p, ws_bytes=8) == 5


def _kv_carried_call(lib, p, rows=0x9000, out_rows=0xC000, n_orig=500, B=1, so=None, cos=None, sin=None,
                     rope_len=0, S=64, ws_bytes=1 << 30):
    return lib.sharpv_prune_kv_carried(0x1000, 0x2000, rows, 0x30000, 0x40000, 64 * 32, 32, so, B, S, n_orig, 64, 2, 32,
                                       0, C.byref(p), 0x5000, 0x6000, 0x70000, 0x80000, 64 * 32, out_rows, None, cos,
                                       sin, rope_len, 0, 0x10000, ws_bytes, None)


def test_prune_kv_carried_rejects_bad_arguments_on_the_host(lib):
    _no_gpu_here()
    p = sharpv.default_params()
    assert lib.sharpv_prune_kv_carried_workspace(1, 64, C.byref(p)) == lib.sharpv_prune_kv_workspace(1, 64, 64, C.byref(p))
    assert _kv_carried_call(lib, p, rows=None) == 1
    assert _kv_carried_call(lib, p, out_rows=None) == 1
    assert _kv_carried_call(lib, p, n_orig=0) == 2
    assert _kv_carried_call(lib, p, B=2) == 1                # a batch needs seq_offsets
    assert _kv_carried_call(lib, p, cos=0xA000) == 1         # one rotary table without the other
    assert _kv_carried_call(lib, p, cos=0xA000, sin=0xB000, rope_len=10) == 2
    assert _kv_carried_call(lib, p, rows=0x9001) == 2
    assert _kv_carried_call(lib, p, ws_bytes=8) == 5
    q = sharpv.default_params(); q.kv_mode = 1
    assert _kv_carried_call(lib, q) == 4                     # per-token decisions only


def test_binding_refuses_to_run_without_a_gpu():
    import torch
    if torch.cuda.is_available():
        pytest.skip("GPU present")
    with pytest.raises(RuntimeError):
        sharpv.prune_tokens(torch.zeros(2, 4, 8))
    with pytest.raises(RuntimeError):
        sharpv.prune_kv(torch.zeros(8, 8), torch.zeros(4, 8), torch.zeros(1, 8, 8), torch.zeros(1, 8, 8))
