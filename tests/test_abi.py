"""Host-side checks of the C-ABI library: it loads, exports what include/pasa.h declares, validates
arguments before touching the GPU, and its host-only beta solver agrees with the paper and the oracle.
No compute call is made here (there is no GPU in this test tier)."""
import ctypes
import math
import os
import re

import pytest

import paper_2503_01873_amd as P
from oracle import pasa_oracle as po

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "pasa.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pasa_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = P.lib()
    names = _declared_functions()
    assert {"pasa_attn_fwd", "pasa_attn_fwd_ex", "pasa_attn_fwd_static", "pasa_attn_fwd_workspace",
            "pasa_attn_fwd_workspace_min", "pasa_prepare_kv",
            "pasa_attn_fwd_prepared", "pasa_attn_fwd_chunk", "pasa_attn_fwd_adaptive", "pasa_shift_keys", "pasa_shift_keys_matrix", "pasa_shift_keys_direct",
            "pasa_optimal_beta", "pasa_invariance_rounded",
            "pasa_status_string", "pasa_version"} <= set(names)
    for n in names:
        assert hasattr(L, n), n
    assert P.pasa_version() >= 100


def test_static_entry_point_checks_sizes_on_the_host():
    # shape errors and sizes beyond the library's fixed workspace are refused before any device is touched
    assert P.pasa_attn_fwd_static(16, 16, 16, 32, 1, 3, 2, 256, 64, 0, 0.125, check=False) == 1      # Hq % Hkv
    assert P.pasa_attn_fwd_static(16, 16, 16, 32, 1, 1, 1, 256, 96, 0, 0.125, check=False) == 2      # d
    assert P.pasa_attn_fwd_workspace_min(14, 5, 9216, 64) > P.STATIC_WORKSPACE_BYTES
    assert P.pasa_attn_fwd_static(16, 16, 16, 32, 14, 5, 5, 9216, 64, 0, 0.125, check=False) == 4
    assert P.pasa_attn_fwd_workspace_min(1, 8, 8192, 128) <= P.STATIC_WORKSPACE_BYTES
    text = open(os.path.join(ROOT, "include", "pasa.h")).read()
    assert "#define PASA_STATIC_WORKSPACE_BYTES (33u << 20)" in text and P.STATIC_WORKSPACE_BYTES == 33 << 20


def test_missing_library_fails_loudly(monkeypatch):
    from paper_2503_01873_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", "/nonexistent/libpasa.so")
    with pytest.raises(FileNotFoundError):
        binding.lib()


def test_status_strings():
    for st in range(5):
        assert P.pasa_status_string(st) not in ("", "unknown status")
    assert P.pasa_status_string(99) == "unknown status"


def test_optimal_beta_matches_paper_and_oracle(golden):
    for b0, want in golden("optimal_beta.txt"):
        got = P.pasa_optimal_beta(float(b0), 128, 0)
        assert f"{got:.6f}" == want
        assert got == pytest.approx(po.optimal_beta(float(b0), 128, "f16"), rel=1e-12)
        # the library's solution is exact: it reproduces its own rounded pair, so the condition holds to the last bit
        assert P.pasa_invariance_rounded(got, 128, 0) == pytest.approx(got / (1 - got), rel=1e-13)
    for b0 in (0.9, 0.99, 0.999):
        assert P.pasa_optimal_beta(b0, 128, 0) == pytest.approx(po.optimal_beta(b0, 128, "f16"), rel=1e-12)
        assert P.pasa_invariance_rounded(b0, 128, 0) == pytest.approx(po.invariance_rounded(b0, 128, "f16"), rel=1e-12)
    # bf16 (8 significand bits): 1 - beta/n rounds to 1, so a = 1 + b and the solution is a fixed point
    b = P.pasa_optimal_beta(1 - 2.0 ** -4, 128, 1)
    assert b == pytest.approx(po.optimal_beta(1 - 2.0 ** -4, 128, "bf16"), rel=1e-12)
    assert P.pasa_invariance_rounded(b, 128, 1) == pytest.approx(b / (1 - b), rel=1e-7)
    assert math.isnan(P.pasa_optimal_beta(1.5, 128, 0))
    assert math.isnan(P.pasa_optimal_beta(0.9, 0, 0))
    assert math.isnan(P.pasa_optimal_beta(0.9, 128, 7))


def test_workspace_size():
    # K'/V tiles, then one fp16 shift vector per key tile (rounded up to 256 bytes), then the counters of the adaptive
    # start (256 bytes here), then one mean block of 32 x d halfs per (KV head, 16 key tiles): the part every call needs
    assert P.pasa_attn_fwd_workspace_min(1, 4, 8192, 128) == 4 * 4 * 8192 * 128 + 2 * 4 * 64 * 128 + 256 + 4 * 4 * 64 * 128
    assert P.pasa_attn_fwd_workspace_min(1, 4, 8192, 96) == 0
    assert P.pasa_attn_fwd_workspace_min(1, 4, 8190, 128) == P.pasa_attn_fwd_workspace_min(1, 4, 8192, 128)   # ragged last tile is padded
    assert P.pasa_attn_fwd_workspace_min(1, 4, 1, 64) == 4 * 4 * 128 * 64 + 512 + 256 + 4 * 64 * 64
    assert P.pasa_attn_fwd_workspace_min(1, 1, 128, 64) == 4 * 128 * 64 + 256 + 256 + 64 * 64
    assert P.pasa_attn_fwd_workspace_min(1, 1, 17 * 128, 64) == 4 * 17 * 128 * 64 + 2 * 17 * 64 + 128 + 256 + 2 * 64 * 64
    # then the region of the key split: 1 MiB where a self-attention call of these sizes fills the chip by itself ...
    assert P.pasa_attn_fwd_workspace(1, 28, 4, 8192, 128) == P.pasa_attn_fwd_workspace_min(1, 4, 8192, 128) + (1 << 20)
    # ... and per split and row d floats + two doubles where it does not: 8 heads x 16 query tiles = 128 workgroups,
    # 32 key tiles -> two ways
    assert P.pasa_attn_fwd_workspace(1, 8, 8, 4096, 128) == P.pasa_attn_fwd_workspace_min(1, 8, 4096, 128) + 2 * 8 * 4096 * (128 * 4 + 16)
    assert P.pasa_attn_fwd_workspace(1, 28, 4, 8192, 96) == 0
    assert P.pasa_attn_fwd_workspace(1, 28, 5, 8192, 128) == 0


# fake, well-aligned non-null addresses: every call below must be rejected on the host before any use
Q, K, V, O, WS = 0x10000, 0x20000, 0x30000, 0x40000, 0x50000
OK_ARGS = dict(B=1, Hq=4, Hkv=2, N=256, d=64, causal=0, scale=0.125)


def _ex(**over):
    a = dict(OK_ARGS)
    ptr = dict(q=Q, k=K, v=V, o=O, ws=WS, wsb=1 << 20, beta=-1.0, variant=P.MIXED, shift_tile=128,
               shift_mode=P.SHIFT_MEAN, io_dtype=P.IO_F16)
    for key, val in over.items():
        (ptr if key in ptr else a)[key] = val
    return P.pasa_attn_fwd_ex(ptr["q"], ptr["k"], ptr["v"], ptr["o"], a["B"], a["Hq"], a["Hkv"], a["N"], a["d"],
                              a["causal"], a["scale"], ptr["ws"], ptr["wsb"], beta=ptr["beta"],
                              variant=ptr["variant"], shift_tile=ptr["shift_tile"], shift_mode=ptr["shift_mode"],
                              io_dtype=ptr["io_dtype"], check=False)


@pytest.mark.parametrize("over,want", [
    (dict(q=0), 1), (dict(k=0), 1), (dict(v=0), 1), (dict(o=0), 1),
    (dict(q=Q + 2), 1), (dict(o=O + 8), 1), (dict(o=Q), 1), (dict(o=K), 1),
    (dict(B=0), 1), (dict(N=0), 1), (dict(N=-128), 1), (dict(Hq=3), 1), (dict(Hkv=0), 1),
    (dict(scale=0.0), 1), (dict(scale=-1.0), 1), (dict(scale=float("nan")), 1), (dict(scale=float("inf")), 1),
    (dict(causal=2), 1), (dict(variant=5), 1), (dict(variant=-1), 1), (dict(variant=P.DIRECT, shift_mode=P.SHIFT_MATRIX), 1), (dict(beta=1.0), 1), (dict(beta=float("nan")), 1),
    (dict(d=96), 2), (dict(d=256), 2), (dict(N=262144 + 128), 2), (dict(shift_tile=64), 2),
    (dict(ws=0), 4), (dict(ws=WS + 16), 4), (dict(wsb=1024), 4),
    (dict(shift_mode=3), 1), (dict(shift_mode=-1), 1), (dict(shift_mode=P.SHIFT_MATRIX, N=200), 2),
    (dict(shift_mode=P.SHIFT_MATRIX_MFMA, N=200), 2), (dict(variant=P.DIRECT, shift_mode=P.SHIFT_MATRIX_MFMA), 1),
    (dict(io_dtype=2), 1), (dict(io_dtype=-1), 1),
])
def test_attn_fwd_ex_rejects_bad_arguments(over, want):
    assert _ex(**over) == want


def test_other_entry_points_reject_bad_arguments():
    assert P.pasa_attn_fwd(0, K, V, O, 1, 4, 2, 256, 64, 0, 0.125, check=False) == 1
    assert P.pasa_attn_fwd(Q, K, V, O, 1, 4, 2, 256, 96, 0, 0.125, check=False) == 2
    assert P.pasa_attn_fwd(Q, K, V, O, 1, 4, 3, 256, 64, 0, 0.125, check=False) == 1
    assert P.pasa_shift_keys(0, O, 1, 2, 256, 64, 0.5, 0.125, check=False) == 1
    assert P.pasa_shift_keys(K, K, 1, 2, 256, 64, 0.5, 0.125, check=False) == 1
    assert P.pasa_shift_keys(K, O, 1, 2, 256, 64, 1.0, 0.125, check=False) == 1
    assert P.pasa_shift_keys(K, O, 1, 2, 256, 32, 0.5, 0.125, check=False) == 2
    assert P.pasa_shift_keys_matrix(K, O, 1, 2, 200, 64, 0.5, 0.125, check=False) == 2    # M is 128 x 128
    assert P.pasa_shift_keys_matrix(K, O, 1, 2, 256, 64, -0.5, 0.125, check=False) == 1
    assert P.pasa_prepare_kv(K, V, 1, 2, 200, 64, 0.125, WS, 1 << 20, shift_mode=P.SHIFT_MATRIX, check=False) == 2
    chunk = dict(B=1, Hq=4, Hkv=2, Nq=100, row0=156, N=256, d=64, causal=1, scale=0.125, workspace=WS,
                 workspace_bytes=1 << 20, check=False)
    assert P.pasa_attn_fwd_chunk(0, O, **chunk) == 1
    assert P.pasa_attn_fwd_chunk(Q, O, **{**chunk, "Nq": 0}) == 1
    assert P.pasa_attn_fwd_chunk(Q, O, **{**chunk, "row0": -1}) == 1
    assert P.pasa_attn_fwd_chunk(Q, O, **{**chunk, "Nq": 262144 + 1}) == 2
    assert P.pasa_attn_fwd_workspace_min(1, 2, 256, 64) == 4 * 2 * 256 * 64 + 512 + 256 + 2 * 64 * 64
    assert P.pasa_attn_fwd_chunk(Q, O, **{**chunk, "workspace_bytes": P.pasa_attn_fwd_workspace_min(1, 2, 256, 64) - 1}) == 4
    assert P.pasa_shift_keys_direct(K, O, 0, 1, 2, 256, 64, 0.5, 0.125, check=False) == 1
    assert P.pasa_shift_keys_direct(K, O, O, 1, 2, 256, 64, 0.5, 0.125, check=False) == 1
    assert P.pasa_attn_fwd_chunk(Q, O, **{**chunk, "N": 200, "shift_mode": P.SHIFT_MATRIX}) == 2
    ad = dict(B=1, Hq=4, Hkv=2, N=256, d=64, causal=0, scale=0.125, workspace=WS, workspace_bytes=1 << 20, check=False)
    CNT = 0x60000
    assert P.pasa_attn_fwd_adaptive(Q, K, V, O, overflow_s=None, **ad) == 1             # the trigger counter is required
    assert P.pasa_attn_fwd_adaptive(Q, K, V, O, overflow_s=CNT, opts_null=True, **ad) == 1
    assert P.pasa_attn_fwd_adaptive(Q, K, V, O, overflow_s=CNT, nonfinite_o=CNT + 8, **ad) == 1
    assert P.pasa_attn_fwd_adaptive(Q, K, V, O, overflow_s=CNT, variant=P.NAIVE16, **ad) == 1
    assert P.pasa_attn_fwd_adaptive(Q, K, V, O, overflow_s=CNT + 4, **ad) == 1           # misaligned counter
    assert P.pasa_attn_fwd_adaptive(Q, K, V, O, overflow_s=CNT, **{**ad, "d": 96}) == 2
    assert P.pasa_attn_fwd_adaptive(Q, K, V, O, overflow_s=CNT, **{**ad, "workspace_bytes": 64}) == 4
    assert P.pasa_prepare_kv(K, V, 1, 2, 256, 64, 0.125, WS, 16, check=False) == 4
    assert P.pasa_prepare_kv(K, 0, 1, 2, 256, 64, 0.125, WS, 1 << 20, check=False) == 1
    assert P.pasa_attn_fwd_prepared(Q, Q, 1, 4, 2, 256, 64, 0, 0.125, WS, 1 << 20, check=False) == 1
    assert P.pasa_attn_fwd_prepared(Q, O, 1, 4, 2, 256, 64, 0, 0.125, 0, 1 << 20, check=False) == 4
    with pytest.raises(P.PasaError):
        P.pasa_attn_fwd_prepared(Q, O, 1, 4, 2, 256, 64, 0, 0.125, 0, 1 << 20)
