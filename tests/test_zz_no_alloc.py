"""The entry point that allocates nothing (pasa_attn_fwd_static) against pasa_attn_fwd_ex, through the C ABI.

Two calls in a row on the same GPU, the second with a smaller input: the library's fixed workspace still holds the
first call's tiles then, and nothing of them may leak into the second result.  Both entry points run the same
kernels on the same inputs, so their outputs have to be equal bit for bit; the first is also held to the oracle.
"""
import numpy as np
import pytest

import paper_2503_01873_amd as P
from oracle import pasa_oracle as po
from workloads import Workload, gen_full

pytestmark = pytest.mark.gpu


def _inputs(seed, B, Hq, Hkv, N, d):
    return gen_full(Workload("static", B, Hq, Hkv, N, d, True, seed, "tiny"))     # N(0,1), keys + 4


def _both(q, k, v, causal, variant):
    import torch
    dev = torch.device("cuda:0")
    B, Hq, N, d = q.shape
    Hkv = k.shape[1]
    scale = float(np.float32(1.0 / np.sqrt(d)))
    tq, tk, tv = (torch.from_numpy(x).to(dev) for x in (q, k, v))
    stream = torch.cuda.current_stream()
    wsb = P.pasa_attn_fwd_workspace(B, Hq, Hkv, N, d)
    ws = torch.empty(wsb, dtype=torch.uint8, device=dev)
    o_ex = torch.full_like(tq, float("nan"))
    P.pasa_attn_fwd_ex(tq, tk, tv, o_ex, B, Hq, Hkv, N, d, causal, scale, ws, wsb, stream, variant=variant)
    o_st = torch.full_like(tq, float("nan"))
    P.pasa_attn_fwd_static(tq, tk, tv, o_st, B, Hq, Hkv, N, d, causal, scale, stream, variant=variant)
    torch.cuda.synchronize()
    return o_ex.cpu().numpy(), o_st.cpu().numpy(), scale


@pytest.mark.parametrize("variant", [P.MIXED, P.STRICT16, P.DIRECT])
def test_static_entry_point_two_calls_second_smaller(variant):
    # first call: several key tiles and a ragged tail, grouped-query heads, d = 128
    q, k, v = _inputs(11, 2, 4, 2, 5 * 128 + 37, 128)
    o_ex, o_st, scale = _both(q, k, v, True, variant)
    assert np.isfinite(o_st).all()
    assert np.array_equal(o_ex.view(np.uint16), o_st.view(np.uint16))
    if variant == P.DIRECT:
        ref = po.direct_bhnd(q, k, v, scale, True, po.default_beta())
    else:
        ref = po.pasa_bhnd(q, k, v, scale, True, po.default_beta(), 128, {P.MIXED: po.MIXED, P.STRICT16: po.STRICT16}[variant])
    err = np.abs(o_st.astype(np.float64) - ref.astype(np.float64)).max()
    assert err <= 2e-3, err
    # second call, smaller in every dimension: the array still holds the tiles of the first
    q2, k2, v2 = _inputs(12, 1, 2, 1, 300, 64)
    o_ex2, o_st2, scale2 = _both(q2, k2, v2, False, variant)
    assert np.isfinite(o_st2).all()
    assert np.array_equal(o_ex2.view(np.uint16), o_st2.view(np.uint16))
    if variant != P.DIRECT:
        ref2 = po.pasa_bhnd(q2, k2, v2, scale2, False, po.default_beta(), 128,
                            {P.MIXED: po.MIXED, P.STRICT16: po.STRICT16}[variant])
        err2 = np.abs(o_st2.astype(np.float64) - ref2.astype(np.float64)).max()
        assert err2 <= 2e-3, err2


def test_static_entry_point_with_a_key_split():
    """Few query heads and many keys: the call splits the keys, with its partial results in what the fixed regions
    leave of the library's array.  (Not compared bit for bit with pasa_attn_fwd_ex here: given another amount of
    workspace that call may split another number of ways, which changes the rounding, not the result.)"""
    import torch
    dev = torch.device("cuda:0")
    q, k, v = _inputs(13, 1, 2, 1, 2200, 64)
    scale = float(np.float32(1.0 / 8.0))
    tq, tk, tv = (torch.from_numpy(x).to(dev) for x in (q, k, v))
    outs = []
    for _ in range(2):                       # twice: the second call finds the first one's partial results in the array
        to = torch.full_like(tq, float("nan"))
        P.pasa_attn_fwd_static(tq, tk, tv, to, 1, 2, 1, 2200, 64, True, scale, torch.cuda.current_stream())
        torch.cuda.synchronize()
        outs.append(to.cpu().numpy())
    assert np.array_equal(outs[0].view(np.uint16), outs[1].view(np.uint16))
    ref = po.pasa_bhnd(q, k, v, scale, True, po.default_beta(), 128, po.MIXED)
    err = np.abs(outs[0].astype(np.float64) - ref.astype(np.float64)).max()
    assert np.isfinite(outs[0]).all() and err <= 2e-3, err


def test_static_entry_point_refuses_what_does_not_fit():
    import torch
    dev = torch.device("cuda:0")
    # 14 x 5 heads of 9216 keys, d = 64: 165 MiB of tiles, beyond the fixed array
    B, Hq, Hkv, N, d = 14, 5, 5, 9216, 64
    assert P.pasa_attn_fwd_workspace_min(B, Hkv, N, d) > P.STATIC_WORKSPACE_BYTES
    t = torch.zeros(16, dtype=torch.float16, device=dev)       # never touched: the size check comes first
    st = P.pasa_attn_fwd_static(t, t, t, t, B, Hq, Hkv, N, d, 0, 0.125, torch.cuda.current_stream(), check=False)
    assert st == 4 and "workspace" in P.pasa_status_string(st)
    # the largest size that fits: exactly 8 Mi elements of keys
    assert P.pasa_attn_fwd_workspace_min(1, 8, 8192, 128) <= P.STATIC_WORKSPACE_BYTES
