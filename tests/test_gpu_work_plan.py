"""Planned causal launches on the GPU: workgroups that walk a list of work items give what one workgroup per item
gives, bit for bit, and that agrees with the oracle."""
import numpy as np
import pytest

import paper_2503_01873_amd as P
from oracle import pasa_oracle as po
from workloads import workload, gen_q_head, gen_kv_head
from gpu_harness import f32

pytestmark = pytest.mark.gpu

BETA = po.default_beta()


def _run(tq, tk, tv, B, Hq, Hkv, N, d, scale, variant, planned):
    import torch
    was = P.pasa_work_plan_enable(planned)
    try:
        to = torch.full_like(tq, float("nan"))
        wsb = P.pasa_attn_fwd_workspace(B, Hq, Hkv, N, d)
        ws = torch.empty(wsb, dtype=torch.uint8, device=tq.device)
        P.pasa_attn_fwd_ex(tq, tk, tv, to, B, Hq, Hkv, N, d, True, scale, ws, wsb, torch.cuda.current_stream(),
                           variant=variant)
        torch.cuda.synchronize()
    finally:
        P.pasa_work_plan_enable(was)
    return to


@pytest.mark.parametrize("variant", [P.MIXED, P.DIRECT, P.S16, P.NAIVE16])
def test_lists_of_items_give_the_same_bits_as_one_workgroup_per_item(variant):
    import torch
    B, Hq, Hkv, N, d = 3, 36, 4, 1280, 128
    places = torch.cuda.get_device_properties(0).multi_processor_count
    plan = P.pasa_work_plan(B, Hq, Hkv, N, 0, N, places)
    assert plan is not None and plan[3], "this shape is meant to follow its plan"
    g = torch.Generator().manual_seed(5)
    tq = torch.randn(B, Hq, N, d, generator=g).half().cuda()
    tk = (torch.randn(B, Hkv, N, d, generator=g) + 1.5).half().cuda()
    tv = torch.randn(B, Hkv, N, d, generator=g).half().cuda()
    scale = f32(d ** -0.5)
    a = _run(tq, tk, tv, B, Hq, Hkv, N, d, scale, variant, True)
    b = _run(tq, tk, tv, B, Hq, Hkv, N, d, scale, variant, False)
    assert bool(torch.isfinite(a).all())
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))


def test_planned_launch_of_the_qwen_shape_at_6144_against_the_oracle():
    import torch
    w = workload(3).with_n(6144)
    places = torch.cuda.get_device_properties(0).multi_processor_count
    plan = P.pasa_work_plan(w.B, w.Hq, w.Hkv, w.N, 0, w.N, places)
    assert plan is not None and plan[3]
    dev = torch.device("cuda:0")
    tq = torch.empty((w.B, w.Hq, w.N, w.d), dtype=torch.float16, device=dev)
    tk = torch.empty((w.B, w.Hkv, w.N, w.d), dtype=torch.float16, device=dev)
    tv = torch.empty_like(tk)
    host = {}
    for hk in range(w.Hkv):
        kk, vv = gen_kv_head(w, 0, hk)
        tk[0, hk].copy_(torch.from_numpy(kk))
        tv[0, hk].copy_(torch.from_numpy(vv))
        host[("kv", hk)] = (kk, vv)
    for h in range(w.Hq):
        qq = gen_q_head(w, 0, h)
        tq[0, h].copy_(torch.from_numpy(qq))
        host[("q", h)] = qq
    scale = f32(w.scale)
    a = _run(tq, tk, tv, w.B, w.Hq, w.Hkv, w.N, w.d, scale, P.MIXED, True)
    b = _run(tq, tk, tv, w.B, w.Hq, w.Hkv, w.N, w.d, scale, P.MIXED, False)
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    worst = 0.0
    for h, r0 in [(0, 0), (9, 2944), (27, w.N - 128)]:
        kk, vv = host[("kv", h // w.group)]
        ref = po.pasa_rows(host[("q", h)][r0:r0 + 128], kk[:r0 + 128], vv[:r0 + 128], scale, True, BETA, 128, po.MIXED, r0)
        got = a[0, h, r0:r0 + 128].cpu().numpy()
        worst = max(worst, float(np.abs(got.astype(np.float64) - ref.astype(np.float64)).max()))
    print("planned launch, max-abs against the emulated oracle %.3e" % worst)
    assert worst <= 2e-3
