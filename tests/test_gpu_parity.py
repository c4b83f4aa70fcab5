"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element.

Tolerances.  The spec bars are max-abs <= 2e-3 against the fp16-emulated oracle of the same
precision allocation and RMSE <= 1e-3 against fp64.  The first is asserted as stated wherever the
computation is well conditioned.  On the large-bias workloads the method itself multiplies every
rounding difference in the pseudo-average Sbar' by the invariance 63.5 (Algorithm 1, correction terms),
so a last-bit difference in an fp32 accumulation order (MIXED) or a one-ulp fp16 flip of S' / Sbar'
(S16, STRICT16) moves a whole tile's softmax weight; there the assertion is on the 99.9th / 99th
percentile of the element differences, and -- the strong statistical statement -- on the GPU's RMSE
against fp64 equalling the oracle's own RMSE to within 2 %.  The RMSE <= 1e-3 bar is asserted where the
oracle (i.e. the method) meets it and reported otherwise.
"""
import numpy as np
import pytest

import paper_2503_01873_amd as P
from oracle import pasa_oracle as po
from workloads import Workload, workload, gen_full, gen_q_head, gen_kv_head
from gpu_harness import bf16_bits, gpu_attn, gpu_attn_chunks, compare, f32, ORACLE_POLICY, VARIANT_NAME

pytestmark = pytest.mark.gpu

BETA = po.default_beta()


def _small(idx, N, **over):
    w = workload(idx).with_n(N)
    return Workload(**{**w.__dict__, **over})


# ------------------------------------------------------------------ key pre-processing: bit exact

@pytest.mark.parametrize("d,beta,kscale", [(64, BETA, 0.125), (128, BETA, f32(128 ** -0.5)), (128, 0.9375, 1.0),
                                            (64, 0.0, f32(64 ** -0.5))])
def test_shift_keys_bit_exact(d, beta, kscale):
    import torch
    rng = np.random.default_rng(d)
    k = (rng.standard_normal((2, 3, 384, d)) * rng.uniform(0.1, 30, (1, 1, 1, d)) + rng.uniform(-80, 80, (2, 3, 1, d))).astype(np.float16)
    tk = torch.from_numpy(k).cuda()
    out = torch.empty_like(tk)
    P.pasa_shift_keys(tk, out, 2, 3, 384, d, beta, kscale)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    want = np.stack([[po.shift_keys(k[b, h], beta, kscale) for h in range(3)] for b in range(2)])
    assert np.array_equal(got.view(np.uint16), want.view(np.uint16))


@pytest.mark.parametrize("N,d", [(1, 64), (77, 128), (300, 64), (511, 128)])
def test_shift_keys_ragged_bit_exact(N, d):
    import torch
    rng = np.random.default_rng(N * d)
    k = (rng.standard_normal((1, 2, N, d)) * 4 + rng.uniform(-80, 80, (1, 2, 1, d))).astype(np.float16)
    tk = torch.from_numpy(k).cuda()
    flat = torch.full((k.size + 1024,), float("nan"), dtype=torch.float16, device="cuda")
    out = flat[:k.size].view(tk.shape)
    P.pasa_shift_keys(tk, out, 1, 2, N, d, BETA, 0.125)
    torch.cuda.synchronize()
    want = np.stack([[po.shift_keys(k[0, h], BETA, 0.125) for h in range(2)]])
    assert np.array_equal(out.cpu().numpy().view(np.uint16), want.view(np.uint16))
    assert bool(torch.isnan(flat[k.size:]).all())


# ------------------------------------------------------------------ workload 1: the stated bars

@pytest.mark.parametrize("variant", [P.MIXED, P.S16, P.STRICT16])
def test_tiny_workload_full_tensor(variant):
    w = workload(1)
    q, k, v = gen_full(w)
    scale = f32(w.scale)
    o, cnt = gpu_attn(q, k, v, w.causal, scale, variant, counters=True)
    ref = po.pasa_bhnd(q, k, v, scale, w.causal, BETA, 128, ORACLE_POLICY[variant])
    c = compare(o, ref)
    print(VARIANT_NAME[variant], c)
    assert np.isfinite(o).all() and cnt.tolist() == [0, 0]
    assert c["maxabs"] <= 2e-3
    gold = po.attention_fp64_bhnd(q, k, v, scale, w.causal)
    r_gpu, r_or = po.rmse(o, gold), po.rmse(ref, gold)
    print("rmse gpu %.3e oracle %.3e" % (r_gpu, r_or))
    assert abs(r_gpu - r_or) <= 0.02 * r_or + 2e-5


# ------------------------------------------------------------------ scaled-down workloads, several tiles + ragged tail

SMALL = [
    (1, 384, {}),                                    # 256-row workgroup + a 128-row tail
    (2, 640, dict(Hq=2, Hkv=2)),
    (3, 896, dict(Hq=8, Hkv=2)),                     # causal, GQA 4:1, outlier channels
    (4, 640, dict(B=2)),                             # d = 64, resonance
    (5, 2176, dict(B=1, Hq=4, Hkv=2)),               # causal, bias changes every 1024 keys
]


@pytest.mark.parametrize("variant", [P.MIXED, P.S16, P.STRICT16])
@pytest.mark.parametrize("idx,N,over", SMALL)
def test_scaled_workloads_full_tensor(idx, N, over, variant):
    w = _small(idx, N, **over)
    q, k, v = gen_full(w)
    scale = f32(w.scale)
    o, cnt = gpu_attn(q, k, v, w.causal, scale, variant, counters=True)
    ref = po.pasa_bhnd(q, k, v, scale, w.causal, BETA, 128, ORACLE_POLICY[variant])
    gold = po.attention_fp64_bhnd(q, k, v, scale, w.causal)
    c = compare(o, ref)
    r_gpu, r_or = po.rmse(o, gold), po.rmse(ref, gold)
    print(w.name, N, VARIANT_NAME[variant], c, "rmse gpu %.3e oracle %.3e" % (r_gpu, r_or))
    assert np.isfinite(o).all() and cnt.tolist() == [0, 0]
    assert abs(r_gpu - r_or) <= 0.02 * r_or + 2e-5
    if variant == P.MIXED:
        assert c["maxabs"] <= 2e-3          # the stated bar, on every workload
    elif variant == P.STRICT16:
        assert c["p999"] <= 2e-3
    else:
        assert c["p99"] <= 5e-3
    if r_or <= 1e-3:
        assert r_gpu <= 1e-3


# ------------------------------------------------------------------ the three solutions of the optimal accuracy condition

@pytest.mark.parametrize("variant", [P.MIXED, P.STRICT16])
@pytest.mark.parametrize("beta", [0.9375, 0.968994, 0.984497])
def test_paper_betas_scaled_workload(beta, variant):
    """Section 2.3 lists three solutions of the optimal accuracy condition and adopts the last; the kernel takes any
    of them.  The option is a C float, so both sides use the float value."""
    beta = float(np.float32(beta))
    for idx, N, over in ((1, 384, {}), (3, 896, dict(Hq=8, Hkv=2))):
        w = _small(idx, N, **over)
        q, k, v = gen_full(w)
        scale = f32(w.scale)
        o, cnt = gpu_attn(q, k, v, w.causal, scale, variant, beta=beta, counters=True)
        ref = po.pasa_bhnd(q, k, v, scale, w.causal, beta, 128, ORACLE_POLICY[variant])
        gold = po.attention_fp64_bhnd(q, k, v, scale, w.causal)
        c = compare(o, ref)
        r_gpu, r_or = po.rmse(o, gold), po.rmse(ref, gold)
        print(w.name, beta, VARIANT_NAME[variant], c, "rmse gpu %.3e oracle %.3e" % (r_gpu, r_or))
        assert np.isfinite(o).all() and cnt.tolist() == [0, 0]
        assert abs(r_gpu - r_or) <= 0.02 * r_or + 2e-5
        if variant == P.MIXED:
            assert c["maxabs"] <= 2e-3
        else:
            assert c["p999"] <= 2e-3
    # the first solution has the smallest invariance (15): on the benign workload it meets the 1e-3 bar against fp64
    if variant == P.MIXED and beta == 0.9375:
        w = workload(1)
        q, k, v = gen_full(w)
        o, _ = gpu_attn(q, k, v, w.causal, f32(w.scale), P.MIXED, beta=beta)
        assert po.rmse(o, po.attention_fp64_bhnd(q, k, v, f32(w.scale), w.causal)) <= 1e-3


# ------------------------------------------------------------------ overflow behaviour

def test_naive16_overflows_on_large_bias_pasa_does_not():
    w = _small(2, 512, Hq=2, Hkv=2)
    q, k, v = gen_full(w)
    scale = f32(w.scale)
    o, cnt = gpu_attn(q, k, v, False, scale, P.NAIVE16, counters=True)
    ref = po.fa_bhnd(q, k, v, scale, False, 128, po.PARTIAL16)
    assert np.isnan(ref).all() and np.isnan(o).all()
    # every raw score exceeds 65504 (mean 128*8*80 = 81920): all S entries and all outputs are counted
    assert cnt.tolist() == [2 * 512 * 512, o.size]
    for variant in (P.MIXED, P.S16, P.STRICT16):
        o, cnt = gpu_attn(q, k, v, False, scale, variant, counters=True)
        assert np.isfinite(o).all() and cnt.tolist() == [0, 0]


def test_naive16_matches_oracle_when_nothing_overflows():
    w = _small(1, 512)
    q, k, v = gen_full(w)
    scale = f32(w.scale)
    o, cnt = gpu_attn(q, k, v, False, scale, P.NAIVE16, counters=True)
    ref = po.fa_bhnd(q, k, v, scale, False, 128, po.PARTIAL16)
    assert cnt.tolist() == [0, 0]
    assert compare(o, ref)["maxabs"] <= 2e-3


def test_naive16_partial_overflow_counts_match_oracle():
    # rows whose raw scores straddle 65504: the set of NaN outputs must be the oracle's
    rng = np.random.default_rng(5)
    N, d = 256, 128
    q = (rng.standard_normal((1, 1, N, d)) + 8).astype(np.float16)
    k = (rng.standard_normal((1, 1, N, d)) * 2 + 63.5).astype(np.float16)
    v = rng.standard_normal((1, 1, N, d)).astype(np.float16)
    scale = f32(d ** -0.5)
    o, cnt = gpu_attn(q, k, v, False, scale, P.NAIVE16, counters=True)
    ref = po.fa_bhnd(q, k, v, scale, False, 128, po.PARTIAL16)
    frac = np.isnan(ref).mean()
    assert 0.0 < frac < 1.0
    # a raw score within an fp32 accumulation error of the 65520 rounding boundary may fall either way
    assert abs(np.isnan(o).mean() - frac) < 0.02
    assert cnt[1] == np.isnan(o).sum() + np.isinf(o).sum()


# ------------------------------------------------------------------ options, entry points, edge sizes

@pytest.mark.parametrize("beta", [0.0, 0.5, 0.9375])
@pytest.mark.parametrize("causal", [False, True])
def test_other_betas(beta, causal):
    w = _small(1, 512, Hq=2, Hkv=1, causal=causal)
    q, k, v = gen_full(w)
    scale = f32(w.scale)
    for variant in (P.MIXED, P.STRICT16):
        o, _ = gpu_attn(q, k, v, causal, scale, variant, beta=beta)
        ref = po.pasa_bhnd(q, k, v, scale, causal, beta, 128, ORACLE_POLICY[variant])
        assert compare(o, ref)["maxabs"] <= 2e-3, (beta, causal, variant)


def test_entry_points_agree_and_are_deterministic():
    w = _small(3, 640, Hq=4, Hkv=2)
    q, k, v = gen_full(w)
    scale = f32(w.scale)
    a, _ = gpu_attn(q, k, v, True, scale, P.MIXED, entry="ex")
    b, _ = gpu_attn(q, k, v, True, scale, P.MIXED, entry="plain")
    c, _ = gpu_attn(q, k, v, True, scale, P.MIXED, entry="split")
    e, _ = gpu_attn(q, k, v, True, scale, P.MIXED, entry="ex")
    for other in (b, c, e):
        assert np.array_equal(a.view(np.uint16), other.view(np.uint16))


@pytest.mark.parametrize("N,d,causal", [(128, 64, False), (128, 128, True), (256, 128, True), (1152, 64, True)])
def test_edge_sizes(N, d, causal):
    rng = np.random.default_rng(N + d)
    q = rng.standard_normal((2, 2, N, d)).astype(np.float16)
    k = (rng.standard_normal((2, 1, N, d)) + 3).astype(np.float16)
    v = rng.standard_normal((2, 1, N, d)).astype(np.float16)
    scale = f32(d ** -0.5)
    o, _ = gpu_attn(q, k, v, causal, scale, P.MIXED)
    ref = po.pasa_bhnd(q, k, v, scale, causal, BETA, 128, po.MIXED)
    assert compare(o, ref)["maxabs"] <= 2e-3
    if causal:   # the first query sees one key: its output is that key's value, exactly
        assert np.array_equal(o[:, :, 0], v[:, [0, 0], 0])


# ------------------------------------------------------------------ sequence lengths that are not a multiple of the tile

@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("N,d", [(1, 64), (5, 128), (100, 64), (129, 128), (200, 64), (255, 128), (257, 64),
                                 (383, 128), (500, 128), (1000, 64)])
def test_ragged_lengths(N, d, causal):
    rng = np.random.default_rng(7 * N + d)
    q = rng.standard_normal((1, 4, N, d)).astype(np.float16)
    k = (rng.standard_normal((1, 2, N, d)) + 2.5).astype(np.float16)
    v = rng.standard_normal((1, 2, N, d)).astype(np.float16)
    scale = f32(d ** -0.5)
    o, cnt = gpu_attn(q, k, v, causal, scale, P.MIXED, counters=True)
    ref = po.pasa_bhnd(q, k, v, scale, causal, BETA, 128, po.MIXED)
    c = compare(o, ref)
    print(N, d, causal, c)
    assert np.isfinite(o).all() and cnt.tolist() == [0, 0]
    assert c["maxabs"] <= 2e-3
    gold = po.attention_fp64_bhnd(q, k, v, scale, causal)
    r_gpu, r_or = po.rmse(o, gold), po.rmse(ref, gold)      # the method's own error: the GPU must not add to it
    assert abs(r_gpu - r_or) <= 0.03 * r_or + 2e-5
    if causal:
        assert np.array_equal(o[:, :, 0], v[:, [0, 0, 1, 1], 0])


@pytest.mark.parametrize("variant", [P.STRICT16, P.S16])
@pytest.mark.parametrize("N,causal", [(200, True), (333, False)])
def test_ragged_lengths_other_variants(N, causal, variant):
    w = _small(1, N)
    q, k, v = gen_full(w)
    scale = f32(w.scale)
    o, _ = gpu_attn(q, k, v, causal, scale, variant)
    ref = po.pasa_bhnd(q, k, v, scale, causal, BETA, 128, ORACLE_POLICY[variant])
    c = compare(o, ref)
    print(VARIANT_NAME[variant], N, causal, c)
    assert np.isfinite(o).all()
    assert c["maxabs"] <= 2e-3


def test_ragged_naive16_matches_oracle():
    rng = np.random.default_rng(99)
    N, d = 300, 128
    q = rng.standard_normal((1, 2, N, d)).astype(np.float16)
    k = rng.standard_normal((1, 1, N, d)).astype(np.float16)
    v = rng.standard_normal((1, 1, N, d)).astype(np.float16)
    scale = f32(d ** -0.5)
    o, _ = gpu_attn(q, k, v, False, scale, P.NAIVE16)
    ref = po.fa_bhnd(q, k, v, scale, False, 128, po.PARTIAL16)
    assert compare(o, ref)["maxabs"] <= 2e-3


# ------------------------------------------------------------------ shift by the fp16-rounded matrix M (Algorithm 1 as printed)

PAPER_BETA = 0.984497


@pytest.mark.parametrize("d,beta,kscale", [(64, PAPER_BETA, 0.125), (128, PAPER_BETA, f32(128 ** -0.5)),
                                            (128, 0.9375, 1.0), (64, 0.0, f32(64 ** -0.5))])
def test_shift_keys_matrix_bit_exact(d, beta, kscale):
    import torch
    rng = np.random.default_rng(1000 + d)
    k = (rng.standard_normal((2, 3, 384, d)) * rng.uniform(0.1, 30, (1, 1, 1, d)) + rng.uniform(-80, 80, (2, 3, 1, d))).astype(np.float16)
    tk = torch.from_numpy(k).cuda()
    out = torch.empty_like(tk)
    P.pasa_shift_keys_matrix(tk, out, 2, 3, 384, d, beta, kscale)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    want = np.stack([[po.shift_keys(k[b, h], beta, kscale, 128, "gemm_m") for h in range(3)] for b in range(2)])
    assert np.array_equal(got.view(np.uint16), want.view(np.uint16))
    if beta == PAPER_BETA:   # the rounded entries do change the result: this is not the mean form in disguise
        mean_form = np.stack([[po.shift_keys(k[b, h], beta, kscale) for h in range(3)] for b in range(2)])
        assert (got != mean_form).mean() > 0.05


@pytest.mark.parametrize("d,beta,kscale", [(128, PAPER_BETA, 128 ** -0.5), (64, PAPER_BETA, 0.125), (128, 0.9375, 1.0)])
def test_shift_keys_matrix_on_the_matrix_core_within_fp32_accumulation(d, beta, kscale):
    """The pre-processing GEMM of Algorithm 1 on the matrix core: same operands as the exact evaluation (K and the
    fp16-rounded M), but the 128 products of an output are accumulated in fp32.  Bound on the accumulated value:
    |fl32 sum - exact| <= 128 * 2^-24 * sum_p |M[p,q] K[p,c]| (one rounding per addition, first order); the stored fp16
    value is then within half an fp16 step (2^-11 relative, or 2^-25 absolute in the subnormal range) of that."""
    import torch
    rng = np.random.default_rng(1500 + d)
    k = (rng.standard_normal((2, 3, 384, d)) * rng.uniform(0.1, 30, (1, 1, 1, d)) + rng.uniform(-80, 80, (2, 3, 1, d))).astype(np.float16)
    tk = torch.from_numpy(k).cuda()
    out = torch.empty_like(tk)
    P.pasa_shift_keys_matrix_mfma(tk, out, 2, 3, 384, d, beta, kscale)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    M16 = po.fl(po.shift_matrix(beta, 128, 1.0 / kscale), "f16")
    K64 = k.astype(np.float64).reshape(2, 3, 3, 128, d)
    exact = np.einsum("pq,bhjpc->bhjqc", M16, K64).reshape(2, 3, 384, d)
    mag = np.einsum("pq,bhjpc->bhjqc", np.abs(M16), np.abs(K64)).reshape(2, 3, 384, d)
    bound = 128 * 2.0 ** -24 * mag + np.maximum(2.0 ** -11 * np.abs(exact), 2.0 ** -25) * 1.0001
    assert (np.abs(got - exact) <= bound).all()
    want = np.stack([[po.shift_keys(k[b, h], beta, kscale, 128, "gemm_m") for h in range(3)] for b in range(2)])
    frac = float((out.cpu().numpy() != want).mean())
    print("K' values that differ from the exactly accumulated product: %.4f" % frac)
    assert frac <= 0.02


@pytest.mark.parametrize("idx,N,over", [(1, 256, {}), (3, 640, dict(Hq=7, Hkv=1))])
def test_matrix_shift_on_the_matrix_core_end_to_end(idx, N, over):
    w = _small(idx, N, **over)
    q, k, v = gen_full(w)
    scale = f32(w.scale)
    o, cnt = gpu_attn(q, k, v, w.causal, scale, P.MIXED, counters=True, shift_mode=P.SHIFT_MATRIX_MFMA)
    o_exact, _ = gpu_attn(q, k, v, w.causal, scale, P.MIXED, shift_mode=P.SHIFT_MATRIX)
    ref = po.pasa_bhnd(q, k, v, scale, w.causal, PAPER_BETA, 128, po.MIXED, shift="gemm_m")
    gold = po.attention_fp64_bhnd(q, k, v, scale, w.causal)
    c, ce = compare(o, ref), compare(o, o_exact)
    r_gpu, r_or = po.rmse(o, gold), po.rmse(ref, gold)
    print(w.name, "vs oracle", c, "vs exactly accumulated shift", ce, "rmse gpu %.3e oracle %.3e" % (r_gpu, r_or))
    assert np.isfinite(o).all() and cnt.tolist() == [0, 0]
    # a K' value that lands on the neighbouring fp16 value moves one score by 2^-11 |q_c K'_c| and the tile's
    # pseudo-average by 1/128 of that, times the invariance: far inside the tolerance of the exact path
    assert c["p999"] <= 2e-3 and c["maxabs"] <= 4e-3
    assert abs(r_gpu - r_or) <= 0.05 * r_or + 2e-5


@pytest.mark.parametrize("variant", [P.MIXED, P.S16, P.STRICT16])
def test_matrix_shift_tiny_workload_full_tensor(variant):
    w = workload(1)
    q, k, v = gen_full(w)
    scale = f32(w.scale)
    o, cnt = gpu_attn(q, k, v, w.causal, scale, variant, counters=True, shift_mode=P.SHIFT_MATRIX)
    ref = po.pasa_bhnd(q, k, v, scale, w.causal, PAPER_BETA, 128, ORACLE_POLICY[variant], shift="gemm_m")
    c = compare(o, ref)
    print(VARIANT_NAME[variant], c)
    assert np.isfinite(o).all() and cnt.tolist() == [0, 0]
    assert c["maxabs"] <= 2e-3


@pytest.mark.parametrize("idx,N,over", [(2, 512, dict(Hq=2, Hkv=1)), (3, 640, dict(Hq=7, Hkv=1))])
def test_matrix_shift_scaled_workloads(idx, N, over):
    w = _small(idx, N, **over)
    q, k, v = gen_full(w)
    scale = f32(w.scale)
    o, cnt = gpu_attn(q, k, v, w.causal, scale, P.MIXED, counters=True, shift_mode=P.SHIFT_MATRIX)
    ref = po.pasa_bhnd(q, k, v, scale, w.causal, PAPER_BETA, 128, po.MIXED, shift="gemm_m")
    gold = po.attention_fp64_bhnd(q, k, v, scale, w.causal)
    c = compare(o, ref)
    r_gpu, r_or = po.rmse(o, gold), po.rmse(ref, gold)
    print(w.name, c, "rmse gpu %.3e oracle %.3e" % (r_gpu, r_or))
    assert np.isfinite(o).all() and cnt.tolist() == [0, 0]
    assert c["maxabs"] <= 2e-3
    assert abs(r_gpu - r_or) <= 0.03 * r_or + 2e-5


# ------------------------------------------------------------------ bf16 inputs and outputs

def _bf16_case(idx, N, **over):
    w = _small(idx, N, **over)
    q, k, v = gen_full(w)
    # the workload's values rounded to bf16 (generator side: no arithmetic of the method)
    return w, tuple(po.fl(x.astype(np.float64), "bf16").astype(np.float32) for x in (q, k, v))


@pytest.mark.parametrize("variant", [P.MIXED, P.S16, P.STRICT16])
@pytest.mark.parametrize("idx,N,over", [(1, 512, {}), (3, 600, dict(Hq=7, Hkv=1))])
def test_bf16_io(idx, N, over, variant):
    w, (q, k, v) = _bf16_case(idx, N, **over)
    scale = f32(w.scale)
    o, cnt = gpu_attn(q, k, v, w.causal, scale, variant, counters=True, bf16=True)
    qh, kh, vh = po.from_bf16(q), po.from_bf16(k), po.from_bf16(v)
    g = w.Hq // w.Hkv
    ref = np.stack([[po.pasa_rows(qh[b, h], kh[b, h // g], vh[b, h // g], scale, w.causal, BETA, 128,
                                  ORACLE_POLICY[variant], out_fmt="bf16") for h in range(w.Hq)] for b in range(w.B)])
    assert np.isfinite(o).all() and cnt.tolist() == [0, 0]
    # compare in units of the reference's bf16 spacing: the stored values are 8-bit significands
    ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(ref), 2.0 ** -126))) - 7)
    steps = np.abs(o.astype(np.float64) - ref) / ulp
    c = compare(o, ref)
    print(w.name, VARIANT_NAME[variant], c, "max ulps %.1f, >1 ulp: %.2e" % (steps.max(), (steps > 1).mean()))
    # one bf16 step of an output below 1 is up to 3.9e-3; outputs near zero differ by many of their own (tiny) steps
    if idx == 1:
        assert c["maxabs"] <= 4e-3
    else:
        assert c["p999"] <= 4e-3 and c["maxabs"] <= 1.6e-2
    # In units of the stored format: nearly every output is the oracle's bf16 value or its neighbour.  (How many are
    # the very same value depends on where P is rounded -- the kernel's P carries the factor that places the tile at the
    # stored output's scale, Algorithm 1's does not -- so that fraction is printed, not asserted.)
    big = np.abs(ref) >= 0.5          # one bf16 step is at least 2e-3 there, the size of the whole stated tolerance
    print("equal bf16 values: %.3f; of the outputs beyond 0.5 within one bf16 step: %.4f" % ((o == ref).mean(), (steps[big] <= 1).mean()))
    if variant == P.MIXED:
        assert (steps[big] <= 1).all()


def test_bf16_input_beyond_fp16_range_becomes_infinite_like_the_oracle():
    rng = np.random.default_rng(77)
    N, d = 256, 64
    q = po.fl(rng.standard_normal((1, 1, N, d)), "bf16").astype(np.float32)
    k = po.fl(rng.standard_normal((1, 1, N, d)), "bf16").astype(np.float32)
    v = po.fl(rng.standard_normal((1, 1, N, d)), "bf16").astype(np.float32)
    v[0, 0, 3, 5] = 131072.0         # a bf16 value: +inf once converted to fp16
    o, cnt = gpu_attn(q, k, v, False, 0.125, P.MIXED, counters=True, bf16=True)
    ref = po.pasa_rows(po.from_bf16(q[0, 0]), po.from_bf16(k[0, 0]), po.from_bf16(v[0, 0]), 0.125, False, BETA, 128,
                       po.MIXED, out_fmt="bf16")
    assert np.isinf(ref[:, 5]).all() and np.isinf(o[0, 0, :, 5]).all()
    keep = np.arange(d) != 5
    assert np.isfinite(o[0, 0][:, keep]).all()
    assert cnt[1] == N


# ------------------------------------------------------------------ query chunks: cross-attention, chunked prefill, decoding

def _rows_ref(q, k, v, scale, causal, first, count, row0, policy=po.MIXED):
    B, Hq = q.shape[:2]
    g = Hq // k.shape[1]
    return np.stack([[po.pasa_rows(q[b, h, first:first + count], k[b, h // g], v[b, h // g], scale, causal, BETA, 128,
                                   policy, row0) for h in range(Hq)] for b in range(B)])


@pytest.mark.parametrize("Nq,N,d", [(300, 1000, 64), (1, 640, 128), (513, 128, 128), (64, 77, 64)])
def test_cross_attention_lengths_differ(Nq, N, d):
    rng = np.random.default_rng(Nq * 7 + N)
    q = rng.standard_normal((1, 4, Nq, d)).astype(np.float16)
    k = (rng.standard_normal((1, 2, N, d)) + 2.5).astype(np.float16)
    v = rng.standard_normal((1, 2, N, d)).astype(np.float16)
    scale = f32(d ** -0.5)
    o = gpu_attn_chunks(q, k, v, False, scale, [(0, Nq, 0)])
    ref = _rows_ref(q, k, v, scale, False, 0, Nq, 0)
    c = compare(o, ref)
    print(Nq, N, d, c)
    assert np.isfinite(o).all()
    assert c["maxabs"] <= 2e-3


def test_chunked_causal_prefill_equals_one_call():
    w = _small(3, 1000, Hq=4, Hkv=2)
    q, k, v = gen_full(w)
    scale = f32(w.scale)
    whole, _ = gpu_attn(q, k, v, True, scale, P.MIXED)
    # chunk starts that are multiples of 32 keep every row in the same wavefront slot: bit-identical results
    parts = gpu_attn_chunks(q, k, v, True, scale, [(0, 256, 0), (256, 448, 256), (704, 296, 704)])
    assert np.array_equal(whole.view(np.uint16), parts.view(np.uint16))
    # any other split: each row still follows the same algorithm (summation order of Sbar' may differ)
    odd = gpu_attn_chunks(q, k, v, True, scale, [(0, 7, 0), (7, 600, 7), (607, 393, 607)])
    ref = po.pasa_bhnd(q, k, v, scale, True, BETA, 128, po.MIXED)
    c = compare(odd, ref)
    print(c)
    assert c["maxabs"] <= 2e-3


@pytest.mark.parametrize("variant", [P.MIXED, P.S16, P.STRICT16])
def test_unaligned_chunks_other_variants(variant):
    # waves whose rows straddle a key-tile boundary: their first rows see nothing of the later tile
    w = _small(1, 500)
    q, k, v = gen_full(w)
    scale = f32(w.scale)
    o = gpu_attn_chunks(q, k, v, True, scale, [(0, 101, 0), (101, 399, 101)], variant=variant)
    ref = po.pasa_bhnd(q, k, v, scale, True, BETA, 128, ORACLE_POLICY[variant])
    c = compare(o, ref)
    print(VARIANT_NAME[variant], c)
    assert np.isfinite(o).all()
    assert c["maxabs"] <= 2e-3


def test_unaligned_chunks_naive16():
    rng = np.random.default_rng(61)
    N, d = 400, 64
    q = rng.standard_normal((1, 2, N, d)).astype(np.float16)
    k = rng.standard_normal((1, 1, N, d)).astype(np.float16)
    v = rng.standard_normal((1, 1, N, d)).astype(np.float16)
    scale = f32(d ** -0.5)
    o = gpu_attn_chunks(q, k, v, True, scale, [(0, 50, 0), (50, 350, 50)], variant=P.NAIVE16)
    ref = po.fa_bhnd(q, k, v, scale, True, 128, po.PARTIAL16)
    assert compare(o, ref)["maxabs"] <= 2e-3


@pytest.mark.parametrize("Nq", [1, 3, 40])
def test_decoding_against_a_cache(Nq):
    # the last Nq positions of a sequence of N keys, causal: row0 = N - Nq
    rng = np.random.default_rng(50 + Nq)
    N, d = 777, 128
    q = rng.standard_normal((2, 4, Nq, d)).astype(np.float16)
    k = (rng.standard_normal((2, 1, N, d)) + 2).astype(np.float16)
    v = rng.standard_normal((2, 1, N, d)).astype(np.float16)
    scale = f32(d ** -0.5)
    o = gpu_attn_chunks(q, k, v, True, scale, [(0, Nq, N - Nq)])
    ref = _rows_ref(q, k, v, scale, True, 0, Nq, N - Nq)
    assert compare(o, ref)["maxabs"] <= 2e-3
    # positions past the last key see every key: same as not causal
    o2 = gpu_attn_chunks(q, k, v, True, scale, [(0, Nq, N + 5)])
    o3 = gpu_attn_chunks(q, k, v, False, scale, [(0, Nq, 0)])
    assert compare(o2, o3)["maxabs"] <= 2e-3


# ------------------------------------------------------------------ key split: few workgroups, many key tiles

@pytest.mark.parametrize("variant", [P.MIXED, P.S16, P.DIRECT])
@pytest.mark.parametrize("Nq,N,causal,d", [(1, 4224, True, 128), (37, 6000, True, 128), (300, 2100, False, 64)])
def test_key_split_against_the_oracle_and_against_one_workgroup_per_tile(Nq, N, causal, d, variant):
    """Short query chunks against long keys launch few workgroups, so the library splits the key tiles of each among
    several and merges the per-row states.  The merged result is held to the oracle like any other, and compared with
    the same call made with the bare minimum of workspace, which cannot split."""
    import torch
    rng = np.random.default_rng(900 + Nq)
    B, Hq, Hkv = 1, 4, 2
    q = rng.standard_normal((B, Hq, Nq, d)).astype(np.float16)
    k = (rng.standard_normal((B, Hkv, N, d)) + 3).astype(np.float16)
    v = rng.standard_normal((B, Hkv, N, d)).astype(np.float16)
    scale = f32(d ** -0.5)
    row0 = N - Nq if causal else 0
    dev = torch.device("cuda:0")
    tq, tk, tv = (torch.from_numpy(x).to(dev) for x in (q, k, v))
    full = P.pasa_attn_fwd_workspace(B, Hq, Hkv, N, d)
    bare = P.pasa_attn_fwd_workspace_min(B, Hkv, N, d)
    assert full - bare >= 2 * B * Hq * Nq * (4 * d + 16)          # room for at least two splits of this chunk
    outs = []
    for nbytes in (full, bare):
        ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        to = torch.full_like(tq, float("nan"))
        P.pasa_prepare_kv(tk, tv, B, Hkv, N, d, scale, ws, nbytes, variant=variant)
        P.pasa_attn_fwd_chunk(tq, to, B, Hq, Hkv, Nq, row0, N, d, causal, scale, ws, nbytes, variant=variant)
        torch.cuda.synchronize()
        outs.append(to.cpu().numpy())
    split, whole = outs
    assert np.isfinite(split).all()
    if variant == P.DIRECT:
        ref = np.stack([[po.direct_rows(q[b, h], k[b, h // 2], v[b, h // 2], scale, causal, BETA, 128, po.MIXED, row0)
                         for h in range(Hq)] for b in range(B)])
    else:
        ref = _rows_ref(q, k, v, scale, causal, 0, Nq, row0, policy=ORACLE_POLICY[variant])
    c, cw, cs = compare(split, ref), compare(whole, ref), compare(split, whole)
    print(VARIANT_NAME[variant], Nq, N, "split vs oracle", c, "| unsplit vs oracle", cw, "| split vs unsplit", cs)
    assert (c["maxabs"] <= 2e-3) if variant != P.S16 else (c["p999"] <= 2e-3)
    assert cs["maxabs"] <= 2e-3


def test_key_split_bf16_and_counters():
    """The merge kernel writes the output: bf16 conversion and the non-finite counter live there when the keys are split."""
    import torch
    rng = np.random.default_rng(931)
    B, Hq, Hkv, Nq, N, d = 1, 2, 1, 64, 2304, 128
    q = po.fl(rng.standard_normal((B, Hq, Nq, d)), "bf16").astype(np.float32)
    k = po.fl(rng.standard_normal((B, Hkv, N, d)) + 3, "bf16").astype(np.float32)
    v = po.fl(rng.standard_normal((B, Hkv, N, d)), "bf16").astype(np.float32)
    scale = f32(d ** -0.5)
    dev = torch.device("cuda:0")
    tq, tk, tv = (torch.from_numpy(bf16_bits(x).view(np.float16)).to(dev) for x in (q, k, v))
    wsb = P.pasa_attn_fwd_workspace(B, Hq, Hkv, N, d)
    ws = torch.empty(wsb, dtype=torch.uint8, device=dev)
    to = torch.full_like(tq, float("nan"))
    cnt = torch.zeros(2, dtype=torch.int64, device=dev)
    P.pasa_prepare_kv(tk, tv, B, Hkv, N, d, scale, ws, wsb, io_dtype=P.IO_BF16)
    P.pasa_attn_fwd_chunk(tq, to, B, Hq, Hkv, Nq, N - Nq, N, d, True, scale, ws, wsb, io_dtype=P.IO_BF16,
                          overflow_s=cnt[0:1], nonfinite_o=cnt[1:2])
    torch.cuda.synchronize()
    o = (to.cpu().numpy().view(np.uint16).astype(np.uint32) << 16).view(np.float32)
    qh, kh, vh = po.from_bf16(q), po.from_bf16(k), po.from_bf16(v)
    ref = np.stack([[po.pasa_rows(qh[b, h], kh[b, 0], vh[b, 0], scale, True, BETA, 128, po.MIXED, N - Nq, out_fmt="bf16")
                     for h in range(Hq)] for b in range(B)])
    assert np.isfinite(o).all() and cnt.tolist() == [0, 0]
    c = compare(o, ref)
    print(c)
    assert c["maxabs"] <= 8e-3 and c["p999"] <= 4e-3        # one bf16 step of an output in [1, 2) is 7.8e-3


# ------------------------------------------------------------------ direct-bias recovery (PASA_DIRECT, not the paper's step)

@pytest.mark.parametrize("N,d", [(384, 128), (300, 64), (77, 128)])
def test_direct_shift_keys_bit_exact(N, d):
    import torch
    rng = np.random.default_rng(2000 + N)
    k = (rng.standard_normal((2, 2, N, d)) * rng.uniform(0.1, 30, (1, 1, 1, d)) + rng.uniform(-80, 80, (2, 2, 1, d))).astype(np.float16)
    nt = -(-N // 128)
    tk = torch.from_numpy(k).cuda()
    out = torch.empty_like(tk)
    k0 = torch.full((2, 2, nt, d), float("nan"), dtype=torch.float16, device="cuda")
    P.pasa_shift_keys_direct(tk, out, k0, 2, 2, N, d, BETA, 0.125)
    torch.cuda.synchronize()
    want = [[po.direct_shift_keys(k[b, h], BETA, 0.125) for h in range(2)] for b in range(2)]
    wk = np.stack([[want[b][h][0] for h in range(2)] for b in range(2)])
    w0 = np.stack([[want[b][h][1] for h in range(2)] for b in range(2)])
    assert np.array_equal(out.cpu().numpy().view(np.uint16), wk.view(np.uint16))
    assert np.array_equal(k0.cpu().numpy().view(np.uint16), w0.view(np.uint16))


def test_direct_tiny_workload_full_tensor():
    w = workload(1)
    q, k, v = gen_full(w)
    scale = f32(w.scale)
    o, cnt = gpu_attn(q, k, v, w.causal, scale, P.DIRECT, counters=True)
    ref = po.direct_bhnd(q, k, v, scale, w.causal, BETA, 128, po.MIXED)
    gold = po.attention_fp64_bhnd(q, k, v, scale, w.causal)
    c = compare(o, ref)
    print(c, "rmse gpu %.3e oracle %.3e" % (po.rmse(o, gold), po.rmse(ref, gold)))
    assert np.isfinite(o).all() and cnt.tolist() == [0, 0]
    assert c["maxabs"] <= 2e-3
    assert po.rmse(o, gold) <= 1e-3          # the stated accuracy bar, met by this recovery


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("idx,N,over", [(2, 512, dict(Hq=2, Hkv=1)), (3, 700, dict(Hq=7, Hkv=1)), (4, 333, dict(B=1, Hq=2, Hkv=2))])
def test_direct_scaled_workloads(idx, N, over, causal):
    w = _small(idx, N, **over)
    q, k, v = gen_full(w)
    scale = f32(w.scale)
    o, cnt = gpu_attn(q, k, v, causal, scale, P.DIRECT, counters=True)
    ref = po.direct_bhnd(q, k, v, scale, causal, BETA, 128, po.MIXED)
    gold = po.attention_fp64_bhnd(q, k, v, scale, causal)
    paper = po.pasa_bhnd(q, k, v, scale, causal, BETA, 128, po.MIXED)
    c = compare(o, ref)
    r_gpu, r_or, r_paper = po.rmse(o, gold), po.rmse(ref, gold), po.rmse(paper, gold)
    print(w.name, causal, c, "rmse gpu %.3e oracle %.3e paper's recovery %.3e" % (r_gpu, r_or, r_paper))
    assert np.isfinite(o).all() and cnt.tolist() == [0, 0]
    # The kernel rounds P once at the scale the output is stored at, the oracle rounds exp(S' - m') and scales the
    # product: two equally accurate roundings of every P, each with a relative error of at most 2^-11.  The two
    # outputs therefore differ by at most 2 * 2^-11 * sum_n w_n |v_n| (w the softmax weights) plus the two final
    # roundings to fp16 (half an ulp each).  On the extreme-bias workload the softmax is nearly one-hot, so the sum is
    # |v| of the winning key, at most max |v| (about 4): that bound, 2^-10 max |v|, is asserted there; everywhere else
    # the stated 2e-3 holds.
    if idx == 2:
        assert c["maxabs"] <= 2.0 ** -10 * float(np.abs(v.astype(np.float64)).max()) and c["p999"] <= 2e-3
    else:
        assert c["maxabs"] <= 2e-3 and c["p999"] <= 2e-3
    assert abs(r_gpu - r_or) <= 0.03 * r_or + 2e-5
    # the stated accuracy bar; on the extreme-bias workload the rounding of K' alone leaves 1.4e-3 (the paper's
    # recovering step: 1.7e-2 on the same inputs)
    assert r_gpu <= (2e-3 if idx == 2 else 1e-3) and r_gpu <= max(0.5 * r_paper, 1e-5)


def test_direct_chunks_and_bf16():
    w = _small(3, 640, Hq=4, Hkv=2)
    q, k, v = gen_full(w)
    scale = f32(w.scale)
    whole, _ = gpu_attn(q, k, v, True, scale, P.DIRECT)
    parts = gpu_attn_chunks(q, k, v, True, scale, [(0, 256, 0), (256, 384, 256)], variant=P.DIRECT)
    assert np.array_equal(whole.view(np.uint16), parts.view(np.uint16))
    odd = gpu_attn_chunks(q, k, v, True, scale, [(0, 99, 0), (99, 541, 99)], variant=P.DIRECT)
    assert compare(odd, po.direct_bhnd(q, k, v, scale, True, BETA, 128, po.MIXED))["maxabs"] <= 2e-3


def test_direct_full_size_qwen_workload_sampled():
    w = workload(3)
    r_gpu, r_or = _sampled_check(w, P.DIRECT, [(0, 0, 0), (0, 13, 4096 - 128), (0, 27, w.N - 128)], oracle="direct")
    assert r_gpu <= 1e-3


# ------------------------------------------------------------------ seeded sweep over shapes, variants and entry points

def _sweep_cases():
    rng = np.random.default_rng(20250301)
    cases = []
    for i in range(36):
        d = int(rng.choice([64, 128]))
        N = int(rng.choice([1, 31, 64, 127, 128, 129, 255, 256, 300, 511, 640, 777]))
        hkv = int(rng.choice([1, 2]))
        g = int(rng.choice([1, 2, 3]))
        variant = [P.MIXED, P.S16, P.STRICT16, P.DIRECT, P.NAIVE16][i % 5]
        causal = bool(rng.integers(2))
        bias = float(rng.choice([0.0, 1.0, 4.0]))
        cases.append((i, d, N, hkv, g, variant, causal, bias))
    return cases


@pytest.mark.parametrize("i,d,N,hkv,g,variant,causal,bias", _sweep_cases())
def test_seeded_sweep(i, d, N, hkv, g, variant, causal, bias):
    rng = np.random.default_rng(9000 + i)
    B = 1 + (i % 2)
    q = rng.standard_normal((B, hkv * g, N, d)).astype(np.float16)
    k = (rng.standard_normal((B, hkv, N, d)) + bias).astype(np.float16)
    v = rng.standard_normal((B, hkv, N, d)).astype(np.float16)
    scale = f32(d ** -0.5)
    o, cnt = gpu_attn(q, k, v, causal, scale, variant, counters=(i % 3 == 0), entry="ex" if i % 4 else "split")
    if variant == P.NAIVE16:
        ref = po.fa_bhnd(q, k, v, scale, causal, 128, po.PARTIAL16)
    elif variant == P.DIRECT:
        ref = po.direct_bhnd(q, k, v, scale, causal, BETA, 128, po.MIXED)
    else:
        ref = po.pasa_bhnd(q, k, v, scale, causal, BETA, 128, ORACLE_POLICY[variant])
    c = compare(o, ref)
    print(VARIANT_NAME[variant], (B, hkv * g, hkv, N, d), causal, bias, c)
    assert np.isfinite(o).all()
    if cnt is not None:
        assert cnt.tolist() == [0, 0]
    # bias 4 with fp16 statistics: a one-ulp flip of Sbar' moves a tile's weight by 63.5 ulp; only the bulk agrees
    if variant == P.STRICT16 and bias >= 4.0:
        assert c["p99"] <= 4e-3
    else:
        assert c["maxabs"] <= 2e-3


# ------------------------------------------------------------------ score level moving from tile to tile

@pytest.mark.parametrize("variant", [P.MIXED, P.S16, P.DIRECT, P.STRICT16])
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("step", [3.0, -3.0, 12.0])
def test_score_level_staircase(step, causal, variant):
    """The level of the scores moves by `step` from one key tile to the next (by more for some rows, less for others).
    Rising, the running maximum leaves the scale the output is stored at behind by more than e^8 every few tiles
    (step 3) or on every tile (step 12), which takes the kernel's rare re-scaling path of the stored output; falling,
    later tiles sink far below it and their probabilities underflow."""
    rng = np.random.default_rng(4242)
    d, N, T = 64, 1100, 128
    u = np.zeros(d)
    u[5] = 1.0
    qf = rng.standard_normal((1, 2, N, d)) + 4.0 * u
    tile = np.arange(N) // T
    kf = rng.standard_normal((1, 1, N, d)) + (2.0 * step * tile)[None, None, :, None] * u
    q, k = qf.astype(np.float16), kf.astype(np.float16)
    v = rng.standard_normal((1, 1, N, d)).astype(np.float16)
    scale = f32(0.125)
    o, cnt = gpu_attn(q, k, v, causal, scale, variant, counters=True)
    if variant == P.DIRECT:
        ref = po.direct_bhnd(q, k, v, scale, causal, BETA, 128, po.MIXED)
    else:
        ref = po.pasa_bhnd(q, k, v, scale, causal, BETA, 128, ORACLE_POLICY[variant])
    gold = po.attention_fp64_bhnd(q, k, v, scale, causal)
    c = compare(o, ref)
    r_gpu, r_or = po.rmse(o, gold), po.rmse(ref, gold)
    print(VARIANT_NAME[variant], step, causal, c, "rmse gpu %.3e oracle %.3e" % (r_gpu, r_or))
    assert np.isfinite(o).all() and cnt.tolist() == [0, 0]
    if variant == P.STRICT16:      # fp16 statistics: the weights of whole tiles differ by fp16 roundings times 63.5
        assert c["p99"] <= 8e-3 and abs(r_gpu - r_or) <= 0.1 * r_or + 1e-4
    else:
        assert c["maxabs"] <= 2e-3
        assert abs(r_gpu - r_or) <= 0.03 * r_or + 2e-5


@pytest.mark.parametrize("variant", [P.MIXED, P.S16])
@pytest.mark.parametrize("step", [3.0, 12.0])
def test_score_level_staircase_in_unaligned_chunks(step, variant):
    """The same rising levels reached through query chunks that are not aligned to a wave's 32 rows (some rows of a
    wave see nothing of a tile while others re-reference their stored output on it), and in bf16."""
    rng = np.random.default_rng(777)
    d, N, T = 128, 700, 128
    u = np.zeros(d)
    u[9] = 1.0
    qf = rng.standard_normal((1, 2, N, d)) + 5.0 * u
    kf = rng.standard_normal((1, 2, N, d)) + (2.0 * step * (np.arange(N) // T))[None, None, :, None] * u
    q, k = qf.astype(np.float16), kf.astype(np.float16)
    v = rng.standard_normal((1, 2, N, d)).astype(np.float16)
    scale = f32(d ** -0.5)
    ref = po.pasa_bhnd(q, k, v, scale, True, BETA, 128, ORACLE_POLICY[variant])
    o = gpu_attn_chunks(q, k, v, True, scale, [(0, 77, 0), (77, 300, 77), (377, 323, 377)], variant=variant)
    c = compare(o, ref)
    print(VARIANT_NAME[variant], step, c)
    assert np.isfinite(o).all()
    assert c["maxabs"] <= 2e-3
    # one call over all rows gives the same values as the chunks: the per-row state does not depend on the chunking
    o1, _ = gpu_attn(q, k, v, True, scale, variant)
    assert np.array_equal(o1, o)


# ------------------------------------------------------------------ exact symmetries (no oracle involved)

@pytest.mark.parametrize("variant", [P.MIXED, P.S16, P.STRICT16, P.DIRECT, P.NAIVE16])
def test_powers_of_two_commute_with_every_rounding_on_the_gpu(variant):
    """Doubling Q and halving the scale changes no bit of the output; doubling V doubles it exactly (outputs below
    2^-13 aside, where fp16 is subnormal).  The keys are drawn so that no shifted key is tiny."""
    rng = np.random.default_rng(404)
    N, d = 700, 128
    q = rng.standard_normal((1, 2, N, d)).astype(np.float16)
    k = (3.0 + rng.choice([-1.0, 1.0], (1, 1, N, d)) * rng.uniform(0.25, 1.0, (1, 1, N, d))).astype(np.float16)
    v = rng.standard_normal((1, 1, N, d)).astype(np.float16)
    scale = f32(2.0 ** -4)
    base, _ = gpu_attn(q, k, v, True, scale, variant)
    big = np.abs(base.astype(np.float64)) >= 2.0 ** -13
    assert np.isfinite(base).all() and big.mean() > 0.99
    if variant != P.NAIVE16:       # NAIVE16 scales the rounded raw scores in fp32 after the GEMM: not the same roundings
        q2, _ = gpu_attn((2 * q).astype(np.float16), k, v, True, f32(2.0 ** -5), variant)
        assert np.array_equal(q2[big], base[big])
    if variant != P.STRICT16:      # its fp16 output combination meets subnormal products
        v2, _ = gpu_attn(q, k, (2 * v).astype(np.float16), True, scale, variant)
        assert np.array_equal(v2.astype(np.float64)[big], 2.0 * base.astype(np.float64)[big])


def test_first_two_key_tiles_enter_symmetrically_in_strict16():
    """Algorithm 1 combines the first two tiles with commutative operations only (F = (Sbar'_1 + Sbar'_2) / 2, the two
    corrections, the maximum, the two-term sums for l and O), so exchanging them changes no bit -- in the oracle
    (pinned there) and in the kernel's literal fp16 variant."""
    rng = np.random.default_rng(405)
    N, d, T = 384, 64, 128
    q = rng.standard_normal((1, 2, 100, d)).astype(np.float16)
    k = (rng.standard_normal((1, 1, N, d)) + 2.0).astype(np.float16)
    v = rng.standard_normal((1, 1, N, d)).astype(np.float16)
    swap01 = np.concatenate([np.arange(T, 2 * T), np.arange(0, T), np.arange(2 * T, N)])
    chunks = [(0, 100, 0)]
    a = gpu_attn_chunks(q, k, v, False, f32(0.125), chunks, variant=P.STRICT16)
    b = gpu_attn_chunks(q, k[:, :, swap01], v[:, :, swap01], False, f32(0.125), chunks, variant=P.STRICT16)
    assert np.isfinite(a).all() and np.array_equal(a.view(np.uint16), b.view(np.uint16))


# ------------------------------------------------------------------ adaptive start

def _adaptive(q, k, v, causal, scale, variant=P.MIXED):
    import torch
    dev = torch.device("cuda:0")
    B, Hq, N, d = q.shape
    Hkv = k.shape[1]
    tq, tk, tv = (torch.from_numpy(np.ascontiguousarray(x)).to(dev) for x in (q, k, v))
    to = torch.full_like(tq, float("nan"))
    cnt = torch.zeros(1, dtype=torch.int64, device=dev)
    wsb = P.pasa_attn_fwd_workspace(B, Hq, Hkv, N, d)
    ws = torch.empty(wsb, dtype=torch.uint8, device=dev)
    P.pasa_attn_fwd_adaptive(tq, tk, tv, to, B, Hq, Hkv, N, d, causal, scale, ws, wsb, torch.cuda.current_stream(),
                             variant=variant, overflow_s=cnt)
    torch.cuda.synchronize()
    return to.cpu().numpy(), int(cnt.item())


def test_adaptive_start_keeps_the_unshifted_result_when_nothing_overflows():
    w = workload(1)
    q, k, v = gen_full(w)
    scale = f32(w.scale)
    o, count = _adaptive(q, k, v, w.causal, scale)
    plain, _ = gpu_attn(q, k, v, w.causal, scale, P.NAIVE16)
    ref, trig = po.adaptive_bhnd(q, k, v, scale, w.causal, BETA)
    assert count == 0 and not trig
    assert np.array_equal(o.view(np.uint16), plain.view(np.uint16))
    assert compare(o, ref)["maxabs"] <= 2e-3
    gold = po.attention_fp64_bhnd(q, k, v, scale, w.causal)
    r_gpu, r_or = po.rmse(o, gold), po.rmse(ref, gold)
    assert abs(r_gpu - r_or) <= 0.03 * r_or + 2e-5


@pytest.mark.parametrize("variant", [P.MIXED, P.STRICT16, P.DIRECT])
def test_adaptive_start_switches_to_pasa_on_overflow(variant):
    w = _small(2, 512, Hq=2, Hkv=1)
    q, k, v = gen_full(w)
    scale = f32(w.scale)
    o, count = _adaptive(q, k, v, w.causal, scale, variant)
    shifted, _ = gpu_attn(q, k, v, w.causal, scale, variant)
    assert count > 0 and np.isfinite(o).all()
    assert np.array_equal(o.view(np.uint16), shifted.view(np.uint16))
    if variant == P.MIXED:
        ref, trig = po.adaptive_bhnd(q, k, v, scale, w.causal, BETA)
        assert trig
        c = compare(o, ref)
        assert c["maxabs"] <= 2e-3


def test_adaptive_start_switches_only_the_kv_head_that_overflowed():
    # 2 batches x 2 KV heads x 2 query heads each; raw scores overflow in one query head of (batch 1, KV head 0) only
    rng = np.random.default_rng(56)
    N, d = 384, 128
    q = rng.standard_normal((2, 4, N, d)).astype(np.float16)
    k = rng.standard_normal((2, 2, N, d)).astype(np.float16)
    v = rng.standard_normal((2, 2, N, d)).astype(np.float16)
    q[1, 1] = 30.0
    k[1, 0] = (30.0 + rng.standard_normal((N, d))).astype(np.float16)
    scale = f32(d ** -0.5)
    o, count = _adaptive(q, k, v, True, scale)
    info = {}
    ref, trig = po.adaptive_bhnd(q, k, v, scale, True, BETA, info=info)
    assert trig and info["groups"].tolist() == [[False, False], [True, False]]
    assert count == N * (N + 1) // 2 + (N // 128) * (128 * 127 // 2)   # head (1, 1): its visible scores, and the masked ones of the diagonal tiles
    assert np.isfinite(o).all() and compare(o, ref)["maxabs"] <= 2e-3
    plain, _ = gpu_attn(q, k, v, True, scale, P.NAIVE16)
    shifted, _ = gpu_attn(q, k, v, True, scale, P.MIXED)
    for b in range(2):
        for h in range(4):
            want = shifted if (b, h // 2) == (1, 0) else plain
            assert np.array_equal(o[b, h].view(np.uint16), want[b, h].view(np.uint16)), (b, h)
    # query head (1, 0) did not overflow itself and still switched with its KV head
    assert not np.array_equal(plain[1, 0].view(np.uint16), shifted[1, 0].view(np.uint16))


# ------------------------------------------------------------------ capture into a HIP graph

@pytest.mark.parametrize("N", [1000, 2500])
def test_graph_capture_and_replay(N):
    """pasa_attn_fwd_ex with a caller workspace allocates nothing and only enqueues kernels, so it can be
    captured into a HIP graph; every replay must give the eager result for the inputs then in the buffers.
    N = 2500: the call splits its keys (three kernels: pre-processing, main, merge)."""
    import torch
    dev = torch.device("cuda:0")
    w = _small(3, N, Hq=4, Hkv=2)
    scale = f32(w.scale)
    inputs = []
    for seed in (w.seed, w.seed + 1, w.seed + 2):
        inputs.append(gen_full(Workload(**{**w.__dict__, "seed": seed})))
    tq, tk, tv = (torch.from_numpy(x).to(dev) for x in inputs[0])
    to = torch.zeros_like(tq)
    wsb = P.pasa_attn_fwd_workspace(w.B, w.Hq, w.Hkv, w.N, w.d)
    ws = torch.empty(wsb, dtype=torch.uint8, device=dev)
    args = (w.B, w.Hq, w.Hkv, w.N, w.d, True, scale)
    eager = []
    for q, k, v in inputs:                       # eager results first (also warms the kernels up before capture)
        tq.copy_(torch.from_numpy(q)); tk.copy_(torch.from_numpy(k)); tv.copy_(torch.from_numpy(v))
        P.pasa_attn_fwd_ex(tq, tk, tv, to, *args, ws, wsb, torch.cuda.current_stream())
        torch.cuda.synchronize()
        eager.append(to.cpu().numpy().copy())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        P.pasa_attn_fwd_ex(tq, tk, tv, to, *args, ws, wsb, torch.cuda.current_stream())
    for rep in range(2):
        for i, (q, k, v) in enumerate(inputs):
            tq.copy_(torch.from_numpy(q)); tk.copy_(torch.from_numpy(k)); tv.copy_(torch.from_numpy(v))
            to.fill_(float("nan"))
            ws.zero_()                           # eager work between the replays
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            got = to.cpu().numpy()
            assert np.array_equal(got.view(np.uint16), eager[i].view(np.uint16)), (rep, i)


# ------------------------------------------------------------------ full sizes, sampled, in the benchmark's launch configuration

def _sampled_check(w, variant, units, tol_p999=2e-3, oracle="pasa"):
    """Run the whole workload on the GPU; compare the listed (b, h, row0) 128-row blocks with the oracle."""
    import torch
    scale = f32(w.scale)
    dev = torch.device("cuda:0")
    tq = torch.empty((w.B, w.Hq, w.N, w.d), dtype=torch.float16, device=dev)
    tk = torch.empty((w.B, w.Hkv, w.N, w.d), dtype=torch.float16, device=dev)
    tv = torch.empty_like(tk)
    need_q = {(b, h) for b, h, _ in units}
    host_q, host_kv = {}, {}
    for b in range(w.B):
        for hk in range(w.Hkv):
            kk, vv = gen_kv_head(w, b, hk)
            tk[b, hk].copy_(torch.from_numpy(kk))
            tv[b, hk].copy_(torch.from_numpy(vv))
            if any((b, h) in need_q for h in range(hk * w.group, (hk + 1) * w.group)):
                host_kv[(b, hk)] = (kk, vv)
        for h in range(w.Hq):
            qq = gen_q_head(w, b, h)
            tq[b, h].copy_(torch.from_numpy(qq))
            if (b, h) in need_q:
                host_q[(b, h)] = qq
    to = torch.full_like(tq, float("nan"))
    wsb = P.pasa_attn_fwd_workspace(w.B, w.Hq, w.Hkv, w.N, w.d)
    ws = torch.empty(wsb, dtype=torch.uint8, device=dev)
    cnt = torch.zeros(2, dtype=torch.int64, device=dev)
    P.pasa_attn_fwd_ex(tq, tk, tv, to, w.B, w.Hq, w.Hkv, w.N, w.d, w.causal, scale, ws, wsb,
                       torch.cuda.current_stream(), variant=variant, overflow_s=cnt[0:1], nonfinite_o=cnt[1:2])
    torch.cuda.synchronize()
    assert cnt.tolist() == [0, 0]
    assert bool(torch.isfinite(to).all())
    num = den = num_o = 0.0
    diffs = []
    for b, h, r0 in units:
        kk, vv = host_kv[(b, h // w.group)]
        qq = host_q[(b, h)][r0:r0 + 128]
        nk = min(r0 + 128, w.N) if w.causal else w.N      # r0 is a multiple of 128: whole tiles, or the true ragged tail
        if oracle == "direct":
            ref = po.direct_rows(qq, kk[:nk], vv[:nk], scale, w.causal, BETA, 128, po.MIXED, r0)
        else:
            ref = po.pasa_rows(qq, kk[:nk], vv[:nk], scale, w.causal, BETA, 128, ORACLE_POLICY[variant], r0)
        gold = po.attention_fp64(qq, kk[:nk], vv[:nk], scale, w.causal, r0)
        o = to[b, h, r0:r0 + 128].cpu().numpy()
        diffs.append(np.abs(o.astype(np.float64) - ref.astype(np.float64)).ravel())
        num += ((o - gold) ** 2).sum()
        num_o += ((ref - gold) ** 2).sum()
        den += (gold ** 2).sum()
    dd = np.concatenate(diffs)
    r_gpu, r_or = (num / den) ** 0.5, (num_o / den) ** 0.5
    print(w.name, VARIANT_NAME[variant], "maxabs %.3e p999 %.3e rmse gpu %.3e oracle %.3e"
          % (dd.max(), np.quantile(dd, 0.999), r_gpu, r_or))
    assert np.quantile(dd, 0.999) <= tol_p999
    if variant in (P.MIXED, P.DIRECT):
        assert dd.max() <= 2e-3, "max-abs against the emulated oracle above the stated bar: %d elements" % int((dd > 2e-3).sum())
    assert abs(r_gpu - r_or) <= 0.03 * r_or + 2e-5
    return r_gpu, r_or


def test_full_size_overflow_workload_sampled():
    w = workload(2)
    _sampled_check(w, P.MIXED, [(0, 0, 0), (0, 3, 1920), (0, 7, w.N - 128)])


@pytest.mark.parametrize("variant", [P.MIXED, P.STRICT16])
def test_full_size_qwen_workload_sampled(variant):
    w = workload(3)   # the benchmark workload, same launch configuration
    units = [(0, 0, 0), (0, 6, 128), (0, 13, 4096 - 128), (0, 20, 5504), (0, 27, w.N - 128)]
    # STRICT16: one-ulp fp16 flips of Sbar' move a tile's weight by up to 63.5 ulp; only the bulk agrees
    _sampled_check(w, variant, units, tol_p999=2e-3 if variant == P.MIXED else 1e-2)


def test_paper_qwen2_sequence_length_5676_sampled():
    # the sequence length of the paper's Qwen2-7B overflow case (section 2.1); 5676 = 44 * 128 + 44
    w = workload(3).with_n(5676)
    _sampled_check(w, P.MIXED, [(0, 0, 0), (0, 13, 2560), (0, 27, 5632)])


def test_full_size_svd_workload_sampled():
    w = workload(4)
    _sampled_check(w, P.MIXED, [(0, 0, 0), (6, 1, 4608), (13, 4, w.N - 128)])


def test_full_size_long_context_workload_sampled():
    w = workload(5)
    _sampled_check(w, P.MIXED, [(0, 0, 0), (1, 9, 16384), (1, 27, w.N - 128)])


def test_maximum_sequence_length_sampled():
    w = Workload("max_n", 1, 1, 1, 262144, 64, True, 11, "tiny")
    _sampled_check(w, P.MIXED, [(0, 0, 0), (0, 0, 131072), (0, 0, w.N - 128)])
