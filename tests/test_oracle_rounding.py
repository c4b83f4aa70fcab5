"""Pins of WHERE the emulated oracle rounds (no GPU).

`pasa_rows` / `fa_rows` / `direct_rows` emulate low precision by computing in fp64 and calling a rounding helper
at the points Algorithm 1 marks "(Precision = FP16)".  A forgotten or misplaced call of that helper leaves the
algebra intact, so none of the algebraic pins sees it.  Here the same algorithms are evaluated once more for
tiny cases, one query row at a time, with numpy's native IEEE scalars (`np.float16`, `np.float32`): every
`+ - * /` on two such scalars is one correctly rounded operation of that type by construction (numpy widens half
operands to fp32, and 24 >= 2*11 + 2 bits make the second rounding harmless), so there is no rounding helper
that could be left out.  Sums that the method takes "inside the matrix engine" (dot products, row sums) are
accumulated exactly with rationals and rounded once.  The oracle has to agree bit for bit.
"""
import math
from fractions import Fraction

import numpy as np
import pytest

from oracle import pasa_oracle as po

H, F32 = np.float16, np.float32
NEG_INF = float("-inf")


def _round_exact(x: Fraction, t):
    """One rounding of an exact rational to scalar type t (through the nearest fp64, which keeps > 2p + 2 bits)."""
    return t(x.numerator / x.denominator)          # int / int is correctly rounded to fp64 in Python


def _dot(a, b, t):
    return _round_exact(sum((Fraction(float(x)) * Fraction(float(y)) for x, y in zip(a, b)), Fraction(0)), t)


def _exp(x, t):
    """exp of a scalar, rounded once to type t."""
    x = float(x)
    return t(0.0) if x == NEG_INF else t(math.exp(x))


def _shifted_keys(K, beta, scale, T):
    """Eq. (11) per tile: exact column sum, then (K - beta * mean) * scale in fp64 operations, one rounding to fp16."""
    N, d = K.shape
    out = np.empty((N, d), H)
    for t0 in range(0, N, T):
        rows = range(t0, min(N, t0 + T))
        for c in range(d):
            total = sum(Fraction(float(K[n, c])) for n in rows)
            mean = float(total) / len(rows)
            for n in rows:
                out[n, c] = H((float(K[n, c]) - beta * mean) * scale)
    return out


def alg1_row(q, K, V, scale, beta, T, causal, pos, tS, tstat, tO):
    """Algorithm 1 for ONE query row at sequence position `pos`, native scalars.  tS: type the score tile leaves
    the first GEMM in; tstat: type of Sbar', F, the Delta terms, m, l; tO: type of P V and O.  P is fp16."""
    N, d = K.shape
    Kp = _shifted_keys(K, beta, scale, T)
    inva = tstat(beta / (1.0 - beta))
    ntile = -(-N // T)
    if causal:
        ntile = min(pos // T + 1, ntile)
    Fbar = m = l = None
    O = None
    for jt in range(ntile):
        keys = list(range(jt * T, min(N, jt * T + T)))
        # (GEMM) attention matrix of the tile
        S = [_dot(q, Kp[n], tS) for n in keys]
        # pseudo-average over all keys of the tile, masked or not
        Sbar = _round_exact(sum(Fraction(float(s)) for s in S) / len(keys), tstat)
        if causal:
            S = [s if n <= pos else tS(NEG_INF) for s, n in zip(S, keys)]
        # softmax pieces: m', P, l'
        mloc = max(S)
        P = [_exp(s - mloc, H) for s in S]                      # the difference is one operation of type tS
        lloc = _round_exact(sum(Fraction(float(p)) for p in P), tstat)
        # (GEMM) temporary output
        Ot = [_round_exact(sum(Fraction(float(p)) * Fraction(float(V[n, c])) for p, n in zip(P, keys)), tO)
              for c in range(d)]
        if jt == 0:                                              # the first tile initialises the state
            Fbar, m, l, O = Sbar, tstat(mloc), lloc, Ot
            continue
        j = jt + 1
        mloc = tstat(mloc)
        # global pseudo-average, Eq. (15), in the order it is printed
        Fnew = ((tstat(j - 1) * Fbar) + Sbar) / tstat(j)
        # correction terms of the maximum: difference first, then the factor beta / (1 - beta)
        dpp = inva * (Fbar - Fnew)
        dpc = inva * (Sbar - Fnew)
        # the maximum
        mnew = max(m + dpp, mloc + dpc)
        # correction terms
        dp = (m - mnew) + dpp
        dc = (mloc - mnew) + dpc
        ep, ec = _exp(dp, tstat), _exp(dc, tstat)
        # running sum and output
        l = (ep * l) + (ec * lloc)
        O = [(tO(ec) * ot) + (tO(ep) * o) for ot, o in zip(Ot, O)]
        m, Fbar = mnew, Fnew
    return np.array([H(float(o) / float(l)) for o in O], H)


def fa_row(q, K, V, scale, T, causal, pos, tS, tstat, tO):
    """Eq. (1)-(8) for one query row: raw scores rounded to tS as they leave the GEMM, then scaled."""
    N, d = K.shape
    ntile = -(-N // T)
    if causal:
        ntile = min(pos // T + 1, ntile)
    m, l, O = tstat(NEG_INF), tstat(0), [tO(0)] * d
    for jt in range(ntile):
        keys = list(range(jt * T, min(N, jt * T + T)))
        Sraw = [_dot(q, K[n], tS) for n in keys]                 # Eq. (1)
        S = [tstat(float(s) * scale) for s in Sraw]              # Eq. (2): the rounded score times the constant, one rounding
        if causal:
            S = [s if n <= pos else tstat(NEG_INF) for s, n in zip(S, keys)]
        mnew = max(m, max(S))                                    # Eq. (4)
        P = [_exp(s - mnew, H) for s in S]                       # Eq. (5)
        e = _exp(m - mnew, tstat)
        l = (e * l) + _round_exact(sum(Fraction(float(p)) for p in P), tstat)           # Eq. (6)
        PV = [_round_exact(sum(Fraction(float(p)) * Fraction(float(V[n, c])) for p, n in zip(P, keys)), tO)
              for c in range(d)]
        O = [(tO(e) * o) + pv for o, pv in zip(O, PV)]           # Eq. (7)
        m = mnew
    return np.array([H(float(o) / float(l)) for o in O], H)      # Eq. (8)


def direct_row(q, K, V, scale, beta, T, causal, pos, tS, tstat, tO):
    """The recovery that is not the paper's (bias added back as scale * q . k0), one query row, native scalars."""
    N, d = K.shape
    ntile = -(-N // T)
    if causal:
        ntile = min(pos // T + 1, ntile)
    Mx = l = O = None
    for jt in range(ntile):
        keys = list(range(jt * T, min(N, jt * T + T)))
        k0 = [H(beta * (float(sum(Fraction(float(K[n, c])) for n in keys)) / len(keys))) for c in range(d)]
        Kp = [[H((float(K[n, c]) - float(k0[c])) * scale) for c in range(d)] for n in keys]
        S = [_dot(q, kp, tS) for kp in Kp]
        c = tstat(scale * float(_dot(q, k0, F32)))              # the fp32 dot product times the constant, one rounding
        if causal:
            S = [s if n <= pos else tS(NEG_INF) for s, n in zip(S, keys)]
        mloc = max(S)
        P = [_exp(s - mloc, H) for s in S]
        lloc = _round_exact(sum(Fraction(float(p)) for p in P), tstat)
        Ot = [_round_exact(sum(Fraction(float(p)) * Fraction(float(V[n, ch])) for p, n in zip(P, keys)), tO)
              for ch in range(d)]
        L = tstat(mloc) + c
        if jt == 0:
            Mx, l, O = L, lloc, Ot
            continue
        Mn = max(Mx, L)
        ep, ec = _exp(Mx - Mn, tstat), _exp(L - Mn, tstat)
        l = (ep * l) + (ec * lloc)
        O = [(tO(ec) * ot) + (tO(ep) * o) for ot, o in zip(Ot, O)]
        Mx = Mn
    return np.array([H(float(o) / float(l)) for o in O], H)


TYPES = {"STRICT16": (po.STRICT16, H, H, H), "MIXED": (po.MIXED, F32, F32, F32), "PARTIAL16": (po.PARTIAL16, H, F32, F32)}


def _case(seed, R, N, d, kbias, amp=1.0):
    rng = np.random.default_rng(seed)
    q = (amp * rng.standard_normal((R, d))).astype(H)
    k = (amp * rng.standard_normal((N, d)) + kbias).astype(H)
    v = rng.standard_normal((N, d)).astype(H)
    return q, k, v


# two and three tiles, T = 2 .. 4, d = 2; ragged tails; one causal case per shape; the paper's adopted beta (its
# invariance 63.504 is NOT an fp16 value, so a missing rounding of it shows) and a small one
CASES = [
    # (N, T, causal, beta)
    (4, 2, False, 0.984497), (6, 2, True, 0.984497), (8, 4, False, 0.984497), (12, 4, True, 0.984497),
    (9, 3, False, 0.9), (11, 4, True, 0.984497), (7, 3, False, 0.75), (12, 4, False, 63.5 / 64.5),
]


@pytest.mark.parametrize("policy", ["STRICT16", "MIXED", "PARTIAL16"])
@pytest.mark.parametrize("N,T,causal,beta", CASES)
def test_pasa_rows_rounds_where_algorithm_1_says(policy, N, T, causal, beta):
    pol, tS, tstat, tO = TYPES[policy]
    d = 2
    scale = 1.0 / math.sqrt(d)
    mismatches = 0
    for seed in range(12):
        q, k, v = _case(1000 * N + seed, N if causal else 5, N, d, kbias=3.0, amp=2.0)
        got = po.pasa_rows(q, k, v, scale, causal, beta, T, pol)
        for r in range(q.shape[0]):
            want = alg1_row(q[r], k, v, scale, beta, T, causal, r, tS, tstat, tO)
            if not np.array_equal(got[r].view(np.uint16), want.view(np.uint16)):
                mismatches += 1
    assert mismatches == 0


@pytest.mark.parametrize("policy", ["PARTIAL16", "STRICT16", "MIXED"])
@pytest.mark.parametrize("N,T,causal", [(4, 2, False), (6, 2, True), (12, 4, False), (11, 4, True), (9, 3, False)])
def test_fa_rows_rounds_where_eq_1_to_8_say(policy, N, T, causal):
    pol, tS, tstat, tO = TYPES[policy]
    d = 2
    scale = 1.0 / math.sqrt(d)
    for seed in range(12):
        q, k, v = _case(7000 * N + seed, N if causal else 5, N, d, kbias=1.0, amp=2.0)
        got = po.fa_rows(q, k, v, scale, causal, T, pol)
        for r in range(q.shape[0]):
            want = fa_row(q[r], k, v, scale, T, causal, r, tS, tstat, tO)
            assert np.array_equal(got[r].view(np.uint16), want.view(np.uint16)), (seed, r)


@pytest.mark.parametrize("policy", ["MIXED", "STRICT16"])
@pytest.mark.parametrize("N,T,causal,d", [(8, 4, False, 2), (12, 4, True, 2), (9, 3, False, 2), (8, 4, False, 16)])
def test_direct_rows_rounds_where_its_docstring_says(policy, N, T, causal, d):
    # d = 16: the dot product q . k0 no longer fits fp32 exactly, so its own rounding to fp32 shows
    pol, tS, tstat, tO = TYPES[policy]
    scale = 1.0 / math.sqrt(d)
    for seed in range(12):
        q, k, v = _case(9000 * N + seed, N if causal else 5, N, d, kbias=3.0, amp=2.0)
        got = po.direct_rows(q, k, v, scale, causal, 63.5 / 64.5, T, pol)
        for r in range(q.shape[0]):
            want = direct_row(q[r], k, v, scale, 63.5 / 64.5, T, causal, r, tS, tstat, tO)
            assert np.array_equal(got[r].view(np.uint16), want.view(np.uint16)), (seed, r)


def test_native_half_scalars_round_every_operation_once():
    """The facts the evaluators above rest on: an operation on two numpy half scalars is ONE correctly rounded fp16
    operation (ties to even), and Eq. (15) taken in its printed order differs from its incremental form in fp16."""
    assert type(H(1) + H(1)) is H and type(F32(1) * F32(1)) is F32
    assert float(H(2049.0)) == 2048.0 and float(H(2051.0)) == 2052.0             # ties to even at spacing 2
    assert float(H(2048) + H(1)) == 2048.0 and float(H(2050) + H(1)) == 2052.0
    assert float(H(1) / H(3)) == 1365 / 4096                                      # 0.333251953125, nearest to 1/3
    # F^2 = 1, Sbar'^3 = -7.75, j = 3.  Printed order: 2 * 1 = 2; 2 - 7.75 = -5.75 (exact); -5.75 / 3 = -1.91666..,
    # spacing 2^-10 in [1, 2): 1962.67 -> 1963.  Incremental: -7.75 - 1 = -8.75; / 3 = -2.91666.., spacing 2^-9 in
    # [2, 4): 1493.33 -> 1493, i.e. -2.916015625; 1 - 2.916015625 = -1962/1024 exactly.
    Fprev, Sbar = H(1.0), H(-7.75)
    assert float(((H(2) * Fprev) + Sbar) / H(3)) == -1963 / 1024
    assert float(Fprev + (Sbar - Fprev) / H(3)) == -1962 / 1024


def test_three_tiles_by_hand_strict16():
    """One query row, d = 1, T = 2, beta = 1/2 (invariance 1), scale = 1, q = 1, keys (2, 2 | 2, 2 | -15.5, -15.5):
    K' = K - mean/2 = (1, 1 | 1, 1 | -7.75, -7.75), every score tile is constant, so P = (1, 1), l' = 2, m' = Sbar' = the
    score.  By hand, every operation rounded to fp16 (spacings: 2^-10 in [1,2), 2^-9 in [2,4), 2^-8 in [4,8), 2^-7 in
    [8,16), 2^-6 in [16,32)):
      tile 1:  F = 1, m = 1, l = 2
      tile 2:  F = (1*1 + 1)/2 = 1, both corrections 0, m = 1, l = 1*2 + 1*2 = 4
      tile 3:  F = ((2*1) - 7.75)/3 = -5.75/3 -> -1963/1024
               dm'_2 = 1 * fl(1 + 1963/1024) = fl(2.9169921875): 1493.5 halves of 2^-8 -> tie -> even -> 2.91796875
               dm'_3 = 1 * fl(-7.75 + 1963/1024) = fl(-5.8330078125) -> -5.83203125
               m_3   = max(fl(1 + 2.91796875), fl(-7.75 - 5.83203125)) = max(3.91796875, -13.578125) = 3.91796875
               dm_2  = fl(fl(1 - 3.91796875) + 2.91796875) = 0
               dm_3  = fl(fl(-7.75 - 3.91796875) + -5.83203125) = fl(-11.671875 - 5.83203125) = fl(-17.50390625) = -17.5
               e^0 = 1, fl(e^-17.5 = 2.5e-8) = 0 (below half of the smallest subnormal 6e-8), l = 1*4 + 0*2 = 4
    The output is (V_1 + V_2 + V_3 + V_4) / 4."""
    q = np.array([[1.0]], H)
    K = np.array([[2.0], [2.0], [2.0], [2.0], [-15.5], [-15.5]], H)
    V = np.array([[1.0], [3.0], [5.0], [-2.0], [100.0], [100.0]], H)
    st = {}
    out = po.pasa_rows(q, K, V, 1.0, False, 0.5, 2, po.STRICT16, info=st)
    assert st["F"][0] == -1963 / 1024
    assert st["m"][0] == 3.91796875
    assert st["l"][0] == 4.0
    assert float(out[0, 0]) == 1.75
    # with fp32 statistics the third tile's weight e^-17.5 survives and F is the fp32 quotient
    out32 = po.pasa_rows(q, K, V, 1.0, False, 0.5, 2, po.MIXED, info=st)
    assert st["F"][0] == float(F32(-5.75) / F32(3))
    assert st["l"][0] == pytest.approx(4.0 + 2 * math.exp(-17.5), rel=1e-6)
    assert float(out32[0, 0]) == 1.75
