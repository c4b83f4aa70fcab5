"""CPU oracle for PASA attention forward (arXiv 2503.01873).  TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the `cpu_baseline` leg of the bench may import this module.  It
shares no code with the HIP library and never calls it.  It is deliberately plain and slow: numpy,
fp64 arithmetic, one rounding per emulated low-precision operation, no fusion, no reordering.

Contents (citations are to the paper's sections / equations / Algorithm 1):

  fl                     round-to-nearest-even into fp16 / fp32 (Table 1 formats), returned as fp64
  optimal_beta           fixed-point solve of the optimal accuracy condition, Eq. (16), (20)-(22)
  invariance_rounded     the practical invariance Inva_1 of Appendix A, Eq. (20)-(21)
  shift_matrix           M = I/alpha - beta*J/(alpha*s2), Eq. (10)
  shift_keys             K' = (K - beta*Kbar)*scale per key tile, Eq. (11) / Alg. 1 pre-processing loop
  attention_fp64         the plain definition softmax(scale*Q K^T) V in fp64 (section 1.1, four steps)
  pasa_rows              Algorithm 1 step by step with a per-quantity precision policy
  fa_rows                plain blocked FlashAttention, Eq. (1)-(8), with the precision allocations of
                         section 1.2 (used for the beta = 0 special case and the overflow baseline)
  direct_rows            NOT the paper's recovering step: the same key shift, but the removed bias is added back
                         as the dot product of the query with the shift vector (Eq. (9) allows any shift), which
                         avoids multiplying the rounding noise of Sbar' by beta/(1-beta).  Kept under its own name.
  rmse                   relative RMSE, Eq. (19)

Pins (tests/test_oracle_*.py): Table 3 and the three printed beta values; Theorem 2.1; Eq. (13), (14);
softmax translation invariance Eq. (9); PASA in fp64 == plain definition for any beta / tile size;
beta = 0 == blocked FlashAttention; brute-force python loops on tiny inputs; Table 4 rows 1 and 4
(100 % NaN for the partially-fp16 allocation, none for PASA).
Accuracy *levels* of the low-precision policies against fp64 are "parity unpinned": the paper's RMSE
values were only plotted (Figures 13 and 14) and did not survive; only the ordering FP32-FA < PASA <
FP16-FP32-FA for non-zero-mean inputs (Appendix D) is checked, softly.

Readings taken where the paper is silent or inconsistent:
  * alpha = sqrt(d); callers pass scale = 1/alpha explicitly.
  * Eq. (6)/(7) are used with exp(m_{j-1} - m_j) (the printed sign would give factors >= 1).
  * Eq. (11)'s "/beta" is "/alpha".
  * The first key tile initialises the state (F = Sbar', m = m', l = l', O = P V) as the remark
    after Eq. (15) says; the printed m_0 = 0 is not used.
  * Every GEMM / row reduction accumulates exactly and is rounded once on output.
  * Causal masking and grouped-query heads are not in the paper: the pseudo-average Sbar' and the key
    tile mean use all keys of a tile; the mask is applied afterwards (legal by Eq. (9): any per-row
    constant may be removed from a row's scores).  Query head h reads KV head h // (Hq // Hkv).
  * In the default shift mode the matrix M is never formed: the tile mean is taken exactly (fp64),
    K' is rounded to fp16 once.  shift="gemm_m" forms M in fp16 and does the GEMM of Alg. 1 literally.
  * A sequence length that is not a multiple of the tile size (the paper's own Qwen2 case has 5676 keys; its
    handling is not stated): the last tile uses its own key count as the divisor of both the key mean and the
    pseudo-average Sbar', so that Eq. (14) still holds for it; the global pseudo-average F weighs it like any
    other tile (F is only a reference level).
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

FP16_MAX = 65504.0  # Table 1

_NP = {"f16": np.float16, "f32": np.float32, "f64": np.float64}


def fl(x, fmt: str) -> np.ndarray:
    """Round x (fp64) to the nearest value of format `fmt`, ties to even; overflow gives +-inf.

    The result is returned widened back to fp64 so that the next operation is again exact-then-rounded.
    """
    x = np.asarray(x, dtype=np.float64)
    if fmt == "f64":
        return x
    if fmt == "bf16":
        return _round_bf16(x)
    with np.errstate(over="ignore", invalid="ignore"):
        return x.astype(_NP[fmt]).astype(np.float64)


def _round_bf16(x: np.ndarray) -> np.ndarray:
    """bfloat16 (Table 1: 8 exponent bits, 8 significand bits with the hidden one) from fp64, one rounding."""
    x = np.asarray(x, dtype=np.float64)
    with np.errstate(over="ignore", invalid="ignore"):
        m, e = np.frexp(x)                                  # x = m * 2^e, 0.5 <= |m| < 1
        lsb = np.maximum(e - 8, -133)                       # weight of the last kept bit; -133: subnormal spacing
        r = np.ldexp(np.rint(np.ldexp(x, -lsb)), lsb)       # rint: ties to even
        r = np.where(np.abs(r) >= 2.0 ** 128, np.copysign(np.inf, x), r)
    return np.where(np.isfinite(x), r, x)


@dataclass(frozen=True)
class Policy:
    """Storage precision of each quantity of Algorithm 1 (section 1.2, Figures 1-3)."""

    S: str     # score tile as it leaves the matrix engine
    P: str     # exp(S - m), the second GEMM's operand
    stat: str  # Sbar', F, all Delta terms, m, l
    O: str     # P V tile and the running output
    K: str = "f16"  # the shifted key tile K' (the first GEMM's operand)


MIXED = Policy("f32", "f16", "f32", "f32")      # fp16 operands, fp32 everything else (Fig. 1 allocation + shift)
STRICT16 = Policy("f16", "f16", "f16", "f16")   # everything fp16 as Algorithm 1 marks it (Fig. 3 allocation)
PARTIAL16 = Policy("f16", "f16", "f32", "f32")  # only S is fp16 (Fig. 2, "FP16-FP32")
EXACT64 = Policy("f64", "f64", "f64", "f64", "f64")  # no rounding at all; for algebraic pins


# ----------------------------------------------------------------------------------------------
# Optimal accuracy condition (section 2.3, Appendix A, B, C)
# ----------------------------------------------------------------------------------------------

def _rounded_ab(beta: float, n: int, tp: str):
    """a, b of Eq. (21): the rounded shifting matrix is a*I - b*J (Eq. (22) of Appendix B)."""
    b = float(fl(beta / n, tp))
    a = float(fl(1.0 - beta / n, tp)) + b
    return a, b


def invariance_rounded(beta: float, n: int, tp: str = "f16") -> float:
    """Inva_1 = b n / (a (a - b n)) + (1 - a) / a, Eq. (20)."""
    a, b = _rounded_ab(beta, n, tp)
    return b * n / (a * (a - b * n)) + (1.0 - a) / a


def optimal_beta(beta0: float, n: int, tp: str = "f16", tol: float = 1e-8, max_iter: int = 1000) -> float:
    """Solve beta/(1-beta) = f(beta) by the fixed-point iteration beta <- f/(1+f), Eq. (16), (22)."""
    beta = float(beta0)
    for _ in range(max_iter):
        f = invariance_rounded(beta, n, tp)
        new = f / (1.0 + f)
        err = abs(new - beta) / abs(beta)
        beta = new
        if err <= tol:
            break
    return beta


def default_beta() -> float:
    """beta whose invariance beta/(1-beta) is exactly 63.5.

    63.5 is fl16 of the invariance of the paper's adopted beta = 0.984497 (Table 3, right); 63.5/64.5
    differs from 0.984497 by 1e-6.  With the matrix M never formed there is no rounded (a, b) pair, so
    the optimal-accuracy condition reduces to "the invariance is exactly representable".
    """
    return 63.5 / 64.5


# ----------------------------------------------------------------------------------------------
# Shifting (steps 1 and 2 of the method)
# ----------------------------------------------------------------------------------------------

def shift_matrix(beta: float, s2: int, alpha: float) -> np.ndarray:
    """Eq. (10) in fp64."""
    return np.eye(s2) / alpha - beta * np.ones((s2, s2)) / (alpha * s2)


def shift_keys(K: np.ndarray, beta: float, scale: float, T: int = 128, mode: str = "mean",
               fmt: str = "f16") -> np.ndarray:
    """K' for every key tile of one head.  K: fp16 [N, d] -> [N, d] rounded to `fmt` (fp16 in the method).

    mode "mean":   K'[n, c] = fl16((K[n, c] - beta * mean_{tile}(K[:, c])) * scale), Eq. (11).
    mode "gemm_m": K'^T = fl16(K^T M16), M16 = fl16(M) entrywise, the literal GEMM of Alg. 1.
    """
    N, d = K.shape
    K64 = K.astype(np.float64)
    if mode == "mean":
        Kp = np.empty((N, d))
        for t0 in range(0, N, T):                           # a ragged last tile uses its own key count
            tile = K64[t0:t0 + T]
            kbar = tile.sum(axis=0, keepdims=True) / tile.shape[0]   # exact: at most 128 fp16 values fit fp64
            Kp[t0:t0 + T] = (tile - beta * kbar) * scale
    elif mode == "gemm_m":
        assert N % T == 0
        M16 = fl(shift_matrix(beta, T, 1.0 / scale), "f16")
        # (K_j^T M)[c, q] = sum_p K_j[p, c] M[p, q]  ->  K'_j = M^T K_j
        Kp = np.einsum("pq,jpc->jqc", M16, K64.reshape(N // T, T, d)).reshape(N, d)
    else:
        raise ValueError(mode)
    with np.errstate(over="ignore"):
        return Kp.astype(_NP[fmt])


# ----------------------------------------------------------------------------------------------
# The plain definition (golden)
# ----------------------------------------------------------------------------------------------

def attention_fp64(Q, K, V, scale: float, causal: bool, row0: int = 0) -> np.ndarray:
    """softmax(scale * Q K^T) V in fp64 for one head; Q holds query rows row0 .. row0+R-1."""
    Q = np.asarray(Q, np.float64)
    K = np.asarray(K, np.float64)
    V = np.asarray(V, np.float64)
    S = (Q @ K.T) * scale
    if causal:
        rows = row0 + np.arange(Q.shape[0])
        S = np.where(np.arange(K.shape[0])[None, :] > rows[:, None], -np.inf, S)
    S = S - S.max(axis=1, keepdims=True)
    P = np.exp(S)
    return (P @ V) / P.sum(axis=1, keepdims=True)


# ----------------------------------------------------------------------------------------------
# Algorithm 1, step by step
# ----------------------------------------------------------------------------------------------

def from_bf16(x) -> np.ndarray:
    """The paper's rule for BF16 inputs: convert them to FP16 and run the method on that.  x holds bf16 values
    (in any wider numpy type); the result is the fp16 array the method then sees."""
    with np.errstate(over="ignore"):
        return np.asarray(x, np.float64).astype(np.float16)


def pasa_rows(Q, K, V, scale: float, causal: bool, beta: float, T: int = 128,
              policy: Policy = MIXED, row0: int = 0, shift: str = "mean", info: dict | None = None,
              out_fmt: str = "f16"):
    """Algorithm 1 for query rows row0 .. row0+R-1 of one head.  Q [R,d], K,V [N,d] fp16 -> fp16 [R,d].

    out_fmt "bf16": the quotient O / l is rounded to the precision O is kept in, then to bf16, and returned as
    float32 values (numpy has no bf16 type).

    Rows are independent: all state (F, m, l, O) is per query row.  If `info` is a dict it receives
    max |S'| over finite entries, the number of non-finite S' entries and of S' entries seen, and the final per-row
    state F, m, l (copies).
    """
    st, pS, pP, pO = policy.stat, policy.S, policy.P, policy.O
    Q64 = np.asarray(Q).astype(np.float64)
    V64 = np.asarray(V).astype(np.float64)
    N, d = K.shape
    R = Q64.shape[0]
    Kp64 = shift_keys(np.asarray(K), beta, scale, T, shift, policy.K).astype(np.float64)
    inva = float(fl(beta / (1.0 - beta), st))
    rows = row0 + np.arange(R)
    ntile = np.minimum(rows // T + 1, -(-N // T)) if causal else np.full(R, -(-N // T))   # positions past the last key see all keys

    F = np.zeros(R)
    m = np.zeros(R)
    l = np.zeros(R)
    O = np.zeros((R, d))
    smax, s_nonfinite, s_seen = 0.0, 0, 0

    with np.errstate(over="ignore", invalid="ignore", divide="ignore"):
        for jt in range(int(ntile.max())):
            a = np.nonzero(ntile > jt)[0]          # rows that still have this tile
            Kt = Kp64[jt * T:(jt + 1) * T]
            Vt = V64[jt * T:(jt + 1) * T]
            Tv = Kt.shape[0]                                            # keys in this tile (< T only in a ragged tail)
            S = fl(Q64[a] @ Kt.T, pS)                                   # first GEMM
            fin = np.isfinite(S)
            s_seen += S.size
            s_nonfinite += int(S.size - fin.sum())
            if fin.any():
                smax = max(smax, float(np.abs(S[fin]).max()))
            Sbar = fl(S.sum(axis=1) / Tv, st)                           # pseudo-average, all keys of the tile
            if causal:
                keys = jt * T + np.arange(Tv)
                S = np.where(keys[None, :] > rows[a][:, None], -np.inf, S)
            mloc = S.max(axis=1)                                        # m'
            P = fl(np.exp(fl(S - mloc[:, None], pS)), pP)
            lloc = fl(P.sum(axis=1), st)                                # l'
            Ot = fl(P @ Vt, pO)                                         # second GEMM
            if jt == 0:
                F[a], m[a], l[a], O[a] = Sbar, mloc, lloc, Ot
                continue
            j = jt + 1
            Fprev = F[a]
            Fnew = fl(fl(fl((j - 1) * Fprev, st) + Sbar, st) / j, st)   # Eq. (15)
            dpp = fl(inva * fl(Fprev - Fnew, st), st)                   # Delta m'_{j-1}
            dpc = fl(inva * fl(Sbar - Fnew, st), st)                    # Delta m'_j
            mnew = np.maximum(fl(m[a] + dpp, st), fl(mloc + dpc, st))   # m_j
            dp = fl(fl(m[a] - mnew, st) + dpp, st)                      # Delta m_{j-1}
            dc = fl(fl(mloc - mnew, st) + dpc, st)                      # Delta m_j
            ep = fl(np.exp(dp), st)
            ec = fl(np.exp(dc), st)
            l[a] = fl(fl(ep * l[a], st) + fl(ec * lloc, st), st)
            O[a] = fl(fl(ec[:, None] * Ot, pO) + fl(ep[:, None] * O[a], pO), pO)
            m[a] = mnew
            F[a] = Fnew
        if out_fmt == "bf16":
            out = fl(fl(O / l[:, None], pO), "bf16").astype(np.float32)
        else:
            out = (O / l[:, None]).astype(np.float16)
    if info is not None:
        info.update(smax=smax, s_nonfinite=s_nonfinite, s_seen=s_seen, F=F.copy(), m=m.copy(), l=l.copy())
    return out


# ----------------------------------------------------------------------------------------------
# Direct-bias recovery (not in the paper; same shift, different recovering step)
# ----------------------------------------------------------------------------------------------

def direct_shift_keys(K: np.ndarray, beta: float, scale: float, T: int = 128):
    """Per key tile: k0 = fl16(beta * mean_tile(K)) and K' = fl16((K - k0) * scale).  Returns (K' [N,d] fp16,
    k0 [ntile,d] fp16).  The shift vector is itself an fp16 vector, so S = S' + scale * Q k0 holds exactly for the
    K' before its own rounding (softmax translation invariance, Eq. (9), with K0 = k0)."""
    N, d = K.shape
    K64 = np.asarray(K).astype(np.float64)
    ntile = -(-N // T)
    Kp = np.empty((N, d))
    k0 = np.empty((ntile, d))
    for jt in range(ntile):
        tile = K64[jt * T:(jt + 1) * T]
        kbar = tile.sum(axis=0) / tile.shape[0]                     # exact sum, one division
        k0[jt] = fl(beta * kbar, "f16")
        Kp[jt * T:(jt + 1) * T] = (tile - k0[jt][None, :]) * scale    # the difference is exact in fp64
    with np.errstate(over="ignore"):
        return Kp.astype(np.float16), k0.astype(np.float16)


def direct_rows(Q, K, V, scale: float, causal: bool, beta: float, T: int = 128, policy: Policy = MIXED,
                row0: int = 0, info: dict | None = None):
    """Blocked attention with the key shift of Eq. (10), (11) and the bias added back directly.

    Per tile j and query row: S' = Q K'_j^T as in Algorithm 1 (so the scores stay small), c_j = scale * (Q . k0_j),
    local maximum m'_j, P = exp(S' - m'_j), and then ordinary online softmax (Eq. (4)-(8)) on the level m'_j + c_j.
    """
    st, pS, pP, pO = policy.stat, policy.S, policy.P, policy.O
    Q64 = np.asarray(Q).astype(np.float64)
    V64 = np.asarray(V).astype(np.float64)
    N, d = K.shape
    R = Q64.shape[0]
    Kp, k0 = direct_shift_keys(np.asarray(K), beta, scale, T)
    Kp64, k064 = Kp.astype(np.float64), k0.astype(np.float64)
    rows = row0 + np.arange(R)
    ntile = np.minimum(rows // T + 1, -(-N // T)) if causal else np.full(R, -(-N // T))
    Mx = np.zeros(R)
    l = np.zeros(R)
    O = np.zeros((R, d))
    smax = 0.0
    with np.errstate(over="ignore", invalid="ignore", divide="ignore"):
        for jt in range(int(ntile.max())):
            a = np.nonzero(ntile > jt)[0]
            Kt = Kp64[jt * T:(jt + 1) * T]
            Vt = V64[jt * T:(jt + 1) * T]
            S = fl(Q64[a] @ Kt.T, pS)
            smax = max(smax, float(np.abs(S[np.isfinite(S)]).max()))
            c = fl(scale * fl(Q64[a] @ k064[jt], "f32"), st)           # the removed bias of this tile, per row
            if causal:
                keys = jt * T + np.arange(Kt.shape[0])
                S = np.where(keys[None, :] > rows[a][:, None], -np.inf, S)
            mloc = S.max(axis=1)
            P = fl(np.exp(fl(S - mloc[:, None], pS)), pP)
            lloc = fl(P.sum(axis=1), st)
            Ot = fl(P @ Vt, pO)
            L = fl(mloc + c, st)                                        # level of this tile's maximum
            if jt == 0:
                Mx[a], l[a], O[a] = L, lloc, Ot
                continue
            Mn = np.maximum(Mx[a], L)
            ep = fl(np.exp(fl(Mx[a] - Mn, st)), st)
            ec = fl(np.exp(fl(L - Mn, st)), st)
            l[a] = fl(fl(ep * l[a], st) + fl(ec * lloc, st), st)
            O[a] = fl(fl(ec[:, None] * Ot, pO) + fl(ep[:, None] * O[a], pO), pO)
            Mx[a] = Mn
        out = (O / l[:, None]).astype(np.float16)
    if info is not None:
        info.update(smax=smax)
    return out


def direct_bhnd(q, k, v, scale, causal, beta, T=128, policy=MIXED) -> np.ndarray:
    B, Hq, N, d = q.shape
    Hkv = k.shape[1]
    out = np.empty((B, Hq, N, d), np.float16)
    for b in range(B):
        for h in range(Hq):
            hk = h // (Hq // Hkv)
            out[b, h] = direct_rows(q[b, h], k[b, hk], v[b, hk], scale, causal, beta, T, policy)
    return out


# ----------------------------------------------------------------------------------------------
# Plain blocked FlashAttention, Eq. (1)-(8)
# ----------------------------------------------------------------------------------------------

def fa_rows(Q, K, V, scale: float, causal: bool, T: int = 128, policy: Policy = PARTIAL16,
            row0: int = 0, info: dict | None = None):
    """Blocked FlashAttention for query rows row0.. of one head, no shifting.

    S_raw = fl_S(Q K_j^T) is rounded as it leaves the matrix engine and only then scaled (Eq. (1), (2)),
    which is where the partially / fully low-precision allocations overflow (section 2.1).  The running
    maximum, sum and output follow Eq. (4)-(8).
    """
    st, pS, pP, pO = policy.stat, policy.S, policy.P, policy.O
    Q64 = np.asarray(Q).astype(np.float64)
    K64 = np.asarray(K).astype(np.float64)
    V64 = np.asarray(V).astype(np.float64)
    N, d = K64.shape
    R = Q64.shape[0]
    rows = row0 + np.arange(R)
    ntile = np.minimum(rows // T + 1, -(-N // T)) if causal else np.full(R, -(-N // T))   # positions past the last key see all keys
    m = np.full(R, -np.inf)
    l = np.zeros(R)
    O = np.zeros((R, d))
    smax, s_nonfinite, s_seen = 0.0, 0, 0
    with np.errstate(over="ignore", invalid="ignore", divide="ignore"):
        for jt in range(int(ntile.max())):
            a = np.nonzero(ntile > jt)[0]
            Sraw = fl(Q64[a] @ K64[jt * T:(jt + 1) * T].T, pS)          # Eq. (1)
            fin = np.isfinite(Sraw)
            s_seen += Sraw.size
            s_nonfinite += int(Sraw.size - fin.sum())
            if fin.any():
                smax = max(smax, float(np.abs(Sraw[fin]).max()))
            S = fl(Sraw * scale, st)                                    # Eq. (2)
            if causal:
                keys = jt * T + np.arange(S.shape[1])
                S = np.where(keys[None, :] > rows[a][:, None], -np.inf, S)
            mnew = np.maximum(m[a], S.max(axis=1))                      # Eq. (4)
            P = fl(np.exp(fl(S - mnew[:, None], st)), pP)               # Eq. (5)
            e = fl(np.exp(fl(m[a] - mnew, st)), st)
            l[a] = fl(fl(e * l[a], st) + fl(P.sum(axis=1), st), st)     # Eq. (6)
            O[a] = fl(fl(e[:, None] * O[a], pO) + fl(P @ V64[jt * T:(jt + 1) * T], pO), pO)  # Eq. (7)
            m[a] = mnew
        out = (O / l[:, None]).astype(np.float16)                       # Eq. (8)
    if info is not None:
        info.update(smax=smax, s_nonfinite=s_nonfinite, s_seen=s_seen)
    return out


# ----------------------------------------------------------------------------------------------
# [B, H, N, d] conveniences and the error metric
# ----------------------------------------------------------------------------------------------

def kv_head(h: int, Hq: int, Hkv: int) -> int:
    return h // (Hq // Hkv)


def attention_fp64_bhnd(q, k, v, scale, causal, block: int = 512) -> np.ndarray:
    """Golden output for whole [B,Hq,N,d] tensors (fp64 result)."""
    B, Hq, N, d = q.shape
    Hkv = k.shape[1]
    out = np.empty((B, Hq, N, d), np.float64)
    for b in range(B):
        for h in range(Hq):
            hk = kv_head(h, Hq, Hkv)
            for r0 in range(0, N, block):
                r1 = min(N, r0 + block)
                nk = r1 if causal else N
                out[b, h, r0:r1] = attention_fp64(q[b, h, r0:r1], k[b, hk, :nk], v[b, hk, :nk], scale, causal, r0)
    return out


def pasa_bhnd(q, k, v, scale, causal, beta, T=128, policy=MIXED, shift="mean") -> np.ndarray:
    B, Hq, N, d = q.shape
    Hkv = k.shape[1]
    out = np.empty((B, Hq, N, d), np.float16)
    for b in range(B):
        for h in range(Hq):
            hk = kv_head(h, Hq, Hkv)
            out[b, h] = pasa_rows(q[b, h], k[b, hk], v[b, hk], scale, causal, beta, T, policy, 0, shift)
    return out


def fa_bhnd(q, k, v, scale, causal, T=128, policy=PARTIAL16) -> np.ndarray:
    B, Hq, N, d = q.shape
    Hkv = k.shape[1]
    out = np.empty((B, Hq, N, d), np.float16)
    for b in range(B):
        for h in range(Hq):
            hk = kv_head(h, Hq, Hkv)
            out[b, h] = fa_rows(q[b, h], k[b, hk], v[b, hk], scale, causal, T, policy)
    return out


def adaptive_bhnd(q, k, v, scale, causal, beta, T=128, policy=MIXED, info=None):
    """The adaptive start the paper leaves to future work (its closing section), in a simple form: run the
    partially low-precision FlashAttention (raw scores stored in fp16, Fig. 2) and keep its result for the query heads
    of a (batch, KV head) unless some raw score of one of them left the fp16 range; only those get PASA (they share
    the shifted keys, so a KV head is the finest unit).  Returns (output, triggered anywhere); info, if a dict,
    receives 'groups': the boolean [B, Hkv] array of the (batch, KV head)s that switched."""
    B, Hq, N, d = q.shape
    Hkv = k.shape[1]
    out = np.empty((B, Hq, N, d), np.float16)
    overflowed = np.zeros((B, Hkv), np.int64)
    for b in range(B):
        for h in range(Hq):
            hk = kv_head(h, Hq, Hkv)
            one = {}
            out[b, h] = fa_rows(q[b, h], k[b, hk], v[b, hk], scale, causal, T, PARTIAL16, 0, one)
            overflowed[b, hk] += one["s_nonfinite"]
    for b in range(B):
        for h in range(Hq):
            hk = kv_head(h, Hq, Hkv)
            if overflowed[b, hk]:
                out[b, h] = pasa_rows(q[b, h], k[b, hk], v[b, hk], scale, causal, beta, T, policy)
    if info is not None:
        info["groups"] = overflowed > 0
    return out, bool(overflowed.any())


def rmse(o, o_gold) -> float:
    """Relative RMSE, Eq. (19): ||O - O_gold||_2 / ||O_gold||_2."""
    o = np.asarray(o, np.float64)
    g = np.asarray(o_gold, np.float64)
    return float(np.linalg.norm((o - g).ravel()) / np.linalg.norm(g.ravel()))
