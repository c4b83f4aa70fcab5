// PASA attention forward for gfx950: device kernels and their launchers.
//
// Two kernels per call.
//
//  pasa_prep_kv   Algorithm 1's pre-processing loop (Eq. (10), (11)) without forming the matrix M:
//                 per 128-key tile, the per-channel mean of K is taken exactly in fp64, K' = (K - beta*mean)*kscale
//                 is rounded once to fp16, and both K' and V are re-tiled so that the main kernel's LDS image of
//                 a tile is a straight copy whose MFMA fragments are single conflict-free 128-bit LDS reads.
//
//  pasa_fwd       Algorithm 1's main loops.  One workgroup = 4 wavefronts = 256 query rows; each wavefront owns
//                 64 query rows and sweeps the key tiles.  Both GEMMs are computed transposed on
//                 v_mfma_f32_32x32x16_f16:
//                     S'^T = K' Q^T      (A = K' fragment from LDS, B = Q fragment held in registers)
//                     O^T += V^T P^T     (A = V^T fragment from LDS, B = P^T taken straight from the S'^T accumulators)
//                 In the transposed accumulator layout a lane holds 64 keys of ONE query row, so the row
//                 statistics (pseudo-average Sbar', maximum m', sum l') are in-lane reductions plus one exchange
//                 with lane^32, and exp(S'-m') converted to fp16 is already the B operand of the second GEMM.
//
// Tile layouts in the workspace (one tile = 128 keys x D channels, fp16, 16-byte chunks):
//   K' tile: chunk index (c/8)*128 + n         holds channels 8*(c/8) .. +7 of key n
//   V  tile: chunk index ((n/16)*2 + h)*D + c  holds, for channel c, the 8 keys 16*(n/16) + {4h..4h+3, 8+4h..8+4h+3}
// The second layout is the key order in which a lane of the 32x32 accumulator holds its S'^T rows.
//
// The matrix cores accumulate in fp32 in every variant; "fp16" quantities are rounded (nearest-even) where
// Algorithm 1 marks them.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pasa_kernels.h"

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef _Float16 h4 __attribute__((ext_vector_type(4)));
typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef float f16v __attribute__((ext_vector_type(16)));
typedef float f2 __attribute__((ext_vector_type(2)));

namespace {

constexpr int T = 128;          // keys per shift tile (s2 of the paper)
constexpr int ROWS_PER_WAVE = 64;
constexpr int WAVES = 4;
constexpr int ROWS_PER_WG = ROWS_PER_WAVE * WAVES;
constexpr float LOG2E = 1.4426950408889634f;

// ---------------------------------------------------------------------------------------------
// fp64 -> fp16 with a single rounding: truncate to fp32 (round to nearest, then step back if that
// rounded away from zero), make the fp32 "odd" when inexact, then
// let the hardware round fp32 -> fp16 to nearest-even.  fp32 has more than two extra bits, so the
// sticky bit makes the second rounding see exactly what a direct rounding would.
// ---------------------------------------------------------------------------------------------
__device__ inline _Float16 double_to_half_rn(double x)
{
    float f = (float)x;                         // nearest
    if ((double)f != x) {
        uint32_t u = __float_as_uint(f);
        if (__builtin_fabs((double)f) > __builtin_fabs(x)) u -= 1u;   // step the magnitude back: now truncated
        f = __uint_as_float(u | 1u);            // sticky bit
    }
    return (_Float16)f;
}

// ---------------------------------------------------------------------------------------------
// Pre-processing kernel.  grid = B*Hkv*(N/128) tiles, 256 threads.
// plain_out != nullptr: write K' in the plain [.., N, D] layout instead (pasa_shift_keys).
// ---------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void pasa_prep_kv(const _Float16* __restrict__ k, const _Float16* __restrict__ v,
                                                    _Float16* __restrict__ kp, _Float16* __restrict__ vt,
                                                    _Float16* __restrict__ plain_out, double beta, double kscale)
{
    constexpr int CH = D / 8;            // 16-byte chunks per key
    constexpr int KL = 256 / CH;         // key lanes
    constexpr int KPT = T / KL;          // keys per thread
    __shared__ double psum[KL][D];
    __shared__ _Float16 vs[T][D + 8];    // +8 halfs: rows start 16 bytes apart in bank space

    const size_t tile = blockIdx.x;
    const _Float16* ksrc = k + tile * (size_t)(T * D);
    const int tid = threadIdx.x;
    const int c8 = tid % CH, kl = tid / CH;

    h8 kv[KPT];
    double s[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int i = 0; i < KPT; ++i) {
        const int n = kl + KL * i;
        kv[i] = *reinterpret_cast<const h8*>(ksrc + n * D + 8 * c8);
#pragma unroll
        for (int e = 0; e < 8; ++e) s[e] += (double)kv[i][e];   // exact: fp16 values, 128 terms
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) psum[kl][8 * c8 + e] = s[e];

    if (v != nullptr) {
        const _Float16* vsrc = v + tile * (size_t)(T * D);
#pragma unroll
        for (int i = 0; i < KPT; ++i) {
            const int n = kl + KL * i;
            *reinterpret_cast<h8*>(&vs[n][8 * c8]) = *reinterpret_cast<const h8*>(vsrc + n * D + 8 * c8);
        }
    }
    __syncthreads();

    double mean[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        double t = 0;
        for (int r = 0; r < KL; ++r) t += psum[r][8 * c8 + e];
        mean[e] = t / (double)T;
    }
#pragma unroll
    for (int i = 0; i < KPT; ++i) {
        const int n = kl + KL * i;
        h8 out;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            // three separately rounded fp64 operations (no contraction): beta*mean, K - that, * kscale
            const double bm = __dmul_rn(beta, mean[e]);
            const double df = __dsub_rn((double)kv[i][e], bm);
            out[e] = double_to_half_rn(__dmul_rn(df, kscale));
        }
        if (plain_out != nullptr)
            *reinterpret_cast<h8*>(plain_out + tile * (size_t)(T * D) + n * D + 8 * c8) = out;
        else
            *reinterpret_cast<h8*>(kp + tile * (size_t)(T * D) + ((size_t)c8 * T + n) * 8) = out;
    }

    if (v != nullptr) {
        _Float16* vdst = vt + tile * (size_t)(T * D);
        for (int chunk = tid; chunk < 16 * D; chunk += 256) {
            const int c = chunk % D;
            const int kh = chunk / D;            // (n/16)*2 + h
            const int nb = (kh >> 1) * 16 + (kh & 1) * 4;
            h8 out;
#pragma unroll
            for (int e = 0; e < 8; ++e) out[e] = vs[nb + (e >> 2) * 8 + (e & 3)][c];
            *reinterpret_cast<h8*>(vdst + (size_t)chunk * 8) = out;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Main kernel
// ---------------------------------------------------------------------------------------------
__device__ inline float xor32(float x) { return __shfl_xor(x, 32, 64); }

__device__ inline float exp_nat(float x) { return __builtin_amdgcn_exp2f(x * LOG2E); }

template <int D, int VAR, bool CAUSAL, bool INSTR>
__global__ __launch_bounds__(256, 1) void pasa_fwd(const _Float16* __restrict__ q, const _Float16* __restrict__ kp,
                                                   const _Float16* __restrict__ vt, _Float16* __restrict__ o,
                                                   int Hq, int Hkv, int N, int nqt, float inva, float scale,
                                                   unsigned long long* ovf_s, unsigned long long* nonfinite_o)
{
    constexpr int KS = D / 16;   // k-steps of S'^T = K' Q^T
    constexpr int CB = D / 32;   // 32-channel row blocks of O^T
    constexpr bool S16 = (VAR != PASA_K_MIXED);                 // S' rounded to fp16 as it leaves the matrix core
    constexpr bool STRICT = (VAR == PASA_K_STRICT16);
    constexpr bool NAIVE = (VAR == PASA_K_NAIVE16);
    constexpr int TILE_HALFS = T * D;

    __shared__ __attribute__((aligned(16))) _Float16 lds_k[TILE_HALFS];
    __shared__ __attribute__((aligned(16))) _Float16 lds_v[TILE_HALFS];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lq = lane & 31, lh = lane >> 5;

    // work decode: longest (last) query tiles first so that causal work drains evenly
    const int wg = blockIdx.x;
    const int qt = nqt - 1 - (wg % nqt);
    const int bh = wg / nqt;
    const int hq = bh % Hq, b = bh / Hq;
    const int hk = hq / (Hq / Hkv);
    const int ntile = N / T;

    const int q0 = qt * ROWS_PER_WG;
    const int qw0 = q0 + wave * ROWS_PER_WAVE;
    const bool wave_valid = qw0 < N;       // N is a multiple of 128 and a wave owns 64 rows: all or nothing
    int last_row_wg = q0 + ROWS_PER_WG - 1;
    if (last_row_wg > N - 1) last_row_wg = N - 1;
    const int J_wg = CAUSAL ? (last_row_wg / T + 1) : ntile;
    const int J_w = wave_valid ? (CAUSAL ? ((qw0 + ROWS_PER_WAVE - 1) / T + 1) : ntile) : 0;

    const _Float16* qbase = q + ((size_t)(b * Hq + hq) * N) * D;
    const _Float16* kbase = kp + ((size_t)(b * Hkv + hk) * ntile) * TILE_HALFS;
    const _Float16* vbase = vt + ((size_t)(b * Hkv + hk) * ntile) * TILE_HALFS;

    // Q fragments: B operand, lane (query lq of block qb, half lh) holds channels 16*ks + 8*lh .. +7
    h8 Qf[2][KS];
    if (wave_valid) {
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                Qf[qb][ks] = *reinterpret_cast<const h8*>(qbase + (size_t)(qw0 + 32 * qb + lq) * D + 16 * ks + 8 * lh);
    } else {
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) Qf[qb][ks] = (h8)(_Float16)0;
    }

    // per-row state (one query row per lane and query block; both halves of the wave hold copies)
    float F[2], m[2], l[2];          // STRICT: values are always fp16-representable
    f16v O[2][CB];                   // fp32 running output (not used by STRICT)
    h2 O16[2][CB][8];                // fp16 running output (STRICT only)
    unsigned long long n_ovf = 0;
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        F[qb] = 0.f;
        m[qb] = NAIVE ? -__builtin_inff() : 0.f;
        l[qb] = 0.f;
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
            O[qb][cb] = (f16v)0.f;
#pragma unroll
            for (int t = 0; t < 8; ++t) O16[qb][cb][t] = (h2)(_Float16)0;
        }
    }

    for (int j = 0; j < J_wg; ++j) {
        __syncthreads();   // everyone is done with the previous tile
        {
            const h8* ks = reinterpret_cast<const h8*>(kbase + (size_t)j * TILE_HALFS);
            const h8* vs = reinterpret_cast<const h8*>(vbase + (size_t)j * TILE_HALFS);
            h8* kd = reinterpret_cast<h8*>(lds_k);
            h8* vd = reinterpret_cast<h8*>(lds_v);
#pragma unroll
            for (int i = 0; i < TILE_HALFS / 8 / 256; ++i) {
                kd[tid + 256 * i] = ks[tid + 256 * i];
                vd[tid + 256 * i] = vs[tid + 256 * i];
            }
        }
        __syncthreads();
        if (j >= J_w) continue;     // wave-uniform; the barriers above are still reached by every wave

        // ---------------- first GEMM: S'^T tile (128 keys x 64 queries) ----------------
        f16v S[2][4];
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int kb = 0; kb < 4; ++kb) S[qb][kb] = (f16v)0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int kb = 0; kb < 4; ++kb) {
                const h8 a = *reinterpret_cast<const h8*>(lds_k + ((2 * ks + lh) * T + 32 * kb + lq) * 8);
                S[0][kb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, Qf[0][ks], S[0][kb], 0, 0, 0);
                S[1][kb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, Qf[1][ks], S[1][kb], 0, 0, 0);
            }

        const bool diag = CAUSAL && (j * T + T - 1 > qw0);
        h8 Pf[2][8];
        float ec_[2], ep_[2];
        bool first = (j == 0);

#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            const int row = qw0 + 32 * qb + lq;
            // ---- S' as stored: fp32, or rounded to fp16 ----
            if (S16) {
#pragma unroll
                for (int kb = 0; kb < 4; ++kb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const float s32 = S[qb][kb][i];
                        if (INSTR) n_ovf += (__builtin_fabsf(s32) >= 65520.f) ? 1u : 0u;
                        float s = (float)(_Float16)s32;
                        if (NAIVE) s = s * scale;          // Eq. (2): static scaling after the GEMM
                        S[qb][kb][i] = s;
                    }
            } else if (INSTR) {
#pragma unroll
                for (int kb = 0; kb < 4; ++kb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) n_ovf += (__builtin_fabsf(S[qb][kb][i]) >= 65520.f) ? 1u : 0u;
            }
            // ---- pseudo-average over all 128 keys of the tile (before masking) ----
            float sbar = 0.f;
            if (!NAIVE) {
                float sum = 0.f;
#pragma unroll
                for (int kb = 0; kb < 4; ++kb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) sum += S[qb][kb][i];
                sum += xor32(sum);
                sbar = sum * (1.0f / T);
                if (STRICT) sbar = (float)(_Float16)sbar;
            }
            // ---- causal mask (diagonal tiles only) ----
            if (diag) {
#pragma unroll
                for (int kb = 0; kb < 4; ++kb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int key = j * T + 32 * kb + 8 * (i >> 2) + 4 * lh + (i & 3);
                        if (key > row) S[qb][kb][i] = -__builtin_inff();
                    }
            }
            // ---- local maximum m' ----
            float mx = -__builtin_inff();
#pragma unroll
            for (int kb = 0; kb < 4; ++kb)
#pragma unroll
                for (int i = 0; i < 16; ++i) mx = __builtin_fmaxf(mx, S[qb][kb][i]);
            mx = __builtin_fmaxf(mx, xor32(mx));

            // ---- reference level for exp: local m' (PASA), running max (plain FlashAttention) ----
            float mref = mx, e_old = 0.f;
            if (NAIVE) {
                const float mnew = __builtin_fmaxf(m[qb], mx);
                e_old = exp_nat(m[qb] - mnew);
                m[qb] = mnew;
                mref = mnew;
            }
            // ---- P = exp(S' - m') rounded to fp16; l' = sum of the rounded P ----
            float lsum = 0.f;
#pragma unroll
            for (int kb = 0; kb < 4; ++kb)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    float x = S[qb][kb][i] - mref;
                    if (STRICT) x = (float)(_Float16)x;
                    const _Float16 p = (_Float16)exp_nat(x);
                    Pf[qb][2 * kb + (i >> 3)][i & 7] = p;
                    lsum += (float)p;
                }
            lsum += xor32(lsum);
            if (STRICT) lsum = (float)(_Float16)lsum;

            // ---- global recovering (step 3) and the running sum (step 4) ----
            if (NAIVE) {
                l[qb] = e_old * l[qb] + lsum;
                ep_[qb] = e_old;
                ec_[qb] = 1.f;
            } else if (first) {
                F[qb] = sbar;
                m[qb] = mx;
                l[qb] = lsum;
                ep_[qb] = 0.f;
                ec_[qb] = 1.f;
            } else if (!STRICT) {
                const float jm1 = (float)j, jj = (float)(j + 1);
                const float Fn = (jm1 * F[qb] + sbar) / jj;
                const float dpp = inva * (F[qb] - Fn);
                const float dpc = inva * (sbar - Fn);
                const float mn = __builtin_fmaxf(m[qb] + dpp, mx + dpc);
                const float dp = (m[qb] - mn) + dpp;
                const float dc = (mx - mn) + dpc;
                const float ep = exp_nat(dp), ec = exp_nat(dc);
                l[qb] = ep * l[qb] + ec * lsum;
                F[qb] = Fn;
                m[qb] = mn;
                ep_[qb] = ep;
                ec_[qb] = ec;
            } else {
                // every operation rounded to fp16, in the order Algorithm 1 states them
                const _Float16 jm1 = (_Float16)(float)j, jj = (_Float16)(float)(j + 1);
                const _Float16 Fo = (_Float16)F[qb], sb = (_Float16)sbar, mo = (_Float16)m[qb], mxh = (_Float16)mx;
                const _Float16 iv = (_Float16)inva;
                const _Float16 Fn = (_Float16)((_Float16)((_Float16)(jm1 * Fo) + sb) / jj);
                const _Float16 dpp = (_Float16)(iv * (_Float16)(Fo - Fn));
                const _Float16 dpc = (_Float16)(iv * (_Float16)(sb - Fn));
                const _Float16 c1 = (_Float16)(mo + dpp), c2 = (_Float16)(mxh + dpc);
                const _Float16 mn = c1 > c2 ? c1 : c2;
                const _Float16 dp = (_Float16)((_Float16)(mo - mn) + dpp);
                const _Float16 dc = (_Float16)((_Float16)(mxh - mn) + dpc);
                const _Float16 ep = (_Float16)exp_nat((float)dp), ec = (_Float16)exp_nat((float)dc);
                const _Float16 lo = (_Float16)l[qb], ln = (_Float16)lsum;
                l[qb] = (float)(_Float16)((_Float16)(ep * lo) + (_Float16)(ec * ln));
                F[qb] = (float)Fn;
                m[qb] = (float)mn;
                ep_[qb] = (float)ep;
                ec_[qb] = (float)ec;
            }
        }

        // ---------------- second GEMM: (P V)^T tile (D channels x 64 queries) ----------------
        f16v Ot[2][CB];
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) Ot[qb][cb] = (f16v)0.f;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk)
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) {
                const h8 a = *reinterpret_cast<const h8*>(lds_v + ((2 * kk + lh) * D + 32 * cb + lq) * 8);
                Ot[0][cb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, Pf[0][kk], Ot[0][cb], 0, 0, 0);
                Ot[1][cb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, Pf[1][kk], Ot[1][cb], 0, 0, 0);
            }

        // ---------------- corrected output update (step 4) ----------------
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            if (!STRICT) {
                const float ec = ec_[qb], ep = ep_[qb];
                if (first) {
#pragma unroll
                    for (int cb = 0; cb < CB; ++cb) O[qb][cb] = Ot[qb][cb];
                } else {
#pragma unroll
                    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                        for (int i = 0; i < 16; ++i) O[qb][cb][i] = ec * Ot[qb][cb][i] + ep * O[qb][cb][i];
                }
            } else {
                const _Float16 ec = (_Float16)ec_[qb], ep = (_Float16)ep_[qb];
                const h2 ec2 = {ec, ec}, ep2 = {ep, ep};
#pragma unroll
                for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                    for (int t = 0; t < 8; ++t) {
                        const h2 ot = {(_Float16)Ot[qb][cb][2 * t], (_Float16)Ot[qb][cb][2 * t + 1]};
                        if (first) {
                            O16[qb][cb][t] = ot;
                        } else {
                            const h2 a1 = ec2 * ot;               // each packed op rounds to fp16 once
                            const h2 a2 = ep2 * O16[qb][cb][t];
                            O16[qb][cb][t] = a1 + a2;
                        }
                    }
            }
        }
    }

    // ---------------- final normalisation and store ----------------
    unsigned long long n_bad = 0;
    if (wave_valid) {
        _Float16* obase = o + ((size_t)(b * Hq + hq) * N) * D;
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            const int row = qw0 + 32 * qb + lq;
#pragma unroll
            for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    h4 out;
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int i = 4 * g + r;
                        _Float16 val;
                        if (!STRICT) {
                            val = (_Float16)(O[qb][cb][i] / l[qb]);
                        } else {
                            val = (_Float16)(O16[qb][cb][i >> 1][i & 1] / (_Float16)l[qb]);
                        }
                        if (INSTR) {
                            const float fv = (float)val;
                            n_bad += (fv != fv || __builtin_fabsf(fv) == __builtin_inff()) ? 1u : 0u;
                        }
                        out[r] = val;
                    }
                    *reinterpret_cast<h4*>(obase + (size_t)row * D + 32 * cb + 8 * g + 4 * lh) = out;
                }
        }
    }
    if (INSTR) {
        if (ovf_s != nullptr && n_ovf) atomicAdd(ovf_s, n_ovf);
        if (nonfinite_o != nullptr && n_bad) atomicAdd(nonfinite_o, n_bad);
    }
}

template <int D, int VAR, bool CAUSAL, bool INSTR>
hipError_t launch_fwd(const PasaLaunch& p)
{
    const int nqt = (p.N + ROWS_PER_WG - 1) / ROWS_PER_WG;
    const dim3 grid((unsigned)(nqt * p.Hq * p.B));
    hipLaunchKernelGGL((pasa_fwd<D, VAR, CAUSAL, INSTR>), grid, dim3(256), 0, p.stream,
                       (const _Float16*)p.q, (const _Float16*)p.kp, (const _Float16*)p.vt, (_Float16*)p.o,
                       p.Hq, p.Hkv, p.N, nqt, p.inva, p.scale, p.overflow_s, p.nonfinite_o);
    return hipGetLastError();
}

template <int D, int VAR>
hipError_t launch_fwd_cv(const PasaLaunch& p)
{
    const bool instr = p.overflow_s != nullptr || p.nonfinite_o != nullptr;
    if (p.causal) return instr ? launch_fwd<D, VAR, true, true>(p) : launch_fwd<D, VAR, true, false>(p);
    return instr ? launch_fwd<D, VAR, false, true>(p) : launch_fwd<D, VAR, false, false>(p);
}

template <int D>
hipError_t launch_fwd_d(const PasaLaunch& p)
{
    switch (p.variant) {
        case PASA_K_MIXED: return launch_fwd_cv<D, PASA_K_MIXED>(p);
        case PASA_K_STRICT16: return launch_fwd_cv<D, PASA_K_STRICT16>(p);
        case PASA_K_NAIVE16: return launch_fwd_cv<D, PASA_K_NAIVE16>(p);
        case PASA_K_S16: return launch_fwd_cv<D, PASA_K_S16>(p);
    }
    return hipErrorInvalidValue;
}

}  // namespace

hipError_t pasa_launch_prep(const void* k, const void* v, void* kp, void* vt, void* plain_out,
                            int B, int Hkv, int N, int d, double beta, double kscale, hipStream_t stream)
{
    const dim3 grid((unsigned)((size_t)B * Hkv * (N / T)));
    if (d == 128)
        hipLaunchKernelGGL(pasa_prep_kv<128>, grid, dim3(256), 0, stream, (const _Float16*)k, (const _Float16*)v,
                           (_Float16*)kp, (_Float16*)vt, (_Float16*)plain_out, beta, kscale);
    else
        hipLaunchKernelGGL(pasa_prep_kv<64>, grid, dim3(256), 0, stream, (const _Float16*)k, (const _Float16*)v,
                           (_Float16*)kp, (_Float16*)vt, (_Float16*)plain_out, beta, kscale);
    return hipGetLastError();
}

hipError_t pasa_launch_fwd(const PasaLaunch& p)
{
    return p.d == 128 ? launch_fwd_d<128>(p) : launch_fwd_d<64>(p);
}
