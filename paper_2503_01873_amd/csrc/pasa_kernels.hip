// PASA attention forward for gfx950: device kernels and their launchers.
//
// Two kernels per call.
//
//  pasa_prep_kv   Algorithm 1's pre-processing loop (Eq. (10), (11)) without forming the matrix M:
//                 per 128-key tile, the per-channel mean of K is taken exactly in fp64, K' = (K - beta*mean)*kscale
//                 is rounded once to fp16, and both K' and V are re-tiled so that the main kernel's LDS image of
//                 a tile is a straight copy whose MFMA fragments are single conflict-free 128-bit LDS reads.
//
//  pasa_fwd       Algorithm 1's main loops.  One workgroup = 8 wavefronts = 256 query rows; each wavefront owns
//                 32 query rows and sweeps the key tiles.  Both GEMMs are computed transposed on
//                 v_mfma_f32_32x32x16_f16:
//                     S'^T = K' Q^T      (A = K' fragment from LDS, B = Q fragment held in registers)
//                     O^T += V^T P^T     (A = V^T fragment from LDS, B = P^T taken straight from the S'^T accumulators)
//                 In the transposed accumulator layout a lane holds 64 keys of ONE query row, so the row
//                 statistics (pseudo-average Sbar', maximum m', sum l') are in-lane reductions plus one exchange
//                 with lane^32, and exp(S'-m') converted to fp16 is already the B operand of the second GEMM.
//
// Workspace: for every (batch, KV head, key tile) the K' tile followed by the V tile, so that one tile pair is
// one contiguous block that is copied to LDS verbatim with direct global->LDS loads, double buffered.
// For PASA_K_MIXED also, per (batch, KV head) and group of 16 key tiles, one "mean block": the per-channel mean over
// 128 key slots of the rounded K' of each of the 16 tiles, split into an fp16 high and an fp16 low part (times 2^11), laid out
// as a 32-row A operand (see pasa_prep_kv) -- by Eq. (12), (14) the pseudo-average of a score row is the query
// times that mean, which the main kernel takes for 16 tiles at a time on the matrix core.
// Tile layouts (one tile = 128 keys x D channels, fp16, 16-byte chunks):
//   K' tile: chunk index (c/8)*128 + n         holds channels 8*(c/8) .. +7 of key n
//   V  tile: chunk index ((n/16)*2 + h)*D + c  holds, for channel c, the 8 keys 16*(n/16) + {4h..4h+3, 8+4h..8+4h+3}
// The second layout is the key order in which a lane of the 32x32 accumulator holds its S'^T rows.
//
// The matrix cores accumulate in fp32 in every variant; "fp16" quantities are rounded (nearest-even) where
// Algorithm 1 marks them.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <atomic>
#include <type_traits>

#include "pasa_kernels.h"

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef _Float16 h4 __attribute__((ext_vector_type(4)));
typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef unsigned short u16x8 __attribute__((ext_vector_type(8)));
typedef unsigned short u16x4 __attribute__((ext_vector_type(4)));

// bf16 inputs are converted to fp16 as they are loaded (the paper's remark on BF16 inputs): round to nearest even,
// values beyond the fp16 range become infinities.
__device__ inline h8 bf16x8_to_h8(u16x8 raw)
{
    h8 out;
#pragma unroll
    for (int e = 0; e < 8; ++e) out[e] = (_Float16)__uint_as_float((unsigned)raw[e] << 16);
    return out;
}

__device__ inline h8 load_h8(const _Float16* p, int is_bf16)
{
    if (is_bf16) return bf16x8_to_h8(*reinterpret_cast<const u16x8*>(p));
    return *reinterpret_cast<const h8*>(p);
}

// fp32 -> bf16 bits, round to nearest even; NaN stays NaN
__device__ inline unsigned short f32_to_bf16_rn(float f)
{
    const unsigned u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (unsigned short)((u >> 16) | 0x40u);
    return (unsigned short)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}
typedef float f16v __attribute__((ext_vector_type(16)));
typedef float f2 __attribute__((ext_vector_type(2)));

namespace {

constexpr int T = 128;          // keys per shift tile (s2 of the paper)
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
// Pre-processing kernel.  grid = (B*Hkv*ceil(N/128) tiles, work groups of a tile), 256 threads.
// plain_out != nullptr: write K' in the plain [.., N, D] layout instead (pasa_shift_keys).
// A ragged last tile is padded with zero keys and zero values in the workspace.
#ifndef PASA_PREP_SPLIT
#define PASA_PREP_SPLIT 4
#endif

// One channel c of the two rows that key tile t owns in its "mean block" (a 32-row x D A operand per 16 tiles, in the
// K' tile's chunk order: chunk (c/8)*32 + row holds channels 8*(c/8)..+7 of row `row`).  Tile t of the group has its
// "high" row at 8*(t/4) + t%4 and its "low" row four rows further down: in the 32x32 accumulator layout the first kind
// of row lands in lanes 0-31 and the second in lanes 32-63 of the same accumulator register.  The last tile of a head
// also clears the rows of the tiles that do not exist.
__device__ inline void write_block_rows(_Float16* blocks, size_t head, int ntile, int t, int c, int D, _Float16 hi, _Float16 lo)
{
    const int nblk = (ntile + 15) / 16;
    const int t16 = t & 15, row = 8 * (t16 >> 2) + (t16 & 3);
    _Float16* blk = blocks + ((head * (size_t)nblk + (size_t)(t >> 4)) * 32) * D;
    blk[((size_t)(c / 8) * 32 + row) * 8 + (c % 8)] = hi;
    blk[((size_t)(c / 8) * 32 + row + 4) * 8 + (c % 8)] = lo;
    if (t == ntile - 1)
        for (int u = t16 + 1; u < 16; ++u) {
            const int ru = 8 * (u >> 2) + (u & 3);
            blk[((size_t)(c / 8) * 32 + ru) * 8 + (c % 8)] = (_Float16)0;
            blk[((size_t)(c / 8) * 32 + ru + 4) * 8 + (c % 8)] = (_Float16)0;
        }
}
// ---------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void pasa_prep_kv(const _Float16* __restrict__ k, const _Float16* __restrict__ v,
                                                    _Float16* __restrict__ wsout,
                                                    _Float16* __restrict__ plain_out, _Float16* __restrict__ k0out,
                                                    _Float16* __restrict__ kmean_out,
                                                    int N, int ntile, double beta, double kscale, int shift_mode,
                                                    int in_bf16, const unsigned long long* gate, int y_off)
{
    // adaptive start: nothing overflowed in this (batch, KV head), its shifted pass is not needed
    if (gate != nullptr && gate[blockIdx.x / ntile] == 0) return;

    // A tile's work is cut into 2*NS blocks (blockIdx.y): NS groups of D/NS channels of K (column means are per
    // channel, so the groups are independent) and NS groups of 128/NS keys of V.  The pass is bound by memory
    // latency and by fp64 arithmetic per thread, not by bandwidth, so it wants many small blocks.
    constexpr int NS = PASA_PREP_SPLIT;
    constexpr int DB = D / NS;           // channels of K per block
    constexpr int CH = DB / 8;           // 16-byte chunks per key within the group
    constexpr int KL = 256 / CH;         // key lanes
    constexpr int KPT = T / KL;          // keys per thread
    constexpr int PARTS = 256 / DB;      // second reduction stage: row groups per channel
    constexpr int TB = T / NS;           // keys of V per block
    constexpr size_t PSUM_BYTES = sizeof(double) * (KL + PARTS + 1) * DB, VS_BYTES = sizeof(_Float16) * TB * (D + 8);
    __shared__ __attribute__((aligned(16))) char lds_raw[PSUM_BYTES > VS_BYTES ? PSUM_BYTES : VS_BYTES];

    const size_t tile = blockIdx.x;                      // (batch, KV head, key tile)
    const size_t head = tile / ntile;
    const int t = (int)(tile % ntile);
    const int nvalid = (N - t * T) < T ? (N - t * T) : T;    // keys of this tile (< 128 only in a ragged last tile)
    const size_t src_off = (head * (size_t)N + (size_t)t * T) * D;
    const int tid = threadIdx.x;

    const int by = blockIdx.y + y_off;     // y_off = NS: only the value blocks are launched
    if (by >= NS) {
        // ---- values: keys [n0, n0 + TB) of the tile, all channels ----
        _Float16 (*vs)[D + 8] = reinterpret_cast<_Float16 (*)[D + 8]>(lds_raw);   // +8 halfs: rows 16 bytes apart in bank space
        const int n0 = (by - NS) * TB;
        const _Float16* vsrc = v + src_off;
        constexpr int VCH = D / 8;
        for (int idx = tid; idx < TB * VCH; idx += 256) {
            const int nl = idx / VCH, c8 = idx % VCH, n = n0 + nl;
            *reinterpret_cast<h8*>(&vs[nl][8 * c8]) =
                n < nvalid ? load_h8(vsrc + (size_t)n * D + 8 * c8, in_bf16) : (h8)(_Float16)0;
        }
        __syncthreads();
        _Float16* vdst = wsout + tile * (size_t)(2 * T * D) + T * D;
        const int chunk0 = (n0 / 16) * 2 * D;            // chunk ((n/16)*2 + h)*D + c; this block owns TB/16*2 values of (n/16)*2+h
        for (int chunk = tid; chunk < (TB / 16) * 2 * D; chunk += 256) {
            const int c = chunk % D;
            const int kh = chunk / D;
            const int nb = (kh >> 1) * 16 + (kh & 1) * 4;    // local key of the first of the 8
            h8 out;
#pragma unroll
            for (int e = 0; e < 8; ++e) out[e] = vs[nb + (e >> 2) * 8 + (e & 3)][c];
            *reinterpret_cast<h8*>(vdst + (size_t)(chunk0 + chunk) * 8) = out;
        }
        return;
    }

    // ---- keys: channels [cg*DB, cg*DB + DB) of the tile, all 128 keys ----
    double (*psum)[DB] = reinterpret_cast<double (*)[DB]>(lds_raw);              // [KL] partial column sums
    double (*psum2)[DB] = psum + KL;                                             // [PARTS] second stage
    double* colv = reinterpret_cast<double*>(psum2 + PARTS);                     // [DB] mean (or sum, or k0) per channel
    const int cg = by;
    const int c8 = tid % CH, kl = tid / CH;
    const int ch0 = cg * DB + 8 * c8;                    // first of this thread's 8 channels
    const _Float16* ksrc = k + src_off;

    h8 kv[KPT];
    double s[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int i = 0; i < KPT; ++i) {
        const int n = kl + KL * i;
        kv[i] = n < nvalid ? load_h8(ksrc + (size_t)n * D + ch0, in_bf16) : (h8)(_Float16)0;
#pragma unroll
        for (int e = 0; e < 8; ++e) s[e] += (double)kv[i][e];   // exact: fp16 values, at most 128 terms
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) psum[kl][8 * c8 + e] = s[e];
    __syncthreads();
    {   // every partial sum is exact in fp64, so the order of the two stages does not matter
        const int c = tid % DB, part = tid / DB;
        double acc = 0;
        for (int r = part; r < KL; r += PARTS) acc += psum[r][c];
        psum2[part][c] = acc;
    }
    __syncthreads();
    if (tid < DB) {
        double tot = 0;
#pragma unroll
        for (int r = 0; r < PARTS; ++r) tot += psum2[r][tid];
        // the tile's own key count, so that Eq. (14) holds for a ragged tile too; the matrix form needs the plain sum
        double val = shift_mode == PASA_PREP_MATRIX ? tot : tot / (double)nvalid;
        // direct-bias recovery: the shift vector k0 = fp16(beta * mean) is itself an fp16 vector
        if (shift_mode == PASA_PREP_DIRECT) {
            const _Float16 k0h = double_to_half_rn(__dmul_rn(beta, val));
            val = (double)k0h;
            k0out[tile * (size_t)D + cg * DB + tid] = k0h;
            // the main kernel reads the vector from the tile's "high" row of a mean block (below); the "low" row is zero
            if (kmean_out != nullptr) write_block_rows(kmean_out, head, ntile, t, cg * DB + tid, D, k0h, (_Float16)0);
        }
        colv[tid] = val;
    }
    __syncthreads();
    double mean[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) mean[e] = colv[8 * c8 + e];
    double rs[8] = {0, 0, 0, 0, 0, 0, 0, 0};     // column sums of the ROUNDED K' over this thread's keys (exact in fp64)
#pragma unroll
    for (int i = 0; i < KPT; ++i) {
        const int n = kl + KL * i;
        h8 out;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            double r;
            if (shift_mode == PASA_PREP_DIRECT) {
                r = __dmul_rn(__dsub_rn((double)kv[i][e], mean[e]), kscale);     // (K - k0) is exact in fp64
            } else if (shift_mode == PASA_PREP_MATRIX) {
                // K'^T = K^T M with M = a I + b (J - I) entrywise rounded to fp16 (Eq. (10), (11) as a GEMM):
                // sum_p M[p,q] K[p,c] = (a - b) K[q,c] + b sum_p K[p,c].  Here beta carries (a - b) and kscale
                // carries b; both products are exact in fp64 and the sum rounds once.
                r = __dadd_rn(__dmul_rn(beta, (double)kv[i][e]), __dmul_rn(kscale, mean[e]));
            } else {
                // three separately rounded fp64 operations (no contraction): beta*mean, K - that, * kscale
                const double bm = __dmul_rn(beta, mean[e]);
                const double df = __dsub_rn((double)kv[i][e], bm);
                r = __dmul_rn(df, kscale);
            }
            out[e] = n < nvalid ? double_to_half_rn(r) : (_Float16)0;   // padding keys: exact zeros
            rs[e] += (double)out[e];
        }
        if (plain_out != nullptr) {
            if (n < nvalid) *reinterpret_cast<h8*>(plain_out + src_off + (size_t)n * D + ch0) = out;
        } else {
            *reinterpret_cast<h8*>(wsout + tile * (size_t)(2 * T * D) + ((size_t)(ch0 / 8) * T + n) * 8) = out;
        }
    }
    if (kmean_out == nullptr || shift_mode == PASA_PREP_DIRECT) return;

    // ---- mean block: column sum of the rounded K' / 128 (an exact scaling), as an fp16 pair hi + lo ----
    __syncthreads();                       // psum is reused
#pragma unroll
    for (int e = 0; e < 8; ++e) psum[kl][8 * c8 + e] = rs[e];
    __syncthreads();
    {
        const int c = tid % DB, part = tid / DB;
        double acc = 0;
        for (int r = part; r < KL; r += PARTS) acc += psum[r][c];
        psum2[part][c] = acc;
    }
    __syncthreads();
    if (tid < DB) {
        double tot = 0;
#pragma unroll
        for (int r = 0; r < PARTS; ++r) tot += psum2[r][tid];
        const double m128 = tot * 0.0078125;                 // 2^-7: exact
        // the low part is stored times 2^11 (undone when the two products are added): unscaled it is an fp16
        // subnormal for every mean below 0.125, and the matrix core reads those as zero
        const _Float16 hi = double_to_half_rn(m128);
        const _Float16 lo = double_to_half_rn((m128 - (double)hi) * 2048.0);
        write_block_rows(kmean_out, head, ntile, t, cg * DB + tid, D, hi, lo);
    }
}

// ---------------------------------------------------------------------------------------------
// Main kernel
// ---------------------------------------------------------------------------------------------
// Value of x in the lane 32 away (lane l <-> lane l^32), without going through the LDS crossbar: the LDS pipe is
// saturated by the other wave group's fragment reads while this is needed.  v_permlane32_swap exchanges lanes 32-63
// of its first operand with lanes 0-31 of its second; with two copies of x that leaves [x_lo, x_lo] and [x_hi, x_hi].
// The s_nop cover the VALU-write -> permlane-read and permlane-write -> VALU-read wait states, which the compiler
// cannot see through inline assembly.
__device__ inline void halves32(float x, float& lo, float& hi)
{
    lo = x;
    hi = x;
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(lo), "+v"(hi));
}
// lanes 32-63 of a <-> lanes 0-31 of b.  Through the builtin, so that the compiler sees the reads: the operands here
// come straight from an MFMA, whose result registers must not be read before the instruction has written them all.
__device__ inline void swap32(float& a, float& b)
{
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(a), __float_as_uint(b), false, false);
    a = __uint_as_float(r[0]);
    b = __uint_as_float(r[1]);
}
__device__ inline float sum32(float x)
{
    float lo, hi;
    halves32(x, lo, hi);
    return lo + hi;
}
__device__ inline float max32(float x)
{
    float lo, hi;
    halves32(x, lo, hi);
    return __builtin_fmaxf(lo, hi);
}

__device__ inline float exp_nat(float x) { return __builtin_amdgcn_exp2f(x * LOG2E); }

__device__ inline h2 pack_rn(float a, float b)
{
    const f2 v = {a, b};
    return __builtin_convertvector(v, h2);     // v_cvt_pk_f16_f32: nearest-even
}

// a + b + acc with the two halves widened exactly (v_dot2_f32_f16 against ones)
__device__ inline float add_pair(h2 v, float acc)
{
    const h2 one = {(_Float16)1, (_Float16)1};
    return __builtin_amdgcn_fdot2(v, one, acc, false);
}

// (acc + a) + b, the same sum with two v_fma_mix_f32 (half * 1.0 + acc, the half read straight from its packed
// register).  v_dot2_f32_f16 takes its turn in the matrix pipeline: beside a wave that issues MFMAs back to back it
// holds its own wave for 24 cycles (a v_fma_mix_f32: 7) while costing the shared issue port little.  Where the vector
// part is short enough for that wait to show (STRICT16; MIXED since its pseudo-average moved to the matrix core) two of
// these are faster than one of those; in the other variants they are slower.  (The compiler folds fma(x, 1, acc) to
// an add with two separate conversions, hence the asm.)
__device__ inline float add_pair_mix(h2 v, float acc)
{
    asm("v_fma_mix_f32 %0, %1, 1.0, %0 op_sel_hi:[1,0,0]" : "+v"(acc) : "v"(v));
    asm("v_fma_mix_f32 %0, %1, 1.0, %0 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "+v"(acc) : "v"(v));
    return acc;
}

// exp of one half of a packed pair: (float)half * log2(e) in one v_fma_mix_f32 (the product rounded once, as a
// conversion followed by a multiplication would), then v_exp_f32
template <int HI>
__device__ inline float exp_nat_half(h2 v)
{
    float x;
    const float k = LOG2E;
    if (HI) asm("v_fma_mix_f32 %0, %1, %2, 0 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(x) : "v"(v), "v"(k));
    else asm("v_fma_mix_f32 %0, %1, %2, 0 op_sel_hi:[1,0,0]" : "=v"(x) : "v"(v), "v"(k));
    return __builtin_amdgcn_exp2f(x);
}

// One wave-wide direct global -> LDS copy of 1 KiB: lane i moves 16 bytes from byte soff + 16*i of the buffer to
// ldst + 16*i.  soff and ldst must be wave-uniform (ldst travels in M0).
// OFF is an immediate added to both addresses, so a wave's consecutive pieces share one M0 value.
// The buffer form (buffer_load ... lds) is used rather than global_load_lds: the compiler treats the latter as a flat
// access that may touch LDS and from then on drains the LDS counter to zero before every use of an LDS fragment,
// which defeats the fragment prefetch of the GEMM loops.  A buffer load out of range returns zeros instead of faulting.
template <int OFF>
__device__ inline void copy_1k_to_lds(__amdgpu_buffer_rsrc_t src, int soff, char* ldst, int lane)
{
    __builtin_amdgcn_raw_ptr_buffer_load_lds(src, (__attribute__((address_space(3))) void*)ldst, 16, lane * 16, soff, OFF, 0);
}

#define PASA_FENCE() __builtin_amdgcn_sched_barrier(0)

// A workgroup is 8 wavefronts and owns 256 query rows, 32 per wavefront.  Wavefronts 0-3 (group A) and 4-7
// (group B) sit pairwise on the four SIMDs and run the same program half a tile apart: time is cut into slots
// separated by workgroup barriers, and in every slot one group is in its matrix part while the other is in its
// vector part, so the MFMA pipe and the VALU of a SIMD are busy at the same time.
//
//   group A:  M(0) V(0) M(1) V(1) ...        group B:  -  M(0) V(0) M(1) ...
//   M(j) = [ O^T += V(j-1)^T P(j-1)^T ,  S'^T = K'(j) Q^T ]
//   V(j) = [ row statistics, global recovering scalars, exponentials -> P(j), row sum ]
//
// LDS holds two K' tiles and two V tiles; tile copies are direct global->LDS loads issued at the start of the vector
// parts, one to two slots before the first matrix part that reads them.
//
// Output accumulation.  STRICT16 keeps Algorithm 1's form: the tile product is rounded to fp16 and combined as
// O = fp16(e^{dm_j} * PV) + fp16(e^{dm_{j-1}} * O).  The fp32 variants accumulate the second GEMM directly onto the
// running output, which is stored at a scale of its own: O_j = e^{Lc_j} * Ostore_j.  The stored output is left alone
// and the tile's P takes the factor instead: with dp = dm_{j-1} and dc = dm_j of Algorithm 1's step 3,
// Lc_j = Lc_{j-1} + dp and P_j = fp16(exp(S' - m'_j + c_j)), c_j = dc - Lc_j, so Ostore_j = Ostore_{j-1} + P_j V_j and
// the running sum l is kept at the same scale (l += rowsum(P_j); the final quotient needs no factor).  c_j is the
// tile's level relative to the stored scale, which is the level of an earlier tile: c_j <= 0 unless the running
// maximum rises.  Only when c_j > 8 is a row's stored output and sum multiplied by e^{-c_j} (then Lc_j = dc, c_j = 0),
// a branch taken on a few tiles at the start of a row at most; so P <= e^8, far inside fp16, and a tile far below the
// running maximum underflows to zero by itself.  Against a rescale of the stored output on every tile this removes 64
// multiplications per tile and lane and three exponentials from the recovering scalars (3.7 % of the kernel time);
// the price is that P is Algorithm 1's exp(S' - m') times e^{c_j} rounded once, not exp(S' - m') rounded and then
// scaled, so outputs agree with a step-by-step evaluation to rounding, not bit for bit.  DIRECT (levels m' + c) and
// NAIVE16 (plain online softmax: P relative to the running maximum, dc = 0) use the same bookkeeping.
template <int D, int VAR, bool CAUSAL, bool INSTR>
__global__ __launch_bounds__(512, 2)
void pasa_fwd(const _Float16* __restrict__ q, const char* __restrict__ ws, _Float16* __restrict__ o,
              const _Float16* __restrict__ kmean, int Hq, int Hkv, int Nq, int row0, int N,
              int nqt, float inva, float scale,
              int io_bf16,
              unsigned long long* ovf_s, unsigned long long* nonfinite_o, unsigned long long* ovf_group,
              const unsigned long long* gate, int nsplit, float* __restrict__ part_o, double* __restrict__ part_lr)
{

    constexpr int KS = D / 16;   // k-steps of S'^T = K' Q^T
    constexpr int CB = D / 32;   // 32-channel row blocks of O^T
    constexpr bool S16 = (VAR != PASA_K_MIXED && VAR != PASA_K_DIRECT);   // S' rounded to fp16 as it leaves the matrix core
    constexpr bool STRICT = (VAR == PASA_K_STRICT16);
    constexpr bool NAIVE = (VAR == PASA_K_NAIVE16);
    constexpr bool DIRECT = (VAR == PASA_K_DIRECT);               // bias added back as scale * (q . k0), no pseudo-average
    // MIXED takes the pseudo-average as q . colmean(K') (Eq. (12), (14)) on the matrix core, 16 tiles at a time,
    // instead of summing 128 scores per row and tile on the vector unit
    // DIRECT takes q . k0 of the tiles the same way (their "mean block" holds the shift vectors, low rows zero)
    constexpr bool MSBAR = (VAR == PASA_K_MIXED || VAR == PASA_K_DIRECT);
    constexpr int KM_BYTES = 64 * D;                            // one mean block: 32 rows x D halfs
    constexpr int SB_OFF = 4 * (T * D * 2) + KM_BYTES;          // per-wave [16 tiles][32 rows] floats behind it
    constexpr int KT_BYTES = T * D * 2;                         // one K' (or V) tile
    constexpr int TILE_BYTES = 2 * KT_BYTES;                    // workspace stride: K' tile then V tile
    constexpr int CPW = KT_BYTES / 1024 / 8;                    // 1 KiB copies per wave per K' (or V) tile
    constexpr int RW = 32, RWG = 256;

    extern __shared__ __attribute__((aligned(1024))) char smem[];   // K'[2] then V[2]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int grp = wave >> 2;
    const int lq = lane & 31, lh = lane >> 5;

    // Work decode.  Workgroups are dispatched in index order and dealt round-robin to the 8 XCDs (index % 8), each
    // with its own L2.  Two goals: (1) every XCD walks its share longest-first -- the query tiles with the most key
    // tiles (the last ones when causal) first -- which keeps the tail of the launch short; (2) the query heads that
    // share one KV head run on the same XCD(s), so that K'/V tiles are fetched into as few L2s as possible.
    // A "group" is the set of Hq/Hkv query heads of one (batch, KV head).
    // Key split (nsplit > 1, for launches with too few workgroups to fill the chip): nsplit workgroups share one
    // (query tile, head); each sweeps a contiguous range of key tiles and leaves its per-row state (stored output, sum,
    // level) in part_o / part_lr for pasa_merge_splits.
    // How the workgroups of a launch reach the compute units was measured with a probe kernel (workgroups of this
    // kernel's LDS size that record their XCC, shader engine and compute unit and spin for a given time): within an XCD
    // they go to its four shader engines in strict rotation, in index order, and each waits for a compute unit of ITS
    // engine (8 per engine); a simulation of exactly that reproduces the probe's end times to 0.4 %.  With the items
    // simply longest first the engine that always gets the first of four carries 5 % more than the one that gets the
    // last (896 causal items of 2 .. 64 tile-steps end 4.5 % behind the mean).  So every other group of four
    // consecutive places of an XCD's list is taken backwards: the engines' loads even out and items that are
    // neighbours in the list stay neighbours in time, which keeps the query heads of a KV head on the same key tiles
    // at the same time (numberings that balance better but scatter the list ran slower: they lose that L2 reuse).
    const int split = blockIdx.x % nsplit;
    int wg = blockIdx.x / nsplit;
    {
        const int nwg = gridDim.x / nsplit, x = wg & 7, r = wg >> 3;
        const int in_xcd = (nwg - x + 7) >> 3;             // workgroups of this XCD
        if ((r & 4) && (r | 3) < in_xcd) wg = ((r ^ 3) << 3) | x;
    }
    const int G = Hq / Hkv;                 // query heads per group
    const int ngroups = (gridDim.x / nsplit) / (nqt * G);
    int qt, grp_id, hin;                    // query tile, group, head within group
    if (ngroups % 8 == 0) {                 // each XCD owns ngroups/8 whole groups
        const int x = wg & 7, r = wg >> 3, per = (ngroups >> 3) * G;
        qt = nqt - 1 - r / per;
        grp_id = x + 8 * ((r % per) / G);
        hin = (r % per) % G;
    } else if (8 % ngroups == 0 && (nqt * G) % (8 / ngroups) == 0) {   // each group is spread over 8/ngroups XCDs
        const int span = 8 / ngroups, x = wg & 7, r = wg >> 3;
        const int i = r * span + (x % span);
        grp_id = x / span;
        qt = nqt - 1 - i / G;
        hin = i % G;
    } else {                                // plain longest-first order
        const int nbh = ngroups * G;
        qt = nqt - 1 - wg / nbh;
        grp_id = (wg % nbh) / G;
        hin = (wg % nbh) % G;
    }
    // adaptive start: nothing overflowed in this (batch, KV head), its shifted pass is not needed (whole workgroup leaves)
    if (gate != nullptr && gate[grp_id] == 0) return;
    const int b = grp_id / Hkv, hk_ = grp_id % Hkv;
    const int hq = hk_ * G + hin;
    const int hk = hk_;
    const int ntile = (N + T - 1) / T;
    const int tail_keys = N % T;           // keys of a ragged last tile (0: none)
    const float inv_tail = 1.0f / (float)(tail_keys ? tail_keys : T);

    // Query row r of the Nq rows given sits at sequence position row0 + r (causal: it sees keys <= its position).
    const int q0 = qt * RWG;
    const int qw0 = q0 + wave * RW;
    const bool wave_valid = qw0 < Nq;      // the wave owns at least one real row
    int last_row_wg = q0 + RWG - 1;
    if (last_row_wg > Nq - 1) last_row_wg = Nq - 1;
    int last_row_w = qw0 + RW - 1;
    if (last_row_w > Nq - 1) last_row_w = Nq - 1;
    auto tiles_seen = [&](int r) {         // key tiles a causal row at position row0 + r reaches
        const int t = (row0 + r) / T + 1;
        return t < ntile ? t : ntile;
    };
    // this workgroup's key tiles [j0, J_wg): all of the tiles its rows see, or -- split -- one range of them, cut at
    // multiples of 16 tiles so that a range starts with a mean block of its own
    const int J_all = CAUSAL ? tiles_seen(last_row_wg) : ntile;
    const int per16 = (((J_all + 15) >> 4) + nsplit - 1) / nsplit;
    const bool splitting = !STRICT && nsplit > 1;      // STRICT16 is never launched split: its fp16 state has no merge rule
    const int j0 = splitting ? (split * per16 * 16 < J_all ? split * per16 * 16 : J_all) : 0;
    const int J_wg = splitting ? (j0 + per16 * 16 < J_all ? j0 + per16 * 16 : J_all) : J_all;
    int J_w = wave_valid ? (CAUSAL ? tiles_seen(last_row_w) : ntile) : 0;
    if (J_w > J_wg) J_w = J_wg;
    const int row = qw0 + lq;
    const bool row_valid = row < Nq;       // rows past the end compute on zero queries and are never stored
    const int pos_w0 = row0 + qw0;         // position of the wave's first row

    const _Float16* qbase = q + ((size_t)(b * Hq + hq) * Nq) * D;
    const char* wsbase = ws + ((size_t)(b * Hkv + hk) * ntile) * TILE_BYTES;
    // raw buffer over this (batch, KV head)'s tiles: at most 2048 tiles of 64 KiB, so every offset fits 32 bits
    const __amdgpu_buffer_rsrc_t wsbuf =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(wsbase), 0, ntile * TILE_BYTES, 0x00020000);

    // mean blocks of this (batch, KV head): block g serves tiles 16g .. 16g+15; one 1 KiB piece per wave (D = 64: waves 0-3)
    const int nblk16 = (ntile + 15) >> 4;
    const __amdgpu_buffer_rsrc_t kmbuf = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<_Float16*>(MSBAR ? kmean + ((size_t)(b * Hkv + hk) * nblk16) * (32 * D) : q), 0, MSBAR ? nblk16 * KM_BYTES : 0,
        0x00020000);
    auto issue_kmean = [&](int g) {
        if (MSBAR && wave * 1024 < KM_BYTES && g < nblk16)
            copy_1k_to_lds<0>(kmbuf, g * KM_BYTES + wave * 1024, smem + 4 * KT_BYTES + wave * 1024, lane);
    };
    auto issue_k = [&](int j) {
        const int src = j * TILE_BYTES;
        char* dst = smem + (j & 1) * KT_BYTES;
#pragma unroll
        for (int i = 0; i < CPW; ++i) copy_1k_to_lds<0>(wsbuf, src + (wave * CPW + i) * 1024, dst + (wave * CPW + i) * 1024, lane);
    };
    issue_k(j0);
    issue_kmean(j0 >> 4);

    // Q fragments: B operand, lane (query lq, half lh) holds channels 16*ks + 8*lh .. +7
    h8 Qf[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
        Qf[ks] = row_valid ? load_h8(qbase + (size_t)row * D + 16 * ks + 8 * lh, io_bf16) : (h8)(_Float16)0;

    // per-row state (one query row per lane; both halves of the wave hold copies)
    float F = 0.f, m = NAIVE ? -__builtin_inff() : 0.f, l = 0.f;   // STRICT: always fp16-representable values
    float Lc = 0.f;                  // log of the scale of the stored output (fp32 variants)
    float ec_s = 1.f, ep_s = 0.f;    // STRICT: factors of the pending output combination
    f16v S[4];                       // S'^T accumulators
    h8 Pf[8];                        // P^T, B operand of the second GEMM
    f16v O[CB];                      // fp32 variants: stored output; STRICT: product of the latest tile
    h2 O16[CB][8];                   // STRICT: running output
    unsigned long long n_ovf = 0;
#pragma unroll
    for (int kb = 0; kb < 4; ++kb) S[kb] = (f16v)0.f;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) Pf[kk] = (h8)(_Float16)0;
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) {
        O[cb] = (f16v)0.f;
#pragma unroll
        for (int t = 0; t < 8; ++t) O16[cb][t] = (h2)(_Float16)0;
    }

    // STRICT: fold the product of tile jt (in O) into the running fp16 output
    auto fold16 = [&](int jt) {
        const _Float16 ec = (_Float16)ec_s, ep = (_Float16)ep_s;
        const h2 ec2 = {ec, ec}, ep2 = {ep, ep};
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const h2 ot = pack_rn(O[cb][2 * t], O[cb][2 * t + 1]);
                const h2 a1 = ec2 * ot;                   // each packed op rounds to fp16 once; first tile: 1 * ot + 0 * 0
                const h2 a2 = ep2 * O16[cb][t];
                O16[cb][t] = a1 + a2;
            }
    };

    // The copies of the even global slot sg are K'(sg/2 + 1) and V(sg/2); each wave owns 2*CPW of their 1 KiB pieces.
    // A wave issues its eight pieces back to back at the start of its vector part (one wave-wide copy each, sharing M0
    // through immediate offsets).
    auto issue_piece = [&](int sg, auto piece_c) {
        constexpr int piece = decltype(piece_c)::value;       // 0 .. 2*CPW-1: K' pieces first, then V pieces
        const int jl = sg >> 1;
        if (piece < CPW) {
            if (jl + 1 < J_wg)
                copy_1k_to_lds<(piece % CPW) * 1024>(wsbuf, (jl + 1) * TILE_BYTES + wave * (CPW * 1024),
                                                     smem + ((jl + 1) & 1) * KT_BYTES + wave * (CPW * 1024), lane);
        } else {
            if (jl < J_wg)
                copy_1k_to_lds<(piece % CPW) * 1024>(wsbuf, jl * TILE_BYTES + KT_BYTES + wave * (CPW * 1024),
                                                     smem + 2 * KT_BYTES + (jl & 1) * KT_BYTES + wave * (CPW * 1024), lane);
        }
    };
    // idx is a constant after unrolling; the switch turns it back into a template argument (an instruction immediate)
    auto issue_copy = [&](int sg, int idx) {
        switch (idx) {
            case 0: issue_piece(sg, std::integral_constant<int, 0>{}); break;
            case 1: issue_piece(sg, std::integral_constant<int, 1>{}); break;
            case 2: issue_piece(sg, std::integral_constant<int, 2 % (2 * CPW)>{}); break;
            case 3: issue_piece(sg, std::integral_constant<int, 3 % (2 * CPW)>{}); break;
            case 4: issue_piece(sg, std::integral_constant<int, 4 % (2 * CPW)>{}); break;
            case 5: issue_piece(sg, std::integral_constant<int, 5 % (2 * CPW)>{}); break;
            case 6: issue_piece(sg, std::integral_constant<int, 6 % (2 * CPW)>{}); break;
            case 7: issue_piece(sg, std::integral_constant<int, 7 % (2 * CPW)>{}); break;
            default: break;
        }
    };
    auto issue_slot = [&](int sg) {
#pragma unroll
        for (int idx = 0; idx < 2 * CPW; ++idx) issue_copy(sg, idx);
    };
    auto drain_copies = [&]() { __builtin_amdgcn_s_waitcnt(0x0F70); };   // vmcnt(0)

    // Barrier b ends slot b-1 and starts slot b.  Group A runs M(j) in slot 2j and V(j) in slot 2j+1; group B runs
    // M(j) in slot 2j+1 and V(j) in slot 2j+2.  Every wave issues its share of the copies K'(j+1), V(j) from its
    // vector part V(j) for group A (slot 2j+1) and V(j-1) for group B (slot 2j) -- the matrix part keeps its MFMA
    // chain free of them -- and drains them before the barrier that starts slot 2j+2, when group A reads them.
    drain_copies();
    __syncthreads();                       // barrier 0: K'(0) is in LDS
    if (grp == 1) {
        issue_slot(2 * j0);
        __syncthreads();                   // barrier 1: group B idles through slot 0
    }

    // Hand-offs between the parts of one wave.
    constexpr bool LAZY = !STRICT;   // fp32 variants: the recovering factor goes to P, not to the stored output
    // The running sum l of the fp32 variants is not taken in the vector part that makes P.
    // d = 128: the row sums of a tile's P are added up in the matrix part that follows, between the MFMAs of the second
    // GEMM (which reads the same P fragments): the wave has issue slots to spare there (an MFMA occupies the matrix core
    // for 32 cycles), while in the vector part every instruction counts.  0.7 % on the headline workload, although the
    // vector part loses 64 of its 330 instructions: the kernel's clock, not its cycle count, is the limit.  (MIXED and
    // DIRECT; S16 and NAIVE16, whose vector part sums with v_dot2_f32_f16, lose 1.2 % by it and keep their sums there.)
    // d = 64: the vector part is 2.7 times as long as the matrix part (the softmax is the same work, the GEMMs half),
    // and the sum moves onto the idle matrix core itself: one more MFMA per k-step of the second GEMM, P^T against a
    // block of ones, accumulates the row sums beside the stored output, at the same scale (every row of the result is
    // the sum).  4 % on the d = 64 workload (the first way is 2 % slower there; this way is 2.4 % slower at d = 128).
    constexpr bool LSUM_MFMA = LAZY && D == 64;
    constexpr bool LSUM_DEFER = LAZY && D == 128 && MSBAR;
    f16v Lacc = (f16v)0.f;
    const h8 ones = (h8)(_Float16)1;
    float pl_d[4] = {0.f, 0.f, 0.f, 0.f};
    constexpr float CMAX = 8.f;      // LAZY: P may exceed 1 by at most e^CMAX before the row re-references its scale
    float cj = 0.f;                  // DIRECT: scale * (q . k0) of the tile in the vector part

    // Both GEMMs run k-step by k-step: the four MFMAs of a k-step share their B operand (the Q or P fragment) and go
    // to the four accumulator blocks in turn, so consecutive MFMAs never depend on each other and the B registers are
    // read four times in a row (measured 1.4 % faster than one dependent chain per accumulator block, with the
    // maxima of finished blocks taken behind the MFMAs of the next).  LDS fragments are fetched PF instructions ahead.
#ifndef PASA_PF
#define PASA_PF 3
#endif
    constexpr int PF = PASA_PF;
    constexpr int NM1 = 4 * KS;      // MFMAs of the first GEMM:  n = kb * KS + ks
    constexpr int NM2 = CB * 8;      // MFMAs of the second GEMM
    auto gemm1 = [&](int jt) {   // S'^T of tile jt: 128 keys x 32 queries; MFMA n: key block n % 4, k-step n / 4
        const _Float16* lds_k = reinterpret_cast<const _Float16*>(smem + (jt & 1) * KT_BYTES);
        auto frag = [&](int n) { return *reinterpret_cast<const h8*>(lds_k + ((2 * (n / 4) + lh) * T + 32 * (n % 4) + lq) * 8); };
        h8 a[PF];
#pragma unroll
        for (int n = 0; n < PF; ++n) a[n] = frag(n);
        PASA_FENCE();
#pragma unroll
        for (int n = 0; n < NM1; ++n) {
            const int kb = n % 4, ks = n / 4;
            if (ks == 0)
                S[kb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[n % PF], Qf[ks], (f16v)0.f, 0, 0, 0);
            else
                S[kb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[n % PF], Qf[ks], S[kb], 0, 0, 0);
            PASA_FENCE();
            if (n + PF < NM1) a[n % PF] = frag(n + PF);
            PASA_FENCE();
        }
    };
    auto gemm2 = [&](int jt) {   // (P V)^T of tile jt: D channels x 32 queries; runs during M(jt+1); MFMA n: channel block n % CB, k-step n / CB
        const _Float16* lds_v = reinterpret_cast<const _Float16*>(smem + 2 * KT_BYTES + (jt & 1) * KT_BYTES);
        auto frag = [&](int n) { return *reinterpret_cast<const h8*>(lds_v + ((2 * (n / CB) + lh) * D + 32 * (n % CB) + lq) * 8); };
        h8 a[PF];
#pragma unroll
        for (int n = 0; n < PF; ++n) a[n] = frag(n);
        PASA_FENCE();
#pragma unroll
        for (int n = 0; n < NM2; ++n) {
            const int cb = n % CB, kk = n / CB;
            if (STRICT && kk == 0)
                O[cb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[n % PF], Pf[kk], (f16v)0.f, 0, 0, 0);
            else
                O[cb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[n % PF], Pf[kk], O[cb], 0, 0, 0);
            PASA_FENCE();
            if (n + PF < NM2) a[n % PF] = frag(n + PF);
            PASA_FENCE();
            if (LSUM_MFMA && cb == CB - 1) {
                Lacc = __builtin_amdgcn_mfma_f32_32x32x16_f16(ones, Pf[kk], Lacc, 0, 0, 0);
                PASA_FENCE();
            }
            if (LSUM_DEFER) {
                // 32 packed pairs over NM2 MFMAs
                constexpr int PER = 32 / NM2;
#pragma unroll
                for (int u = 0; u < PER; ++u) {
                    const int pr = n * PER + u;          // pair pr: Pf[pr / 4], elements 2 * (pr % 4), + 1
                    const h2 p2 = {Pf[pr / 4][2 * (pr % 4)], Pf[pr / 4][2 * (pr % 4) + 1]};
                    pl_d[pr & 3] = add_pair_mix(p2, pl_d[pr & 3]);
                }
                PASA_FENCE();
            }
        }
        if (LSUM_DEFER) {
            l += sum32((pl_d[0] + pl_d[1]) + (pl_d[2] + pl_d[3]));
            pl_d[0] = pl_d[1] = pl_d[2] = pl_d[3] = 0.f;
        }
    };

    for (int j = j0; j <= J_wg; ++j) {
        // =========================== matrix part M(j) ===========================
        const bool do_g2 = (j > j0 && j - 1 < J_w), do_g1 = (j < J_w);
        const bool tail = (tail_keys != 0) && (j == ntile - 1); // ragged last tile: padding keys are masked
        const bool diag = (CAUSAL && (j * T + T - 1 > pos_w0)) || tail;   // tile j needs the mask for this wave
        __builtin_amdgcn_s_setprio(1);
        // ---- pseudo-averages of the next 16 tiles: rows of A are the high and low parts of the tiles' mean keys ----
        if (MSBAR && ((j & 15) == 0 || j == j0) && do_g1) {
            const _Float16* lds_km = reinterpret_cast<const _Float16*>(smem + 4 * KT_BYTES);
            f16v acc = (f16v)0.f;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(*reinterpret_cast<const h8*>(lds_km + ((2 * ks + lh) * 32 + lq) * 8),
                                                             Qf[ks], acc, 0, 0, 0);
            // lanes 0-31 hold q . hi of tile i in element i, lanes 32-63 q . lo of the same tile; after the exchange
            // element i + 8 -> i the sum is tile i in lanes 0-31 and tile i + 8 in lanes 32-63
            float* sb = reinterpret_cast<float*>(smem + SB_OFF + wave * 2048);
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                float x = acc[i], y = acc[i + 8];
                swap32(x, y);
                sb[(i + 8 * lh) * 32 + lq] = x + y * 0.00048828125f;      // low parts are stored times 2^11
            }
        }
        // ---- pending product of tile j-1 ----
        if (do_g2) gemm2(j - 1);
        // ---- S'(j) ----
        if (do_g1) gemm1(j);
        __builtin_amdgcn_s_setprio(0);
        if (grp == 1) drain_copies();
        __syncthreads();
        // This wave's share of the tile copies first: they have the whole vector part to land (issued later, among the
        // exponentials, their latency showed at the drain before the next barrier: 3.8 % of the kernel's cycles).
        issue_slot(grp ? 2 * j + 2 : 2 * j);
        if (MSBAR && (j & 15) == 8) issue_kmean((j >> 4) + 1);   // read from M(16 * ((j >> 4) + 1)) on, free since M(j - 8)
        PASA_FENCE();

        // =========================== vector part V(j) ===========================
        if (j < J_w) {
            const bool first = (j == j0);
            if (STRICT && do_g2) fold16(j - 1);      // O <- fp16(e^{dm_j} PV) + fp16(e^{dm_{j-1}} O) for the product of tile j-1
            // ---- S' as stored: fp32, or rounded to fp16 ----
            // STRICT16 keeps the rounded scores packed two per register and works on them with packed fp16
            // instructions (same roundings, half the instructions and registers)
            h2 Sh[4][8];
            if (STRICT) {
#pragma unroll
                for (int kb = 0; kb < 4; ++kb)
#pragma unroll
                    for (int t = 0; t < 8; ++t) {
                        if (INSTR)
                            n_ovf += ((__builtin_fabsf(S[kb][2 * t]) >= 65520.f) ? 1u : 0u) +
                                     ((__builtin_fabsf(S[kb][2 * t + 1]) >= 65520.f) ? 1u : 0u);
                        Sh[kb][t] = pack_rn(S[kb][2 * t], S[kb][2 * t + 1]);
                    }
            } else if (S16) {
#pragma unroll
                for (int kb = 0; kb < 4; ++kb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const float s32 = S[kb][i];
                        if (INSTR) n_ovf += (__builtin_fabsf(s32) >= 65520.f) ? 1u : 0u;
                        float sv = (float)(_Float16)s32;
                        if (NAIVE) sv = sv * scale;          // Eq. (2): static scaling after the GEMM
                        S[kb][i] = sv;
                    }
            } else if (INSTR) {
#pragma unroll
                for (int kb = 0; kb < 4; ++kb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) n_ovf += (__builtin_fabsf(S[kb][i]) >= 65520.f) ? 1u : 0u;
            }
            // ---- pseudo-average over all 128 keys of the tile (before masking) ----
            float sbar = 0.f;
            if (MSBAR) {
                const float v = reinterpret_cast<const float*>(smem + SB_OFF + wave * 2048)[(j & 15) * 32 + lq];
                if (DIRECT) cj = scale * v;                    // the bias the shift removed from this tile's scores
                else sbar = tail ? v * ((float)T * inv_tail) : v;   // stored per 128 key slots; a ragged last tile divides by its own key count
            } else if (!NAIVE && !DIRECT) {
                float ps[4];
#pragma unroll
                for (int kb = 0; kb < 4; ++kb) {
                    if (STRICT) {          // fp16 values summed in fp32
                        ps[kb] = 0.f;
#pragma unroll
                        for (int t = 0; t < 8; ++t) ps[kb] = add_pair_mix(Sh[kb][t], ps[kb]);
                        continue;
                    }
                    ps[kb] = S[kb][0];
#pragma unroll
                    for (int i = 1; i < 16; ++i) ps[kb] += S[kb][i];
                }
                // padding keys of a ragged last tile have K' = 0 and add nothing; the divisor is the tile's own key count
                const float sum = sum32((ps[0] + ps[1]) + (ps[2] + ps[3]));
                sbar = sum * (tail ? inv_tail : 1.0f / T);
                if (STRICT) sbar = (float)(_Float16)sbar;
            }
            // ---- mask: keys after the query (causal, diagonal tiles) or past the end (ragged last tile) ----
            if (diag) {
                int last_key = N - 1;
                if (CAUSAL && row0 + row < last_key) last_key = row0 + row;
#pragma unroll
                for (int kb = 0; kb < 4; ++kb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int key = j * T + 32 * kb + 8 * (i >> 2) + 4 * lh + (i & 3);
                        if (key > last_key) {
                            if (STRICT) Sh[kb][i >> 1][i & 1] = (_Float16)(-__builtin_inff());
                            else S[kb][i] = -__builtin_inff();
                        }
                    }
            }
            // ---- local maximum m' ----
            float pm[4];
#pragma unroll
            for (int kb = 0; kb < 4; ++kb) {
                if (STRICT) {
                    h2 mm = Sh[kb][0];
#pragma unroll
                    for (int t = 1; t < 8; ++t) mm = __builtin_elementwise_max(mm, Sh[kb][t]);
                    pm[kb] = __builtin_fmaxf((float)mm[0], (float)mm[1]);
                    continue;
                }
                pm[kb] = S[kb][0];
#pragma unroll
                for (int i = 1; i < 16; ++i) pm[kb] = __builtin_fmaxf(pm[kb], S[kb][i]);
            }
            const float mx = max32(__builtin_fmaxf(__builtin_fmaxf(pm[0], pm[1]), __builtin_fmaxf(pm[2], pm[3])));
            // A wave whose rows straddle a tile boundary (chunks not aligned to 32 rows) reaches tile j although its
            // first rows see none of it: those rows keep their state and add nothing.
            const bool unseen = CAUSAL && diag && (row0 + row < j * T);
            // ---- reference level for exp: local m' (PASA), running max (plain FlashAttention) ----
            float mref = unseen ? 0.f : mx;
            float c_adj = 0.f;    // LAZY: log of the factor this tile's P carries (its level relative to the stored scale)
            bool resc = false;    // LAZY: this row re-references its stored output and sum to the level of tile j
            float lc_resc = 0.f;  // LAZY: log of the factor that does it
            if (NAIVE) {
                // plain online softmax (Eq. (4)-(8)) on the running maximum, the stored output handled as in MIXED:
                // its log scale moves by m_{j-1} - m_j, P carries the factor, no per-tile rescale
                const float mnew = __builtin_fmaxf(m, mx);
                const bool keep = first || unseen;
                const float lcn = Lc + (m - mnew), c = -lcn;
                resc = !keep && c > CMAX;
                lc_resc = lcn;
                c_adj = (keep || resc) ? 0.f : c;
                Lc = first ? 0.f : unseen ? Lc : resc ? 0.f : lcn;
                m = mnew;
                mref = mnew;
            }
            // ---- fp32 variants: global recovering (step 3) and the factor of the output or of P now, before the
            // exponentials.  Only the running sum needs l'; the rest is a chain of dependent scalar operations whose
            // latency is hidden when the exponentials that follow can issue in between. ----
            bool l_keep = false;             // STRICT16: this row's state is not touched by this tile
            if (STRICT) {
                // Step 3 with every operation rounded to fp16, in the order Algorithm 1 states them; computed before
                // the exponentials and without branches (the first tile and rows that see nothing of the tile select
                // their values at the end) so that the latency of this chain is hidden.  The factors of the output
                // combination go to ep_s / ec_s (the pending product of tile j-1 has been folded in above).
                const _Float16 jm1 = (_Float16)(float)(j - j0), jn = (_Float16)(float)(j - j0 + 1);
                const _Float16 Fo = (_Float16)F, sb = (_Float16)sbar, mo = (_Float16)m, mxh = (_Float16)mx;
                const _Float16 iv = (_Float16)inva;
                const _Float16 Fn = (_Float16)((_Float16)((_Float16)(jm1 * Fo) + sb) / jn);
                const _Float16 dpp = (_Float16)(iv * (_Float16)(Fo - Fn));
                const _Float16 dpc = (_Float16)(iv * (_Float16)(sb - Fn));
                const _Float16 c1 = (_Float16)(mo + dpp), c2 = (_Float16)(mxh + dpc);
                const _Float16 mn = c1 > c2 ? c1 : c2;
                const _Float16 dp = (_Float16)((_Float16)(mo - mn) + dpp);
                const _Float16 dc = (_Float16)((_Float16)(mxh - mn) + dpc);
                const _Float16 ep = (_Float16)exp_nat((float)dp), ec = (_Float16)exp_nat((float)dc);
                l_keep = unseen;
                F = first ? sbar : unseen ? F : (float)Fn;
                m = first ? mx : unseen ? m : (float)mn;
                ep_s = first ? 0.f : unseen ? 1.f : (float)ep;     // unseen: O <- fp16(0 * 0) + fp16(1 * O)
                ec_s = first ? 1.f : unseen ? 0.f : (float)ec;
            } else if (DIRECT) {
                // ordinary online softmax on the level m' + c of this tile's maximum; same bookkeeping as below
                const float lev = mx + cj;
                const float mn = __builtin_fmaxf(m, lev);
                const float dp = m - mn;
                const float dc = lev - mn;
                const bool keep = first || unseen;
                const float lcn = Lc + dp, c = dc - lcn;
                resc = !keep && c > CMAX;
                lc_resc = -c;
                c_adj = (keep || resc) ? 0.f : c;
                Lc = first ? 0.f : unseen ? Lc : resc ? dc : lcn;
                m = first ? lev : unseen ? m : mn;
            } else if (!STRICT && !NAIVE) {
                // Written without branches (the first tile and rows that see nothing of the tile select their values at
                // the end) so that it stays in one block with the exponentials.
                // F is only a reference level (it cancels between the two correction terms), so Eq. (15)'s division by
                // j is a multiplication by the hardware's reciprocal of j here
                const float jm1 = (float)(j - j0), rj = __builtin_amdgcn_rcpf((float)(j - j0 + 1));
                const float Fn = (jm1 * F + sbar) * rj;
                const float dpp = inva * (F - Fn);
                const float dpc = inva * (sbar - Fn);
                const float mn = __builtin_fmaxf(m + dpp, mx + dpc);
                const float dp = (m - mn) + dpp;
                const float dc = (mx - mn) + dpc;
                const bool keep = first || unseen;        // no recovering step for this row
                // the stored output keeps its scale (its log moves by dp with the frame); the tile's P takes the factor
                // e^c that places it there, unless that is too large: then the row's output and sum move to this tile
                const float lcn = Lc + dp, c = dc - lcn;
                resc = !keep && c > CMAX;
                lc_resc = -c;
                c_adj = (keep || resc) ? 0.f : c;
                Lc = first ? 0.f : unseen ? Lc : resc ? dc : lcn;
                F = first ? sbar : unseen ? F : Fn;
                m = first ? mx : unseen ? m : mn;
            }
            if (LAZY && __builtin_amdgcn_ballot_w64(resc) != 0ull) {
                // rare (the running maximum rose by more than CMAX above the stored scale); the pending product of
                // tile j-1 is already in O.  The empty asm keeps this a branch instead of 64 selects on every tile.
                asm volatile("" ::: "memory");
                const float r = resc ? exp_nat(lc_resc) : 1.f;
#pragma unroll
                for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) O[cb][i] *= r;
                l *= r;
                if (LSUM_MFMA) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) Lacc[i] *= r;
                }
            }
            // ---- P = exp(S' - m' [+ c]) rounded to fp16; l' = sum of the rounded P ----
            float lsum = 0.f;
            {
                const float nml = (c_adj - mref) * LOG2E;
                float pl[4];
#pragma unroll
                for (int kb = 0; kb < 4; ++kb) {
                    pl[kb] = 0.f;
#pragma unroll
                    for (int t2 = 0; t2 < 8; ++t2) {
                        float e0, e1;
                        if (STRICT) {   // the difference is itself rounded to fp16 before the exponential
                            const _Float16 mh = (_Float16)mref;      // exact: m' is one of the fp16 scores (or 0)
                            const h2 d2 = Sh[kb][t2] - (h2){mh, mh};
                            e0 = exp_nat_half<0>(d2);
                            e1 = exp_nat_half<1>(d2);
                        } else {        // exp(s - m) = 2^(s*log2e - m*log2e), one fused multiply-add per element
                            e0 = __builtin_amdgcn_exp2f(__builtin_fmaf(S[kb][2 * t2], LOG2E, nml));
                            e1 = __builtin_amdgcn_exp2f(__builtin_fmaf(S[kb][2 * t2 + 1], LOG2E, nml));
                        }
                        const h2 p2 = pack_rn(e0, e1);
                        Pf[2 * kb + (t2 >> 2)][2 * (t2 & 3)] = p2[0];
                        Pf[2 * kb + (t2 >> 2)][2 * (t2 & 3) + 1] = p2[1];
                        if (!LSUM_MFMA && !LSUM_DEFER) pl[kb] = (STRICT || MSBAR) ? add_pair_mix(p2, pl[kb]) : add_pair(p2, pl[kb]);
                    }
                }
                if (!LSUM_MFMA && !LSUM_DEFER) lsum = sum32((pl[0] + pl[1]) + (pl[2] + pl[3]));
                if (STRICT) lsum = (float)(_Float16)lsum;
            }

            // ---- the running sum (step 4); STRICT16: the whole of step 3 and 4 in fp16 ----
            if (LAZY) {
                l += lsum;                     // the sum is kept at the stored output's scale (first tile: l was 0)
            } else {
                // fp16, each operation rounded: l = fp16(fp16(e^{dm_{j-1}} l) + fp16(e^{dm_j} l')); first tile: l = l'
                const _Float16 lo = (_Float16)l, ln = (_Float16)lsum;
                const float ln_all = (float)(_Float16)((_Float16)((_Float16)ep_s * lo) + (_Float16)((_Float16)ec_s * ln));
                l = first ? lsum : l_keep ? l : ln_all;
            }
        }
        if (grp == 0) drain_copies();
        __syncthreads();
    }
    if (grp == 0) __syncthreads();         // group B's last barrier

    if (LSUM_MFMA) l = Lacc[0];            // every row of the block is the sum
    // ---------------- key split: leave the row state for the merge ----------------
    if (!STRICT && part_o != nullptr) {
        if (wave_valid) {
            const size_t rows_all = (size_t)(gridDim.x / nsplit) / nqt * Nq;                     // B * Hq * Nq
            const size_t grow = (size_t)(b * Hq + hq) * Nq + row;                                // global row index
            // level of the stored output: running maximum in its frame, the frame's offset, the stored scale (exact in fp64)
            const bool none = !(J_w > j0) || !(l > 0.f);
            if (row_valid && lh == 0) {
                part_lr[((size_t)split * rows_all + grow) * 2] = none ? 0.0 : (double)l;
                part_lr[((size_t)split * rows_all + grow) * 2 + 1] =
                    none ? -__builtin_inf() : (double)m + (double)inva * (double)F + (double)Lc;
            }
            float* pbase = part_o + ((size_t)split * rows_all + grow) * D;
            if (row_valid && !none) {
#pragma unroll
                for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                    for (int gq = 0; gq < 4; ++gq) {
                        float4 v4 = {O[cb][4 * gq], O[cb][4 * gq + 1], O[cb][4 * gq + 2], O[cb][4 * gq + 3]};
                        *reinterpret_cast<float4*>(pbase + 32 * cb + 8 * gq + 4 * lh) = v4;
                    }
            }
        }
        if (INSTR) {
            if (ovf_s != nullptr && n_ovf) atomicAdd(ovf_s, n_ovf);
            if (ovf_group != nullptr && n_ovf) atomicAdd(ovf_group + grp_id, n_ovf);
        }
        return;
    }

    // ---------------- final normalisation and store ----------------
    unsigned long long n_bad = 0;
    if (wave_valid) {
        if (STRICT) fold16(J_w - 1);
        const float oscale = STRICT ? 0.f : 1.0f / l;
        _Float16* obase = o + ((size_t)(b * Hq + hq) * Nq) * D;
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                h4 out;
                u16x4 outb;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int i = 4 * gq + r;
                    // fp32 variants: the fp32 quotient is rounded once, to the output type; STRICT16: the fp16
                    // quotient of Algorithm 1's last line, converted when the output is bf16
                    const float v32 = STRICT ? (float)(_Float16)(O16[cb][i >> 1][i & 1] / (_Float16)l) : O[cb][i] * oscale;
                    const _Float16 val = (_Float16)v32;
                    outb[r] = f32_to_bf16_rn(v32);
                    if (INSTR && row_valid) {
                        const float fv = io_bf16 ? __uint_as_float((unsigned)outb[r] << 16) : (float)val;
                        n_bad += (fv != fv || __builtin_fabsf(fv) == __builtin_inff()) ? 1u : 0u;
                    }
                    out[r] = val;
                }
                _Float16* dst = obase + (size_t)row * D + 32 * cb + 8 * gq + 4 * lh;
                if (row_valid) {
                    if (io_bf16) *reinterpret_cast<u16x4*>(dst) = outb;
                    else *reinterpret_cast<h4*>(dst) = out;
                }
            }
    }
    if (INSTR) {
        if (ovf_s != nullptr && n_ovf) atomicAdd(ovf_s, n_ovf);
        if (ovf_group != nullptr && n_ovf) atomicAdd(ovf_group + grp_id, n_ovf);
        if (nonfinite_o != nullptr && n_bad) atomicAdd(nonfinite_o, n_bad);
    }
}

// Merge of the key splits of one call: per query row, the splits' stored outputs and sums are brought to the highest of
// their levels (the log-sum-exp rule on R = m + Inva * F + Lc, the absolute level a split's stored output refers to)
// and added; then Algorithm 1's final quotient.  One thread per 8 channels of a row.
template <int D>
__global__ __launch_bounds__(256) void pasa_merge_splits(const float* __restrict__ part_o, const double* __restrict__ part_lr,
                                                         _Float16* __restrict__ o, size_t rows_all, int nsplit, int io_bf16,
                                                         unsigned long long* nonfinite_o)
{
    constexpr int TPR = D / 8;                       // threads per row
    const size_t grow = (size_t)blockIdx.x * (256 / TPR) + threadIdx.x / TPR;
    if (grow >= rows_all) return;
    const int c0 = (threadIdx.x % TPR) * 8;
    double rmax = -__builtin_inf();
    for (int s = 0; s < nsplit; ++s) {
        const double r = part_lr[((size_t)s * rows_all + grow) * 2 + 1];
        rmax = r > rmax ? r : rmax;
    }
    float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    float lsum = 0.f;
    for (int s = 0; s < nsplit; ++s) {
        const double r = part_lr[((size_t)s * rows_all + grow) * 2 + 1];
        if (!(r > -__builtin_inf())) continue;       // this split saw none of the row's keys (its output is not written)
        const float wgt = __builtin_amdgcn_exp2f((float)(r - rmax) * LOG2E);
        lsum += wgt * (float)part_lr[((size_t)s * rows_all + grow) * 2];
        const float4* src = reinterpret_cast<const float4*>(part_o + ((size_t)s * rows_all + grow) * D + c0);
        const float4 a = src[0], b4 = src[1];
        acc[0] += wgt * a.x; acc[1] += wgt * a.y; acc[2] += wgt * a.z; acc[3] += wgt * a.w;
        acc[4] += wgt * b4.x; acc[5] += wgt * b4.y; acc[6] += wgt * b4.z; acc[7] += wgt * b4.w;
    }
    const float inv = 1.0f / lsum;
    h8 out;
    u16x8 outb;
    unsigned n_bad = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const float v32 = acc[e] * inv;
        out[e] = (_Float16)v32;
        outb[e] = f32_to_bf16_rn(v32);
        const float fv = io_bf16 ? __uint_as_float((unsigned)outb[e] << 16) : (float)out[e];
        n_bad += (fv != fv || __builtin_fabsf(fv) == __builtin_inff()) ? 1u : 0u;
    }
    if (io_bf16) *reinterpret_cast<u16x8*>(o + grow * D + c0) = outb;
    else *reinterpret_cast<h8*>(o + grow * D + c0) = out;
    if (nonfinite_o != nullptr && n_bad) atomicAdd(nonfinite_o, (unsigned long long)n_bad);
}

template <int D, int VAR, bool CAUSAL, bool INSTR>
hipError_t launch_fwd(const PasaLaunch& p)
{
    constexpr int RWG = 256;
    constexpr int LDS_BYTES = 4 * (T * D * 2) + ((VAR == PASA_K_MIXED || VAR == PASA_K_DIRECT) ? 64 * D + 8 * 2048 : 0);
    const int nqt = (p.Nq + RWG - 1) / RWG;
    const int nsplit = (VAR == PASA_K_STRICT16 || p.nsplit < 1) ? 1 : p.nsplit;   // fp16 state has no merge rule
    const dim3 grid((unsigned)(nqt * p.Hq * p.B * nsplit));
    auto kern = pasa_fwd<D, VAR, CAUSAL, INSTR>;
    // the dynamic LDS limit of this instantiation is raised once per device, not on every launch
    static std::atomic<unsigned long long> lds_limit_set{0ull};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const unsigned long long bit = 1ull << (dev & 63);
    if (!(lds_limit_set.load(std::memory_order_acquire) & bit)) {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
        if (e != hipSuccess) return e;
        lds_limit_set.fetch_or(bit, std::memory_order_release);
    }
    hipLaunchKernelGGL(kern, grid, dim3(512), LDS_BYTES, p.stream, (const _Float16*)p.q, (const char*)p.ws,
                       (_Float16*)p.o, (const _Float16*)p.kmean, p.Hq, p.Hkv, p.Nq, p.row0, p.N, nqt, p.inva, p.scale, p.io_bf16, p.overflow_s,
                       nsplit > 1 ? nullptr : p.nonfinite_o, p.overflow_group, p.gate, nsplit,
                       nsplit > 1 ? (float*)p.part_o : nullptr, nsplit > 1 ? (double*)p.part_lr : nullptr);
    e = hipGetLastError();
    if (e != hipSuccess || nsplit == 1) return e;
    const size_t rows_all = (size_t)p.B * p.Hq * p.Nq;
    constexpr int RPB = 256 / (D / 8);                          // rows per block of the merge
    hipLaunchKernelGGL(pasa_merge_splits<D>, dim3((unsigned)((rows_all + RPB - 1) / RPB)), dim3(256), 0, p.stream,
                       (const float*)p.part_o, (const double*)p.part_lr, (_Float16*)p.o, rows_all, nsplit, p.io_bf16,
                       p.nonfinite_o);
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
        case PASA_K_DIRECT: return launch_fwd_cv<D, PASA_K_DIRECT>(p);
    }
    return hipErrorInvalidValue;
}

}  // namespace

hipError_t pasa_launch_prep(const void* k, const void* v, void* ws, void* plain_out,
                            int B, int Hkv, int N, int d, double beta, double kscale, int shift_mode, int in_bf16,
                            void* k0out, void* kmean_out, const unsigned long long* gate, hipStream_t stream)
{
    const int ntile = (N + T - 1) / T;
    const int y_off = k == nullptr ? PASA_PREP_SPLIT : 0;     // no keys given: the value blocks alone
    const dim3 grid((unsigned)((size_t)B * Hkv * ntile), (v != nullptr && k != nullptr ? 2u : 1u) * PASA_PREP_SPLIT);   // y: key channel groups, then value key groups
    if (d == 128)
        hipLaunchKernelGGL(pasa_prep_kv<128>, grid, dim3(256), 0, stream, (const _Float16*)k, (const _Float16*)v,
                           (_Float16*)ws, (_Float16*)plain_out, (_Float16*)k0out, (_Float16*)kmean_out, N, ntile, beta, kscale, shift_mode, in_bf16, gate, y_off);
    else
        hipLaunchKernelGGL(pasa_prep_kv<64>, grid, dim3(256), 0, stream, (const _Float16*)k, (const _Float16*)v,
                           (_Float16*)ws, (_Float16*)plain_out, (_Float16*)k0out, (_Float16*)kmean_out, N, ntile, beta, kscale, shift_mode, in_bf16, gate, y_off);
    return hipGetLastError();
}

namespace {
__global__ void pasa_zero_u64(unsigned long long* p, int n)
{
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) p[i] = 0ull;
}
}  // namespace

hipError_t pasa_launch_zero(unsigned long long* p, int n, hipStream_t stream)
{
    hipLaunchKernelGGL(pasa_zero_u64, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, p, n);
    return hipGetLastError();
}

hipError_t pasa_launch_fwd(const PasaLaunch& p)
{
    return p.d == 128 ? launch_fwd_d<128>(p) : launch_fwd_d<64>(p);
}
