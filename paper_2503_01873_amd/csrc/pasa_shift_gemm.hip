// Algorithm 1's pre-processing loop as the paper prints it: the batched GEMM K'^T = K^T M on the matrix core, M the
// shifting matrix of Eq. (10) with every entry rounded to fp16 first (diagonal a, off-diagonal b).  Kept beside the
// default pre-processing kernel (which takes the tile mean by reduction) so that the paper's "one batched GEMM instead
// of a reduction on the vector unit" has a measured cost on this GPU, and a measured accuracy: the matrix core
// accumulates the 128 products of an output element in fp32, the other paths accumulate them exactly.
//
//  pasa_shift_gemm_k    one workgroup per (batch, KV head, key tile), one wavefront per 32 channels:
//                       (K'^T)[c, q] = sum_p K[p, c] M[p, q],  A = K^T fragment (32 channels x 16 keys, gathered from
//                       the LDS copy of the tile), B = M fragment (16 x 32, built in registers: b everywhere, a where
//                       p == q), v_mfma_f32_32x32x16_f16, one rounding of the fp32 sum to fp16.  Writes the K' tile in
//                       the workspace's fragment order (or the plain [N, d] layout).
//  pasa_kmean_of_tiles  per tile, the per-channel mean over 128 key slots of the K' just written, as the fp16 pair
//                       (high, low * 2^11) in the mean block that PASA_K_MIXED reads.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pasa_kernels.h"

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef _Float16 h4 __attribute__((ext_vector_type(4)));
typedef float f16v __attribute__((ext_vector_type(16)));
typedef unsigned short u16x8 __attribute__((ext_vector_type(8)));

namespace {

constexpr int T = 128;

__device__ inline _Float16 half_of_double(double x)     // one rounding (truncate to fp32 with a sticky bit, then to fp16)
{
    float f = (float)x;
    if ((double)f != x) {
        uint32_t u = __float_as_uint(f);
        if (__builtin_fabs((double)f) > __builtin_fabs(x)) u -= 1u;
        f = __uint_as_float(u | 1u);
    }
    return (_Float16)f;
}

template <int D>
__global__ __launch_bounds__(256) void pasa_shift_gemm_k(const _Float16* __restrict__ k, _Float16* __restrict__ wsout,
                                                         _Float16* __restrict__ plain_out, int ntile, float a16, float b16,
                                                         int in_bf16)
{
    constexpr int CBS = D / 32;                 // 32-channel blocks = wavefronts that work
    __shared__ __attribute__((aligned(16))) _Float16 ks_lds[T][D + 8];   // +8 halfs: rows 16 bytes apart in bank space

    const size_t tile = blockIdx.x;
    const size_t head = tile / ntile;
    const int t = (int)(tile % ntile);
    const size_t src_off = (head * (size_t)ntile * T + (size_t)t * T) * D;     // N = ntile * 128 (whole tiles only)
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lq = lane & 31, lh = lane >> 5;

    for (int idx = tid; idx < T * (D / 8); idx += 256) {
        const int n = idx / (D / 8), c8 = idx % (D / 8);
        h8 val;
        if (in_bf16) {
            const u16x8 raw = *reinterpret_cast<const u16x8*>(k + src_off + (size_t)n * D + 8 * c8);
#pragma unroll
            for (int e = 0; e < 8; ++e) val[e] = (_Float16)__uint_as_float((unsigned)raw[e] << 16);
        } else {
            val = *reinterpret_cast<const h8*>(k + src_off + (size_t)n * D + 8 * c8);
        }
        *reinterpret_cast<h8*>(&ks_lds[n][8 * c8]) = val;
    }
    __syncthreads();
    if (wave >= CBS) return;

    const int cb = wave;
    const _Float16 ah = (_Float16)a16, bh = (_Float16)b16;
    f16v acc[4];
#pragma unroll
    for (int qb = 0; qb < 4; ++qb) acc[qb] = (f16v)0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
        // A: channel 32*cb + lq, keys 16*ks + 8*lh .. +7
        h8 afrag;
#pragma unroll
        for (int e = 0; e < 8; ++e) afrag[e] = ks_lds[16 * ks + 8 * lh + e][32 * cb + lq];
#pragma unroll
        for (int qb = 0; qb < 4; ++qb) {
            // B: column q = 32*qb + lq, rows p = 16*ks + 8*lh .. +7: the diagonal entry where p == q
            const int hit = 32 * qb + lq - 16 * ks - 8 * lh;
            h8 bfrag;
#pragma unroll
            for (int e = 0; e < 8; ++e) bfrag[e] = (e == hit) ? ah : bh;
            acc[qb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(afrag, bfrag, acc[qb], 0, 0, 0);
        }
    }
    // acc[qb][i]: key 32*qb + lq, channel 32*cb + 8*(i/4) + 4*lh + i%4 -- four consecutive channels per group of i
#pragma unroll
    for (int qb = 0; qb < 4; ++qb) {
        const int n = 32 * qb + lq;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            h4 out;
#pragma unroll
            for (int r = 0; r < 4; ++r) out[r] = (_Float16)acc[qb][4 * g + r];      // fp32 -> fp16, nearest even
            const int c0 = 32 * cb + 8 * g + 4 * lh;
            if (plain_out != nullptr)
                *reinterpret_cast<h4*>(plain_out + src_off + (size_t)n * D + c0) = out;
            else
                *reinterpret_cast<h4*>(wsout + tile * (size_t)(2 * T * D) + ((size_t)(c0 / 8) * T + n) * 8 + (c0 % 8)) = out;
        }
    }
}

template <int D>
__global__ __launch_bounds__(256) void pasa_kmean_of_tiles(const _Float16* __restrict__ ws, _Float16* __restrict__ kmean_out,
                                                           int ntile)
{
    // thread = (channel chunk c8, key group): sums 8 channels over its keys exactly in fp64, then LDS reduction
    constexpr int CH = D / 8, KL = 256 / CH, KPT = T / KL;
    __shared__ double psum[KL][D];
    const size_t tile = blockIdx.x;
    const size_t head = tile / ntile;
    const int t = (int)(tile % ntile);
    const int tid = threadIdx.x, c8 = tid % CH, kl = tid / CH;
    const _Float16* kt = ws + tile * (size_t)(2 * T * D);
    double s[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int i = 0; i < KPT; ++i) {
        const h8 val = *reinterpret_cast<const h8*>(kt + ((size_t)c8 * T + kl + KL * i) * 8);
#pragma unroll
        for (int e = 0; e < 8; ++e) s[e] += (double)val[e];
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) psum[kl][8 * c8 + e] = s[e];
    __syncthreads();
    if (tid < D) {
        double tot = 0;
        for (int r = 0; r < KL; ++r) tot += psum[r][tid];
        const double m128 = tot * 0.0078125;
        const _Float16 hi = half_of_double(m128);
        const _Float16 lo = half_of_double((m128 - (double)hi) * 2048.0);
        const int nblk = (ntile + 15) / 16;
        const int t16 = t & 15, row = 8 * (t16 >> 2) + (t16 & 3), c = tid;
        _Float16* blk = kmean_out + ((head * (size_t)nblk + (size_t)(t >> 4)) * 32) * D;
        blk[((size_t)(c / 8) * 32 + row) * 8 + (c % 8)] = hi;
        blk[((size_t)(c / 8) * 32 + row + 4) * 8 + (c % 8)] = lo;
        if (t == ntile - 1)
            for (int u = t16 + 1; u < 16; ++u) {
                const int ru = 8 * (u >> 2) + (u & 3);
                blk[((size_t)(c / 8) * 32 + ru) * 8 + (c % 8)] = (_Float16)0;
                blk[((size_t)(c / 8) * 32 + ru + 4) * 8 + (c % 8)] = (_Float16)0;
            }
    }
}

}  // namespace

hipError_t pasa_launch_shift_gemm(const void* k, void* ws, void* plain_out, int B, int Hkv, int N, int d, double a16,
                                 double b16, int in_bf16, void* kmean_out, hipStream_t stream)
{
    const int ntile = N / T;                   // the caller has checked N % 128 == 0
    const dim3 grid((unsigned)((size_t)B * Hkv * ntile));
    if (d == 128)
        hipLaunchKernelGGL(pasa_shift_gemm_k<128>, grid, dim3(256), 0, stream, (const _Float16*)k, (_Float16*)ws,
                           (_Float16*)plain_out, ntile, (float)a16, (float)b16, in_bf16);
    else
        hipLaunchKernelGGL(pasa_shift_gemm_k<64>, grid, dim3(256), 0, stream, (const _Float16*)k, (_Float16*)ws,
                           (_Float16*)plain_out, ntile, (float)a16, (float)b16, in_bf16);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || kmean_out == nullptr || plain_out != nullptr) return e;
    if (d == 128)
        hipLaunchKernelGGL(pasa_kmean_of_tiles<128>, grid, dim3(256), 0, stream, (const _Float16*)ws, (_Float16*)kmean_out, ntile);
    else
        hipLaunchKernelGGL(pasa_kmean_of_tiles<64>, grid, dim3(256), 0, stream, (const _Float16*)ws, (_Float16*)kmean_out, ntile);
    return hipGetLastError();
}
