// Measurement tool (not part of libpasa): what the vector instructions of the attention kernel's vector part cost
// on a SIMD whose other wavefront issues MFMAs back to back -- the situation of the two wave groups of pasa_fwd,
// where one group is in its matrix part while the other is in its vector part.
//
// One workgroup per CU.  With 4 wavefronts (one per SIMD) every wavefront runs the vector instruction under test
// ("alone").  With 8 (two per SIMD) wavefronts 0-3 run it and wavefronts 4-7 run v_mfma_f32_32x32x16_f16, as one
// dependent chain or as 2 or 4 independent chains, at the default or at a raised wave priority.  Printed: shader
// cycles per vector instruction as the issuing wavefront sees them, and cycles per MFMA of the other wavefront.
//
// What it shows on MI355X: the MFMA wavefront is never slowed (32 cycles per MFMA, chained or not); a full-rate
// vector instruction takes 5 cycles alone and 7 beside it (an MFMA occupies the shared issue port for about 8 of its
// 32 cycles); v_exp_f32 takes 9 and 11; v_dot2_f32_f16 takes 5 alone but 24 beside the MFMAs -- it executes in the
// matrix pipeline and waits for a gap -- while costing the issue port little.  A second part measures the LDS read
// rate of a CU for the kernel's fragment reads (ds_read_b128).
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <stdlib.h>

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef float f16v __attribute__((ext_vector_type(16)));

#define CHECK(x)                                                                      \
    do {                                                                              \
        hipError_t e_ = (x);                                                          \
        if (e_ != hipSuccess) {                                                       \
            fprintf(stderr, "%s failed: %s\n", #x, hipGetErrorString(e_));            \
            exit(1);                                                                  \
        }                                                                             \
    } while (0)

enum { OP_EXP, OP_FMA, OP_CVT, OP_DOT2, OP_MAX3, OP_ADD, OP_FMAMIX, OP_PKADD16, OP_LOOP_DOT2, OP_LOOP_MIX, OP_N };
static const char* NAMES[OP_N] = {"v_exp_f32", "v_fma_f32", "v_cvt_pk_f16_f32", "v_dot2c_f32_f16", "v_max3_f32",
                                  "v_add_f32", "v_fma_mix_f32", "v_pk_add_f16",
                                  "P loop: 2 fma, 2 exp, cvt_pk, dot2c", "P loop: 2 fma, 2 exp, cvt_pk, 2 fma_mix"};
static const int PER_BODY[OP_N] = {16, 16, 16, 16, 16, 16, 16, 16, 48, 56};

// 16 independent instructions (or the exponential loop of the kernel over 16 scores); every value stays in registers
template <int OP>
__device__ __forceinline__ void body(float (&x)[16], float k)
{
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        if (OP == OP_EXP) asm volatile("v_exp_f32 %0, %0" : "+v"(x[i]));
        if (OP == OP_FMA) asm volatile("v_fma_f32 %0, %0, %1, %1" : "+v"(x[i]) : "v"(k));
        if (OP == OP_CVT) asm volatile("v_cvt_pk_f16_f32 %0, %0, %1" : "+v"(x[i]) : "v"(k));
        if (OP == OP_DOT2) asm volatile("v_dot2c_f32_f16 %0, %1, %1" : "+v"(x[i]) : "v"(k));
        if (OP == OP_MAX3) asm volatile("v_max3_f32 %0, %0, %1, %1" : "+v"(x[i]) : "v"(k));
        if (OP == OP_ADD) asm volatile("v_add_f32 %0, %0, %1" : "+v"(x[i]) : "v"(k));
        if (OP == OP_FMAMIX) asm volatile("v_fma_mix_f32 %0, %1, 1.0, %0 op_sel_hi:[1,0,0]" : "+v"(x[i]) : "v"(k));
        if (OP == OP_PKADD16) asm volatile("v_pk_add_f16 %0, %0, %1" : "+v"(x[i]) : "v"(k));
    }
    if (OP == OP_LOOP_DOT2 || OP == OP_LOOP_MIX) {
        float acc = 0.f;
#pragma unroll
        for (int i = 0; i < 16; i += 2) {
            asm volatile("v_fma_f32 %0, %0, %1, %1" : "+v"(x[i]) : "v"(k));
            asm volatile("v_fma_f32 %0, %0, %1, %1" : "+v"(x[i + 1]) : "v"(k));
            asm volatile("v_exp_f32 %0, %0" : "+v"(x[i]));
            asm volatile("v_exp_f32 %0, %0" : "+v"(x[i + 1]));
            asm volatile("v_cvt_pk_f16_f32 %0, %0, %1" : "+v"(x[i]) : "v"(x[i + 1]));
            if (OP == OP_LOOP_DOT2) {
                asm volatile("v_dot2c_f32_f16 %0, %1, %1" : "+v"(acc) : "v"(x[i]));
            } else {
                asm volatile("v_fma_mix_f32 %0, %1, 1.0, %0 op_sel_hi:[1,0,0]" : "+v"(acc) : "v"(x[i]));
                asm volatile("v_fma_mix_f32 %0, %1, 1.0, %0 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "+v"(acc) : "v"(x[i]));
            }
        }
        x[15] += acc;
    }
}

template <int OP, int NW, int PRIO, int CH>
__global__ __launch_bounds__(NW * 64, 1) void run(const h8* tab, long long* out, float* sink, int iters)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float x[16];
    for (int i = 0; i < 16; ++i) x[i] = -0.001f * (float)(lane + i);
    const float k = 0.999f;
    const h8 a = tab[lane], b = tab[64 + lane];
    f16v c0 = (f16v)0.f, c1 = (f16v)0.f, c2 = (f16v)0.f, c3 = (f16v)0.f;
    __syncthreads();
    const long long t0 = __builtin_readcyclecounter();
    if (NW == 8 && wave >= 4) {
        if (PRIO) __builtin_amdgcn_s_setprio(1);
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {      // 16 MFMAs per iteration in CH independent accumulator chains
                c0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c0, 0, 0, 0);
                if (CH == 4) {
                    c1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c1, 0, 0, 0);
                    c2 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c2, 0, 0, 0);
                    c3 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c3, 0, 0, 0);
                } else if (CH == 2) {
                    c1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c1, 0, 0, 0);
                    c0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c0, 0, 0, 0);
                    c1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c1, 0, 0, 0);
                } else {
                    c0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c0, 0, 0, 0);
                    c0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c0, 0, 0, 0);
                    c0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c0, 0, 0, 0);
                }
            }
        }
    } else {
        for (int it = 0; it < iters; ++it) {
            body<OP>(x, k);
            body<OP>(x, k);
        }
    }
    const long long t1 = __builtin_readcyclecounter();
    if (blockIdx.x == 0 && lane == 0) out[wave] = t1 - t0;
    float r = c0[0] + c1[1] + c2[2] + c3[3];
    for (int i = 0; i < 16; ++i) r += x[i];
    if (r == 12345.678f) sink[threadIdx.x] = r;   // keeps every value live
}

template <int OP, int PRIO, int CH>
static void beside(const h8* tab, long long* out, float* sink, int iters, int ncu)
{
    long long h[8];
    run<OP, 8, PRIO, CH><<<ncu, 512>>>(tab, out, sink, iters);
    CHECK(hipDeviceSynchronize());
    CHECK(hipMemcpy(h, out, sizeof(h), hipMemcpyDeviceToHost));
    printf("   %d chain(s) prio %d: %5.2f | %5.2f", CH, PRIO, h[0] / (2.0 * PER_BODY[OP] * iters), h[4] / (16.0 * iters));
}

template <int OP>
static void one(const h8* tab, long long* out, float* sink, int ncu)
{
    const int iters = 4000;
    long long h[8];
    run<OP, 4, 0, 4><<<ncu, 256>>>(tab, out, sink, iters);
    CHECK(hipDeviceSynchronize());
    CHECK(hipMemcpy(h, out, sizeof(h), hipMemcpyDeviceToHost));
    printf("%-42s alone %5.2f;  beside MFMAs (cycles per instruction | per MFMA):", NAMES[OP], h[0] / (2.0 * PER_BODY[OP] * iters));
    beside<OP, 0, 4>(tab, out, sink, iters, ncu);
    beside<OP, 1, 4>(tab, out, sink, iters, ncu);
    beside<OP, 1, 1>(tab, out, sink, iters, ncu);
    printf("\n");
    fflush(stdout);
}

// LDS read rate of a CU: NW wavefronts issue ds_read_b128 in the fragment pattern of the attention kernel (lanes 0-31
// read 512 contiguous bytes, lanes 32-63 another 512), DEPTH reads in flight per wavefront.
typedef float f4 __attribute__((ext_vector_type(4)));
template <int NW, int DEPTH>
__global__ __launch_bounds__(NW * 64, 1) void lds_rate(long long* out, float* sink, int iters)
{
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int i = threadIdx.x; i < 65536 / 4; i += NW * 64) reinterpret_cast<float*>(smem)[i] = (float)i;
    __syncthreads();
    const char* base = smem + (lane & 31) * 16 + (lane >> 5) * 2048 + (wave & 3) * 4096;
    const long long t0 = __builtin_readcyclecounter();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 16; u += DEPTH) {
            f4 v[DEPTH];
#pragma unroll
            for (int d = 0; d < DEPTH; ++d) v[d] = *reinterpret_cast<const f4*>(base + (((u + d) & 3) * 512 + ((u + d) >> 2) * 16384));
#pragma unroll
            for (int d = 0; d < DEPTH; ++d) asm volatile("" ::"v"(v[d]));
        }
    }
    const long long t1 = __builtin_readcyclecounter();
    if (blockIdx.x == 0 && lane == 0) out[wave & 7] = t1 - t0;
    if (t1 == 12345) sink[threadIdx.x] = 1.f;
}

template <int NW, int DEPTH>
static void lds_one(long long* out, float* sink, int ncu)
{
    const int iters = 2000;
    CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(lds_rate<NW, DEPTH>), hipFuncAttributeMaxDynamicSharedMemorySize, 65536));
    lds_rate<NW, DEPTH><<<ncu, NW * 64, 65536>>>(out, sink, iters);
    CHECK(hipDeviceSynchronize());
    long long h[8];
    CHECK(hipMemcpy(h, out, sizeof(h), hipMemcpyDeviceToHost));
    const double per = (double)h[0] / (16.0 * iters);
    printf("ds_read_b128: %2d wavefronts per CU, %d in flight each: %6.2f cycles per read per wavefront = %6.1f bytes/clk per CU\n",
           NW, DEPTH, per, NW * 1024.0 / per);
}

int main()
{
    hipDeviceProp_t prop;
    CHECK(hipGetDeviceProperties(&prop, 0));
    const int ncu = prop.multiProcessorCount;
    printf("%s, %d CUs; shader cycles per instruction of wavefront 0 of workgroup 0\n", prop.gcnArchName, ncu);
    h8* tab;
    long long* out;
    float* sink;
    CHECK(hipMalloc(&tab, 128 * sizeof(h8)));
    CHECK(hipMemset(tab, 0, 128 * sizeof(h8)));
    CHECK(hipMalloc(&out, 8 * sizeof(long long)));
    CHECK(hipMemset(out, 0, 8 * sizeof(long long)));
    CHECK(hipMalloc(&sink, 512 * sizeof(float)));
    one<OP_ADD>(tab, out, sink, ncu);
    one<OP_FMA>(tab, out, sink, ncu);
    one<OP_MAX3>(tab, out, sink, ncu);
    one<OP_CVT>(tab, out, sink, ncu);
    one<OP_FMAMIX>(tab, out, sink, ncu);
    one<OP_PKADD16>(tab, out, sink, ncu);
    one<OP_EXP>(tab, out, sink, ncu);
    one<OP_DOT2>(tab, out, sink, ncu);
    one<OP_LOOP_DOT2>(tab, out, sink, ncu);
    one<OP_LOOP_MIX>(tab, out, sink, ncu);
    lds_one<4, 1>(out, sink, ncu);
    lds_one<4, 4>(out, sink, ncu);
    lds_one<8, 1>(out, sink, ncu);
    lds_one<8, 4>(out, sink, ncu);
    lds_one<16, 4>(out, sink, ncu);
    CHECK(hipFree(tab));
    CHECK(hipFree(out));
    CHECK(hipFree(sink));
    return 0;
}
