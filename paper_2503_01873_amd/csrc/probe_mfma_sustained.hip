// Measurement tool (not part of libpasa): the fp16 MFMA rate this GPU sustains when nothing but
// v_mfma_f32_32x32x16_f16 runs, as a function of the operand data.  The published peak (2.5 PFLOP/s) assumes
// the 2.4 GHz boost clock; with operands that toggle like real activations the power management holds the
// shader clock well below that, which bounds what any attention kernel can reach on this machine.
//
// Every wavefront issues a long run of independent MFMAs (four accumulator chains) on operand fragments kept in
// registers; one wavefront per SIMD (256 threads per workgroup) or two (512), one workgroup per CU.
#include <hip/hip_runtime.h>
#include <math.h>
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

template <int NW>
__global__ __launch_bounds__(NW * 64, 2) void mfma_run(const h8* tab, long long* cycles, float* sink, int iters)
{
    const int lane = threadIdx.x & 63;
    h8 a[8], b[8];
    for (int i = 0; i < 8; ++i) {
        a[i] = tab[i * 64 + lane];
        b[i] = tab[(8 + i) * 64 + lane];
    }
    f16v c0 = (f16v)0.f, c1 = (f16v)0.f, c2 = (f16v)0.f, c3 = (f16v)0.f;
    __syncthreads();
    const long long r0 = __builtin_amdgcn_s_memrealtime();   // constant 100 MHz counter
    const long long t0 = __builtin_readcyclecounter();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            c0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[u], b[u], c0, 0, 0, 0);
            c1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[(u + 1) & 7], b[u], c1, 0, 0, 0);
            c2 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[(u + 2) & 7], b[(u + 3) & 7], c2, 0, 0, 0);
            c3 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[(u + 5) & 7], b[(u + 6) & 7], c3, 0, 0, 0);
        }
    }
    const long long t1 = __builtin_readcyclecounter();
    const long long r1 = __builtin_amdgcn_s_memrealtime();
    if (blockIdx.x == 0 && lane == 0) {
        cycles[threadIdx.x >> 6] = t1 - t0;
        cycles[8 + (threadIdx.x >> 6)] = r1 - r0;
    }
    const float r = c0[0] + c1[1] + c2[2] + c3[3];
    if (r == 12345.678f) sink[threadIdx.x] = r;   // keeps the accumulators live
}

template <int NW>
static void run(const char* name, const h8* tab, long long* cycles, float* sink, int ncu)
{
    const int iters = 2000;
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    mfma_run<NW><<<ncu, NW * 64>>>(tab, cycles, sink, iters);
    CHECK(hipDeviceSynchronize());
    CHECK(hipEventRecord(e0));
    mfma_run<NW><<<ncu, NW * 64>>>(tab, cycles, sink, iters);
    CHECK(hipEventRecord(e1));
    CHECK(hipEventSynchronize(e1));
    float ms;
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    long long h[16];
    CHECK(hipMemcpy(h, cycles, sizeof(h), hipMemcpyDeviceToHost));
    const double n_mfma = (double)ncu * NW * iters * 32;
    const double tflops = n_mfma * 32768 / ms / 1e9;
    // a SIMD retires one 32x32x16 MFMA (32768 FLOP) per 32 cycles when the pipe never idles, so the rate implies the clock
    const double clock_ghz = tflops * 1e12 / ((double)ncu * 4 * 1024) / 1e9;
    printf("%-28s %d wave(s)/SIMD  %8.3f ms  %7.0f TFLOP/s  %5.1f %% of 2500  implied shader clock >= %.2f GHz"
           "   [wave 0: cycle counter %lld, 100 MHz counter %lld, ratio %.2f]\n", name,
           NW / 4, ms, tflops, tflops / 25.0, clock_ghz, h[0], h[8], (double)h[0] / (double)(h[8] ? h[8] : 1));
}

int main()
{
    hipDeviceProp_t prop;
    CHECK(hipGetDeviceProperties(&prop, 0));
    const int ncu = prop.multiProcessorCount;
    printf("device: %s, %d CUs, reported max clock %.2f GHz\n", prop.gcnArchName, ncu, prop.clockRate / 1e6);
    const int n = 16 * 64 * 8;
    _Float16* h = (_Float16*)malloc(n * sizeof(_Float16));
    h8* tab;
    long long* cycles;
    float* sink;
    CHECK(hipMalloc(&tab, n * sizeof(_Float16)));
    CHECK(hipMalloc(&cycles, 4096));
    CHECK(hipMalloc(&sink, 8192));
    for (int mode = 0; mode < 3; ++mode) {
        srand(1);
        for (int i = 0; i < n; ++i) {
            float v = 0.f;
            if (mode == 1) v = 1.f;
            if (mode == 2) {   // standard normal (Box-Muller)
                const double u1 = (rand() + 1.0) / (RAND_MAX + 2.0), u2 = (rand() + 1.0) / (RAND_MAX + 2.0);
                v = (float)(sqrt(-2.0 * log(u1)) * cos(6.283185307179586 * u2));
            }
            h[i] = (_Float16)v;
        }
        CHECK(hipMemcpy(tab, h, n * sizeof(_Float16), hipMemcpyHostToDevice));
        const char* nm = mode == 0 ? "all-zero operands" : mode == 1 ? "all-one operands" : "N(0,1) random operands";
        run<4>(nm, tab, cycles, sink, ncu);
        run<8>(nm, tab, cycles, sink, ncu);
    }
    return 0;
}
