// Measurement tool (not part of libpasa): how does the GPU hand the workgroups of a launch out to its compute units?
// The attention kernel's work order (pasa_fwd, work decode) is built on the answer.
//
// Launches workgroups with the attention kernel's footprint (512 threads, 152 KiB of LDS: one per compute unit at a
// time).  Workgroup g records the XCC, shader engine and compute unit it runs on (hardware-ID registers) and the
// wall-clock times at which it starts and ends, and in between waits len[g] microseconds, len[] being the lengths of
// the causal work items of `heads` query heads x `tiles` query tiles in the kernel's own numbering (plain longest-first
// or with the snake).  Prints: whether the XCC is g % 8; the engine sequence of the first XCD; the load every
// (XCC, engine) received; the measured end time, and the end time a simulation of the rule "within an XCD the engines
// take the workgroups in strict rotation, in index order, each workgroup waiting for a free unit of its engine" gives.
//
// usage: dispatch_probe [heads = 28] [query tiles = 32] [snake = 1]
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <stdlib.h>

#include <algorithm>
#include <map>
#include <vector>

#define CHECK(x)                                                                  \
    do {                                                                          \
        hipError_t e_ = (x);                                                      \
        if (e_ != hipSuccess) {                                                   \
            fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_));               \
            return 1;                                                             \
        }                                                                         \
    } while (0)

__global__ __launch_bounds__(512) void probe(const int* len, unsigned* hwid, unsigned* xcc, unsigned long long* t0,
                                             unsigned long long* t1)
{
    extern __shared__ char smem[];
    if (threadIdx.x == 0) {
        unsigned h, x;
        asm volatile("s_getreg_b32 %0, hwreg(HW_REG_HW_ID)" : "=s"(h));
        asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(x));
        hwid[blockIdx.x] = h;
        xcc[blockIdx.x] = x;
        const unsigned long long s = wall_clock64();
        t0[blockIdx.x] = s;
        const unsigned long long want = (unsigned long long)len[blockIdx.x] * 100ull;   // the wall clock runs at 100 MHz
        while (wall_clock64() - s < want) __builtin_amdgcn_s_sleep(8);                  // ends after len us whatever happens
        t1[blockIdx.x] = wall_clock64();
        smem[0] = 1;
    }
    __syncthreads();
}

int main(int argc, char** argv)
{
    const int heads = argc > 1 ? atoi(argv[1]) : 28, nqt = argc > 2 ? atoi(argv[2]) : 32, snake = argc > 3 ? atoi(argv[3]) : 1;
    if (heads < 4 || heads % 4 != 0 || nqt < 1 || heads * nqt > 65536 || (nqt * (heads / 4)) % 2 != 0) {
        fprintf(stderr, "heads: a multiple of 4 (four KV heads); heads / 4 * tiles even\n");
        return 2;
    }
    const int n = heads * nqt, G = heads / 4;
    std::vector<int> len(n);
    for (int g = 0; g < n; ++g) {                   // the kernel's decode for four (batch, KV head) groups
        int wg = g;
        const int x = wg & 7, r0 = wg >> 3, in_xcd = (n - x + 7) >> 3;
        if (snake && (r0 & 4) && (r0 | 3) < in_xcd) wg = ((r0 ^ 3) << 3) | x;
        const int r = wg >> 3, i = r * 2 + (x % 2);
        const int qt = nqt - 1 - i / G;
        len[g] = 4 * (2 * qt + 2) + 8;              // microseconds: 4 per tile-step (two key tiles per query tile) + 8 fixed
    }
    int* dlen;
    unsigned *dh, *dx;
    unsigned long long *d0, *d1;
    CHECK(hipMalloc(&dlen, n * 4));
    CHECK(hipMalloc(&dh, n * 4));
    CHECK(hipMalloc(&dx, n * 4));
    CHECK(hipMalloc(&d0, n * 8));
    CHECK(hipMalloc(&d1, n * 8));
    CHECK(hipMemcpy(dlen, len.data(), n * 4, hipMemcpyHostToDevice));
    CHECK(hipFuncSetAttribute((const void*)probe, hipFuncAttributeMaxDynamicSharedMemorySize, 155648));
    for (int rep = 0; rep < 2; ++rep) {             // the second launch is the one that counts
        hipLaunchKernelGGL(probe, dim3(n), dim3(512), 155648, 0, dlen, dh, dx, d0, d1);
        CHECK(hipDeviceSynchronize());
    }
    std::vector<unsigned> h(n), x(n);
    std::vector<unsigned long long> t0(n), t1(n);
    CHECK(hipMemcpy(h.data(), dh, n * 4, hipMemcpyDeviceToHost));
    CHECK(hipMemcpy(x.data(), dx, n * 4, hipMemcpyDeviceToHost));
    CHECK(hipMemcpy(t0.data(), d0, n * 8, hipMemcpyDeviceToHost));
    CHECK(hipMemcpy(t1.data(), d1, n * 8, hipMemcpyDeviceToHost));
    const unsigned long long base = *std::min_element(t0.begin(), t0.end());
    const double end_us = (*std::max_element(t1.begin(), t1.end()) - base) / 100.0;

    int xcc_ok = 0, rot_ok = 0, rot_all = 0;
    std::map<std::pair<int, int>, long> load;
    std::map<std::pair<int, int>, std::map<int, int>> units;
    std::vector<int> first_seq;
    std::vector<int> rot(8 * 4, -1);
    for (int g = 0; g < n; ++g) {
        const int xc = x[g] & 15, se = (h[g] >> 13) & 7, cu = (h[g] >> 8) & 15;
        xcc_ok += xc == (g & 7);
        load[{xc, se}] += len[g];
        units[{xc, se}][cu]++;
        if ((g & 7) == 0 && first_seq.size() < 16) first_seq.push_back(se);
        const int p = g >> 3;                       // place in the XCD's list
        if (p < 4) rot[(g & 7) * 4 + p] = se;       // the first four places fix the XCD's rotation
        else {
            ++rot_all;
            rot_ok += rot[(g & 7) * 4 + (p & 3)] == se;
        }
    }
    // simulation of the rule
    long sim_end = 0;
    int per_engine = 0;
    for (auto& u : units) per_engine = std::max(per_engine, (int)u.second.size());
    for (int xc = 0; xc < 8; ++xc) {
        std::vector<std::vector<long>> busy(4, std::vector<long>(per_engine, 0));
        int p = 0;
        for (int g = xc; g < n; g += 8, ++p) {
            auto& q = busy[p & 3];
            *std::min_element(q.begin(), q.end()) += len[g];
        }
        for (auto& q : busy) sim_end = std::max(sim_end, *std::max_element(q.begin(), q.end()));
    }
    long total = 0;
    for (int v : len) total += v;
    printf("workgroups %d (%d heads x %d query tiles, %s order), %zu (XCC, engine) pairs, up to %d compute units each\n", n, heads, nqt,
           snake ? "snake" : "plain longest-first", load.size(), per_engine);
    printf("workgroup g on XCC g %% 8: %d of %d\n", xcc_ok, n);
    printf("engines of the first XCD's workgroups, in index order:");
    for (int s : first_seq) printf(" %d", s);
    printf("\nworkgroups whose engine is the one the rotation of their XCD's first four predicts: %d of %d\n", rot_ok, rot_all);
    long lo = 1L << 60, hi = 0;
    for (auto& l : load) {
        lo = std::min(lo, l.second);
        hi = std::max(hi, l.second);
    }
    printf("load per (XCC, engine), us of work: min %ld max %ld mean %.1f\n", lo, hi, (double)total / (double)load.size());
    printf("end of the launch: measured %.2f us, simulated by the rule %ld us (+ %.2f us), mean load per compute unit %.1f us\n", end_us,
           sim_end, end_us - (double)sim_end, (double)total / (double)(load.size() * per_engine));
    return 0;
}
