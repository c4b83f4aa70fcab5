// Internal interface between the C-ABI host layer and the device code.  Not installed.
#ifndef PASA_KERNELS_H
#define PASA_KERNELS_H

#include <hip/hip_runtime.h>

// kernel precision variants; values equal the public pasa_variant enumerators
enum { PASA_K_MIXED = 0, PASA_K_STRICT16 = 1, PASA_K_NAIVE16 = 2, PASA_K_S16 = 3 };

struct PasaLaunch {
    const void* q;
    const void* ws;   // per (batch, KV head, key tile): shifted-key tile then value tile, fragment-major layout
    void* o;
    int B, Hq, Hkv, N, d;   // N: keys
    int Nq, row0;           // query rows given, and the sequence position of the first of them
    int causal;
    int variant;
    int io_bf16;      // q is read and o is written as bf16 (converted to / from the fp16 the method computes in)
    float inva;       // beta/(1-beta), already rounded to the statistics precision
    float scale;      // only used by PASA_K_NAIVE16 (static scaling after the first GEMM)
    unsigned long long* overflow_s;
    unsigned long long* nonfinite_o;
    hipStream_t stream;
};

// Shift + re-tile K (and re-tile V when v != nullptr).  plain_out != nullptr: K' goes there in the
// plain [B,Hkv,N,d] layout and ws is not written.
// in_bf16: k and v hold bf16 and are converted to fp16 as they are loaded (outputs stay fp16).
// matrix_mode == 0: K' = fp16((K - beta * tile mean) * kscale).
// matrix_mode == 1: K' = fp16(beta * K + kscale * tile sum), i.e. the product with the fp16-rounded shifting
//                   matrix a I + b (J - I) when beta carries a - b and kscale carries b (N % 128 == 0 only).
hipError_t pasa_launch_prep(const void* k, const void* v, void* ws, void* plain_out,
                            int B, int Hkv, int N, int d, double beta, double kscale, int matrix_mode, int in_bf16,
                            hipStream_t stream);

hipError_t pasa_launch_fwd(const PasaLaunch& p);

#endif
