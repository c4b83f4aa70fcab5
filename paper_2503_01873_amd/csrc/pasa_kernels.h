// Internal interface between the C-ABI host layer and the device code.  Not installed.
#ifndef PASA_KERNELS_H
#define PASA_KERNELS_H

#include <hip/hip_runtime.h>

// kernel precision variants; values equal the public pasa_variant enumerators
enum { PASA_K_MIXED = 0, PASA_K_STRICT16 = 1, PASA_K_NAIVE16 = 2, PASA_K_S16 = 3, PASA_K_DIRECT = 4 };
// how the pre-processing kernel forms K'
enum { PASA_PREP_MEAN = 0, PASA_PREP_MATRIX = 1, PASA_PREP_DIRECT = 2 };

struct PasaLaunch {
    const void* q;
    const void* ws;   // per (batch, KV head, key tile): shifted-key tile then value tile, fragment-major layout
    void* o;
    const void* kmean;  // PASA_K_MIXED: per (batch, KV head, 16 key tiles) the mean block, 32 x d halfs;
                        // PASA_K_DIRECT: the same blocks holding the tiles' shift vectors k0
    int B, Hq, Hkv, N, d;   // N: keys
    int Nq, row0;           // query rows given, and the sequence position of the first of them
    int causal;
    int variant;
    int io_bf16;      // q is read and o is written as bf16 (converted to / from the fp16 the method computes in)
    float inva;       // beta/(1-beta), already rounded to the statistics precision
    float scale;      // only used by PASA_K_NAIVE16 (static scaling after the first GEMM)
    unsigned long long* overflow_s;
    unsigned long long* nonfinite_o;
    unsigned long long* overflow_group;   // non-null: the overflow count is also added to entry b * Hkv + hk of this array
    const unsigned long long* gate;   // non-null: one device counter per (batch, KV head); a workgroup does nothing
                                      // unless the counter of its own (batch, KV head) is non-zero
    int nsplit;       // > 1: the key tiles of every (query tile, head) are swept by nsplit workgroups, whose per-row states
                      // go to part_o ([nsplit, B*Hq*Nq, d] floats) and part_lr ([nsplit, B*Hq*Nq, 2] doubles: sum, level)
                      // and are merged by a second kernel; ignored by PASA_K_STRICT16
    void* part_o;
    void* part_lr;
    hipStream_t stream;
};

// Shift + re-tile K (and re-tile V when v != nullptr).  plain_out != nullptr: K' goes there in the
// plain [B,Hkv,N,d] layout and ws is not written.
// in_bf16: k and v hold bf16 and are converted to fp16 as they are loaded (outputs stay fp16).
// gate: non-null: one device counter per (batch, KV head); a head's tiles are left untouched unless its counter is non-zero.
// PASA_PREP_MEAN:   K' = fp16((K - beta * tile mean) * kscale).
// PASA_PREP_MATRIX: K' = fp16(beta * K + kscale * tile sum), i.e. the product with the fp16-rounded shifting
//                   matrix a I + b (J - I) when beta carries a - b and kscale carries b (N % 128 == 0 only).
// PASA_PREP_DIRECT: k0 = fp16(beta * tile mean) goes to k0out ([B, Hkv, tiles, d]) and K' = fp16((K - k0) * kscale).
// k == nullptr: only V is re-tiled (the keys come from pasa_launch_shift_gemm).
// kmean_out != nullptr: also the mean blocks of the rounded K' ([B, Hkv, ceil(tiles/16), 32, d] halfs) that
// PASA_K_MIXED reads; with PASA_PREP_DIRECT the blocks hold the shift vectors k0 instead (what PASA_K_DIRECT reads).
hipError_t pasa_launch_prep(const void* k, const void* v, void* ws, void* plain_out,
                            int B, int Hkv, int N, int d, double beta, double kscale, int shift_mode, int in_bf16,
                            void* k0out, void* kmean_out, const unsigned long long* gate, hipStream_t stream);

// Algorithm 1's pre-processing loop as printed: K'^T = K^T M on the matrix core, M = a on the diagonal and b elsewhere
// (both fp16 values), fp32 accumulation, one rounding to fp16.  N % 128 == 0.  Writes the K' tiles of the workspace
// (or, plain_out != nullptr, the plain [B,Hkv,N,d] layout) and, kmean_out != nullptr, the mean blocks of that K'.
hipError_t pasa_launch_shift_gemm(const void* k, void* ws, void* plain_out, int B, int Hkv, int N, int d, double a16,
                                 double b16, int in_bf16, void* kmean_out, hipStream_t stream);

hipError_t pasa_launch_fwd(const PasaLaunch& p);

// Sets n 64-bit words to zero with a small kernel (not a memset, so that the call may sit in a captured graph).
hipError_t pasa_launch_zero(unsigned long long* p, int n, hipStream_t stream);

#endif
