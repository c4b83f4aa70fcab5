/*
 * libpasa -- PASA (online pseudo-average shifting attention, arXiv 2503.01873) forward pass for
 * AMD MI355X (gfx950).  C ABI: plain pointers and sizes, no C++ types, no exceptions.
 *
 * What is computed (paper section 1.1 problem statement, Algorithm 1):
 *     O = softmax(scale * Q K^T) V      per (batch, query head), optionally causal,
 * evaluated FlashAttention-style over key tiles of 128 keys.  Each key tile is shifted by beta times
 * its own mean along the sequence and scaled (Eq. (10), (11)), which leaves every softmax row unchanged
 * (Eq. (9)); a per-row global recovering step re-aligns the running maximum, sum and output across
 * tiles (Eq. (13)-(15), Algorithm 1 steps 1-4) so that half-precision scores stay far below 65504.
 * N need not be a multiple of 128: a ragged last tile uses its own key count as the divisor of the tile
 * mean and of the pseudo-average, which keeps Eq. (14) valid for it (the paper does not state this case).
 *
 * Layouts.  q, o: [B, Hq, N, d];  k, v: [B, Hkv, N, d].  IEEE fp16 (or bf16, see pasa_io_dtype), row-major, contiguous, DEVICE
 * pointers, 16-byte aligned.  Query head h reads KV head h / (Hq / Hkv) (grouped-query attention; the
 * paper does not discuss it).  causal != 0: key n is visible to query r iff n <= r.
 *
 * Ownership.  The caller owns every buffer, including the workspace.  The library keeps no device
 * state between calls.  q, k, v are only read; o is only written and must not alias an input.
 *
 * Streams.  `stream` is a hipStream_t passed as void* (NULL = the default stream).  Every entry point
 * only enqueues work and returns; it never synchronises the device.
 *
 * Errors.  Every function returning int returns a pasa_status.  All argument checking happens on the
 * host before anything is enqueued; on error nothing has been launched.
 */
#ifndef PASA_H
#define PASA_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PASA_OK = 0,
    PASA_EINVAL = 1,       /* null or misaligned pointer, non-positive size, Hq % Hkv != 0, bad scale / beta / variant */
    PASA_EUNSUPPORTED = 2, /* d not in {64, 128}, a length > 262144, shift_tile != 128, PASA_SHIFT_MATRIX with N % 128 != 0 */
    PASA_ELAUNCH = 3,      /* the HIP runtime refused an allocation or a launch */
    PASA_EWORKSPACE = 4    /* workspace missing, misaligned or smaller than pasa_attn_fwd_workspace() */
} pasa_status;

/* Precision allocation of the tile loop (paper section 1.2).  The matrix cores always accumulate in
 * fp32; "fp16" below means the value is rounded to fp16 (nearest-even) where Algorithm 1 marks it. */
typedef enum {
    PASA_MIXED = 0,    /* K' and P fp16 (the GEMM operands); S', row statistics and O fp32 */
    PASA_STRICT16 = 1, /* Algorithm 1 as printed: S', P, Sbar', F, all Delta terms, m, l, P V and O rounded to fp16 */
    PASA_NAIVE16 = 2,  /* no shift (beta forced to 0): raw S = Q K^T rounded to fp16, then scaled; rest fp32.
                          This is the partially low-precision FlashAttention that overflows (section 2.1, Table 4). */
    PASA_S16 = 3,      /* shifted like MIXED, S' rounded to fp16 as it leaves the matrix core, statistics and O fp32 */
    PASA_DIRECT = 4    /* NOT the paper's recovering step ("direct-bias recovery").  Same idea of a shifted K' so that the
                          scores stay small, precision allocation of MIXED, but the shift vector of a tile is the fp16
                          vector k0 = fp16(beta * mean_tile(K)), K' = fp16((K - k0) * scale), and the removed bias is
                          added back as scale * (q . k0) (legal by Eq. (9): any shift leaves softmax unchanged)
                          followed by ordinary online softmax (Eq. (4)-(8)).  There is no pseudo-average Sbar' and no
                          factor beta/(1-beta), so the rounding noise of K' is not amplified.  The other shift modes do
                          not apply to it. */
} pasa_variant;

/* How the key pre-processing loop of Algorithm 1 forms K' (Eq. (10), (11)). */
typedef enum {
    PASA_SHIFT_MEAN = 0,   /* K' = fp16((K - beta * mean_tile(K)) * scale): mean by reduction in fp64, one rounding.
                              The shifting matrix is never formed, so its entries are never rounded. */
    PASA_SHIFT_MATRIX = 1, /* Algorithm 1 as printed: K'^T = K^T M with every entry of M = I/alpha - beta J/(128 alpha),
                              alpha = 1/scale, rounded to fp16 first (the rounding that section 2.3 and Eq. (20)-(22)
                              analyse); the product is exact (fp64) and rounded to fp16 once.  Evaluated as
                              (a - b) K + b sum_tile(K) with a, b the rounded diagonal and off-diagonal entry, which
                              is the same contraction.  Needs N % 128 == 0. */
    PASA_SHIFT_MATRIX_MFMA = 2 /* The same product as a batched GEMM on the matrix core, the way Algorithm 1's pre-processing
                              loop prints it: v_mfma_f32_32x32x16_f16 with K^T and the rounded M as operands, the 128
                              products of an output accumulated in fp32, one rounding to fp16.  Differs from
                              PASA_SHIFT_MATRIX by the fp32 accumulation only (a fraction of a per cent of the K' values
                              land on the neighbouring fp16 value).  Needs N % 128 == 0; not combined with the adaptive
                              entry point. */
} pasa_shift_mode;

/* Element type of q, k, v and o.  The method computes in fp16: bf16 inputs are converted to fp16 as they are loaded
 * (round to nearest even; magnitudes beyond 65504 become infinities), as the paper prescribes for BF16 inputs, and
 * the output is rounded to bf16 when it is stored. */
typedef enum { PASA_IO_F16 = 0, PASA_IO_BF16 = 1 } pasa_io_dtype;

typedef struct {
    float beta;        /* shift fraction of Eq. (10).  < 0: library default -- by mean 63.5/64.5 (invariance beta/(1-beta) =
                          63.5, the fp16 value of the invariance of the paper's adopted beta), by matrix the paper's
                          adopted beta = 0.984497 (Table 3);  0: plain FlashAttention;  otherwise must lie in [0, 1). */
    int variant;       /* a pasa_variant */
    int shift_tile;    /* keys per pseudo-average group; 0 or 128 (the only supported size) */
    unsigned long long* overflow_s;  /* optional DEVICE counter (caller zeroes it): score-tile entries whose magnitude
                                        exceeds 65504 where they would be stored as fp16.  NULL: not counted. */
    unsigned long long* nonfinite_o; /* optional DEVICE counter (caller zeroes it): inf/NaN entries written to o. */
    int shift_mode;    /* a pasa_shift_mode */
    int io_dtype;      /* a pasa_io_dtype; applies to q, k, v, o of the call it is passed to (the workspace is always
                          fp16, so pasa_prepare_kv and the calls that use its workspace may differ in it) */
} pasa_opts;

/* Default configuration: PASA_MIXED, default beta.  Allocates and frees its workspace in stream order
 * (hipMallocAsync / hipFreeAsync).  scale multiplies Q K^T (normally 1/sqrt(d)); finite and > 0. */
int pasa_attn_fwd(const void* q, const void* k, const void* v, void* o,
                  int B, int Hq, int Hkv, int N, int d, int causal, float scale, void* stream);

/* Bytes of device workspace pasa_attn_fwd_ex needs for these sizes: shifted keys K' and re-tiled values, both fp16
 * (4*B*Hkv*ceil(N/128)*128*d bytes), then one fp16 shift vector per key tile (2*B*Hkv*ceil(N/128)*d bytes, rounded up
 * to a multiple of 256; written by PASA_DIRECT's pre-processing, in plain order), then one 64-bit counter per (batch, KV head) (8*B*Hkv
 * bytes, rounded up to a multiple of 256; used by pasa_attn_fwd_adaptive only), then for every (batch, KV head) and
 * group of 16 key tiles the per-channel means of the rounded K' of those tiles as fp16 pairs (64*d bytes per group,
 * B*Hkv*ceil(ceil(N/128)/16) groups; PASA_MIXED takes the pseudo-average of Eq. (14) as the query times that mean,
 * Eq. (12); for PASA_DIRECT the same blocks hold the tiles' shift vectors k0 instead); these regions together are pasa_attn_fwd_workspace_min().  Last comes the
 * region of the key split: when a call would launch fewer than 192 workgroups (one per 256 query rows of a head) on the
 * 256 compute units, the key tiles of every workgroup are divided among up to 16 workgroups in pieces of 16 tiles,
 * each leaves per query row its unnormalised output (d floats) and two doubles (running sum, level), and a second
 * kernel merges them with the log-sum-exp rule (the same algebra that lets the method run as ring attention, section
 * 2.2).  The region is sized for a call with N query rows (at least 1 MiB, so that short query chunks can split);
 * a call given less than that splits fewer ways or not at all, and one given less than pasa_attn_fwd_workspace_min()
 * fails with PASA_EWORKSPACE.  Not used by PASA_STRICT16 (its fp16 state has no merge rule in Algorithm 1) nor by the
 * adaptive entry point.  Returns 0 if the sizes are invalid. */
size_t pasa_attn_fwd_workspace(int B, int Hq, int Hkv, int N, int d);

/* The part of the workspace every call needs (all regions but the key split's). */
size_t pasa_attn_fwd_workspace_min(int B, int Hkv, int N, int d);

/* As pasa_attn_fwd, with options and a caller-provided workspace (DEVICE pointer, 256-byte aligned,
 * pasa_attn_fwd_workspace() bytes -- at least pasa_attn_fwd_workspace_min(); contents on return are unspecified).  opts == NULL means
 * {beta = -1, PASA_MIXED, 128, NULL, NULL, PASA_SHIFT_MEAN, PASA_IO_F16}.  Performs no allocation. */
int pasa_attn_fwd_ex(const void* q, const void* k, const void* v, void* o,
                     int B, int Hq, int Hkv, int N, int d, int causal, float scale,
                     const pasa_opts* opts, void* workspace, size_t workspace_bytes, void* stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc): pasa_attn_fwd_ex with its workspace in a fixed array of PASA_STATIC_WORKSPACE_BYTES of
 * device memory that belongs to the library (one copy per GPU the library is used on, held until the process ends).
 * Calls no hipMalloc / hipFree and no allocating routine.  PASA_EWORKSPACE if
 * pasa_attn_fwd_workspace_min(B, Hkv, N, d) exceeds PASA_STATIC_WORKSPACE_BYTES (e.g. B*Hkv*N*d > 8 Mi elements
 * for N % 128 == 0; the key split uses what the fixed regions leave of the array); otherwise arguments, options and
 * errors as pasa_attn_fwd_ex.  The device that is current at
 * the call must be the stream's.  The first call on a device looks the array's address up (no allocation, but make
 * it before a capture begins).  All calls on one GPU share the one array: calls that may overlap in time on one GPU
 * (different streams, or different threads) race on it and must be serialised by the caller; the array keeps the
 * previous call's contents, none of which a later call reads. */
#define PASA_STATIC_WORKSPACE_BYTES (33u << 20)
int pasa_attn_fwd_static(const void* q, const void* k, const void* v, void* o,
                         int B, int Hq, int Hkv, int N, int d, int causal, float scale,
                         const pasa_opts* opts, void* stream);

/* The two halves of pasa_attn_fwd_ex as separate calls, for callers that attend to the same keys and
 * values more than once (several query chunks against one K/V): pasa_prepare_kv runs Algorithm 1's
 * pre-processing loop (key shift, Eq. (11)) and re-tiles K' and V into `workspace`;
 * pasa_attn_fwd_prepared runs the main loops of Algorithm 1 against such a workspace.  Both calls must be
 * given the same B, Hkv, N, d, scale and opts (beta, variant); pasa_attn_fwd_prepared does not read k or v.
 * It reads the prepared regions and may write the key-split region at the end of the workspace, so calls that use
 * one workspace must not overlap in time.  Same argument rules, workspace size and error codes as pasa_attn_fwd_ex. */
int pasa_prepare_kv(const void* k, const void* v, int B, int Hkv, int N, int d, float scale,
                    const pasa_opts* opts, void* workspace, size_t workspace_bytes, void* stream);
int pasa_attn_fwd_prepared(const void* q, void* o, int B, int Hq, int Hkv, int N, int d, int causal, float scale,
                           const pasa_opts* opts, void* workspace, size_t workspace_bytes, void* stream);

/* The main loops of Algorithm 1 for a chunk of queries against a prepared workspace of N keys (the problem
 * statement of section 1.1 allows different query and key lengths S1 != S2; the paper does not elaborate).
 * q, o: [B, Hq, Nq, d].  Query row r sits at sequence position row0 + r: with causal != 0 it sees the keys
 * n <= row0 + r (row0 = N - Nq aligns the last query with the last key; positions past N - 1 see all keys);
 * with causal == 0 every row sees all N keys and row0 is ignored.  Covers cross-attention, prefill in chunks and
 * decoding against a cache.  pasa_attn_fwd_prepared(..., N, ...) is the case Nq = N, row0 = 0.  A row's result
 * does not depend on the other rows of its chunk: splitting a sequence at multiples of 32 rows gives bit-identical
 * output, any other split the same up to the fp32 summation order of the pseudo-average.  PASA_EINVAL for
 * Nq <= 0 or row0 < 0; otherwise the rules of pasa_attn_fwd_prepared. */
int pasa_attn_fwd_chunk(const void* q, void* o, int B, int Hq, int Hkv, int Nq, int row0, int N, int d, int causal,
                        float scale, const pasa_opts* opts, void* workspace, size_t workspace_bytes, void* stream);

/* An adaptive start of PASA (the paper's closing section names it as future work and gives no mechanism; this is
 * a simple one).  Pass 1 runs the partially low-precision FlashAttention without any shift (PASA_NAIVE16: raw
 * scores rounded to fp16, section 2.1) into o and counts the raw scores that left the fp16 range: in total in
 * *opts->overflow_s, and per (batch, KV head) in counters of its own inside the workspace.  Pass 2 runs
 * opts->variant (not PASA_NAIVE16) into o, but the workgroups of a (batch, KV head) whose counter is zero return at
 * once -- decided on the device, no host synchronisation.  So the query heads of a (batch, KV head) in which nothing
 * overflowed keep the unshifted result, and those of a (batch, KV head) in which some raw score of some query head
 * overflowed get the PASA result (the shifted keys are shared by the query heads of a KV head, so that is the
 * finest unit).  opts and opts->overflow_s (a DEVICE counter the caller has zeroed; it reports the total) are
 * required, opts->nonfinite_o must be NULL.  Otherwise the rules of pasa_attn_fwd_ex. */
int pasa_attn_fwd_adaptive(const void* q, const void* k, const void* v, void* o,
                           int B, int Hq, int Hkv, int N, int d, int causal, float scale,
                           const pasa_opts* opts, void* workspace, size_t workspace_bytes, void* stream);

/* Key pre-processing alone (Algorithm 1's first loop, Eq. (11)): writes, for every 128-key tile,
 * K'[n, c] = fp16((K[n, c] - beta * mean_tile(K[:, c])) * kscale) to kprime in the plain [B, Hkv, N, d]
 * layout.  The mean and the arithmetic are fp64 and the result is rounded once.  For tests and tools;
 * the attention entry points do this internally in their own tiled layout. */
int pasa_shift_keys(const void* k, void* kprime, int B, int Hkv, int N, int d,
                    double beta, double kscale, void* stream);

/* The same with PASA_SHIFT_MATRIX: K'^T = fp16(K^T M16), M16 the entrywise fp16 rounding of Eq. (10)'s M with
 * alpha = 1/kscale.  N must be a multiple of 128. */
int pasa_shift_keys_matrix(const void* k, void* kprime, int B, int Hkv, int N, int d,
                           double beta, double kscale, void* stream);

/* The same contraction on the matrix core (PASA_SHIFT_MATRIX_MFMA): fp32 accumulation, one rounding to fp16. */
int pasa_shift_keys_matrix_mfma(const void* k, void* kprime, int B, int Hkv, int N, int d,
                                double beta, double kscale, void* stream);

/* The shift of PASA_DIRECT: k0[b, h, t, :] = fp16(beta * mean of key tile t) ([B, Hkv, ceil(N/128), d], DEVICE, written)
 * and K' = fp16((K - k0) * kscale) in the plain layout. */
int pasa_shift_keys_direct(const void* k, void* kprime, void* k0, int B, int Hkv, int N, int d,
                           double beta, double kscale, void* stream);

/* Host-only, fp64: solves the optimal accuracy condition beta/(1-beta) = f(beta) (Eq. (16), (20)-(22)) by
 * fixed-point iteration from beta0, for a shifting matrix of size n rounded to format tp
 * (0 = fp16, 1 = bf16).  Returns NaN for invalid arguments. */
double pasa_optimal_beta(double beta0, int n, int tp);

/* Host-only: the practical invariance Inva_1 of Eq. (20) for the given beta. */
double pasa_invariance_rounded(double beta, int n, int tp);

const char* pasa_status_string(int status);
int pasa_version(void);

#ifdef __cplusplus
}
#endif
#endif /* PASA_H */
