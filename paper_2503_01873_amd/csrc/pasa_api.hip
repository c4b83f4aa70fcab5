// libpasa host layer: the C ABI declared in include/pasa.h.
// Argument validation, the optimal-beta solve (host, fp64) and kernel dispatch.  No kernels here; the only device
// object is the fixed workspace of pasa_attn_fwd_static.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include <mutex>

#include "pasa.h"
#include "pasa_kernels.h"

namespace {

constexpr int kShiftTile = 128;
constexpr int kMaxN = 262144;   // tile counters stay exactly representable in fp16 (STRICT16 statistics)

bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// Round x to a binary floating-point format with `prec` significand bits (including the hidden one),
// minimum normal exponent emin and maximum exponent emax (value < 2^(emax+1)); ties to even; gradual
// underflow; overflow to infinity.  fp16: (11, -14, 15).  bf16: (8, -126, 127).
double round_to_format(double x, int prec, int emin, int emax)
{
    if (x == 0.0 || isnan(x) || isinf(x)) return x;
    int e;
    frexp(x, &e);            // x = m * 2^e with 0.5 <= |m| < 1, so the leading bit has weight 2^(e-1)
    int lsb = e - prec;      // weight of the last kept bit
    if (lsb < emin - (prec - 1)) lsb = emin - (prec - 1);   // subnormal range: fixed spacing
    const double r = ldexp(nearbyint(ldexp(x, -lsb)), lsb); // nearbyint: ties to even in the default mode
    if (fabs(r) >= ldexp(1.0, emax + 1)) return copysign(INFINITY, x);
    return r;
}

double fl_tp(double x, int tp) { return tp == 0 ? round_to_format(x, 11, -14, 15) : round_to_format(x, 8, -126, 127); }

// The entries of the rounded shifting matrix of Appendix A: off-diagonal -b with b = fl(beta / n), diagonal
// a - b with a - b = fl(1 - beta / n) (Eq. (21)).  Both are step functions of beta.
struct RoundedPair {
    double a, b;
    bool operator==(const RoundedPair& o) const { return a == o.a && b == o.b; }
};

RoundedPair rounded_pair(double beta, int n, int tp)
{
    const double b = fl_tp(beta / n, tp);
    return {fl_tp(1.0 - beta / n, tp) + b, b};
}

// Eq. (20): the invariance that a*I - b*J really has, from its exact inverse (Theorem 2.1 with lambda = b / a).
double invariance_of_pair(const RoundedPair& p, int n)
{
    const double bn = p.b * n;
    return bn / (p.a * (p.a - bn)) + (1.0 - p.a) / p.a;
}

int check_shape(int B, int Hq, int Hkv, int N, int d)
{
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || N <= 0 || d <= 0) return PASA_EINVAL;
    if (Hq % Hkv != 0) return PASA_EINVAL;
    if (d != 64 && d != 128) return PASA_EUNSUPPORTED;
    if (N > kMaxN) return PASA_EUNSUPPORTED;
    return PASA_OK;
}

}  // namespace

extern "C" {

const char* pasa_status_string(int status)
{
    switch (status) {
        case PASA_OK: return "ok";
        case PASA_EINVAL: return "invalid argument";
        case PASA_EUNSUPPORTED:
            return "unsupported size (d must be 64 or 128, N <= 262144, shift tile 128, N % 128 == 0 for the matrix shift)";
        case PASA_ELAUNCH: return "HIP runtime refused an allocation or a kernel launch";
        case PASA_EWORKSPACE: return "workspace missing, misaligned or too small";
        default: return "unknown status";
    }
}

int pasa_version(void) { return 100; }

double pasa_invariance_rounded(double beta, int n, int tp)
{
    if (!(beta >= 0.0) || !(beta < 1.0) || n <= 0 || (tp != 0 && tp != 1)) return NAN;
    return invariance_of_pair(rounded_pair(beta, n, tp), n);
}

double pasa_optimal_beta(double beta0, int n, int tp)
{
    if (!(beta0 > 0.0) || !(beta0 < 1.0) || n <= 0 || (tp != 0 && tp != 1)) return NAN;
    // The optimal accuracy condition beta / (1 - beta) = f(beta) (Eq. (16)) has a right-hand side that only depends on
    // the rounded pair (a, b), which is constant on intervals of beta.  On such an interval the condition is solved in
    // closed form, beta* = f / (1 + f); beta* is a solution iff it lies in the interval it was computed for, i.e. iff
    // rounding at beta* gives the same pair again.  Starting from the pair of beta0 and moving to the pair of the
    // candidate until it reproduces itself visits the same intervals as the iteration of Eq. (22) and ends exactly.
    RoundedPair pair = rounded_pair(beta0, n, tp);
    double beta = beta0;
    for (int visited = 0; visited < 256; ++visited) {
        const double f = invariance_of_pair(pair, n);
        beta = f / (1.0 + f);
        const RoundedPair again = rounded_pair(beta, n, tp);
        if (again == pair) return beta;
        pair = again;
    }
    return beta;     // no self-consistent interval found within the budget: the last candidate, as the iteration would give
}

}  // extern "C"

namespace {

// Workspace layout: the K'/V tiles, then (written by PASA_DIRECT's pre-processing) one fp16 shift vector of d halfs per
// tile in plain order, then (used by the adaptive entry point only) one 64-bit overflow counter per (batch, KV head),
// then one block of 32 x d halfs per 16 key tiles (PASA_MIXED: the tiles' mean keys; PASA_DIRECT: their shift vectors),
// then the region of the key split: per split and query row two doubles (sum, level) and the stored output (d floats).
size_t tiles_bytes(int B, int Hkv, int N, int d)
{
    const size_t ntile = ((size_t)N + kShiftTile - 1) / kShiftTile;      // a ragged last tile is padded
    return (size_t)4 * (size_t)B * (size_t)Hkv * ntile * kShiftTile * (size_t)d;
}

size_t k0_bytes(int B, int Hkv, int N, int d)
{
    const size_t ntile = ((size_t)N + kShiftTile - 1) / kShiftTile;
    const size_t raw = (size_t)2 * (size_t)B * (size_t)Hkv * ntile * (size_t)d;
    return (raw + 255) / 256 * 256;
}

size_t group_counter_bytes(int B, int Hkv)
{
    return ((size_t)8 * (size_t)B * (size_t)Hkv + 255) / 256 * 256;
}

size_t kmean_bytes(int B, int Hkv, int N, int d)
{
    const size_t ntile = ((size_t)N + kShiftTile - 1) / kShiftTile;
    return (size_t)B * (size_t)Hkv * ((ntile + 15) / 16) * 64 * (size_t)d;     // a multiple of 256
}

size_t kmean_offset(int B, int Hkv, int N, int d)
{
    return tiles_bytes(B, Hkv, N, d) + k0_bytes(B, Hkv, N, d) + group_counter_bytes(B, Hkv);
}

// Everything but the key-split region: what a call needs at least.
size_t workspace_min_bytes(int B, int Hkv, int N, int d)
{
    return kmean_offset(B, Hkv, N, d) + kmean_bytes(B, Hkv, N, d);
}

// Key split.  A launch of fewer than 192 workgroups (256 query rows of one head each) leaves compute units idle; then
// the key tiles of every workgroup are divided among up to 256 / workgroups of them, in pieces of 16 tiles, at most 16.
constexpr int kComputeUnits = 256;      // MI355X
constexpr int kSplitBelow = 192;
constexpr int kMaxSplit = 16;
constexpr size_t kSplitFloorBytes = (size_t)1 << 20;   // always there, so that short query chunks (decoding) can split

int wanted_splits(int B, int Hq, int Nq, int N)
{
    const long units = ((long)Nq + 255) / 256 * Hq * B;
    const int nblk16 = (int)((((long)N + kShiftTile - 1) / kShiftTile + 15) / 16);
    if (units >= kSplitBelow || nblk16 < 2) return 1;
    long ns = kComputeUnits / units;
    if (ns > nblk16) ns = nblk16;
    if (ns > kMaxSplit) ns = kMaxSplit;
    return ns < 2 ? 1 : (int)ns;
}

size_t split_row_bytes(int d) { return (size_t)d * 4 + 16; }

size_t split_region_bytes(int B, int Hq, int N, int d)
{
    const int ns = wanted_splits(B, Hq, N, N);
    size_t need = ns > 1 ? (size_t)ns * (size_t)B * Hq * N * split_row_bytes(d) : 0;
    if (need < kSplitFloorBytes) need = kSplitFloorBytes;
    return (need + 255) / 256 * 256;
}

}  // namespace

extern "C" {

size_t pasa_attn_fwd_workspace(int B, int Hq, int Hkv, int N, int d)
{
    if (check_shape(B, Hq, Hkv, N, d) != PASA_OK) return 0;
    return workspace_min_bytes(B, Hkv, N, d) + split_region_bytes(B, Hq, N, d);
}

size_t pasa_attn_fwd_workspace_min(int B, int Hkv, int N, int d)
{
    if (check_shape(B, Hkv, Hkv, N, d) != PASA_OK) return 0;
    return workspace_min_bytes(B, Hkv, N, d);
}

}  // extern "C"

namespace {

// Entries of the shifting matrix M = I/alpha - beta J/(alpha T) of Eq. (10), alpha = 1/kscale, each rounded to
// fp16: a on the diagonal, b elsewhere.  The pre-processing kernel takes a - b and b.
void rounded_shift_matrix(double beta, double kscale, double* a_minus_b, double* b)
{
    const double alpha = 1.0 / kscale;
    const double off = beta / (alpha * (double)kShiftTile);
    const double a16 = round_to_format(1.0 / alpha - off, 11, -14, 15);
    const double b16 = round_to_format(0.0 - off, 11, -14, 15);
    *a_minus_b = a16 - b16;    // exact: both are fp16 values
    *b = b16;
}

int shift_keys_common(const void* k, void* kprime, int B, int Hkv, int N, int d, double beta, double kscale,
                      int shift_mode, void* k0out, void* stream)
{
    const int st = check_shape(B, Hkv, Hkv, N, d);
    if (st != PASA_OK) return st;
    if (k == nullptr || kprime == nullptr || !aligned(k, 16) || !aligned(kprime, 16) || k == kprime) return PASA_EINVAL;
    if (!(beta >= 0.0) || !(beta < 1.0) || !isfinite(kscale) || !(kscale > 0.0)) return PASA_EINVAL;
    double c1 = beta, c2 = kscale;
    if (shift_mode == PASA_PREP_MATRIX) {
        if (N % kShiftTile != 0) return PASA_EUNSUPPORTED;   // M is a full 128 x 128 matrix
        rounded_shift_matrix(beta, kscale, &c1, &c2);
    }
    if (shift_mode == PASA_PREP_DIRECT && (k0out == nullptr || !aligned(k0out, 16) || k0out == kprime || k0out == k))
        return PASA_EINVAL;
    const hipError_t e = pasa_launch_prep(k, nullptr, nullptr, kprime, B, Hkv, N, d, c1, c2, shift_mode, 0, k0out,
                                          nullptr, nullptr, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? PASA_OK : PASA_ELAUNCH;
}

}  // namespace

extern "C" {

int pasa_shift_keys(const void* k, void* kprime, int B, int Hkv, int N, int d, double beta, double kscale, void* stream)
{
    return shift_keys_common(k, kprime, B, Hkv, N, d, beta, kscale, PASA_PREP_MEAN, nullptr, stream);
}

int pasa_shift_keys_matrix(const void* k, void* kprime, int B, int Hkv, int N, int d, double beta, double kscale,
                           void* stream)
{
    return shift_keys_common(k, kprime, B, Hkv, N, d, beta, kscale, PASA_PREP_MATRIX, nullptr, stream);
}

int pasa_shift_keys_matrix_mfma(const void* k, void* kprime, int B, int Hkv, int N, int d, double beta, double kscale,
                                void* stream)
{
    const int st = check_shape(B, Hkv, Hkv, N, d);
    if (st != PASA_OK) return st;
    if (k == nullptr || kprime == nullptr || !aligned(k, 16) || !aligned(kprime, 16) || k == kprime) return PASA_EINVAL;
    if (!(beta >= 0.0) || !(beta < 1.0) || !isfinite(kscale) || !(kscale > 0.0)) return PASA_EINVAL;
    if (N % kShiftTile != 0) return PASA_EUNSUPPORTED;
    double amb, b16;
    rounded_shift_matrix(beta, kscale, &amb, &b16);
    const hipError_t e = pasa_launch_shift_gemm(k, nullptr, kprime, B, Hkv, N, d, amb + b16, b16, 0, nullptr,
                                                static_cast<hipStream_t>(stream));
    return e == hipSuccess ? PASA_OK : PASA_ELAUNCH;
}

int pasa_shift_keys_direct(const void* k, void* kprime, void* k0, int B, int Hkv, int N, int d, double beta, double kscale,
                           void* stream)
{
    return shift_keys_common(k, kprime, B, Hkv, N, d, beta, kscale, PASA_PREP_DIRECT, k0, stream);
}

namespace {

// Resolved numeric parameters of one call.
struct Params {
    int variant;
    double beta;      // shift fraction used by the pre-processing kernel (matrix mode: a - b)
    double kscale;    // factor folded into K' (matrix mode: b)
    int matrix_mode;  // K' by the fp16-rounded shifting matrix instead of by the tile mean
    int mfma_shift;   // ... and that product on the matrix core (fp32 accumulation) instead of exactly
    int io_bf16;      // q, k, v, o hold bf16
    float inva;       // beta/(1-beta) rounded to the statistics precision
    unsigned long long* overflow_s;
    unsigned long long* nonfinite_o;
    const unsigned long long* gate;   // set by the adaptive entry point only
};

int resolve(const pasa_opts* opts, float scale, Params* out)
{
    if (!isfinite(scale) || !(scale > 0.f)) return PASA_EINVAL;
    pasa_opts op = {-1.f, PASA_MIXED, kShiftTile, nullptr, nullptr, PASA_SHIFT_MEAN, PASA_IO_F16};
    if (opts != nullptr) op = *opts;
    if (op.variant < PASA_MIXED || op.variant > PASA_DIRECT) return PASA_EINVAL;
    if (op.shift_mode != PASA_SHIFT_MEAN && op.shift_mode != PASA_SHIFT_MATRIX && op.shift_mode != PASA_SHIFT_MATRIX_MFMA)
        return PASA_EINVAL;
    if (op.variant == PASA_DIRECT && op.shift_mode != PASA_SHIFT_MEAN) return PASA_EINVAL;   // it has its own shift
    if (op.io_dtype != PASA_IO_F16 && op.io_dtype != PASA_IO_BF16) return PASA_EINVAL;
    if (op.shift_tile != 0 && op.shift_tile != kShiftTile) return PASA_EUNSUPPORTED;
    if (!(op.beta < 1.f)) return PASA_EINVAL;              // also rejects NaN
    // beta and the invariance beta/(1-beta) in fp64.  Default by mean: the invariance is exactly 63.5.  Default by
    // matrix: the paper's adopted solution of the optimal accuracy condition for fp16 and n = 128 (Table 3).
    const double beta_default = op.shift_mode != PASA_SHIFT_MEAN ? 0.984497 : 63.5 / 64.5;
    double beta = op.beta < 0.f ? beta_default : (double)op.beta;
    double kscale = (double)scale;
    if (op.variant == PASA_NAIVE16) {   // no shift, static scaling applied after the first GEMM (Eq. (1), (2))
        beta = 0.0;
        kscale = 1.0;
    }
    const double inva_d = beta / (1.0 - beta);
    out->variant = op.variant;
    out->beta = beta;
    out->kscale = kscale;
    out->io_bf16 = op.io_dtype == PASA_IO_BF16;
    out->matrix_mode = op.shift_mode != PASA_SHIFT_MEAN && op.variant != PASA_NAIVE16;
    out->mfma_shift = out->matrix_mode && op.shift_mode == PASA_SHIFT_MATRIX_MFMA;
    if (out->matrix_mode) rounded_shift_matrix(beta, kscale, &out->beta, &out->kscale);
    out->inva = op.variant == PASA_STRICT16 ? (float)round_to_format(inva_d, 11, -14, 15) : (float)inva_d;
    out->overflow_s = op.overflow_s;
    out->nonfinite_o = op.nonfinite_o;
    out->gate = nullptr;
    return PASA_OK;
}

int check_workspace(const void* ws, size_t bytes, size_t need)
{
    return (ws == nullptr || !aligned(ws, 256) || bytes < need) ? PASA_EWORKSPACE : PASA_OK;
}

}  // namespace

}  // extern "C"

namespace {

int prepare_kv_impl(const void* k, const void* v, int B, int Hkv, int N, int d, float scale, const pasa_opts* opts,
                    void* workspace, size_t workspace_bytes, void* stream, const unsigned long long* gate)
{
    if (k == nullptr || v == nullptr || !aligned(k, 16) || !aligned(v, 16)) return PASA_EINVAL;
    Params pr;
    int st = resolve(opts, scale, &pr);
    if (st != PASA_OK) return st;
    pr.gate = gate;
    st = check_shape(B, Hkv, Hkv, N, d);
    if (st != PASA_OK) return st;
    if (pr.matrix_mode && N % kShiftTile != 0) return PASA_EUNSUPPORTED;   // M is a full 128 x 128 matrix
    const size_t need = workspace_min_bytes(B, Hkv, N, d);
    st = check_workspace(workspace, workspace_bytes, need);
    if (st != PASA_OK) return st;
    const int mode = pr.variant == PASA_DIRECT ? PASA_PREP_DIRECT : pr.matrix_mode ? PASA_PREP_MATRIX : PASA_PREP_MEAN;
    void* k0out = static_cast<char*>(workspace) + tiles_bytes(B, Hkv, N, d);
    void* kmean = (pr.variant == PASA_MIXED || pr.variant == PASA_DIRECT)
                      ? static_cast<char*>(workspace) + kmean_offset(B, Hkv, N, d) : nullptr;
    if (pr.mfma_shift) {
        // V by the re-tiling blocks of the pre-processing kernel, K' by the GEMM (pr.beta carries a - b, pr.kscale b)
        hipError_t e2 = pasa_launch_prep(nullptr, v, workspace, nullptr, B, Hkv, N, d, 0.0, 1.0, PASA_PREP_MEAN, pr.io_bf16,
                                         nullptr, nullptr, pr.gate, static_cast<hipStream_t>(stream));
        if (e2 == hipSuccess)
            e2 = pasa_launch_shift_gemm(k, workspace, nullptr, B, Hkv, N, d, pr.beta + pr.kscale, pr.kscale, pr.io_bf16,
                                        kmean, static_cast<hipStream_t>(stream));
        return e2 == hipSuccess ? PASA_OK : PASA_ELAUNCH;
    }
    const hipError_t e = pasa_launch_prep(k, v, workspace, nullptr, B, Hkv, N, d, pr.beta, pr.kscale, mode, pr.io_bf16,
                                          k0out, kmean, pr.gate, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? PASA_OK : PASA_ELAUNCH;
}

}  // namespace

extern "C" {

int pasa_prepare_kv(const void* k, const void* v, int B, int Hkv, int N, int d, float scale, const pasa_opts* opts,
                    void* workspace, size_t workspace_bytes, void* stream)
{
    return prepare_kv_impl(k, v, B, Hkv, N, d, scale, opts, workspace, workspace_bytes, stream, nullptr);
}

int pasa_attn_fwd_prepared(const void* q, void* o, int B, int Hq, int Hkv, int N, int d, int causal, float scale,
                           const pasa_opts* opts, void* workspace, size_t workspace_bytes, void* stream)
{
    return pasa_attn_fwd_chunk(q, o, B, Hq, Hkv, N, 0, N, d, causal, scale, opts, workspace, workspace_bytes, stream);
}

}  // extern "C"

namespace {

int fwd_chunk_impl(const void* q, void* o, int B, int Hq, int Hkv, int Nq, int row0, int N, int d, int causal,
                   float scale, const pasa_opts* opts, void* workspace, size_t workspace_bytes, void* stream,
                   unsigned long long* overflow_group, const unsigned long long* gate)
{
    if (q == nullptr || o == nullptr || !aligned(q, 16) || !aligned(o, 16) || o == q) return PASA_EINVAL;
    if (causal != 0 && causal != 1) return PASA_EINVAL;
    if (Nq <= 0 || row0 < 0) return PASA_EINVAL;
    Params pr;
    int st = resolve(opts, scale, &pr);
    if (st != PASA_OK) return st;
    st = check_shape(B, Hq, Hkv, N, d);
    if (st != PASA_OK) return st;
    if (Nq > kMaxN || row0 > kMaxN) return PASA_EUNSUPPORTED;
    if (pr.matrix_mode && N % kShiftTile != 0) return PASA_EUNSUPPORTED;
    const size_t need = workspace_min_bytes(B, Hkv, N, d);
    st = check_workspace(workspace, workspace_bytes, need);
    if (st != PASA_OK) return st;
    PasaLaunch p;
    p.q = q; p.ws = workspace; p.o = o;
    p.kmean = static_cast<const char*>(workspace) + kmean_offset(B, Hkv, N, d);
    p.B = B; p.Hq = Hq; p.Hkv = Hkv; p.N = N; p.d = d;
    p.Nq = Nq; p.row0 = causal ? row0 : 0;
    p.causal = causal;
    p.variant = pr.variant;
    p.io_bf16 = pr.io_bf16;
    p.inva = pr.inva;
    p.scale = scale;
    p.overflow_s = pr.overflow_s;
    p.nonfinite_o = pr.nonfinite_o;
    p.overflow_group = overflow_group;
    p.gate = gate;
    // key split: as many ways as the rule wants and the bytes behind the fixed regions hold
    int ns = (gate != nullptr || pr.variant == PASA_STRICT16) ? 1 : wanted_splits(B, Hq, Nq, N);
    const size_t rows_all = (size_t)B * Hq * Nq, room = workspace_bytes - need;
    while (ns > 1 && (size_t)ns * rows_all * split_row_bytes(d) > room) --ns;
    p.nsplit = ns;
    char* split_base = static_cast<char*>(workspace) + need;
    p.part_lr = split_base;                                              // [ns][rows][2] doubles
    p.part_o = split_base + (size_t)ns * rows_all * 16;                  // [ns][rows][d] floats
    p.stream = static_cast<hipStream_t>(stream);
    return pasa_launch_fwd(p) == hipSuccess ? PASA_OK : PASA_ELAUNCH;
}

}  // namespace

extern "C" {

int pasa_attn_fwd_chunk(const void* q, void* o, int B, int Hq, int Hkv, int Nq, int row0, int N, int d, int causal,
                        float scale, const pasa_opts* opts, void* workspace, size_t workspace_bytes, void* stream)
{
    return fwd_chunk_impl(q, o, B, Hq, Hkv, Nq, row0, N, d, causal, scale, opts, workspace, workspace_bytes, stream,
                          nullptr, nullptr);
}

int pasa_attn_fwd_adaptive(const void* q, const void* k, const void* v, void* o, int B, int Hq, int Hkv, int N, int d,
                           int causal, float scale, const pasa_opts* opts, void* workspace, size_t workspace_bytes,
                           void* stream)
{
    // every check of both passes first, so that nothing is enqueued on error
    if (q == nullptr || k == nullptr || v == nullptr || o == nullptr) return PASA_EINVAL;
    if (!aligned(q, 16) || !aligned(k, 16) || !aligned(v, 16) || !aligned(o, 16)) return PASA_EINVAL;
    if (o == q || o == k || o == v) return PASA_EINVAL;
    if (causal != 0 && causal != 1) return PASA_EINVAL;
    if (opts == nullptr || opts->overflow_s == nullptr || !aligned(opts->overflow_s, 8)) return PASA_EINVAL;
    if (opts->nonfinite_o != nullptr || opts->variant == PASA_NAIVE16) return PASA_EINVAL;
    if (opts->shift_mode == PASA_SHIFT_MATRIX_MFMA) return PASA_EINVAL;    // the GEMM pre-pass has no per-head gate
    Params pr;
    int st = resolve(opts, scale, &pr);
    if (st != PASA_OK) return st;
    st = check_shape(B, Hq, Hkv, N, d);
    if (st != PASA_OK) return st;
    if (pr.matrix_mode && N % kShiftTile != 0) return PASA_EUNSUPPORTED;
    st = check_workspace(workspace, workspace_bytes, workspace_min_bytes(B, Hkv, N, d));
    if (st != PASA_OK) return st;
    // the per-(batch, KV head) counters live behind the tiles and the shift vectors; cleared by a small kernel
    unsigned long long* group_cnt = reinterpret_cast<unsigned long long*>(
        static_cast<char*>(workspace) + tiles_bytes(B, Hkv, N, d) + k0_bytes(B, Hkv, N, d));
    if (pasa_launch_zero(group_cnt, B * Hkv, static_cast<hipStream_t>(stream)) != hipSuccess) return PASA_ELAUNCH;
    // pass 1: no shift, raw scores rounded to fp16, counting those that leave the fp16 range -- in total (the
    // caller's counter) and per (batch, KV head)
    pasa_opts first = *opts;
    first.variant = PASA_NAIVE16;
    first.shift_mode = PASA_SHIFT_MEAN;
    first.beta = -1.f;
    st = prepare_kv_impl(k, v, B, Hkv, N, d, scale, &first, workspace, workspace_bytes, stream, nullptr);
    if (st != PASA_OK) return st;
    st = fwd_chunk_impl(q, o, B, Hq, Hkv, N, 0, N, d, causal, scale, &first, workspace, workspace_bytes, stream,
                        group_cnt, nullptr);
    if (st != PASA_OK) return st;
    // pass 2: the caller's variant; the workgroups of a (batch, KV head) whose counter is zero leave at once, so its
    // query heads keep the result of pass 1
    pasa_opts second = *opts;
    second.overflow_s = nullptr;
    st = prepare_kv_impl(k, v, B, Hkv, N, d, scale, &second, workspace, workspace_bytes, stream, group_cnt);
    if (st != PASA_OK) return st;
    return fwd_chunk_impl(q, o, B, Hq, Hkv, N, 0, N, d, causal, scale, &second, workspace, workspace_bytes, stream,
                          nullptr, group_cnt);
}

int pasa_attn_fwd_ex(const void* q, const void* k, const void* v, void* o, int B, int Hq, int Hkv, int N, int d,
                     int causal, float scale, const pasa_opts* opts, void* workspace, size_t workspace_bytes,
                     void* stream)
{
    // all checks of both halves first, so that nothing is enqueued on error
    if (q == nullptr || k == nullptr || v == nullptr || o == nullptr) return PASA_EINVAL;
    if (!aligned(q, 16) || !aligned(k, 16) || !aligned(v, 16) || !aligned(o, 16)) return PASA_EINVAL;
    if (o == q || o == k || o == v) return PASA_EINVAL;
    if (causal != 0 && causal != 1) return PASA_EINVAL;
    Params pr;
    int st = resolve(opts, scale, &pr);
    if (st != PASA_OK) return st;
    st = check_shape(B, Hq, Hkv, N, d);
    if (st != PASA_OK) return st;
    if (pr.matrix_mode && N % kShiftTile != 0) return PASA_EUNSUPPORTED;
    st = check_workspace(workspace, workspace_bytes, workspace_min_bytes(B, Hkv, N, d));
    if (st != PASA_OK) return st;
    st = pasa_prepare_kv(k, v, B, Hkv, N, d, scale, opts, workspace, workspace_bytes, stream);
    if (st != PASA_OK) return st;
    return pasa_attn_fwd_prepared(q, o, B, Hq, Hkv, N, d, causal, scale, opts, workspace, workspace_bytes, stream);
}

int pasa_attn_fwd(const void* q, const void* k, const void* v, void* o, int B, int Hq, int Hkv, int N, int d,
                  int causal, float scale, void* stream)
{
    // validate before allocating anything: run the checks of the _ex entry point against a dummy workspace size
    const int st = check_shape(B, Hq, Hkv, N, d);
    if (q == nullptr || k == nullptr || v == nullptr || o == nullptr) return PASA_EINVAL;
    if (st != PASA_OK) return st;
    const size_t need = pasa_attn_fwd_workspace(B, Hq, Hkv, N, d);
    hipStream_t s = static_cast<hipStream_t>(stream);
    void* ws = nullptr;
    if (hipMallocAsync(&ws, need, s) != hipSuccess || ws == nullptr) {
        (void)hipGetLastError();
        return PASA_ELAUNCH;
    }
    const int rc = pasa_attn_fwd_ex(q, k, v, o, B, Hq, Hkv, N, d, causal, scale, nullptr, ws, need, stream);
    if (hipFreeAsync(ws, s) != hipSuccess) {
        (void)hipGetLastError();
        return rc == PASA_OK ? PASA_ELAUNCH : rc;
    }
    return rc;
}

}  // extern "C"

// ---------------------------------------------------------------------------------------------
// The entry point that allocates nothing.  Its workspace (shifted keys, re-tiled values, shift vectors) is this
// fixed array in device memory; every GPU the library is used on holds its own copy at its own address until the
// process ends.  In host code the array's name only stands for the symbol: the address on the current device comes
// from hipGetSymbolAddress, once per device, and only that address is handed to the kernels.
// ---------------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[PASA_STATIC_WORKSPACE_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices];   // device address of `scratch` on each GPU, filled on the first call there

int static_scratch(void** out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        return PASA_ELAUNCH;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) {
            (void)hipGetLastError();
            return PASA_ELAUNCH;
        }
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return PASA_OK;
}

}  // namespace

extern "C" int pasa_attn_fwd_static(const void* q, const void* k, const void* v, void* o, int B, int Hq, int Hkv, int N,
                                    int d, int causal, float scale, const pasa_opts* opts, void* stream)
{
    const int st = check_shape(B, Hq, Hkv, N, d);
    if (st != PASA_OK) return st;
    // sizes beyond the fixed array are refused before anything else is looked at; what the fixed regions leave of the
    // array serves the key split
    const size_t need = workspace_min_bytes(B, Hkv, N, d);
    if (need == 0 || need > (size_t)PASA_STATIC_WORKSPACE_BYTES) return PASA_EWORKSPACE;
    void* ws = nullptr;
    const int sp = static_scratch(&ws);
    if (sp != PASA_OK) return sp;
    // every byte of the workspace that the main kernel reads is rewritten by the pre-processing kernel of the same
    // call (the padding keys of a ragged last tile included), so nothing has to be cleared between calls
    return pasa_attn_fwd_ex(q, k, v, o, B, Hq, Hkv, N, d, causal, scale, opts, ws, (size_t)PASA_STATIC_WORKSPACE_BYTES,
                            stream);
}
