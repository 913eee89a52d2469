// extern "C" entry points of libmaddness: argument checks, then the launchers.
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <atomic>

#include "common.h"

namespace maddness {

static thread_local char g_error[512] = "";

int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof(g_error), fmt, ap);
    va_end(ap);
    return code;
}

static thread_local const char *g_kernel_family = nullptr;
static thread_local const char *g_kernel_instance = nullptr;
static thread_local char g_kernel_text[320] = "";

void note_kernel(const char *family, const char *instance)
{
    if (g_kernel_family) return;
    g_kernel_family = family;
    g_kernel_instance = instance;
}

// every launching entry point starts with this
static void begin_call() { g_kernel_family = g_kernel_instance = nullptr; }

int check_hip(hipError_t e, const char *what)
{
    if (e == hipSuccess) return MADDNESS_OK;
    return fail(MADDNESS_E_HIP, "%s: %s", what, hipGetErrorString(e));
}

const DeviceInfo &device_info()
{
    static DeviceInfo info = [] {
        DeviceInfo d{256, 65536};
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) == hipSuccess) {
            if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
                d.cus = v;
            if (hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) == hipSuccess &&
                v > 0)
                d.lds_per_block = v;
        }
        return d;
    }();
    return info;
}

// The switches of maddness_set_option, all 0 at start ("the library chooses").
constexpr int kOptions = 4;
static std::atomic<int32_t> g_options[kOptions];

int32_t option(int which) { return g_options[which].load(std::memory_order_relaxed); }

bool vector_scan_only() { return option(MADDNESS_OPT_KERNELS) >= MADDNESS_KERNELS_NO_MATRIX_CORES; }

namespace {

bool aligned(const void *p, size_t a) { return reinterpret_cast<uintptr_t>(p) % a == 0; }

bool general_kernels_only() { return option(MADDNESS_OPT_KERNELS) == MADDNESS_KERNELS_GENERAL; }

int check_params(const maddness_params *p, bool need_tree, bool need_protos)
{
    if (!p) return fail(MADDNESS_E_INVAL, "params is NULL");
    if (p->D < 1) return fail(MADDNESS_E_INVAL, "params.D = %d, must be >= 1", p->D);
    if (p->C < 1 || p->C > MADDNESS_MAX_C)
        return fail(MADDNESS_E_UNSUPPORTED, "params.C = %d, supported range is 1..%d", p->C, MADDNESS_MAX_C);
    if (need_tree) {
        if (!p->split_dims || !p->thresholds)
            return fail(MADDNESS_E_INVAL, "params.split_dims / params.thresholds is NULL");
        if (!aligned(p->split_dims, 4) || !aligned(p->thresholds, 4))
            return fail(MADDNESS_E_ALIGN, "params.split_dims / params.thresholds not 4-byte aligned");
    }
    if (need_protos) {
        if (!p->prototypes) return fail(MADDNESS_E_INVAL, "params.prototypes is NULL");
        if (!aligned(p->prototypes, 4)) return fail(MADDNESS_E_ALIGN, "params.prototypes not 4-byte aligned");
    }
    return MADDNESS_OK;
}

int check_A(const void *A, int32_t dtype, int32_t layout, int64_t N, int64_t lda, int D, MatrixA &desc)
{
    if (dtype < MADDNESS_F32 || dtype > MADDNESS_U8) return fail(MADDNESS_E_INVAL, "dtype = %d is not a maddness_dtype", dtype);
    if (layout != MADDNESS_ROW_MAJOR && layout != MADDNESS_COL_MAJOR)
        return fail(MADDNESS_E_INVAL, "layout = %d is not a maddness_layout", layout);
    if (N < 0) return fail(MADDNESS_E_INVAL, "N = %lld is negative", (long long)N);
    if (layout == MADDNESS_ROW_MAJOR && lda < D)
        return fail(MADDNESS_E_INVAL, "lda = %lld is smaller than D = %d", (long long)lda, D);
    if (layout == MADDNESS_COL_MAJOR && lda < N)
        return fail(MADDNESS_E_INVAL, "lda = %lld is smaller than N = %lld (A stored by columns)", (long long)lda,
                    (long long)N);
    if (N > 0 && !A) return fail(MADDNESS_E_INVAL, "A is NULL");
    desc.data = A; desc.dtype = dtype; desc.col_major = layout == MADDNESS_COL_MAJOR; desc.ld = lda;
    if (!aligned(A, (size_t)desc.elem_bytes()))
        return fail(MADDNESS_E_ALIGN, "A not aligned to its element size (%d bytes)", desc.elem_bytes());
    return MADDNESS_OK;
}

int check_scan(int32_t C, int32_t M, int64_t N, const uint8_t *luts, const float *scale,
               const float *offset, const float *out, int64_t ldo, const uint16_t *acc)
{
    if (C < 1 || C > MADDNESS_MAX_C)
        return fail(MADDNESS_E_UNSUPPORTED, "C = %d, supported range is 1..%d", C, MADDNESS_MAX_C);
    if (M < 1) return fail(MADDNESS_E_INVAL, "M = %d, must be >= 1", M);
    if (N < 0) return fail(MADDNESS_E_INVAL, "N = %lld is negative", (long long)N);
    if (!luts || !scale || !offset) return fail(MADDNESS_E_INVAL, "luts / scale / offset is NULL");
    if (N > 0 && !out && !acc) return fail(MADDNESS_E_INVAL, "both out and acc are NULL");
    if (out && ldo < M) return fail(MADDNESS_E_INVAL, "ldo = %lld is smaller than M = %d", (long long)ldo, M);
    if (!aligned(scale, 4) || !aligned(offset, 4) || !aligned(out, 4))
        return fail(MADDNESS_E_ALIGN, "scale / offset / out not 4-byte aligned");
    if (!aligned(acc, 2)) return fail(MADDNESS_E_ALIGN, "acc not 2-byte aligned");
    return MADDNESS_OK;
}

}  // namespace
}  // namespace maddness

using namespace maddness;

extern "C" {

static int encode_checked(const maddness_params *params, const void *A, int32_t dtype, int32_t layout,
                          int64_t N, int64_t lda, uint8_t *codes, void *stream)
{
    begin_call();
    int rc = check_params(params, true, false);
    if (rc != MADDNESS_OK) return rc;
    MatrixA desc;
    if ((rc = check_A(A, dtype, layout, N, lda, params->D, desc)) != MADDNESS_OK) return rc;
    if (N == 0) return MADDNESS_OK;
    if (!codes) return fail(MADDNESS_E_INVAL, "codes is NULL");
    if (!general_kernels_only()) {
        rc = desc.col_major ? launch_encode_cols(*params, desc, N, codes, static_cast<hipStream_t>(stream))
                            : launch_encode_rows(*params, desc, N, codes, static_cast<hipStream_t>(stream));
        if (rc != 1) return rc;
    }
    return launch_encode(*params, desc, N, codes, static_cast<hipStream_t>(stream));
}

int maddness_encode(const maddness_params *params, const float *A, int64_t N, int64_t lda,
                    uint8_t *codes, void *stream)
{
    return encode_checked(params, A, MADDNESS_F32, MADDNESS_ROW_MAJOR, N, lda, codes, stream);
}

int maddness_encode_typed(const maddness_params *params, const void *A, int32_t dtype, int32_t layout,
                          int64_t N, int64_t lda, uint8_t *codes, void *stream)
{
    return encode_checked(params, A, dtype, layout, N, lda, codes, stream);
}

size_t maddness_build_luts_workspace(int32_t D, int32_t C, int32_t M)
{
    if (D < 1 || C < 1 || M < 1) return 0;
    return build_luts_workspace_bytes(D, C, M);
}

static int build_luts_checked(const maddness_params *params, const float *B, int32_t M, int64_t ldb,
                              uint8_t *luts, float *scale, float *offset, void *workspace,
                              size_t workspace_bytes, bool pooled, void *stream)
{
    begin_call();
    int rc = check_params(params, false, true);
    if (rc != MADDNESS_OK) return rc;
    if (M < 1) return fail(MADDNESS_E_INVAL, "M = %d, must be >= 1", M);
    if (ldb < M) return fail(MADDNESS_E_INVAL, "ldb = %lld is smaller than M = %d", (long long)ldb, M);
    if (!B || !luts || !scale || !offset) return fail(MADDNESS_E_INVAL, "B / luts / scale / offset is NULL");
    if (!aligned(B, 4) || !aligned(scale, 4) || !aligned(offset, 4))
        return fail(MADDNESS_E_ALIGN, "B / scale / offset not 4-byte aligned");
    const size_t need = build_luts_workspace_bytes(params->D, params->C, M);
    if (!workspace || workspace_bytes < need)
        return fail(MADDNESS_E_UNSUPPORTED, "workspace of %zu bytes given, %zu needed", workspace_bytes, need);
    if (!aligned(workspace, 8)) return fail(MADDNESS_E_ALIGN, "workspace not 8-byte aligned");
    return launch_build_luts(*params, B, M, ldb, luts, scale, offset, workspace, pooled,
                             static_cast<hipStream_t>(stream));
}

int maddness_build_luts(const maddness_params *params, const float *B, int32_t M, int64_t ldb,
                        uint8_t *luts, float *scale, float *offset, void *workspace,
                        size_t workspace_bytes, void *stream)
{
    return build_luts_checked(params, B, M, ldb, luts, scale, offset, workspace, workspace_bytes, false, stream);
}

int maddness_build_luts_pooled(const maddness_params *params, const float *B, int32_t M, int64_t ldb,
                               uint8_t *luts, float *scale, float *offset, void *workspace,
                               size_t workspace_bytes, void *stream)
{
    return build_luts_checked(params, B, M, ldb, luts, scale, offset, workspace, workspace_bytes, true, stream);
}

int maddness_build_luts_static(const maddness_params *params, const float *B, int32_t M, int64_t ldb,
                               uint8_t *luts, float *scale, float *offset, void *stream)
{
    // argument errors first, as in maddness_build_luts (the workspace cannot be wrong yet)
    int rc = check_params(params, false, true);
    if (rc != MADDNESS_OK) return rc;
    if (M < 1) return fail(MADDNESS_E_INVAL, "M = %d, must be >= 1", M);
    const size_t need = build_luts_workspace_bytes(params->D, params->C, M);
    if (need > (size_t)MADDNESS_STATIC_WORKSPACE_BYTES)
        return fail(MADDNESS_E_UNSUPPORTED,
                    "tables of C = %d codebooks and M = %d columns need a workspace of %zu bytes; "
                    "maddness_build_luts_static holds %zu (use maddness_build_luts with a workspace of your own)",
                    params->C, M, need, (size_t)MADDNESS_STATIC_WORKSPACE_BYTES);
    void *workspace = nullptr;
    if ((rc = static_workspace(&workspace)) != MADDNESS_OK) return rc;
    return build_luts_checked(params, B, M, ldb, luts, scale, offset, workspace, MADDNESS_STATIC_WORKSPACE_BYTES,
                              false, stream);
}

static int check_averaged(int32_t C)
{
    if (C % 16 != 0)
        return fail(MADDNESS_E_UNSUPPORTED, "averaged aggregation works on blocks of 16 codebooks: C must be a multiple of 16");
    return MADDNESS_OK;
}

static int scan_checked(int32_t C, int32_t M, const uint8_t *codes, int64_t N, const uint8_t *luts,
                 const float *scale, const float *offset, float *out, int64_t ldo, uint16_t *acc,
                 bool averaged, void *stream)
{
    begin_call();
    int rc = check_scan(C, M, N, luts, scale, offset, out, ldo, acc);
    if (rc != MADDNESS_OK) return rc;
    if (averaged && (rc = check_averaged(C)) != MADDNESS_OK) return rc;
    if (N == 0) return MADDNESS_OK;
    if (!codes) return fail(MADDNESS_E_INVAL, "codes is NULL");
    if (!general_kernels_only()) {
        if (!averaged && !vector_scan_only()) {
            rc = launch_scan_mfma(C, M, codes, N, luts, scale, offset, out, ldo, acc, static_cast<hipStream_t>(stream));
            if (rc != 1) return rc;
        }
        rc = launch_scan_rows(C, M, codes, N, luts, scale, offset, out, ldo, acc, averaged,
                              static_cast<hipStream_t>(stream));
        if (rc != 1) return rc;
    }
    return launch_scan(nullptr, nullptr, codes, C, M, N, luts, scale, offset, out, ldo, acc, nullptr,
                       averaged, static_cast<hipStream_t>(stream));
}

static int encode_scan_checked(const maddness_params *params, const void *A, int32_t dtype, int32_t layout,
                               int64_t N, int64_t lda, int32_t M, const uint8_t *luts, const float *scale,
                               const float *offset, float *out, int64_t ldo, uint16_t *acc, uint8_t *codes,
                               bool averaged, void *stream)
{
    begin_call();
    int rc = check_params(params, true, false);
    if (rc != MADDNESS_OK) return rc;
    MatrixA desc;
    if ((rc = check_A(A, dtype, layout, N, lda, params->D, desc)) != MADDNESS_OK) return rc;
    if ((rc = check_scan(params->C, M, N, luts, scale, offset, out, ldo, acc)) != MADDNESS_OK) return rc;
    if (averaged && (rc = check_averaged(params->C)) != MADDNESS_OK) return rc;
    if (N == 0) return MADDNESS_OK;
    if (!general_kernels_only()) {
        hipStream_t st = static_cast<hipStream_t>(stream);
        rc = desc.col_major
                 ? launch_fused_cols(*params, desc, N, M, luts, scale, offset, out, ldo, acc, codes, averaged, st)
                 : launch_fused_rows(*params, desc, N, M, luts, scale, offset, out, ldo, acc, codes, averaged, st);
        if (rc != 1) return rc;
    }
    return launch_scan(params, &desc, nullptr, params->C, M, N, luts, scale, offset, out, ldo, acc, codes,
                       averaged, static_cast<hipStream_t>(stream));
}

int maddness_scan(int32_t C, int32_t M, const uint8_t *codes, int64_t N, const uint8_t *luts,
                  const float *scale, const float *offset, float *out, int64_t ldo, uint16_t *acc,
                  void *stream)
{
    return scan_checked(C, M, codes, N, luts, scale, offset, out, ldo, acc, false, stream);
}

int maddness_scan_averaged(int32_t C, int32_t M, const uint8_t *codes, int64_t N, const uint8_t *luts,
                           const float *scale, const float *offset, float *out, int64_t ldo,
                           uint16_t *acc, void *stream)
{
    return scan_checked(C, M, codes, N, luts, scale, offset, out, ldo, acc, true, stream);
}

int maddness_encode_scan(const maddness_params *params, const float *A, int64_t N, int64_t lda,
                         int32_t M, const uint8_t *luts, const float *scale, const float *offset,
                         float *out, int64_t ldo, uint16_t *acc, uint8_t *codes, void *stream)
{
    return encode_scan_checked(params, A, MADDNESS_F32, MADDNESS_ROW_MAJOR, N, lda, M, luts, scale, offset, out,
                               ldo, acc, codes, false, stream);
}

int maddness_encode_scan_typed(const maddness_params *params, const void *A, int32_t dtype, int32_t layout,
                               int64_t N, int64_t lda, int32_t M, const uint8_t *luts, const float *scale,
                               const float *offset, float *out, int64_t ldo, uint16_t *acc, uint8_t *codes,
                               void *stream)
{
    return encode_scan_checked(params, A, dtype, layout, N, lda, M, luts, scale, offset, out, ldo, acc, codes,
                               false, stream);
}

int maddness_encode_scan_averaged(const maddness_params *params, const float *A, int64_t N, int64_t lda,
                                  int32_t M, const uint8_t *luts, const float *scale,
                                  const float *offset, float *out, int64_t ldo, uint16_t *acc,
                                  uint8_t *codes, void *stream)
{
    return encode_scan_checked(params, A, MADDNESS_F32, MADDNESS_ROW_MAJOR, N, lda, M, luts, scale, offset, out,
                               ldo, acc, codes, true, stream);
}

// common checks of the two learning calls; returns the widest subspace in *dmax
static int check_learn(const float *A, int64_t N, int64_t lda, int32_t D, int32_t C, const int32_t *bounds, int32_t *dmax)
{
    if (D < 1) return fail(MADDNESS_E_INVAL, "D = %d, must be >= 1", D);
    if (C < 1 || C > MADDNESS_MAX_C) return fail(MADDNESS_E_UNSUPPORTED, "C = %d, supported range is 1..%d", C, MADDNESS_MAX_C);
    if (N < 1) return fail(MADDNESS_E_INVAL, "N = %lld training rows, must be >= 1", (long long)N);
    if (N >= (1LL << 29)) return fail(MADDNESS_E_UNSUPPORTED, "N = %lld training rows, at most 2^29 - 1", (long long)N);
    if (lda < D) return fail(MADDNESS_E_INVAL, "lda = %lld is smaller than D = %d", (long long)lda, D);
    if (!A || !bounds) return fail(MADDNESS_E_INVAL, "A_train / subspace_bounds is NULL");
    if (!aligned(A, 4)) return fail(MADDNESS_E_ALIGN, "A_train not 4-byte aligned");
    *dmax = 0;
    for (int c = 0; c < C; ++c) {
        const int lo = bounds[2 * c], hi = bounds[2 * c + 1];
        if (lo < 0 || hi <= lo || hi > D)
            return fail(MADDNESS_E_INVAL, "subspace of codebook %d is [%d, %d): must be non-empty and inside [0, %d)", c, lo, hi, D);
        if (hi - lo > *dmax) *dmax = hi - lo;
    }
    return MADDNESS_OK;
}

size_t maddness_learn_trees_workspace(int64_t N, int32_t D, int32_t C, const int32_t *subspace_bounds)
{
    int32_t dmax = 0;
    if (N < 1 || D < 1 || C < 1 || C > MADDNESS_MAX_C || !subspace_bounds) return 0;
    for (int c = 0; c < C; ++c) {
        const int w = subspace_bounds[2 * c + 1] - subspace_bounds[2 * c];
        if (w < 1) return 0;
        if (w > dmax) dmax = w;
    }
    return learn_trees_workspace_bytes(N, C, dmax);
}

int maddness_learn_trees(const float *A_train, int64_t N, int64_t lda, int32_t D, int32_t C,
                         const int32_t *subspace_bounds, int32_t *split_dims, float *thresholds,
                         uint8_t *train_codes, void *workspace, size_t workspace_bytes, void *stream)
{
    begin_call();
    int32_t dmax = 0;
    int rc = check_learn(A_train, N, lda, D, C, subspace_bounds, &dmax);
    if (rc != MADDNESS_OK) return rc;
    if (!split_dims || !thresholds) return fail(MADDNESS_E_INVAL, "split_dims / thresholds is NULL");
    if (!aligned(split_dims, 4) || !aligned(thresholds, 4)) return fail(MADDNESS_E_ALIGN, "split_dims / thresholds not 4-byte aligned");
    if (dmax > learn_max_subspace_width())
        return fail(MADDNESS_E_UNSUPPORTED, "a subspace of %d columns: the GPU learner takes at most %d", dmax,
                    learn_max_subspace_width());
    const size_t need = learn_trees_workspace_bytes(N, C, dmax);
    if (!workspace || workspace_bytes < need)
        return fail(MADDNESS_E_UNSUPPORTED, "workspace of %zu bytes given, %zu needed", workspace_bytes, need);
    if (!aligned(workspace, 256)) return fail(MADDNESS_E_ALIGN, "workspace not 256-byte aligned");
    return launch_learn_trees(A_train, N, lda, C, subspace_bounds, dmax, split_dims, thresholds, train_codes, workspace,
                              static_cast<hipStream_t>(stream));
}

size_t maddness_learn_prototypes_workspace(int32_t D, int32_t C)
{
    if (D < 1 || C < 1 || C > MADDNESS_MAX_C) return 0;
    return learn_prototypes_workspace_bytes(D, C);
}

int maddness_learn_prototypes(const uint8_t *train_codes, const float *A_train, int64_t N, int64_t lda, int32_t D,
                              int32_t C, const int32_t *subspace_bounds, int32_t ridge, double lambda,
                              float *prototypes, void *workspace, size_t workspace_bytes, void *stream)
{
    begin_call();
    int32_t dmax = 0;
    int rc = check_learn(A_train, N, lda, D, C, subspace_bounds, &dmax);
    if (rc != MADDNESS_OK) return rc;
    if (!train_codes || !prototypes) return fail(MADDNESS_E_INVAL, "train_codes / prototypes is NULL");
    if (!aligned(prototypes, 4)) return fail(MADDNESS_E_ALIGN, "prototypes not 4-byte aligned");
    if (ridge && !(lambda > 0.0)) return fail(MADDNESS_E_INVAL, "lambda = %g: the ridge penalty must be positive", lambda);
    const size_t need = learn_prototypes_workspace_bytes(D, C);
    if (!workspace || workspace_bytes < need)
        return fail(MADDNESS_E_UNSUPPORTED, "workspace of %zu bytes given, %zu needed", workspace_bytes, need);
    if (!aligned(workspace, 256)) return fail(MADDNESS_E_ALIGN, "workspace not 256-byte aligned");
    return launch_learn_prototypes(train_codes, A_train, N, lda, D, C, subspace_bounds, ridge != 0, lambda, prototypes,
                                   workspace, static_cast<hipStream_t>(stream));
}

int maddness_set_option(int32_t opt, int32_t value)
{
    bool ok;
    switch (opt) {
    case MADDNESS_OPT_KERNELS: ok = value >= MADDNESS_KERNELS_AUTO && value <= MADDNESS_KERNELS_GENERAL; break;
    case MADDNESS_OPT_PHASED_ROWS: ok = value == 0 || value >= 2; break;
    case MADDNESS_OPT_COLS_RUN: ok = value == 0 || value == 1 || value == 2 || value == 4; break;
    case MADDNESS_OPT_MAX_WORKGROUPS: ok = value >= 0; break;
    default: return fail(MADDNESS_E_INVAL, "option %d is not a maddness_option", opt);
    }
    if (!ok) return fail(MADDNESS_E_INVAL, "value %d is not valid for option %d", value, opt);
    g_options[opt].store(value, std::memory_order_relaxed);
    return MADDNESS_OK;
}

int32_t maddness_get_option(int32_t opt)
{
    if (opt < 0 || opt >= kOptions) return -1;
    return option(opt);
}

const char *maddness_last_error(void) { return g_error; }

const char *maddness_last_kernel(void)
{
    if (!g_kernel_family) return "";
    const char *args = g_kernel_instance ? strrchr(g_kernel_instance, '[') : nullptr;
    snprintf(g_kernel_text, sizeof(g_kernel_text), "%s%s%s", g_kernel_family, args ? " " : "", args ? args : "");
    return g_kernel_text;
}

}  // extern "C"
