// h(B): table construction (Section 3, "Table Construction", with the dense
// prototype matrix of Section 4.3) and 8-bit quantisation (Appendix A).
//
// The contraction T = P B (16 C x D times D x M) is the one dense piece of the
// method and runs on the fp64 matrix cores (v_mfma_f64_16x16x4_f64): products of
// two fp32 numbers are exact in fp64, so the tables differ from an fp64
// reference only by summation order (~1e-16 relative) and the 8-bit entries are
// reproducible to the byte except for values within that distance of a rounding
// boundary.  The contraction is tiny (2 * 16 C D M flops, 0.13 GFLOP at C = 32,
// D = 512, M = 256), so three small launches are enough.
#include "common.h"

namespace maddness {
namespace {

// Workspace of maddness_build_luts_static, the entry point for callers that cannot
// allocate: one array per GPU, held until the process ends.  In host code the name
// `scratch` is only a handle for hipGetSymbolAddress, never a device address.
static __device__ __align__(256) unsigned char scratch[MADDNESS_STATIC_WORKSPACE_BYTES];

typedef double double4_t __attribute__((ext_vector_type(4)));

// One workgroup of KSPLIT wavefronts per (codebook, tile of 16 output columns);
// wavefront w contracts the slice d = 4 (w + KSPLIT i) + 0..3 of the inner
// dimension, eight steps' worth of loads in flight at a time, and the partial
// tiles are added in wavefront order through LDS.
// Operand layout of v_mfma_f64_16x16x4_f64: lane l supplies A[i = l % 16][k = l / 16]
// and B[k = l / 16][j = l % 16]; it receives D[i = 4 r + l / 16][j = l % 16] in
// accumulator element r = 0..3.
constexpr int KSPLIT = 4;

__global__ __launch_bounds__(64 * KSPLIT) void lut_gemm_kernel(const float *__restrict__ P,
                                                               const float *__restrict__ B, int D, int M,
                                                               int64_t ldb, double *__restrict__ T)
{
    __shared__ double part[KSPLIT][4][64];
    const int c = blockIdx.x;
    const int lane = threadIdx.x & 63;
    const int w = threadIdx.x >> 6;
    const int i = lane & 15;
    const int kk = lane >> 4;
    const int m = blockIdx.y * 16 + i;
    const bool m_ok = m < M;
    const float *prow = P + ((size_t)c * 16 + i) * D;
    double4_t acc = {0.0, 0.0, 0.0, 0.0};
    constexpr int UNROLL = 8;
    for (int d0 = 4 * w; d0 < D; d0 += 4 * KSPLIT * UNROLL) {
        float av[UNROLL], bv[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int d = d0 + 4 * KSPLIT * u + kk;
            const bool ok = d < D;
            av[u] = ok ? prow[d] : 0.0f;
            bv[u] = (ok && m_ok) ? B[(size_t)d * ldb + m] : 0.0f;
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u)
            acc = __builtin_amdgcn_mfma_f64_16x16x4f64((double)av[u], (double)bv[u], acc, 0, 0, 0);
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) part[w][r][lane] = acc[r];
    __syncthreads();
    if (w == 0 && m_ok) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            double s = part[0][r][lane];
#pragma unroll
            for (int q = 1; q < KSPLIT; ++q) s += part[q][r][lane];
            T[((size_t)c * 16 + 4 * r + kk) * M + m] = s;
        }
    }
}

// Per output column: table minima, the widest range, the power-of-two scale.
// A block covers 32 columns; its 16 slices share out the codebooks, the widest
// range is reduced through LDS, and slice 0 then adds the minima in codebook
// order (the order the definition of beta is written in).
constexpr int STAT_COLS = 32;
constexpr int STAT_SLICES = 16;

__global__ __launch_bounds__(STAT_COLS * STAT_SLICES) void lut_stats_kernel(
    const double *__restrict__ T, int C, int M, double *__restrict__ delta, int *__restrict__ lexp,
    float *__restrict__ scale, float *__restrict__ offset)
{
    __shared__ double rmax[STAT_SLICES][STAT_COLS];
    const int tx = threadIdx.x % STAT_COLS;
    const int ty = threadIdx.x / STAT_COLS;
    const int m = blockIdx.x * STAT_COLS + tx;
    double r = 0.0;
    if (m < M) {
        for (int c = ty; c < C; c += STAT_SLICES) {
            const double *t = T + (size_t)c * 16 * M + m;
            double lo = t[0], hi = t[0];
#pragma unroll
            for (int k = 1; k < 16; ++k) {
                const double v = t[(size_t)k * M];
                lo = v < lo ? v : lo;
                hi = v > hi ? v : hi;
            }
            const double e = hi - lo;
            r = e > r ? e : r;
            delta[(size_t)c * M + m] = lo;
        }
    }
    rmax[ty][tx] = r;
    __syncthreads();   // also makes this block's writes to delta visible to slice 0
    if (ty != 0 || m >= M) return;
#pragma unroll
    for (int q = 1; q < STAT_SLICES; ++q) r = rmax[q][tx] > r ? rmax[q][tx] : r;
    double beta = 0.0;
    for (int c = 0; c < C; ++c) beta += delta[(size_t)c * M + m];
    int l = 0;
    if (r > 0.0 && isfinite(r)) {
        // r = f 2^e with f in [0.5, 1); r 2^l <= 255 = (255/256) 2^8
        int e;
        const double f = frexp(r, &e);
        l = (f <= 255.0 / 256.0) ? 8 - e : 7 - e;
        l = l > 126 ? 126 : (l < -126 ? -126 : l);
    }
    lexp[m] = l;
    scale[m] = ldexpf(1.0f, -l);
    offset[m] = (float)beta;
}

// Pooled variant (Appendix A as printed), step 1: one block per codebook finds
// the minimum and maximum of the codebook's tables over all columns and entries.
__global__ __launch_bounds__(256) void lut_pooled_minmax_kernel(const double *__restrict__ T, int M,
                                                                double *__restrict__ cb_min,
                                                                double *__restrict__ cb_range)
{
    __shared__ double lo_s[256], hi_s[256];
    const int c = blockIdx.x;
    const double *t = T + (size_t)c * 16 * M;
    const int n = 16 * M;
    double lo = t[0], hi = t[0];
    for (int i = threadIdx.x; i < n; i += 256) {
        const double v = t[i];
        lo = v < lo ? v : lo;
        hi = v > hi ? v : hi;
    }
    lo_s[threadIdx.x] = lo;
    hi_s[threadIdx.x] = hi;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) {
            lo_s[threadIdx.x] = lo_s[threadIdx.x + s] < lo_s[threadIdx.x] ? lo_s[threadIdx.x + s] : lo_s[threadIdx.x];
            hi_s[threadIdx.x] = hi_s[threadIdx.x + s] > hi_s[threadIdx.x] ? hi_s[threadIdx.x + s] : hi_s[threadIdx.x];
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        cb_min[c] = lo_s[0];
        cb_range[c] = hi_s[0] - lo_s[0];
    }
}

// Step 2 (one block): the widest range gives the scale, the minima are added in
// codebook order; delta[c][m] and lexp[m] are filled so that the quantise kernel
// of the per-column variant can be used unchanged.
__global__ __launch_bounds__(256) void lut_pooled_finish_kernel(const double *__restrict__ cb_min,
                                                                const double *__restrict__ cb_range, int C,
                                                                int M, double *__restrict__ delta,
                                                                int *__restrict__ lexp, float *__restrict__ scale,
                                                                float *__restrict__ offset)
{
    double r = 0.0, beta = 0.0;
    for (int c = 0; c < C; ++c) {   // every thread computes the same two numbers
        r = cb_range[c] > r ? cb_range[c] : r;
        beta += cb_min[c];
    }
    int l = 0;
    if (r > 0.0 && isfinite(r)) {
        int e;
        const double f = frexp(r, &e);
        l = (f <= 255.0 / 256.0) ? 8 - e : 7 - e;
        l = l > 126 ? 126 : (l < -126 ? -126 : l);
    }
    for (int m = threadIdx.x; m < M; m += 256) {
        lexp[m] = l;
        scale[m] = ldexpf(1.0f, -l);
        offset[m] = (float)beta;
    }
    for (int i = threadIdx.x; i < C * M; i += 256) delta[i] = cb_min[i / M];
}

__global__ __launch_bounds__(256) void lut_quantize_kernel(const double *__restrict__ T,
                                                           const double *__restrict__ delta,
                                                           const int *__restrict__ lexp, int C, int M,
                                                           uint8_t *__restrict__ luts)
{
    const int m = blockIdx.x * blockDim.x + threadIdx.x;
    const int row = blockIdx.y;  // c * 16 + k
    if (m >= M) return;
    const int c = row >> 4;
    double q = rint(ldexp(T[(size_t)row * M + m] - delta[(size_t)c * M + m], lexp[m]));
    q = (q >= 0.0) ? q : 0.0;  // NaN -> 0
    q = q > 255.0 ? 255.0 : q;
    luts[(size_t)row * M + m] = (uint8_t)q;
}

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

}  // namespace

// Workspace: T [C][16][M], delta [C][M], per-codebook min and range [2][C] (pooled
// variant), then lexp [M].
size_t build_luts_workspace_bytes(int32_t D, int32_t C, int32_t M)
{
    (void)D;
    return align_up(sizeof(double) * ((size_t)C * 16 * M + (size_t)C * M + 2 * (size_t)C) +
                        sizeof(int) * (size_t)M,
                    256);
}

int launch_build_luts(const maddness_params &p, const float *B, int32_t M, int64_t ldb,
                      uint8_t *luts, float *scale, float *offset, void *workspace, bool pooled,
                      hipStream_t stream)
{
    const int C = p.C;
    double *T = static_cast<double *>(workspace);
    double *delta = T + (size_t)C * 16 * M;
    double *cb_min = delta + (size_t)C * M;
    double *cb_range = cb_min + C;
    int *lexp = reinterpret_cast<int *>(cb_range + C);

    note_kernel(pooled ? "lut_gemm_kernel + lut_pooled_minmax_kernel + lut_pooled_finish_kernel + lut_quantize_kernel"
                       : "lut_gemm_kernel + lut_stats_kernel + lut_quantize_kernel", nullptr);
    hipLaunchKernelGGL(lut_gemm_kernel, dim3(C, (M + 15) / 16), dim3(64 * KSPLIT), 0, stream, p.prototypes, B,
                       p.D, M, ldb, T);
    int rc = check_hip(hipGetLastError(), "launch lut_gemm_kernel");
    if (rc != MADDNESS_OK) return rc;
    if (pooled) {
        hipLaunchKernelGGL(lut_pooled_minmax_kernel, dim3(C), dim3(256), 0, stream, T, M, cb_min, cb_range);
        rc = check_hip(hipGetLastError(), "launch lut_pooled_minmax_kernel");
        if (rc != MADDNESS_OK) return rc;
        hipLaunchKernelGGL(lut_pooled_finish_kernel, dim3(1), dim3(256), 0, stream, cb_min, cb_range, C, M,
                           delta, lexp, scale, offset);
        rc = check_hip(hipGetLastError(), "launch lut_pooled_finish_kernel");
    } else {
        hipLaunchKernelGGL(lut_stats_kernel, dim3((M + STAT_COLS - 1) / STAT_COLS),
                           dim3(STAT_COLS * STAT_SLICES), 0, stream, T, C, M, delta, lexp, scale, offset);
        rc = check_hip(hipGetLastError(), "launch lut_stats_kernel");
    }
    if (rc != MADDNESS_OK) return rc;
    hipLaunchKernelGGL(lut_quantize_kernel, dim3((M + 255) / 256, C * 16), dim3(256), 0, stream, T,
                       delta, lexp, C, M, luts);
    return check_hip(hipGetLastError(), "launch lut_quantize_kernel");
}

// The address of `scratch` on the current device, looked up once per device (every GPU
// holds its own copy of the array at its own address).
int static_workspace(void **workspace)
{
    constexpr int kMaxDevices = 64;
    static std::mutex mutex;
    static void *address[kMaxDevices] = {};
    int dev = -1;
    if (int rc = check_hip(hipGetDevice(&dev), "hipGetDevice"); rc != MADDNESS_OK) return rc;
    if (dev < 0 || dev >= kMaxDevices)
        return fail(MADDNESS_E_UNSUPPORTED, "device ordinal %d: maddness_build_luts_static keeps an address for %d devices",
                    dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(mutex);
    if (!address[dev]) {
        void *ptr = nullptr;
        if (int rc = check_hip(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)), "hipGetSymbolAddress(scratch)");
            rc != MADDNESS_OK)
            return rc;
        address[dev] = ptr;
    }
    *workspace = address[dev];
    return MADDNESS_OK;
}

}  // namespace maddness
