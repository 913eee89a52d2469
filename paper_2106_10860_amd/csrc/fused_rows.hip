// Fused encode+scan for the wide-output case (one tile of up to 256 output
// columns whose uint8 tables all fit in LDS next to a small staging area).
//
// Every wavefront works on its own rows with no workgroup barrier after the
// tables are loaded:
//   1. rows of A arrive with coalesced 16-byte non-temporal loads, one group of
//      RPI = 64 / C rows ahead of the one being processed (registers are the
//      prefetch buffer), and are copied to a wavefront-private LDS area;
//   2. lane (r, c) picks its four split values out of that area and walks tree c
//      (Algorithm 1, Section 4.1) with the 15 thresholds held in registers;
//   3. the 4-bit codes are packed eight to a register across lanes and read
//      back as scalars, so that for each row the address of table row
//      (c, code) is wavefront-uniform: lane l reads the 32-bit word that holds
//      output columns 4l..4l+3 and the 64 lanes read 256 consecutive bytes;
//   4. the four bytes are added into two registers of two 16-bit sums each
//      (Section 4.4 as an exact sum), then alpha f + beta (Section 1.1) and one
//      coalesced 16-byte store per lane.
#include "common.h"
#include "device_common.h"

namespace maddness {
namespace {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef unsigned u2 __attribute__((ext_vector_type(2)));

struct RowsArgs {
    const float *A;
    int64_t lda;
    int D;
    int64_t N;
    const int32_t *split_dims;
    const float *thresholds;
    const uint8_t *luts;
    const float *scale;
    const float *offset;
    int M;
    float *out;
    int64_t ldo;
    uint16_t *acc;
    uint8_t *codes_out;
    int64_t n_groups;  // ceil(N / RPI)
};

// Value of `v` in the lane `n` places up within the same row of 16 lanes.
template <int N_>
__device__ __forceinline__ unsigned from_lane_above(unsigned v)
{
    return (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x100 + N_ /* row_shl:N */, 0xF, 0xF, true);
}

template <int C, int DV, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void fused_rows_kernel(const RowsArgs a)
{
    static_assert(C == 16 || C == 32 || C == 64, "codebooks per row group");
    constexpr int RPI = 64 / C;      // rows per wavefront iteration
    constexpr int ROWF = DV * 256;   // floats of staging per row
    constexpr int CW = C / 8;        // 32-bit words of packed codes per row

    extern __shared__ __align__(16) unsigned char smem[];
    uint32_t *lut = reinterpret_cast<uint32_t *>(smem);  // [C * 16][64] words
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    float *stage = reinterpret_cast<float *>(smem + C * 16 * 256) + wave * (RPI * ROWF);

    for (int row = wave; row < C * 16; row += WAVES) {
        uint32_t w = 0;
        if (4 * lane < a.M) w = *reinterpret_cast<const uint32_t *>(a.luts + (size_t)row * a.M + 4 * lane);
        lut[row * 64 + lane] = w;
    }

    const int c = lane & (C - 1);
    const int rsub = lane / C;
    Tree tr;
    load_tree(tr, a.split_dims + 4 * c, a.thresholds + 16 * c, a.D);
    const float *st = stage + rsub * ROWF;
    const bool col_on = 4 * lane < a.M;
    f4 sc = {0.f, 0.f, 0.f, 0.f}, of = {0.f, 0.f, 0.f, 0.f};
    if (col_on) {
        sc = *reinterpret_cast<const f4 *>(a.scale + 4 * lane);
        of = *reinterpret_cast<const f4 *>(a.offset + 4 * lane);
    }
    __syncthreads();

    const int64_t gstride = (int64_t)gridDim.x * WAVES;
    int64_t g = (int64_t)blockIdx.x * WAVES + wave;
    f4 pre[RPI][DV];

    auto issue_loads = [&](int64_t gg) {
#pragma unroll
        for (int r = 0; r < RPI; ++r) {
            const int64_t row = gg * RPI + r;
#pragma unroll
            for (int i = 0; i < DV; ++i) {
                const int col4 = lane + 64 * i;
                f4 v = {0.f, 0.f, 0.f, 0.f};
                if (row < a.N && 4 * col4 < a.D)
                    v = __builtin_nontemporal_load(reinterpret_cast<const f4 *>(a.A + row * a.lda) + col4);
                pre[r][i] = v;
            }
        }
    };

    if (g < a.n_groups) issue_loads(g);
    while (g < a.n_groups) {
#pragma unroll
        for (int r = 0; r < RPI; ++r)
#pragma unroll
            for (int i = 0; i < DV; ++i)
                *reinterpret_cast<f4 *>(stage + r * ROWF + 4 * (lane + 64 * i)) = pre[r][i];
        const int64_t gn = g + gstride;
        if (gn < a.n_groups) issue_loads(gn);
        wave_lds_fence();
        const float x0 = st[tr.j0], x1 = st[tr.j1], x2 = st[tr.j2], x3 = st[tr.j3];
        const unsigned code = hash_regs(tr, x0, x1, x2, x3);
        wave_lds_fence();

        // eight codes per register: lanes whose index is a multiple of 8 end up
        // with codebooks c..c+7 of their row, codebook c in the low nibble
        unsigned p = code | (from_lane_above<1>(code) << 4);
        p |= from_lane_above<2>(p) << 8;
        p |= from_lane_above<4>(p) << 16;

        if (a.codes_out && (lane & 7) == 0) {
            const int64_t row = g * RPI + rsub;
            if (row < a.N)
                *reinterpret_cast<uint32_t *>(a.codes_out + row * (C / 2) + (c >> 3) * 4) = p;
        }

#pragma unroll
        for (int r = 0; r < RPI; ++r) {
            const int64_t row = g * RPI + r;
            if (row >= a.N) break;
            unsigned cw[CW];
#pragma unroll
            for (int q = 0; q < CW; ++q) cw[q] = (unsigned)__builtin_amdgcn_readlane((int)p, r * C + 8 * q);
            uint32_t acc_e = 0, acc_o = 0;
#pragma unroll
            for (int cc = 0; cc < C; cc += 2) {
                const unsigned k0 = (cw[cc >> 3] >> (4 * (cc & 7))) & 15u;
                const unsigned k1 = (cw[cc >> 3] >> (4 * (cc & 7) + 4)) & 15u;
                const uint32_t y0 = lut[(cc * 16 + k0) * 64 + lane];
                const uint32_t y1 = lut[((cc + 1) * 16 + k1) * 64 + lane];
                acc_e += (y0 & 0x00FF00FFu) + (y1 & 0x00FF00FFu);
                acc_o += __builtin_amdgcn_perm(y0, y0, 0x0c030c01u) + __builtin_amdgcn_perm(y1, y1, 0x0c030c01u);
            }
            if (col_on) {
                const uint32_t s0 = acc_e & 0xFFFFu, s1 = acc_o & 0xFFFFu, s2 = acc_e >> 16, s3 = acc_o >> 16;
                if (a.out) {
                    f4 v;
                    v.x = fmaf((float)s0, sc.x, of.x);
                    v.y = fmaf((float)s1, sc.y, of.y);
                    v.z = fmaf((float)s2, sc.z, of.z);
                    v.w = fmaf((float)s3, sc.w, of.w);
                    __builtin_nontemporal_store(v, reinterpret_cast<f4 *>(a.out + row * a.ldo) + lane);
                }
                if (a.acc) {
                    u2 w = {s0 | (s1 << 16), s2 | (s3 << 16)};
                    *reinterpret_cast<u2 *>(a.acc + row * a.M + 4 * lane) = w;
                }
            }
        }
        g = gn;
    }
}

template <int C, int DV, int WAVES>
int launch_variant(const RowsArgs &a, hipStream_t stream)
{
    constexpr int RPI = 64 / C;
    const size_t lds = (size_t)C * 16 * 256 + (size_t)WAVES * RPI * DV * 256 * 4;
    const DeviceInfo &dev = device_info();
    if (lds > (size_t)dev.lds_per_block) return 1;
    static bool attr_set = false;
    if (!attr_set) {
        int rc = check_hip(hipFuncSetAttribute(reinterpret_cast<const void *>(fused_rows_kernel<C, DV, WAVES>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize,
                                               dev.lds_per_block),
                           "hipFuncSetAttribute(MaxDynamicSharedMemorySize)");
        if (rc != MADDNESS_OK) return rc;
        attr_set = true;
    }
    const int64_t blocks_needed = (a.n_groups + WAVES - 1) / WAVES;
    const int per_cu = (int)((size_t)dev.lds_per_block / lds);
    const int64_t max_grid = (int64_t)dev.cus * (per_cu < 1 ? 1 : per_cu);
    const int grid = (int)(blocks_needed < max_grid ? blocks_needed : max_grid);
    hipLaunchKernelGGL((fused_rows_kernel<C, DV, WAVES>), dim3(grid), dim3(WAVES * 64), lds, stream, a);
    return check_hip(hipGetLastError(), "launch fused_rows_kernel");
}

bool aligned16(const void *p) { return reinterpret_cast<uintptr_t>(p) % 16 == 0; }

}  // namespace

// Returns MADDNESS_OK when the launch was made, 1 when the shape is not one this
// kernel covers (the caller then uses the general kernel), or an error status.
int launch_fused_rows(const maddness_params &p, const float *A, int64_t N, int64_t lda, int32_t M,
                      const uint8_t *luts, const float *scale, const float *offset, float *out,
                      int64_t ldo, uint16_t *acc, uint8_t *codes, hipStream_t stream)
{
    const int C = p.C, D = p.D;
    if (M % 4 != 0 || M > 256 || M <= 64) return 1;
    if (D % 4 != 0 || lda % 4 != 0 || !aligned16(A)) return 1;
    if (out && (ldo % 4 != 0 || !aligned16(out))) return 1;
    if (acc && reinterpret_cast<uintptr_t>(acc) % 8 != 0) return 1;
    if (codes && reinterpret_cast<uintptr_t>(codes) % 4 != 0) return 1;
    if (!aligned16(scale) || !aligned16(offset) || reinterpret_cast<uintptr_t>(luts) % 4 != 0) return 1;

    RowsArgs a{};
    a.A = A; a.lda = lda; a.D = D; a.N = N;
    a.split_dims = p.split_dims; a.thresholds = p.thresholds;
    a.luts = luts; a.scale = scale; a.offset = offset; a.M = M;
    a.out = out; a.ldo = ldo; a.acc = acc; a.codes_out = codes;
    const int RPI = 64 / C;
    a.n_groups = (N + RPI - 1) / RPI;
    if (C == 32 && D <= 256) return launch_variant<32, 1, 8>(a, stream);
    if (C == 32 && D <= 512) return launch_variant<32, 2, 8>(a, stream);
    if (C == 16 && D <= 256) return launch_variant<16, 1, 8>(a, stream);
    if (C == 16 && D <= 512) return launch_variant<16, 2, 4>(a, stream);
    return 1;
}

}  // namespace maddness
