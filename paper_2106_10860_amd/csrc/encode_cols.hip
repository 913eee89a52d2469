// Encode, and fused encode+scan, for an input matrix stored by columns.
//
// Algorithm 1 (Section 4.1) reads four elements of a row per codebook, so with A
// stored by columns only the 4 C split columns are touched: O(C) elements per
// row instead of O(D) (Section 5.2), each column read as one contiguous run.
//
// A lane owns a row here (a wavefront takes 64 consecutive rows), so that the
// four loads per codebook are coalesced along the column; the tree of the
// codebook is the same for all lanes and sits in scalar registers.  A lane packs
// the codes of its row into C / 8 registers.  In the fused kernel the wavefront
// then goes through its 64 rows one by one: the codes of row r are read from
// lane r into scalars and the table scan proceeds exactly as in the kernels for
// row-major input (lane = four output columns, tables in LDS).
#include "rows_common.h"

namespace maddness {
namespace {

using namespace rows;

// Codebooks whose loads are issued together (4 loads each, 64 elements wide).
constexpr int kChunk = 4;

__device__ __forceinline__ float uniform(float v)
{
    return __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(v)));
}

template <int MODE, int C, int WAVES, bool AVG, int DT>
__global__ __launch_bounds__(WAVES * 64) void cols_kernel(const RowsArgs a)
{
    static_assert(MODE == kFused || MODE == kEncode, "modes");
    static_assert(C % 8 == 0 && C % kChunk == 0, "codebooks");
    static_assert(MODE == kEncode || C == 16 || C == 32, "the table scan exists for 16 and 32 codebooks");
    constexpr int CW = C / 8;
    typedef unsigned cvec __attribute__((ext_vector_type(CW)));

    extern __shared__ __align__(16) unsigned char smem[];
    uint32_t *lut = reinterpret_cast<uint32_t *>(smem);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    const bool col_on = 4 * lane < a.M;
    f4 sc = {0.f, 0.f, 0.f, 0.f}, of = {0.f, 0.f, 0.f, 0.f};
    if constexpr (MODE == kFused) {
        // LDS layout [code k][codebook c][64 words], as in the row-major kernels
        for (int row = wave; row < C * 16; row += WAVES) {
            uint32_t w = 0;
            if (col_on) w = *reinterpret_cast<const uint32_t *>(a.luts + (size_t)row * a.M + 4 * lane);
            lut[((row & 15) * C + (row >> 4)) * 64 + lane] = w;
        }
        if (col_on) {
            sc = *reinterpret_cast<const f4 *>(a.scale + 4 * lane);
            of = *reinterpret_cast<const f4 *>(a.offset + 4 * lane);
        }
        __syncthreads();
    }

    const int64_t n_groups = (a.N + 63) >> 6;
    const int64_t gstride = (int64_t)gridDim.x * WAVES;
    for (int64_t g = (int64_t)blockIdx.x * WAVES + wave; g < n_groups; g += gstride) {
        const int64_t n = g * 64 + lane;
        const bool row_on = n < a.N;
        const int64_t nn = row_on ? n : a.N - 1;   // lanes past the end repeat the last row: loads stay in bounds

        unsigned cwv[CW];
#pragma unroll
        for (int q = 0; q < CW; ++q) cwv[q] = 0;
#pragma unroll
        for (int c0 = 0; c0 < C; c0 += kChunk) {
            float x[kChunk][4];
#pragma unroll
            for (int u = 0; u < kChunk; ++u) {
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    int j = a.split_dims[4 * (c0 + u) + t];
                    j = __builtin_amdgcn_readfirstlane(min(max(j, 0), a.D - 1));
                    x[u][t] = widen_at<DT>(a.A, (int64_t)j * a.lda + nn);
                }
            }
#pragma unroll
            for (int u = 0; u < kChunk; ++u) {
                Tree tr;
#pragma unroll
                for (int i = 0; i < 15; ++i) tr.t[i] = uniform(a.thresholds[16 * (c0 + u) + i]);
                const unsigned code = hash_regs(tr, x[u][0], x[u][1], x[u][2], x[u][3]);
                cwv[(c0 + u) >> 3] |= code << (4 * ((c0 + u) & 7));
            }
        }

        if (a.codes_out && row_on) {
            cvec v;
#pragma unroll
            for (int q = 0; q < CW; ++q) v[q] = cwv[q];
            *reinterpret_cast<cvec *>(a.codes_out + n * (C / 2)) = v;
        }

        if constexpr (MODE == kFused) {
            const int64_t left = a.N - g * 64;
            const int rows_here = left < 64 ? (int)left : 64;
            for (int r = 0; r < rows_here; ++r) {
                unsigned cw[CW];
#pragma unroll
                for (int q = 0; q < CW; ++q) cw[q] = (unsigned)__builtin_amdgcn_readlane((int)cwv[q], r);
                uint32_t acc_e = 0, acc_o = 0;
                scan_row_addtid<C, AVG>(cw, acc_e, acc_o);
                if (col_on) store_row(a, g * 64 + r, lane, acc_e, acc_o, sc, of, 0, AVG ? C : 0);
            }
        }
    }
}

template <int MODE, int C, int WAVES, bool AVG, int DT>
int launch_cols(const RowsArgs &a, int blocks_per_cu, hipStream_t stream)
{
    const size_t lds = MODE == kFused ? (size_t)C * 16 * 256 : 0;
    const DeviceInfo &dev = device_info();
    if (lds > (size_t)dev.lds_per_block) return 1;
    if (int rc = allow_full_lds<cols_kernel<MODE, C, WAVES, AVG, DT>>(); rc != MADDNESS_OK) return rc;
    const int64_t n_groups = (a.N + 63) / 64;
    const int64_t blocks_needed = (n_groups + WAVES - 1) / WAVES;
    const int64_t max_grid = (int64_t)dev.cus * blocks_per_cu;
    const int grid = (int)(blocks_needed < max_grid ? blocks_needed : max_grid);
    hipLaunchKernelGGL((cols_kernel<MODE, C, WAVES, AVG, DT>), dim3(grid), dim3(WAVES * 64), lds, stream, a);
    return check_hip(hipGetLastError(), "launch cols_kernel");
}

template <int MODE, int C, int WAVES, bool AVG>
int launch_cols_typed(const RowsArgs &a, int dtype, int blocks_per_cu, hipStream_t stream)
{
    switch (dtype) {
    case MADDNESS_F32: return launch_cols<MODE, C, WAVES, AVG, kF32>(a, blocks_per_cu, stream);
    case MADDNESS_F16: return launch_cols<MODE, C, WAVES, AVG, kF16>(a, blocks_per_cu, stream);
    case MADDNESS_BF16: return launch_cols<MODE, C, WAVES, AVG, kBF16>(a, blocks_per_cu, stream);
    default: return launch_cols<MODE, C, WAVES, AVG, kU8>(a, blocks_per_cu, stream);
    }
}

// A wavefront takes 64 rows at a time: with few rows most of the chip would idle,
// and the general kernels do better.
constexpr int64_t kMinRows = 1 << 16;

}  // namespace

int launch_encode_cols(const maddness_params &p, const MatrixA &A, int64_t N, uint8_t *codes,
                       hipStream_t stream)
{
    const int C = p.C;
    if (!A.col_major || N < kMinRows) return 1;
    if ((C != 16 && C != 32 && C != 64) || !aligned_to(codes, C / 2)) return 1;
    RowsArgs a{};
    a.A = A.data; a.lda = A.ld; a.D = p.D; a.N = N;
    a.split_dims = p.split_dims; a.thresholds = p.thresholds;
    a.codes_out = codes;
    if (C == 16) return launch_cols_typed<kEncode, 16, 4, false>(a, A.dtype, 4, stream);
    if (C == 32) return launch_cols_typed<kEncode, 32, 4, false>(a, A.dtype, 4, stream);
    return launch_cols_typed<kEncode, 64, 4, false>(a, A.dtype, 4, stream);
}

int launch_fused_cols(const maddness_params &p, const MatrixA &A, int64_t N, int32_t M,
                      const uint8_t *luts, const float *scale, const float *offset, float *out,
                      int64_t ldo, uint16_t *acc, uint8_t *codes, bool averaged, hipStream_t stream)
{
    const int C = p.C;
    if (!A.col_major || N < kMinRows) return 1;
    if (!tables_ok(C, M, luts, scale, offset, out, ldo, acc)) return 1;   // C in {16, 32}, 64 < M <= 256
    if (codes && !aligned_to(codes, C / 2)) return 1;
    RowsArgs a{};
    a.A = A.data; a.lda = A.ld; a.D = p.D; a.N = N;
    a.split_dims = p.split_dims; a.thresholds = p.thresholds;
    a.luts = luts; a.scale = scale; a.offset = offset; a.M = M;
    a.out = out; a.ldo = ldo; a.acc = acc; a.codes_out = codes;
    if (C == 32)
        return averaged ? launch_cols_typed<kFused, 32, 16, true>(a, A.dtype, 1, stream)
                        : launch_cols_typed<kFused, 32, 16, false>(a, A.dtype, 1, stream);
    return averaged ? launch_cols_typed<kFused, 16, 16, true>(a, A.dtype, 1, stream)
                    : launch_cols_typed<kFused, 16, 16, false>(a, A.dtype, 1, stream);
}

}  // namespace maddness
