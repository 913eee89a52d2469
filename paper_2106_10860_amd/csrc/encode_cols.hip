// Encode, and fused encode+scan, for an input matrix stored by columns.
//
// Algorithm 1 (Section 4.1) reads four elements of a row per codebook, so with A
// stored by columns only the 4 C split columns are touched: O(C) elements per
// row instead of O(D) (Section 5.2), each column read as one contiguous run.
//
// A lane owns RPL consecutive rows here and a wavefront 64 RPL ("a group"), so
// that every load instruction fetches 64 RPL consecutive elements of one column;
// the tree of a codebook is the same for all lanes and sits in scalar registers.
// A lane packs the codes of each of its rows into C / 8 registers.
//
// In the fused kernel the wavefront then goes through the rows of the group one
// by one: the codes of a row are read from its lane into scalars and the table
// scan proceeds exactly as in the kernels for row-major input (lane = four
// output columns, tables in LDS).  While it scans one group it encodes the next:
// the codebooks are taken in chunks, and between the scans of a few rows the
// trees of one chunk are walked and the loads of the following chunk are issued,
// so the column reads (HBM) overlap the table scan (instruction issue).
#include "cols_common.h"

namespace maddness {
namespace {

using namespace rows;
using namespace cols;

// CHUNK: codebooks whose loads are issued together (4 loads each); RPL: rows per lane;
// PIPE (fused mode, M = 256, fp32 output only): encode the next group while scanning.
template <int MODE, int C, int WAVES, bool AVG, int DT, int CHUNK, int RPL, bool PIPE>
__global__ __launch_bounds__(WAVES * 64) void cols_kernel(const RowsArgs a)
{
    static_assert(MODE == kFused || MODE == kEncode, "modes");
    static_assert(C % 8 == 0 && 8 % CHUNK == 0, "a chunk of codebooks lies within one word of codes");
    static_assert(MODE == kEncode || C == 16 || C == 32, "the table scan exists for 16 and 32 codebooks");
    constexpr int CW = C / 8;
    constexpr int NCHUNK = C / CHUNK;
    constexpr int GROUP = 64 * RPL;   // rows a wavefront takes at a time
    static_assert(64 % NCHUNK == 0 || MODE == kEncode, "lanes per chunk step");

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

    const int64_t n_groups = (a.N + GROUP - 1) / GROUP;
    const int64_t gstride = (int64_t)gridDim.x * WAVES;
    ColsEncoder<C, DT, CHUNK, RPL> enc(a);

    int64_t g = (int64_t)blockIdx.x * WAVES + wave;
    if constexpr (MODE == kEncode) {
        for (; g < n_groups; g += gstride) {
            enc.encode_group(g * GROUP, lane);
            enc.store_codes(a.codes_out);
        }
    } else {
        // scan of the rows of lanes [l0, l1) of group g, whose codes are in cwc
        unsigned cwc[RPL][CW];
        auto scan_lanes = [&](int64_t g_, int l0, int l1) INLINE_LAMBDA {
            for (int l = l0; l < l1; ++l) {
#pragma unroll
                for (int r = 0; r < RPL; ++r) {
                    unsigned cw[CW];
#pragma unroll
                    for (int q = 0; q < CW; ++q) cw[q] = (unsigned)__builtin_amdgcn_readlane((int)cwc[r][q], l);
                    uint32_t acc_e = 0, acc_o = 0;
                    scan_row_addtid<C, AVG>(cw, acc_e, acc_o);
                    if (col_on) store_row(a, g_ * GROUP + RPL * l + r, lane, acc_e, acc_o, sc, of, 0, AVG ? C : 0);
                }
            }
        };
        auto encode_group = [&](int64_t g_) INLINE_LAMBDA {
            enc.encode_group(g_ * GROUP, lane);
            enc.store_codes(a.codes_out);
        };
        auto take_codes = [&]() INLINE_LAMBDA {
#pragma unroll
            for (int r = 0; r < RPL; ++r)
#pragma unroll
                for (int q = 0; q < CW; ++q) cwc[r][q] = enc.cwn[r][q];
        };
        auto lanes_of = [&](int64_t g_) INLINE_LAMBDA {   // lanes that hold rows of the matrix
            const int64_t left = (a.N - g_ * GROUP) / RPL;
            return left < 64 ? (int)left : 64;
        };

        if constexpr (!PIPE) {
            for (; g < n_groups; g += gstride) {
                encode_group(g);
                take_codes();
                scan_lanes(g, 0, lanes_of(g));
            }
        } else {
            // While group g is scanned, the next group of this wavefront is encoded: per
            // chunk of codebooks, the loads are issued, then the rows of 64 / NCHUNK lanes
            // are scanned, then the trees are walked.  Every lane stores (M = 256, fp32
            // output only), so between the loads and their first use lies straight-line
            // code with a fixed number of stores: the wait the compiler puts before the
            // walk is for the loads alone and leaves the stores in flight (memory
            // operations complete in order).  A group that has a successor is full.
            if (g >= n_groups) return;
            encode_group(g);
            constexpr int LPS = 64 / NCHUNK;
            for (int64_t gn = g + gstride; gn < n_groups; gn += gstride) {
                take_codes();
                enc.n0 = gn * GROUP + RPL * lane;
                enc.nq = enc.n0 < a.N ? enc.n0 : a.N - RPL;
#pragma unroll
                for (int r = 0; r < RPL; ++r) enc.word[r] = 0;
#pragma unroll 1
                for (int k = 0; k < NCHUNK; ++k) {
                    enc.issue(k);
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int i = 0; i < LPS; ++i) {
                        const int l = k * LPS + i;
#pragma unroll
                        for (int r = 0; r < RPL; ++r) {
                            unsigned cw[CW];
#pragma unroll
                            for (int q = 0; q < CW; ++q)
                                cw[q] = (unsigned)__builtin_amdgcn_readlane((int)cwc[r][q], l);
                            uint32_t acc_e = 0, acc_o = 0;
                            scan_row_addtid<C, AVG>(cw, acc_e, acc_o);
                            store_row(a, g * GROUP + RPL * l + r, lane, acc_e, acc_o, sc, of, 0, AVG ? C : 0, true);
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                    // the loaded values are first touched here, after the scans
#pragma unroll
                    for (int u = 0; u < CHUNK; ++u)
#pragma unroll
                        for (int t = 0; t < 4; ++t)
#pragma unroll
                            for (int r = 0; r < RPL; ++r) asm volatile("" : "+v"(enc.x_nxt[u][t][r]));
                    enc.walk(k, enc.tr_nxt, enc.x_nxt);
                }
                enc.store_codes(a.codes_out);
                g = gn;
            }
            take_codes();
            scan_lanes(g, 0, lanes_of(g));
        }
    }
}

#ifndef MADDNESS_COLS_CHUNK_ENCODE
#define MADDNESS_COLS_CHUNK_ENCODE 2
#endif
#ifndef MADDNESS_COLS_CHUNK_FUSED
#define MADDNESS_COLS_CHUNK_FUSED 1
#endif
#ifndef MADDNESS_COLS_ENCODE_WAVES
#define MADDNESS_COLS_ENCODE_WAVES 4
#endif
#ifndef MADDNESS_COLS_ENCODE_BLOCKS_PER_CU
#define MADDNESS_COLS_ENCODE_BLOCKS_PER_CU 4
#endif
#ifndef MADDNESS_COLS_FUSED_GROUPS_PER_WAVE
#define MADDNESS_COLS_FUSED_GROUPS_PER_WAVE 1
#endif

template <int MODE, int C, int WAVES, bool AVG, int DT, int RPL, bool PIPE>
int launch_cols_variant(const RowsArgs &a, int blocks_per_cu, hipStream_t stream)
{
    constexpr int CHUNK = MODE == kFused ? MADDNESS_COLS_CHUNK_FUSED : MADDNESS_COLS_CHUNK_ENCODE;
    const size_t lds = MODE == kFused ? (size_t)C * 16 * 256 : 0;
    const DeviceInfo &dev = device_info();
    if (lds > (size_t)dev.lds_per_block) return 1;
    if (int rc = allow_full_lds<cols_kernel<MODE, C, WAVES, AVG, DT, CHUNK, RPL, PIPE>>(); rc != MADDNESS_OK) return rc;
    const int64_t n_groups = (a.N + 64 * RPL - 1) / (64 * RPL);
    const int64_t blocks_needed = (n_groups + WAVES - 1) / WAVES;
    const int64_t max_grid = (int64_t)dev.cus * blocks_per_cu;
    const int grid = (int)(blocks_needed < max_grid ? blocks_needed : max_grid);
    note_kernel("cols_kernel", __PRETTY_FUNCTION__);
    hipLaunchKernelGGL((cols_kernel<MODE, C, WAVES, AVG, DT, CHUNK, RPL, PIPE>), dim3(grid), dim3(WAVES * 64), lds, stream,
                       a);
    return check_hip(hipGetLastError(), "launch cols_kernel");
}

template <int MODE, int C, int WAVES, bool AVG, int DT, int RPL>
int launch_cols(const RowsArgs &a, int blocks_per_cu, hipStream_t stream)
{
    if constexpr (MODE == kFused) {
        // all 64 lanes store fp32 and nothing else: the pipelined variant applies
        if (a.M == 256 && a.out && !a.acc)
            return launch_cols_variant<MODE, C, WAVES, AVG, DT, RPL, true>(a, blocks_per_cu, stream);
    }
    return launch_cols_variant<MODE, C, WAVES, AVG, DT, RPL, false>(a, blocks_per_cu, stream);
}

template <int MODE, int C, int WAVES, bool AVG, int RPL>
int launch_cols_typed(const RowsArgs &a, int dtype, int blocks_per_cu, hipStream_t stream)
{
    switch (dtype) {
    case MADDNESS_F32: return launch_cols<MODE, C, WAVES, AVG, kF32, RPL>(a, blocks_per_cu, stream);
    case MADDNESS_F16: return launch_cols<MODE, C, WAVES, AVG, kF16, RPL>(a, blocks_per_cu, stream);
    case MADDNESS_BF16: return launch_cols<MODE, C, WAVES, AVG, kBF16, RPL>(a, blocks_per_cu, stream);
    default: return launch_cols<MODE, C, WAVES, AVG, kU8, RPL>(a, blocks_per_cu, stream);
    }
}

// A wavefront takes at least 64 rows at a time: with few rows most of the chip
// would idle, and the general kernels do better.
constexpr int64_t kMinRows = 1 << 16;

// Runs of rpl rows are loaded as one vector: column stride a multiple of rpl
// elements, base aligned to rpl elements.
bool runs_ok(const MatrixA &A, int rpl)
{
    return A.ld % rpl == 0 && aligned_to(A.data, (size_t)rpl * A.elem_bytes());
}

// A with its first `rows` rows taken off (stored by columns: a pointer offset)
MatrixA tail_of(const MatrixA &A, int64_t rows)
{
    MatrixA t = A;
    t.data = static_cast<const unsigned char *>(A.data) + rows * A.elem_bytes();
    return t;
}

template <int C, bool AVG>
int launch_fused_cols_rpl(const RowsArgs &a, const MatrixA &A, int64_t N, hipStream_t stream)
{
    // Longer runs read DRAM better (N = 2^20, C = 32, M = 256, fp32: 0.416 ms with runs
    // of 4 rows, 0.412 with 2, 0.447 with 1; binary16: 0.338 / 0.372 / 0.433), as long
    // as every wavefront of the chip still gets a group.
    const int64_t waves = (int64_t)device_info().cus * 16;
    const int64_t want = MADDNESS_COLS_FUSED_GROUPS_PER_WAVE;
    // MADDNESS_OPT_COLS_RUN fixes the run length (tests reach every variant at small sizes with it)
    if (const int rpl = option(MADDNESS_OPT_COLS_RUN)) {
        if (rpl == 4 && runs_ok(A, 4)) return launch_cols_typed<kFused, C, 16, AVG, 4>(a, A.dtype, 1, stream);
        if (rpl == 2 && runs_ok(A, 2)) return launch_cols_typed<kFused, C, 16, AVG, 2>(a, A.dtype, 1, stream);
        if (rpl == 1) return launch_cols_typed<kFused, C, 16, AVG, 1>(a, A.dtype, 1, stream);
    }
    if (runs_ok(A, 4) && N >= want * waves * 256) return launch_cols_typed<kFused, C, 16, AVG, 4>(a, A.dtype, 1, stream);
    if (runs_ok(A, 2) && N >= want * waves * 128) return launch_cols_typed<kFused, C, 16, AVG, 2>(a, A.dtype, 1, stream);
    return launch_cols_typed<kFused, C, 16, AVG, 1>(a, A.dtype, 1, stream);
}

}  // namespace

int launch_encode_cols(const maddness_params &p, const MatrixA &A, int64_t N, uint8_t *codes,
                       hipStream_t stream)
{
    const int C = p.C;
    if (!A.col_major || N < kMinRows || !runs_ok(A, 4)) return 1;
    if ((C != 16 && C != 32 && C != 64) || !aligned_to(codes, C / 2)) return 1;
    const int64_t Nq = N & ~(int64_t)3;
    RowsArgs a{};
    a.A = A.data; a.lda = A.ld; a.D = p.D; a.N = Nq;
    a.split_dims = p.split_dims; a.thresholds = p.thresholds;
    a.codes_out = codes;
    constexpr int W = MADDNESS_COLS_ENCODE_WAVES, B = MADDNESS_COLS_ENCODE_BLOCKS_PER_CU;
    int rc;
    if (C == 16) rc = launch_cols_typed<kEncode, 16, W, false, 4>(a, A.dtype, B, stream);
    else if (C == 32) rc = launch_cols_typed<kEncode, 32, W, false, 4>(a, A.dtype, B, stream);
    else rc = launch_cols_typed<kEncode, 64, W, false, 4>(a, A.dtype, B, stream);
    if (rc != MADDNESS_OK || Nq == N) return rc;
    return launch_encode(p, tail_of(A, Nq), N - Nq, codes + Nq * (C / 2), stream);
}

int launch_fused_cols(const maddness_params &p, const MatrixA &A, int64_t N, int32_t M,
                      const uint8_t *luts, const float *scale, const float *offset, float *out,
                      int64_t ldo, uint16_t *acc, uint8_t *codes, bool averaged, hipStream_t stream)
{
    const int C = p.C;
    if (!A.col_major || N < kMinRows) return 1;
    // whole runs of four rows (whatever run length is chosen); the rest goes to the general kernel
    const int64_t Nq = N & ~(int64_t)3;
    // the exact sum on the matrix cores where that kernel takes the shape (bound by HBM, where
    // the kernel below is bound by the vector ALUs)
    int rc = 1;
    if (!averaged && !vector_scan_only())
        rc = launch_fused_mfma(p, A, Nq, M, luts, scale, offset, out, ldo, acc, codes, stream);
    if (rc == 1) {
        if (!tables_ok(C, M, luts, scale, offset, out, ldo, acc)) return 1;   // C in {16, 32}, 64 < M <= 256
        if (codes && !aligned_to(codes, C / 2)) return 1;
        RowsArgs a{};
        a.A = A.data; a.lda = A.ld; a.D = p.D; a.N = Nq;
        a.split_dims = p.split_dims; a.thresholds = p.thresholds;
        a.luts = luts; a.scale = scale; a.offset = offset; a.M = M;
        a.out = out; a.ldo = ldo; a.acc = acc; a.codes_out = codes;
        if (C == 32)
            rc = averaged ? launch_fused_cols_rpl<32, true>(a, A, Nq, stream)
                          : launch_fused_cols_rpl<32, false>(a, A, Nq, stream);
        else
            rc = averaged ? launch_fused_cols_rpl<16, true>(a, A, Nq, stream)
                          : launch_fused_cols_rpl<16, false>(a, A, Nq, stream);
    }
    if (rc != MADDNESS_OK || Nq == N) return rc;
    const MatrixA tail = tail_of(A, Nq);
    return launch_scan(&p, &tail, nullptr, C, M, N - Nq, luts, scale, offset, out ? out + Nq * ldo : nullptr, ldo,
                       acc ? acc + Nq * M : nullptr, codes ? codes + Nq * (C / 2) : nullptr, averaged, stream);
}

}  // namespace maddness
