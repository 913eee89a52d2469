// Row-streaming kernels for the wide-output case: one tile of up to 256 output
// columns whose uint8 tables all fit in LDS (16 C M bytes, C = 16 or 32), in
// three modes - fused encode+scan, encode only, scan only.
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
//      output columns 4l..4l+3 and the 64 lanes read 256 consecutive bytes
//      (ds_read_addtid_b32: scalar base in M0, no vector address arithmetic);
//   4. the four bytes are added into two registers of two 16-bit sums each
//      (Section 4.4 as an exact sum), then alpha f + beta (Section 1.1) and one
//      coalesced 16-byte store per lane.
// HBM efficiency on this chip drops when much more than ~16-32 KiB of loads per
// CU are in flight, so the fused and encode modes run few wavefronts per CU
// with one group of rows of prefetch each.
#include "rows_common.h"

namespace maddness {
namespace {

using namespace rows;

template <int MODE, int C, int DV, int WAVES, int RPI = 64 / C, bool AVG = false, int DT = kF32>
__global__ __launch_bounds__(WAVES * 64) void rows_kernel(const RowsArgs a)
{
    static_assert(C == 16 || C == 32 || C == 64, "codebooks per row group");
    // RPI: rows per wavefront iteration (encode); lanes beyond RPI * C repeat the
    // work of the first ones when RPI < 64 / C
    static_assert(RPI >= 1 && RPI * C <= 64, "rows per iteration");
    constexpr int ROWB = DV * 1024;  // bytes of staging per row (DV pieces of 16 bytes per lane)
    constexpr int ES = elem_size(DT);
    constexpr int CW = C / 8;        // 32-bit words of packed codes per row
    constexpr int LUT_BYTES = (MODE == kEncode) ? 0 : C * 16 * 256;

    extern __shared__ __align__(16) unsigned char smem[];
    uint32_t *lut = reinterpret_cast<uint32_t *>(smem);  // [C * 16][64] words
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    const bool col_on = 4 * lane < a.M;
    f4 sc = {0.f, 0.f, 0.f, 0.f}, of = {0.f, 0.f, 0.f, 0.f};
    // The tables into LDS, layout [code k][codebook c][64 words]: table row (c, k) of the input
    // goes to word offset (k * C + c) * 64.  Eight loads per lane in flight (all 32 of a lane at once
    // were slower: 11.7 against 10.5 us for the fused call on 10000 rows, C = 32).
    auto load_tables_to_lds = [&]() INLINE_LAMBDA {
        constexpr int ROWS = C * 16;
        for (int row0 = wave; row0 < ROWS; row0 += 8 * WAVES) {
            uint32_t w[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int row = row0 + u * WAVES;
                w[u] = 0;
                if (col_on && row < ROWS) w[u] = *reinterpret_cast<const uint32_t *>(a.luts + (size_t)row * a.M + 4 * lane);
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int row = row0 + u * WAVES;
                if (row < ROWS) lut[((row & 15) * C + (row >> 4)) * 64 + lane] = w[u];
            }
        }
        if (col_on) {
            sc = *reinterpret_cast<const f4 *>(a.scale + 4 * lane);
            of = *reinterpret_cast<const f4 *>(a.offset + 4 * lane);
        }
        __syncthreads();
    };
    if constexpr (MODE == kScan) load_tables_to_lds();

    if constexpr (MODE == kScan) {
        // one row per iteration; the packed codes of the next row are fetched
        // (same address in every lane) while the current row is scanned
        typedef unsigned cvec __attribute__((ext_vector_type(CW)));
        const int64_t stride = (int64_t)gridDim.x * WAVES;
        int64_t row = (int64_t)blockIdx.x * WAVES + wave;
        cvec next = {};
        if (row < a.N) next = *reinterpret_cast<const cvec *>(a.codes_in + row * (C / 2));
        while (row < a.N) {
            const cvec cur = next;
            const int64_t rn = row + stride;
            if (rn < a.N) next = *reinterpret_cast<const cvec *>(a.codes_in + rn * (C / 2));
            unsigned cw[CW];
#pragma unroll
            for (int q = 0; q < CW; ++q) cw[q] = (unsigned)__builtin_amdgcn_readfirstlane((int)cur[q]);
            uint32_t acc_e = 0, acc_o = 0;
            scan_row_addtid<C, AVG>(cw, acc_e, acc_o);
            if (col_on) store_row(a, row, lane, acc_e, acc_o, sc, of, 0, AVG ? C : 0);
            row = rn;
        }
    } else {
        unsigned char *stage = smem + LUT_BYTES + wave * (RPI * ROWB);
        const int c = lane & (C - 1);
        const int rsub = (lane / C) % RPI;
        Tree tr;
        load_tree(tr, a.split_dims + 4 * c, a.thresholds + 16 * c, a.D);
        const unsigned char *st = stage + rsub * ROWB;
        const unsigned char *A_bytes = static_cast<const unsigned char *>(a.A);
        const int row_bytes = a.D * ES;

        const int64_t gstride = (int64_t)gridDim.x * WAVES;
        int64_t g = (int64_t)blockIdx.x * WAVES + wave;
        f4 pre[RPI][DV];

        auto issue_loads = [&](int64_t gg) INLINE_LAMBDA {
#pragma unroll
            for (int r = 0; r < RPI; ++r) {
                const int64_t row = gg * RPI + r;
#pragma unroll
                for (int i = 0; i < DV; ++i) {
                    const int col4 = lane + 64 * i;
                    f4 v = {0.f, 0.f, 0.f, 0.f};
                    if (row < a.N && 16 * col4 < row_bytes)
                        v = __builtin_nontemporal_load(reinterpret_cast<const f4 *>(A_bytes + row * a.lda * ES) + col4);
                    pre[r][i] = v;
                }
            }
        };

        // the first rows are on their way (and the tree was asked for above) while the tables are fetched:
        // with few rows per wavefront the kernel is a chain of memory latencies, and this takes one link out
        // (1000 rows of 320 floats, C = 16, M = 128: 7.3 instead of 8.3 us)
        if (g < a.n_groups) issue_loads(g);
        if constexpr (MODE == kFused) load_tables_to_lds();
        while (g < a.n_groups) {
#pragma unroll
            for (int r = 0; r < RPI; ++r)
#pragma unroll
                for (int i = 0; i < DV; ++i)
                    *reinterpret_cast<f4 *>(stage + r * ROWB + 16 * (lane + 64 * i)) = pre[r][i];
            const int64_t gn = g + gstride;
            if (gn < a.n_groups) issue_loads(gn);
            wave_lds_fence();
            const float x0 = widen_at<DT>(st, tr.j0), x1 = widen_at<DT>(st, tr.j1), x2 = widen_at<DT>(st, tr.j2),
                        x3 = widen_at<DT>(st, tr.j3);
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

            if constexpr (MODE == kFused) {
#pragma unroll
                for (int r = 0; r < RPI; ++r) {
                    const int64_t row = g * RPI + r;
                    if (row >= a.N) break;
                    unsigned cw[CW];
#pragma unroll
                    for (int q = 0; q < CW; ++q)
                        cw[q] = (unsigned)__builtin_amdgcn_readlane((int)p, r * C + 8 * q);
                    uint32_t acc_e = 0, acc_o = 0;
                    scan_row_addtid<C, AVG>(cw, acc_e, acc_o);
                    if (col_on) store_row(a, row, lane, acc_e, acc_o, sc, of, 0, AVG ? C : 0);
                }
            }
            g = gn;
        }
    }
}

template <int MODE, int C, int DV, int WAVES, int RPI = 64 / C, bool AVG = false, int DT = kF32>
int launch_variant(const RowsArgs &a, int blocks_per_cu, hipStream_t stream)
{
    const size_t lds = (MODE == kEncode ? 0 : (size_t)C * 16 * 256) +
                       (MODE == kScan ? 0 : (size_t)WAVES * RPI * DV * 256 * 4);
    const DeviceInfo &dev = device_info();
    if (lds > (size_t)dev.lds_per_block) return 1;
    if (int rc = allow_full_lds<rows_kernel<MODE, C, DV, WAVES, RPI, AVG, DT>>(); rc != MADDNESS_OK) return rc;
    const int64_t units = (MODE == kScan) ? a.N : a.n_groups;  // work items a wavefront takes in turn
    const int64_t blocks_needed = (units + WAVES - 1) / WAVES;
    const int64_t max_grid = (int64_t)dev.cus * blocks_per_cu;
    const int grid = (int)(blocks_needed < max_grid ? blocks_needed : max_grid);
    note_kernel("rows_kernel", __PRETTY_FUNCTION__);
    hipLaunchKernelGGL((rows_kernel<MODE, C, DV, WAVES, RPI, AVG, DT>), dim3(grid), dim3(WAVES * 64), lds, stream, a);
    return check_hip(hipGetLastError(), "launch rows_kernel");
}


// ---------------------------------------------------------------------------
// Tables larger than LDS (C = 64, or C = 32 with more than 256 output columns):
// a workgroup takes a block of WAVES * rw rows through phases.
//   E   every wavefront encodes its rw rows as above (register prefetch, staging
//       in the LDS area that later holds the tables) and leaves the packed codes
//       (C / 2 bytes per row) in LDS;
//   S   for each tile of MT output columns (all C codebooks; TILE_KB = 16 C MT / 1024
//       is 128 or 64): the workgroup loads the tile (16-byte pieces, several in
//       flight per thread); then every wavefront goes through its rows,
//       64 / (MT / 4) at a time: a lane owns 4 columns of one row, expands that
//       row's codes to table addresses itself, and sums, dequantises and stores its
//       4 outputs.
// The tile is re-loaded once per block of rows, so the block is made as large as
// the LDS left beside the tile allows (64 rows per wavefront).  E (HBM-bound) and S
// (LDS/VALU-bound) of one workgroup do not overlap; with 64 KiB tiles two workgroups
// share a CU and the phases of one overlap those of the other.
// ---------------------------------------------------------------------------
template <bool ENCODE, int C, int DV, int WAVES, int TILE_KB, bool AVG = false>
__global__ __launch_bounds__(WAVES * 64) __attribute__((amdgpu_waves_per_eu(4, 4)))   // 16 wavefronts per CU: at most 128 registers
void tiled_rows_kernel(const RowsArgs a, const int rw)
{
    static_assert(C == 32 || C == 64, "codebooks");
    static_assert(TILE_KB == 128 || TILE_KB == 64, "one or two workgroups per CU");
    constexpr int RPI = 64 / C;           // rows per encode step
    constexpr int TILE_BYTES = TILE_KB * 1024;
    constexpr int MT = TILE_BYTES / (16 * C);   // output columns per tile
    constexpr int LPR = MT / 4;           // lanes per row in the scan
    constexpr int RPP = 64 / LPR;         // rows per scan step
    constexpr int ROWF = DV * 256;
    static_assert(WAVES * RPI * ROWF * 4 <= TILE_BYTES, "staging must fit the tile area");
    constexpr int CB = C / 2;             // bytes of packed codes per row
    constexpr int CW = C / 8;             // ... in 32-bit words

    extern __shared__ __align__(16) unsigned char smem[];
    const unsigned char *tile = smem;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    unsigned char *stage = smem + wave * (RPI * ROWF * 4);
    unsigned char *my_codes = smem + TILE_BYTES + (size_t)wave * rw * CB;   // room for rw rows

    const int c = lane & (C - 1);
    Tree tr = {};
    if constexpr (ENCODE) load_tree(tr, a.split_dims + 4 * c, a.thresholds + 16 * c, a.D);
    const int n_col_tiles = (a.M + MT - 1) / MT;

    const int64_t rows_per_block = (int64_t)WAVES * rw;
    const int64_t n_blocks = (a.N + rows_per_block - 1) / rows_per_block;

    for (int64_t blk = blockIdx.x; blk < n_blocks; blk += gridDim.x) {
        const int64_t row0 = blk * rows_per_block + (int64_t)wave * rw;
        if constexpr (ENCODE) {
            // ---- E ----
            encode_rows_to_lds<C, DV>(a, tr, stage, my_codes, row0, rw, lane);
        } else {
            // packed codes of this wavefront's rows: 16 bytes per lane and step
            const int total16 = rw * CB / 16;
            for (int i = lane; i < total16; i += 64) {
                const int64_t row = row0 + (i * 16) / CB;
                uint4 v = make_uint4(0u, 0u, 0u, 0u);
                if (row < a.N) v = *reinterpret_cast<const uint4 *>(a.codes_in + row0 * CB + (size_t)i * 16);
                *reinterpret_cast<uint4 *>(my_codes + i * 16) = v;
            }
        }
        __syncthreads();   // the staging area becomes the table tile

        // ---- S ----
        for (int ct = 0; ct < n_col_tiles; ++ct) {
            const int col0 = ct * MT;
            {
                // C * 16 table rows of MT bytes = MT / 16 pieces of 16 bytes each;
                // piece idx = u * threads + tid, a uniform base plus a per-thread offset
                constexpr int PPR = MT / 16;                     // pieces per table row
                constexpr int PIECES = C * 16 * PPR;
                constexpr int PER_THREAD = PIECES / (WAVES * 64);
                static_assert(PIECES % (WAVES * 64) == 0, "tile pieces per thread");
                constexpr int ROWS_PER_STEP = WAVES * 64 / PPR;  // table rows covered by one u
                const unsigned toff = (unsigned)(tid / PPR) * (unsigned)a.M + 16u * (tid % PPR);
                const bool piece_on = col0 + 16 * (tid % PPR) < a.M;
#pragma unroll
                for (int u0 = 0; u0 < PER_THREAD; u0 += 4) {
                    uint4 v[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const uint8_t *ubase = a.luts + (size_t)((u0 + u) * ROWS_PER_STEP) * a.M + col0;
                        v[u] = make_uint4(0u, 0u, 0u, 0u);
                        if (piece_on) v[u] = *reinterpret_cast<const uint4 *>(ubase + toff);
                    }
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        *reinterpret_cast<uint4 *>(smem + ((u0 + u) * (WAVES * 64) + tid) * 16) = v[u];
                }
            }
            const int g = lane & (LPR - 1);
            const int col = col0 + 4 * g;
            const bool col_on = col < a.M;
            f4 sc = {0.f, 0.f, 0.f, 0.f}, of = {0.f, 0.f, 0.f, 0.f};
            if (col_on) {
                sc = *reinterpret_cast<const f4 *>(a.scale + col);
                of = *reinterpret_cast<const f4 *>(a.offset + col);
            }
            __syncthreads();
            const unsigned char *lane_tile = tile + 4 * g;
#pragma unroll 1
            for (int r0 = 0; r0 < rw; r0 += RPP) {
                const int rl = r0 + lane / LPR;
                const int64_t row = row0 + rl;
                // this row's packed codes, eight per register
                unsigned cw[CW];
#pragma unroll
                for (int q4 = 0; q4 < CW; q4 += 4) {
                    const uint4 t = *reinterpret_cast<const uint4 *>(my_codes + rl * CB + 4 * q4);
                    cw[q4] = t.x; cw[q4 + 1] = t.y; cw[q4 + 2] = t.z; cw[q4 + 3] = t.w;
                }
                uint32_t acc_e = 0, acc_o = 0;
                auto word = [&](int cc) INLINE_LAMBDA {
                    const unsigned k = (cw[cc >> 3] >> (4 * (cc & 7))) & 15u;
                    return *reinterpret_cast<const uint32_t *>(lane_tile + (cc * 16 + k) * MT);
                };
                if constexpr (!AVG) {
#pragma unroll
                    for (int cc = 0; cc < C; cc += 2) {
                        const uint32_t y0 = word(cc), y1 = word(cc + 1);
                        acc_e += (y0 & 0x00FF00FFu) + (y1 & 0x00FF00FFu);
                        acc_o += __builtin_amdgcn_perm(y0, y0, 0x0c030c01u) + __builtin_amdgcn_perm(y1, y1, 0x0c030c01u);
                    }
                } else {
                    // pairwise averages in blocks of 16 codebooks (Appendix D)
#pragma unroll
                    for (int c0 = 0; c0 < C; c0 += 16) {
                        uint32_t y[16];
#pragma unroll
                        for (int u = 0; u < 16; ++u) y[u] = word(c0 + u);
#pragma unroll
                        for (int span = 1; span < 16; span *= 2)
#pragma unroll
                            for (int u = 0; u < 16; u += 2 * span)
                                y[u] = __builtin_amdgcn_lerp(y[u], y[u + span], 0x01010101u);
                        acc_e += y[0] & 0x00FF00FFu;
                        acc_o += __builtin_amdgcn_perm(y[0], y[0], 0x0c030c01u);
                    }
                }
                if (col_on && row < a.N) store_row(a, row, g, acc_e, acc_o, sc, of, col0, AVG ? C : 0);
            }
            __syncthreads();
        }
    }
}

// Fewest rows for which fp32 rows with C = 32 go to the phased matrix-core kernel although
// their tables would fit in LDS.
#ifndef MADDNESS_PHASED_MIN_ROWS
#define MADDNESS_PHASED_MIN_ROWS 262144
#endif
// ... and for which they are encoded by its first phase alone.
#ifndef MADDNESS_ENCODE_PHASED_MIN_ROWS
#define MADDNESS_ENCODE_PHASED_MIN_ROWS 262144
#endif

// Fused kernel for tables larger than LDS: two workgroups of 8 wavefronts per CU with
// 64 KiB tiles (3.72 ms for 2^21 rows of the stress workload) against one of 16 with
// 128 KiB tiles (4.03 ms): the streaming phase of one overlaps the scan of the other.
// Starting the two half a period apart on purpose changed nothing.
#ifndef MADDNESS_TILED_KB
#define MADDNESS_TILED_KB 64
#define MADDNESS_TILED_WAVES 8
#endif
// TILE_KB = 128: one workgroup per CU; 64: two.
template <bool ENCODE, int C, int DV, int WAVES, int TILE_KB, bool AVG = false>
int launch_tiled(const RowsArgs &a, hipStream_t stream)
{
    constexpr int RPI = 64 / C;
    constexpr int RPP = 64 / ((TILE_KB * 1024 / (16 * C)) / 4);
    constexpr int STEP = RPI > RPP ? RPI : RPP;   // both are powers of two
    constexpr int PER_CU = 128 / TILE_KB;
    const DeviceInfo &dev = device_info();
    const int tile_bytes = TILE_KB * 1024;
    int rw = (dev.lds_per_block / PER_CU - tile_bytes) / (WAVES * (C / 2));
    if (rw > 64) rw = 64;
    rw = rw / STEP * STEP;
    if (rw < STEP) return 1;
    const size_t lds = (size_t)tile_bytes + (size_t)WAVES * rw * (C / 2);
    if (int rc = allow_full_lds<tiled_rows_kernel<ENCODE, C, DV, WAVES, TILE_KB, AVG>>(); rc != MADDNESS_OK) return rc;
    const int64_t rows_per_block = (int64_t)WAVES * rw;
    const int64_t blocks_needed = (a.N + rows_per_block - 1) / rows_per_block;
    const int64_t max_grid = (int64_t)dev.cus * PER_CU;
    const int grid = (int)(blocks_needed < max_grid ? blocks_needed : max_grid);
    note_kernel("tiled_rows_kernel", __PRETTY_FUNCTION__);
    hipLaunchKernelGGL((tiled_rows_kernel<ENCODE, C, DV, WAVES, TILE_KB, AVG>), dim3(grid), dim3(WAVES * 64), lds,
                       stream, a, rw);
    return check_hip(hipGetLastError(), "launch tiled_rows_kernel");
}

// encode-only launches for the narrow element types
template <int C, int DT>
int encode_narrow_dt(const RowsArgs &a, bool one_piece, hipStream_t stream)
{
    constexpr int RPI = 64 / C;
    // a wavefront has one group of RPI rows in flight: where that is no more than 1 KiB, eight instead of four
    // workgroups per CU (uint8 rows, N = 2^20, D = 512, C = 32: 0.10 instead of 0.13 ms; rows of 1 KiB, two per
    // group, are slower that way: 0.192 against 0.185 ms)
    const int per_cu = RPI * a.D * elem_size(DT) <= 1024 ? 8 : 4;
    return one_piece ? launch_variant<kEncode, C, 1, 4, RPI, false, DT>(a, per_cu, stream)
                     : launch_variant<kEncode, C, 2, 4, RPI, false, DT>(a, 4, stream);
}

int encode_narrow(const RowsArgs &a, int C, int dtype, bool one_piece, hipStream_t stream)
{
    switch (dtype) {
    case MADDNESS_F16:
        return C == 32 ? encode_narrow_dt<32, kF16>(a, one_piece, stream) : encode_narrow_dt<64, kF16>(a, one_piece, stream);
    case MADDNESS_BF16:
        return C == 32 ? encode_narrow_dt<32, kBF16>(a, one_piece, stream) : encode_narrow_dt<64, kBF16>(a, one_piece, stream);
    default:
        return C == 32 ? encode_narrow_dt<32, kU8>(a, one_piece, stream) : encode_narrow_dt<64, kU8>(a, one_piece, stream);
    }
}

// rows of 16-byte pieces: row length and stride are multiples of 16 bytes
bool rows_ok(int D, const MatrixA &A)
{
    const int es = A.elem_bytes();
    return !A.col_major && (D * es) % 16 == 0 && (A.ld * es) % 16 == 0 && aligned_to(A.data, 16);
}

}  // namespace

// Each launcher returns MADDNESS_OK when the launch was made, 1 when the shape is
// not one these kernels cover (the caller then uses the general kernels), or an
// error status.

int launch_fused_rows(const maddness_params &p, const MatrixA &A, int64_t N, int32_t M,
                      const uint8_t *luts, const float *scale, const float *offset, float *out,
                      int64_t ldo, uint16_t *acc, uint8_t *codes, bool averaged, hipStream_t stream)
{
    const int C = p.C, D = p.D;
    if (!rows_ok(D, A) || (codes && !aligned_to(codes, 4))) {
        // rows that are not whole aligned 16-byte pieces: many fp32 rows go to the phased kernel's form
        // for any shape
        if (A.plain() && !averaged && !vector_scan_only())
            return launch_fused_mfma(p, A, N, M, luts, scale, offset, out, ldo, acc, codes, stream);
        return 1;
    }
    RowsArgs a{};
    a.A = A.data; a.lda = A.ld; a.D = D; a.N = N;
    a.split_dims = p.split_dims; a.thresholds = p.thresholds;
    a.luts = luts; a.scale = scale; a.offset = offset; a.M = M;
    a.out = out; a.ldo = ldo; a.acc = acc; a.codes_out = codes;
    if (A.dtype != MADDNESS_F32) {
        // narrow elements: with fewer bytes to read than to write the one-kernel-per-wavefront
        // design is bound by the vector ALUs; the phased kernel with the scan on the matrix
        // cores is bound by HBM
        if (!averaged && !vector_scan_only()) {
            const int rc = launch_fused_mfma(p, A, N, M, luts, scale, offset, out, ldo, acc, codes, stream);
            if (rc != 1) return rc;
        }
        // C = 32 with the tables in LDS, rows of at most 2 KiB
        if (C != 32 || averaged || !tables_ok(C, M, luts, scale, offset, out, ldo, acc)) return 1;
        const int row_bytes = D * A.elem_bytes();
        if (row_bytes > 2048) return 1;
        a.n_groups = N;
        const bool one = row_bytes <= 1024;
        switch (A.dtype) {
        case MADDNESS_F16:
            return one ? launch_variant<kFused, 32, 1, 16, 1, false, kF16>(a, 1, stream)
                       : launch_variant<kFused, 32, 2, 16, 1, false, kF16>(a, 1, stream);
        case MADDNESS_BF16:
            return one ? launch_variant<kFused, 32, 1, 16, 1, false, kBF16>(a, 1, stream)
                       : launch_variant<kFused, 32, 2, 16, 1, false, kBF16>(a, 1, stream);
        default:
            return one ? launch_variant<kFused, 32, 1, 16, 1, false, kU8>(a, 1, stream)
                       : launch_variant<kFused, 32, 2, 16, 1, false, kU8>(a, 1, stream);
        }
    }
    // tables larger than LDS: the exact scan runs on the matrix cores; the averaged one,
    // and few rows, over column tiles in LDS
    const bool big = (C == 64 && M > 64) || (C == 32 && M > 256);
    if (big && !averaged && !vector_scan_only()) {
        const int rc = launch_fused_mfma(p, A, N, M, luts, scale, offset, out, ldo, acc, codes, stream);
        if (rc != 1) return rc;
    }
    if (big && M % 16 == 0 && aligned_to(luts, 16) && aligned_to(scale, 16) && aligned_to(offset, 16) &&
        (!out || (ldo % 4 == 0 && aligned_to(out, 16))) && (!acc || aligned_to(acc, 8))) {
        if (C == 64 && D <= 1024)
            return averaged ? launch_tiled<true, 64, 4, MADDNESS_TILED_WAVES, MADDNESS_TILED_KB, true>(a, stream)
                            : launch_tiled<true, 64, 4, MADDNESS_TILED_WAVES, MADDNESS_TILED_KB>(a, stream);
        if (C == 32 && D <= 512 && !averaged) return launch_tiled<true, 32, 2, MADDNESS_TILED_WAVES, MADDNESS_TILED_KB>(a, stream);
        return 1;
    }
    // every other shape with C = 32 or 64 (longer rows, few or oddly many columns): the
    // phased kernel again, where it applies
    auto other_shapes = [&]() -> int {
        if (averaged || vector_scan_only()) return 1;
        return launch_fused_mfma(p, A, N, M, luts, scale, offset, out, ldo, acc, codes, stream);
    };
    // Many rows of C = 32 or 16: the phased kernel again.  The chip as a whole first reads, then
    // writes, which HBM serves faster than the mixture of the kernels below (N = 2^20,
    // D = 512, M = 256: 0.515 against 0.534 ms; 0.075 against 0.069 ms at N = 2^17), as long
    // as the rows of the output start on 128-byte lines (it writes a row in pieces of 256 bytes).
    if ((C == 32 || C == 16) && N >= MADDNESS_PHASED_MIN_ROWS && (!out || ldo % 32 == 0))
        if (const int rc = other_shapes(); rc != 1) return rc;
    if (!tables_ok(C, M, luts, scale, offset, out, ldo, acc)) return other_shapes();
    const int RPI = 64 / C;
    a.n_groups = (N + RPI - 1) / RPI;
    if (C == 32 && D <= 256 && !averaged) return launch_variant<kFused, 32, 1, 8>(a, 1, stream);
    if (C == 32 && D <= 512) {
        // 128 KiB of tables leave 32 KiB of staging: 16 wavefronts with one row each
        // hide latency better than 8 with two (0.545 ms against 0.576 ms at
        // N = 2^20, M = 256), at the same 32 KiB of loads in flight per CU
        a.n_groups = N;
        return averaged ? launch_variant<kFused, 32, 2, 16, 1, true>(a, 1, stream)
                        : launch_variant<kFused, 32, 2, 16, 1>(a, 1, stream);
    }
    if (averaged) return 1;
    if (C == 16 && D <= 256) return launch_variant<kFused, 16, 1, 8>(a, 1, stream);
    if (C == 16 && D <= 512) return launch_variant<kFused, 16, 2, 8>(a, 1, stream);
    return other_shapes();
}

int launch_encode_rows(const maddness_params &p, const MatrixA &A, int64_t N, uint8_t *codes,
                       hipStream_t stream)
{
    const int C = p.C, D = p.D;
    if (!rows_ok(D, A) || !aligned_to(codes, 4) || (C != 16 && C != 32 && C != 64 && C % 8 != 0)) {
        // any other shape of many fp32 rows: the first phase of the phased kernel in its form for any shape
        if (A.plain() && N >= MADDNESS_ENCODE_PHASED_MIN_ROWS) return launch_encode_phased(p, A, N, codes, stream);
        return 1;
    }
    if (N < 4096) return 1;
    // many fp32 rows: the first phase of the phased kernel (0.305 against 0.347 ms at
    // N = 2^20, D = 512, C = 32; the narrow types are better off below); it also takes the
    // other multiples of 8 codebooks
    if (A.dtype == MADDNESS_F32 && N >= MADDNESS_ENCODE_PHASED_MIN_ROWS)
        if (const int rc = launch_encode_phased(p, A, N, codes, stream); rc != 1) return rc;
    if (C != 16 && C != 32 && C != 64) return 1;
    RowsArgs a{};
    a.A = A.data; a.lda = A.ld; a.D = D; a.N = N;
    a.split_dims = p.split_dims; a.thresholds = p.thresholds;
    a.codes_out = codes;
    const int RPI = 64 / C;
    a.n_groups = (N + RPI - 1) / RPI;
    if (A.dtype != MADDNESS_F32) {
        // narrow elements: C = 32 or 64, rows of at most 2 KiB
        const int row_bytes = D * A.elem_bytes();
        if ((C != 32 && C != 64) || row_bytes > 2048) return 1;
        return encode_narrow(a, C, A.dtype, row_bytes <= 1024, stream);
    }
    if (C == 64 && D <= 1024) return launch_variant<kEncode, 64, 4, 4>(a, 2, stream);
    if (C == 32 && D <= 512) return launch_variant<kEncode, 32, 2, 4>(a, 4, stream);
    if (C == 32 && D <= 1024) return launch_variant<kEncode, 32, 4, 4>(a, 2, stream);
    if (C == 16 && D <= 512) return launch_variant<kEncode, 16, 2, 4>(a, 1, stream);
    return 1;
}

int launch_scan_rows(int32_t C, int32_t M, const uint8_t *codes, int64_t N, const uint8_t *luts,
                     const float *scale, const float *offset, float *out, int64_t ldo, uint16_t *acc,
                     bool averaged, hipStream_t stream)
{
    if (!aligned_to(codes, 16)) return 1;
    RowsArgs a{};
    a.N = N; a.codes_in = codes;
    a.luts = luts; a.scale = scale; a.offset = offset; a.M = M;
    a.out = out; a.ldo = ldo; a.acc = acc;
    const bool big = (C == 64 && M > 64) || (C == 32 && M > 256);
    if (big && M % 16 == 0 && aligned_to(luts, 16) && aligned_to(scale, 16) && aligned_to(offset, 16) &&
        (!out || (ldo % 4 == 0 && aligned_to(out, 16))) && (!acc || aligned_to(acc, 8))) {
        if (C == 64)
            return averaged ? launch_tiled<false, 64, 1, 16, 128, true>(a, stream)
                            : launch_tiled<false, 64, 1, 16, 128>(a, stream);
        if (averaged) return 1;
        return launch_tiled<false, 32, 1, 16, 128>(a, stream);
    }
    if (!tables_ok(C, M, luts, scale, offset, out, ldo, acc)) return 1;
    if (C == 32)
        return averaged ? launch_variant<kScan, 32, 1, 16, 2, true>(a, 1, stream)
                        : launch_variant<kScan, 32, 1, 16>(a, 1, stream);
    if (C == 16)
        return averaged ? launch_variant<kScan, 16, 1, 16, 4, true>(a, 1, stream)
                        : launch_variant<kScan, 16, 1, 16>(a, 1, stream);
    return 1;
}

}  // namespace maddness
