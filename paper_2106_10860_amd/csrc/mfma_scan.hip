// The exact table scan on the matrix cores, codes read from memory: a wavefront
// keeps the tables of its output columns in registers for the whole kernel and
// streams over the rows.  See mfma_common.h for the formulation.
#include "mfma_common.h"

namespace maddness {
namespace {

using namespace mfma;

struct MfmaScanArgs {
    const uint8_t *codes;   // [N][C / 2]
    const uint8_t *luts;    // [C][16][M]
    const float *scale;
    const float *offset;
    ScanOut o;
    int64_t N;
    int codebooks;          // the any-shape form: the real number of codebooks (<= the kernel's C); rows of codes
                            // are (codebooks + 1) / 2 bytes
};

// The dequantised results of one step of a workgroup (16 rows, or 32 with NT = 2, times its
// 4 blocks of columns) collected in LDS and written out row by row: a store instruction then
// covers 1 KiB (512 bytes) of one row instead of 256 (128) bytes of four rows.  For outputs
// whose rows do not start on 128-byte lines, where the direct stores end inside lines and run
// at a third to a half of their rate.  All 4 wavefronts take part in every step (barriers).
// ODD: any number of codebooks up to C (the others padded with zero codes and entries), any M,
// any pitch and alignment of codes, tables and outputs: codes and tables are read byte by byte,
// rows are written as ranges of floats in aligned 16-byte pieces (store_dense_rows): the 16 or 32
// consecutive rows of a step as one range when there is no padding between them, else row by row.
template <int KG, int NT, bool ODD = false>
__device__ __forceinline__ void scan_gathered(const MfmaScanArgs &a, const v4i *one_hot, float *tile, int lane, int wave)
{
    constexpr int C = 4 * KG;
    constexpr int CW = C / 8;
    constexpr int SPAN = 16 * NT;
    constexpr int GPS = NT == 2 ? 2 : 1;            // groups of 16 rows per step
    constexpr int TILE_LD = 4 * SPAN + 4;           // floats per tile row (4 of padding)
    typedef unsigned cvec __attribute__((ext_vector_type(CW)));
    typedef float piece __attribute__((ext_vector_type(NT)));
    const int j = lane & 15, g = lane >> 4;
    const int col0 = blockIdx.y * 4 * SPAN;          // first column of the workgroup
    const int col = col0 + wave * SPAN + NT * j;     // first of this lane's NT columns
    const bool col_on = col < a.o.M;
    const bool active = col0 + wave * SPAN < a.o.M;  // the wavefront has columns
    const int n_cols = a.o.M - col0 < 4 * SPAN ? a.o.M - col0 : 4 * SPAN;

    v4i B[NT][KG];
    float sc[NT], of[NT];
    if (active) load_tables<KG, NT, ODD, ODD>(B, a.luts, a.o.M, col, col_on, g, a.codebooks);
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const bool on = ODD ? col + t < a.o.M : col_on;
        sc[t] = on ? a.scale[col + t] : 0.f;
        of[t] = on ? a.offset[col + t] : 0.f;
    }
    const ScanOut acc_only{nullptr, 0, a.o.acc, a.o.M};
    const int64_t n_groups = (a.N + 15) >> 4;
    // rows without padding between them, all columns in this workgroup: the rows of a step are one range of floats
    const bool dense = ODD && a.o.out && a.o.ldo == a.o.M && gridDim.y == 1;
    const float inv_M = 1.0f / (float)a.o.M;
    auto load_codes = [&](int64_t rg) INLINE_LAMBDA {
        const int64_t row = rg * 16 + j;
        cvec v = {};
        if constexpr (ODD) {
            const int bytes = (a.codebooks + 1) / 2;
            if (row < a.N) {
                // whole words of the row as (unaligned) 32-bit loads, the last one to three bytes one by one
                const uint8_t *src = a.codes + row * bytes;
#pragma unroll
                for (int q = 0; q < CW; ++q) {
                    if (4 * q + 4 <= bytes) {
                        uint32_t w;
                        __builtin_memcpy(&w, src + 4 * q, 4);
                        v[q] = w;
                    } else {
#pragma unroll
                        for (int t = 0; t < 3; ++t)
                            if (4 * q + t < bytes) v[q] |= (unsigned)src[4 * q + t] << (8 * t);
                    }
                }
            }
        } else {
            // (rows are C / 2 bytes apart and only the base is known to be 16-byte aligned: copied as
            // words, so that no wider alignment than a word's is assumed of a row)
            if (row < a.N) __builtin_memcpy(&v, reinterpret_cast<const uint32_t *>(a.codes + row * (C / 2)), sizeof(uint32_t) * CW);
        }
        return v;
    };
    // step s of this workgroup: groups GPS (blockIdx.x + s gridDim.x) + 0 .. GPS - 1, i.e. 16 GPS
    // consecutive rows
    for (int64_t rg = (int64_t)GPS * blockIdx.x; rg < n_groups; rg += (int64_t)GPS * gridDim.x) {
        if (active) {
            v4i acc[GPS][NT];
            if constexpr (GPS == 2) scan16x2<KG, NT>(load_codes(rg), load_codes(rg + 1), B, g, one_hot, acc[0], acc[1]);
            else scan16<KG, NT>(load_codes(rg), B, g, one_hot, acc[0]);
            if (col_on) {
#pragma unroll
                for (int q = 0; q < GPS; ++q) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        piece v;
#pragma unroll
                        for (int t = 0; t < NT; ++t) v[t] = fmaf((float)acc[q][t][r], sc[t], of[t]);
                        *reinterpret_cast<piece *>(tile + (q * 16 + 4 * g + r) * TILE_LD + wave * SPAN + NT * j) = v;
                    }
                    if (a.o.acc) {
                        const int64_t r0 = (rg + q) * 16;
                        if constexpr (ODD) {
#pragma unroll
                            for (int r = 0; r < 4; ++r)
#pragma unroll
                                for (int t = 0; t < NT; ++t)
                                    if (r0 + 4 * g + r < a.N && col + t < a.o.M)
                                        a.o.acc[(r0 + 4 * g + r) * a.o.M + col + t] = (uint16_t)acc[q][t][r];
                        } else {
                            store16<NT>(acc_only, acc[q], [r0](int k) { return r0 + k; }, a.N, g, col, sc, of);
                        }
                    }
                }
            }
        }
        __syncthreads();
        // row r of the step goes out through wavefront r % 4, NT columns per lane and instruction
        if (ODD && dense) {
            // the 16 GPS consecutive rows of the step are one range of floats
            const int64_t first = rg * 16, left = a.N - first;
            store_dense_rows(a.o.out + first * a.o.M, left < 16 * GPS ? (int)left : 16 * GPS, a.o.M, inv_M, tile, TILE_LD, 0,
                             (int)threadIdx.x, 256);
        } else
        for (int r = wave; r < 16 * GPS; r += 4) {
            const int64_t row = rg * 16 + r;
            if (row >= a.N) break;
            float *dst = a.o.out + row * a.o.ldo + col0;
            if constexpr (ODD) {
                // a row (its columns of this workgroup) as a range of its own
                if (!a.o.out) continue;
                store_dense_rows<true>(dst, 1, n_cols, 0.f, tile, TILE_LD, r, lane, 64);
            } else {
                for (int c = lane; c < n_cols / NT; c += 64)
                    __builtin_nontemporal_store(*reinterpret_cast<const piece *>(tile + r * TILE_LD + NT * c),
                                                reinterpret_cast<piece *>(dst + NT * c));
            }
        }
        __syncthreads();   // the tile is rewritten in the next step
    }
}

// KG: groups of four codebooks (C = 4 KG); NT: column tiles per wavefront (4 or 2);
// GATHER: results through LDS, whole rows written (above).
template <int KG, int NT, bool GATHER = false, bool ODD = false>
__global__ __launch_bounds__(256, 2) void mfma_scan_kernel(const MfmaScanArgs a)
{
    static_assert(!ODD || GATHER, "the any-shape form writes whole rows through LDS");
    static_assert(NT == 4 || NT == 2, "tiles per wavefront");
    static_assert(KG % 2 == 0, "whole words of packed codes");
    constexpr int C = 4 * KG;
    constexpr int CW = C / 8;          // 32-bit words of packed codes per row
    constexpr int SPAN = 16 * NT;      // output columns per wavefront
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int j = lane & 15, g = lane >> 4;
    __shared__ v4i one_hot[16];
    fill_one_hot_table(one_hot, threadIdx.x);
    __syncthreads();
    if constexpr (GATHER) {
        __shared__ __align__(16) float tile[(NT == 2 ? 32 : 16) * (4 * SPAN + 4)];
        scan_gathered<KG, NT, ODD>(a, one_hot, tile, lane, wave);
        return;
    }
    // blocks of SPAN columns for the 4 wavefronts; with fewer than 4 blocks in all,
    // `share` wavefronts hold the same block and take every share-th group of rows
    const int col_blocks = (a.o.M + SPAN - 1) / SPAN;
    const int share = col_blocks >= 3 ? 1 : (col_blocks == 2 ? 2 : 4);
    const int blocks_here = 4 / share;
    const int c0 = (blockIdx.y * blocks_here + wave % blocks_here) * SPAN;   // first column of this wavefront
    if (c0 >= a.o.M) return;                        // no barriers below
    const int col = c0 + NT * j;                    // first of this lane's NT columns
    const bool col_on = col < a.o.M;                // M is a multiple of NT

    v4i B[NT][KG];
    load_tables<KG, NT>(B, a.luts, a.o.M, col, col_on, g);
    float sc[NT], of[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        sc[t] = col_on ? a.scale[col + t] : 0.f;
        of[t] = col_on ? a.offset[col + t] : 0.f;
    }

    // rows, 16 at a time; the codes of the next group are fetched ahead
    typedef unsigned cvec __attribute__((ext_vector_type(CW)));
    const int64_t n_groups = (a.N + 15) >> 4;
    auto load_codes = [&](int64_t rg) INLINE_LAMBDA {
        const int64_t row = rg * 16 + j;
        // (rows are C / 2 bytes apart and only the base is known to be 16-byte aligned: copied as
        // words, so that no wider alignment than a word's is assumed of a row)
        cvec v = {};
        if (row < a.N) __builtin_memcpy(&v, reinterpret_cast<const uint32_t *>(a.codes + row * (C / 2)), sizeof(uint32_t) * CW);
        return v;
    };
    int64_t rg = (int64_t)blockIdx.x * share + wave / blocks_here;
    const int64_t stride = (int64_t)gridDim.x * share;
    if constexpr (NT == 2) {
        // two groups per step: four independent accumulation chains for the matrix pipe
        cvec next0 = {}, next1 = {};
        if (rg < n_groups) next0 = load_codes(rg);
        if (rg + stride < n_groups) next1 = load_codes(rg + stride);
        for (; rg + stride < n_groups; rg += 2 * stride) {
            const cvec cw0 = next0, cw1 = next1;
            if (rg + 2 * stride < n_groups) next0 = load_codes(rg + 2 * stride);
            if (rg + 3 * stride < n_groups) next1 = load_codes(rg + 3 * stride);
            v4i acc0[NT], acc1[NT];
            scan16x2<KG, NT>(cw0, cw1, B, g, one_hot, acc0, acc1);
            if (col_on) {
                const int64_t r1 = rg + stride;
                store16<NT>(a.o, acc0, [rg](int k) { return rg * 16 + k; }, a.N, g, col, sc, of);
                store16<NT>(a.o, acc1, [r1](int k) { return r1 * 16 + k; }, a.N, g, col, sc, of);
            }
        }
        if (rg < n_groups) {   // an odd group left over; its codes are in next0
            v4i acc[NT];
            scan16<KG, NT>(next0, B, g, one_hot, acc);
            if (col_on) store16<NT>(a.o, acc, [rg](int k) { return rg * 16 + k; }, a.N, g, col, sc, of);
        }
    } else {
        cvec next = {};
        if (rg < n_groups) next = load_codes(rg);
        for (; rg < n_groups; rg += stride) {
            const cvec cw = next;
            if (rg + stride < n_groups) next = load_codes(rg + stride);
            v4i acc[NT];
            scan16<KG, NT>(cw, B, g, one_hot, acc);
            if (col_on) store16<NT>(a.o, acc, [rg](int k) { return rg * 16 + k; }, a.N, g, col, sc, of);
        }
    }
}

template <int KG, int NT, bool ODD = false>
int launch_mfma(const MfmaScanArgs &a, hipStream_t stream)
{
    const DeviceInfo &dev = device_info();
    const int span = 16 * NT * 4;                       // columns per workgroup of 4 wavefronts
    const int gy = (a.o.M + span - 1) / span;
    const int col_blocks = (a.o.M + 16 * NT - 1) / (16 * NT);
    if constexpr (ODD) {
        const int64_t n_steps = ((a.N + 15) / 16 + (NT == 2 ? 1 : 0)) / (NT == 2 ? 2 : 1);
        int64_t gx = (int64_t)dev.cus * 2 / gy;
        if (gx < 1) gx = 1;
        if (gx > n_steps) gx = n_steps;
        note_kernel("mfma_scan_kernel, any shape", __PRETTY_FUNCTION__);
        hipLaunchKernelGGL((mfma_scan_kernel<KG, NT, true, true>), dim3((unsigned)gx, (unsigned)gy), dim3(256), 0, stream, a);
        return check_hip(hipGetLastError(), "launch mfma_scan_kernel");
    }
    // fp32 output rows that do not start on 128-byte lines, at least 3 blocks of columns (no
    // sharing of blocks among wavefronts): whole rows through LDS
    if (a.o.out && col_blocks >= 3 && (a.o.ldo % 32 != 0 || !aligned_to(a.o.out, 128))) {
        const int64_t n_steps = ((a.N + 15) / 16 + (NT == 2 ? 1 : 0)) / (NT == 2 ? 2 : 1);
        int64_t gx = (int64_t)dev.cus * 2 / gy;
        if (gx < 1) gx = 1;
        if (gx > n_steps) gx = n_steps;
        note_kernel("mfma_scan_kernel, gathered stores", __PRETTY_FUNCTION__);
        hipLaunchKernelGGL((mfma_scan_kernel<KG, NT, true>), dim3((unsigned)gx, (unsigned)gy), dim3(256), 0, stream, a);
        return check_hip(hipGetLastError(), "launch mfma_scan_kernel");
    }
    const int share = col_blocks >= 3 ? 1 : (col_blocks == 2 ? 2 : 4);   // as in the kernel
    const int64_t n_groups = (a.N + 15) / 16;
    int64_t gx = (int64_t)dev.cus * 2 / gy;             // two workgroups per CU in all
    if (gx < 1) gx = 1;
    if (gx * share > n_groups) gx = (n_groups + share - 1) / share;
    note_kernel("mfma_scan_kernel", __PRETTY_FUNCTION__);
    hipLaunchKernelGGL((mfma_scan_kernel<KG, NT>), dim3((unsigned)gx, (unsigned)gy), dim3(256), 0, stream, a);
    return check_hip(hipGetLastError(), "launch mfma_scan_kernel");
}

}  // namespace

// Returns MADDNESS_OK after a launch, 1 if the shape is not covered.
int launch_scan_mfma(int32_t C, int32_t M, const uint8_t *codes, int64_t N, const uint8_t *luts,
                     const float *scale, const float *offset, float *out, int64_t ldo, uint16_t *acc,
                     hipStream_t stream)
{
    // whole words of packed codes per row; the tables are read once per workgroup, which
    // only pays with many rows
    if (C > 64 || N < 16384) return 1;
    const int NT = C <= 32 ? 4 : 2;
    MfmaScanArgs a{codes, luts, scale, offset, ScanOut{out, ldo, acc, M}, N, C};
    if (C % 8 != 0 || !aligned_to(codes, 16) || M % NT != 0 || !aligned_to(luts, NT) ||
        (out && (ldo % NT != 0 || !aligned_to(out, 4 * NT))) || (acc && !aligned_to(acc, 2 * NT))) {
        // any other shape: padded to 16, 32 or 64 codebooks, everything read and written in the smallest units;
        // worth it from a few blocks of columns on (M = 10 is faster in the general kernel, which does no padded work)
        if (M <= 16) return 1;
        if (C <= 16) return launch_mfma<4, 4, true>(a, stream);
        if (C <= 32) return launch_mfma<8, 4, true>(a, stream);
        return launch_mfma<16, 2, true>(a, stream);
    }
    switch (C) {
    case 8: return launch_mfma<2, 4>(a, stream);
    case 16: return launch_mfma<4, 4>(a, stream);
    case 24: return launch_mfma<6, 4>(a, stream);
    case 32: return launch_mfma<8, 4>(a, stream);
    case 40: return launch_mfma<10, 2>(a, stream);
    case 48: return launch_mfma<12, 2>(a, stream);
    case 56: return launch_mfma<14, 2>(a, stream);
    default: return launch_mfma<16, 2>(a, stream);
    }
}

}  // namespace maddness
