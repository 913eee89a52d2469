// Pieces shared by the row-streaming kernels (rows stored by rows: fused_rows.hip;
// rows stored by columns: encode_cols.hip): argument block, the per-row table scan
// and the dequantising store.
#pragma once

#include "common.h"
#include "device_common.h"
#include "scan_asm.inc"

namespace maddness {
namespace rows {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef unsigned u2 __attribute__((ext_vector_type(2)));

enum Mode { kFused = 0, kEncode = 1, kScan = 2 };

struct RowsArgs {
    const void *A;     // elements of the kernel's element type
    int64_t lda;       // row stride (fused_rows.hip) or column stride (encode_cols.hip) in elements
    int D;
    int64_t N;
    const int32_t *split_dims;
    const float *thresholds;
    const uint8_t *codes_in;
    const uint8_t *luts;
    const float *scale;
    const float *offset;
    int M;
    float *out;
    int64_t ldo;
    uint16_t *acc;
    uint8_t *codes_out;
    int64_t n_groups;  // ceil(N / RPI)
    int codebooks;     // phased kernel with padding only: the real number of codebooks, < the kernel's C
};

// Value of `v` in the lane `n` places up within the same row of 16 lanes.
template <int N_>
__device__ __forceinline__ unsigned from_lane_above(unsigned v)
{
    return (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x100 + N_ /* row_shl:N */, 0xF, 0xF, true);
}

// Sum over the C codebooks of the table words selected by the (wavefront-
// uniform) packed codes cw: even output columns accumulate in acc_e, odd ones in
// acc_o (two 16-bit sums per register).  The tables are laid out as
// [code][codebook][64 words] and the lookups are issued as ds_read_addtid_b32
// (address = M0 + immediate + 4 * lane): no vector instruction is spent on
// addresses.  Instruction text and schedule:
// gen_scan_asm.py.  All 64 lanes must be active; the tables must start at LDS
// address 0.
template <int C, bool AVG>
__device__ __forceinline__ void scan_row_addtid(const unsigned (&cw)[C / 8], uint32_t &acc_e, uint32_t &acc_o)
{
    static_assert(C == 16 || C == 32, "generated for 16 and 32 codebooks");
    uint32_t x0, x1, x2, x3, x4, x5, x6, x7, te, to, e, o;
    unsigned st;
    const unsigned mask = 0x00FF00FFu, sel = 0x0c030c01u;
#define MADDNESS_SCAN_OUTS                                                                                  \
    [ae] "+v"(acc_e), [ao] "+v"(acc_o), [x0] "=&v"(x0), [x1] "=&v"(x1), [x2] "=&v"(x2), [x3] "=&v"(x3),       \
        [x4] "=&v"(x4), [x5] "=&v"(x5), [x6] "=&v"(x6), [x7] "=&v"(x7), [te] "=&v"(te), [to] "=&v"(to),       \
        [e] "=&v"(e), [o] "=&v"(o), [st] "=&s"(st)
    if constexpr (!AVG && C == 32) {
        asm volatile(MADDNESS_SCAN_ASM_C32
                     : MADDNESS_SCAN_OUTS
                     : [c0] "s"(cw[0]), [c1] "s"(cw[1]), [c2] "s"(cw[2]), [c3] "s"(cw[3]), [mask] "s"(mask),
                       [sel] "s"(sel)
                     : "m0", "scc", "memory");
    } else if constexpr (!AVG) {
        asm volatile(MADDNESS_SCAN_ASM_C16
                     : MADDNESS_SCAN_OUTS
                     : [c0] "s"(cw[0]), [c1] "s"(cw[1]), [mask] "s"(mask), [sel] "s"(sel)
                     : "m0", "scc", "memory");
    } else {
        // pairwise averages in blocks of 16 codebooks (Appendix D): the
        // accumulators receive the sum of the block averages
        uint32_t l1, l2, l3;
        const unsigned ones = 0x01010101u;
        if constexpr (C == 32) {
            asm volatile(MADDNESS_SCAN_AVG_ASM_C32
                         : MADDNESS_SCAN_OUTS, [l1] "=&v"(l1), [l2] "=&v"(l2), [l3] "=&v"(l3)
                         : [c0] "s"(cw[0]), [c1] "s"(cw[1]), [c2] "s"(cw[2]), [c3] "s"(cw[3]), [mask] "s"(mask),
                           [sel] "s"(sel), [ones] "s"(ones)
                         : "m0", "scc", "memory");
        } else {
            asm volatile(MADDNESS_SCAN_AVG_ASM_C16
                         : MADDNESS_SCAN_OUTS, [l1] "=&v"(l1), [l2] "=&v"(l2), [l3] "=&v"(l3)
                         : [c0] "s"(cw[0]), [c1] "s"(cw[1]), [mask] "s"(mask), [sel] "s"(sel), [ones] "s"(ones)
                         : "m0", "scc", "memory");
        }
    }
#undef MADDNESS_SCAN_OUTS
}

// alpha f + beta and the stores of one row's four columns per lane.  avg_C = 0:
// the fields of acc_e / acc_o are the exact sums.  avg_C = C > 0 (aggregation by
// averages, blocks of U = 16): the fields are sums of block averages; the estimate
// of the sum is 16 times that minus the expected excess C log2(16) / 4 = C
// (Theorem D.1), and the optional uint16 output receives 16 times the field.
// out_only: the caller knows that only the fp32 output is wanted (no branches).
__device__ __forceinline__ void store_row(const RowsArgs &a, int64_t row, int lane, uint32_t acc_e,
                                          uint32_t acc_o, const f4 &sc, const f4 &of, int col0 = 0,
                                          int avg_C = 0, bool out_only = false)
{
    uint32_t s0 = acc_e & 0xFFFFu, s1 = acc_o & 0xFFFFu, s2 = acc_e >> 16, s3 = acc_o >> 16;
    if (avg_C) { s0 *= 16u; s1 *= 16u; s2 *= 16u; s3 *= 16u; }
    if (out_only || a.out) {
        f4 v;
        v.x = fmaf((float)((int)s0 - avg_C), sc.x, of.x);
        v.y = fmaf((float)((int)s1 - avg_C), sc.y, of.y);
        v.z = fmaf((float)((int)s2 - avg_C), sc.z, of.z);
        v.w = fmaf((float)((int)s3 - avg_C), sc.w, of.w);
        __builtin_nontemporal_store(v, reinterpret_cast<f4 *>(a.out + row * a.ldo + col0) + lane);
    }
    if (!out_only && a.acc) {
        u2 w = {s0 | (s1 << 16), s2 | (s3 << 16)};
        *reinterpret_cast<u2 *>(a.acc + row * a.M + col0 + 4 * lane) = w;
    }
}

// Encode phase of the kernels that keep the codes of a block of rows in LDS: the
// wavefront streams n_rows rows of A starting at row0 (row-major, elements of type DT
// widened when they are compared; 16-byte non-temporal loads, DV per lane and row, PF
// groups of RPI = 64 / C rows in flight in registers), stages
// each group in its private LDS area `stage` (RPI * DV KiB), walks the trees (lane =
// (row of the group, codebook), tree `tr` of that codebook in registers) and leaves the
// packed codes in `my_codes` (C / 2 bytes per row), and in a.codes_out when that is set.
// The wavefront's k-th row is row0 + k * row_stride of the matrix and its codes go to
// slot k * code_stride of my_codes.  n_rows is a multiple of RPI; rows past the end of
// the matrix read as zeros.
// STORE: also to a.codes_out when that is set (else the caller copies them from LDS).
// PAD: codebooks a.codebooks .. C - 1 do not exist; their codes are 0 (the caller gives their lanes any tree).
// UNALIGNED (fp32): rows start on any 4-byte boundary and end anywhere; the aligned pieces that cover
// a row are read (DV KiB of staging must hold the row plus 12 bytes).
template <int C, int DV, int DT = kF32, bool STORE = true, bool PAD = false, bool UNALIGNED = false, int PF = 1>
__device__ __forceinline__ void encode_rows_to_lds(const RowsArgs &a, const Tree &tr, unsigned char *stage,
                                                   unsigned char *my_codes, int64_t row0, int n_rows, int lane,
                                                   int64_t row_stride = 1, int code_stride = 1)
{
    constexpr int RPI = 64 / C;
    constexpr int ROWB = DV * 1024;
    constexpr int CB = C / 2;
    constexpr int ES = elem_size(DT);
    const int c = lane & (C - 1);
    const int rsub = lane / C;
    const unsigned char *st = stage + rsub * ROWB;
    const unsigned char *A_bytes = static_cast<const unsigned char *>(a.A);
    const int row_bytes = a.D * ES;
    // UNALIGNED: row n begins (a0 + n s4) mod 16 bytes after a 16-byte boundary; s4 is a multiple of 4,
    // so that only n mod 4 matters
    const unsigned a0 = (unsigned)reinterpret_cast<uintptr_t>(A_bytes) & 15u, s4 = (unsigned)(a.lda * ES) & 15u;
    f4 pre[PF][RPI][DV];
    auto issue_loads = [&](int gi, int slot) INLINE_LAMBDA {
#pragma unroll
        for (int r = 0; r < RPI; ++r) {
            const int64_t row = row0 + (gi * RPI + r) * row_stride;
#pragma unroll
            for (int i = 0; i < DV; ++i) {
                const int col4 = lane + 64 * i;
                f4 v = {0.f, 0.f, 0.f, 0.f};
                if constexpr (!UNALIGNED) {
                    if (row < a.N && 16 * col4 < row_bytes)
                        v = __builtin_nontemporal_load(reinterpret_cast<const f4 *>(A_bytes + row * a.lda * ES) + col4);
                } else {
                    // the aligned 16-byte pieces that cover the row: the first may begin up to 12 bytes before
                    // it and the last end up to 12 bytes after it, inside the 16 bytes that hold the row's
                    // first / last element (such a piece never leaves the page its valid bytes are on)
                    const int shift = (int)((a0 + ((unsigned)row & 3u) * s4) & 15u);
                    if (row < a.N && 16 * col4 < shift + row_bytes)
                        v = __builtin_nontemporal_load(reinterpret_cast<const f4 *>(A_bytes + row * a.lda * ES - shift) + col4);
                }
                pre[slot][r][i] = v;
            }
        }
    };
    const int n_groups = n_rows / RPI;
#pragma unroll
    for (int s = 0; s < PF; ++s)
        if (s < n_groups) issue_loads(s, s);
#pragma unroll 1
    for (int g0 = 0; g0 < n_groups; g0 += PF) {
#pragma unroll
        for (int s = 0; s < PF; ++s) {
            const int gi = g0 + s;
            if (PF > 1 && gi >= n_groups) break;
#pragma unroll
            for (int r = 0; r < RPI; ++r)
#pragma unroll
                for (int i = 0; i < DV; ++i)
                    *reinterpret_cast<f4 *>(stage + r * ROWB + 16 * (lane + 64 * i)) = pre[s][r][i];
            if (gi + PF < n_groups) issue_loads(gi + PF, s);
            wave_lds_fence();
            const unsigned char *rowp = st;
            if constexpr (UNALIGNED) {
                // the row begins `shift` bytes into its first piece
                const int64_t row = row0 + (gi * RPI + rsub) * row_stride;
                rowp = st + ((a0 + ((unsigned)row & 3u) * s4) & 15u);
            }
            const float x0 = widen_at<DT>(rowp, tr.j0), x1 = widen_at<DT>(rowp, tr.j1), x2 = widen_at<DT>(rowp, tr.j2),
                        x3 = widen_at<DT>(rowp, tr.j3);
            unsigned code = hash_regs(tr, x0, x1, x2, x3);
            if constexpr (PAD) code = c < a.codebooks ? code : 0u;
            wave_lds_fence();
            unsigned q = code | (from_lane_above<1>(code) << 4);
            q |= from_lane_above<2>(q) << 8;
            q |= from_lane_above<4>(q) << 16;
            if ((lane & 7) == 0) {
                const int rl = gi * RPI + rsub;
                *reinterpret_cast<uint32_t *>(my_codes + rl * code_stride * CB + (c >> 3) * 4) = q;
                const int64_t row = row0 + rl * row_stride;
                if (STORE && a.codes_out && row < a.N)
                    *reinterpret_cast<uint32_t *>(a.codes_out + row * CB + (c >> 3) * 4) = q;
            }
        }
    }
}

// Host-side shape checks shared by the launchers.
inline bool aligned_to(const void *p, size_t n) { return reinterpret_cast<uintptr_t>(p) % n == 0; }

inline bool tables_ok(int C, int M, const uint8_t *luts, const float *scale, const float *offset,
               const float *out, int64_t ldo, const uint16_t *acc)
{
    if (C != 16 && C != 32) return false;
    if (M % 4 != 0 || M > 256 || M <= 64) return false;  // narrower outputs leave most lanes idle
    if (out && (ldo % 4 != 0 || !aligned_to(out, 16))) return false;
    if (acc && !aligned_to(acc, 8)) return false;
    return aligned_to(scale, 16) && aligned_to(offset, 16) && aligned_to(luts, 4);
}

}  // namespace rows
}  // namespace maddness
