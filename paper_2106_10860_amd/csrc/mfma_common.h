// Pieces of the table scan on the matrix cores shared by the scan-only kernel
// (mfma_scan.hip) and the fused kernel for tables larger than LDS (fused_mfma.hip).
//
// f sums, for a row and an output column, the table entries its C codes select
// (Section 4.4).  Written with the one-hot code matrix G of Section 4.3 that is
// the product G T of a (rows x 16 C) 0/1 matrix with the (16 C x M) table
// matrix: a dense contraction in which 15 of 16 products are by zero, and still
// the cheaper way here - on the vector ALUs the sum costs 3 instructions per
// four looked-up bytes (unpacking bytes into 16-bit fields), which bounds the
// scan well below the HBM rate, whereas v_mfma_i32_16x16x64_i8 contracts 64
// (codebook, code) pairs for 16 rows x 16 columns in 16 cycles.  The arithmetic
// is exact: the operands are the one-hot bytes 0 / 1 and the table bytes shifted
// into the signed range (t - 128, the same bits as t ^ 0x80), the accumulator is
// 32 bits wide and starts at 128 C, which puts the shift back.
//
// Operand layout of the instruction (checked on the hardware): lane i + 16 g
// supplies, in 4 registers, 16 bytes of row i of A for the 16 values of k in
// group g; lane j + 16 g the same for column j of B; lane l receives, in register
// r, element (4 (l / 16) + r, l % 16) of the result.  Here a group of k is one
// codebook and the byte index is the code: lane (i, g) holds the one-hot code of
// (row i, codebook 4 G + g) for G = 0 .. C / 4 - 1, lane (j, g) the 16 entries of
// that codebook for one output column.
//
// A wavefront keeps the table entries of NT * 16 output columns in registers
// (NT * C registers) and takes the rows 16 at a time; tile t of the wavefront
// holds the columns congruent to t modulo NT, so that a lane ends up with NT
// consecutive columns of a row and stores them with one instruction.
#pragma once

#include "rows_common.h"

namespace maddness {
namespace mfma {

using rows::aligned_to;
using rows::f4;
using rows::u2;

typedef int v4i __attribute__((ext_vector_type(4)));

// Transposes a 4 x 4 byte matrix held in four registers (w[b] = row b) in place:
// afterwards w[t] holds column t, byte b taken from the old w[b].
__device__ __forceinline__ void transpose4x4(uint32_t (&w)[4])
{
    // bytes of (lo, hi) pairs: first interleave rows 0/1 and 2/3, then combine halves
    const uint32_t a = __builtin_amdgcn_perm(w[1], w[0], 0x05010400u);   // w0.b0 w1.b0 w0.b1 w1.b1
    const uint32_t b = __builtin_amdgcn_perm(w[1], w[0], 0x07030602u);   // w0.b2 w1.b2 w0.b3 w1.b3
    const uint32_t c = __builtin_amdgcn_perm(w[3], w[2], 0x05010400u);
    const uint32_t d = __builtin_amdgcn_perm(w[3], w[2], 0x07030602u);
    w[0] = __builtin_amdgcn_perm(c, a, 0x05040100u);   // a.b0 a.b1 c.b0 c.b1
    w[1] = __builtin_amdgcn_perm(c, a, 0x07060302u);   // a.b2 a.b3 c.b2 c.b3
    w[2] = __builtin_amdgcn_perm(d, b, 0x05040100u);
    w[3] = __builtin_amdgcn_perm(d, b, 0x07060302u);
}

// The 16 bytes 0 / 1 with a one at position `code` (0 .. 15), as four registers: read
// from a 256-byte table in LDS (entry e = the one-hot vector of e).  Built with vector
// instructions the same operand costs 8 of them, which made the vector ALU, not the
// matrix cores, the limit of the scan; the LDS reads are conflict-free (entry e lies in
// banks 4 e .. 4 e + 3) and run beside the matrix instructions.
__device__ __forceinline__ void fill_one_hot_table(v4i *table, int tid)
{
    if (tid < 16) {
        const unsigned long long p = 1ull << ((tid & 7) * 8);
        const int lo = (int)(unsigned)p, hi = (int)(unsigned)(p >> 32);
        table[tid] = tid < 8 ? v4i{lo, hi, 0, 0} : v4i{0, 0, lo, hi};
    }
}

// Outputs of the scan (either may be null) and the dequantisation of one lane's columns.
struct ScanOut {
    float *out;
    int64_t ldo;
    uint16_t *acc;
    int M;
};

// The table entries of columns col .. col + NT - 1 (col = c0 + NT j) for all codebooks
// into B; lane (j, g) holds codebook 4 G + g of tile t in B[t][G].  Lanes with
// col_on == false get arbitrary finite contents (their results are never stored).
// PAD: only `codebooks` (< 4 KG) codebooks exist; the others get zero entries, which together
// with their code 0 add nothing to the sums.
// BYTES: M need not be a multiple of NT and the tables need no alignment: entries are read
// byte by byte, those of columns >= M as zero.
template <int KG, int NT, bool PAD = false, bool BYTES = false>
__device__ __forceinline__ void load_tables(v4i (&B)[NT][KG], const uint8_t *luts, int M, int col, bool col_on, int g,
                                            int codebooks = 0)
{
    // entry (codebook 4 G + g, code b) of column col sits at offset (64 G + 16 g + b) M + col.
    // The offset is carried along (and hidden from the optimiser once per group): computed
    // afresh for each of the 16 KG loads, the addresses get hoisted out of the caller's loops
    // and spill.
    size_t off = (size_t)(16 * g) * M + col;
#pragma unroll
    for (int G = 0; G < KG; ++G) {
        asm volatile("" : "+v"(off));
        uint32_t w[16];   // w[b]: entries of code b for the lane's NT columns
#pragma unroll
        for (int b = 0; b < 16; ++b) {
            const uint8_t *src = luts + off + (size_t)b * M;
            uint32_t v = 0;
            if (col_on && (!PAD || 4 * G + g < codebooks)) {
                if constexpr (BYTES) {
#pragma unroll
                    for (int t = 0; t < NT; ++t)
                        if (col + t < M) v |= (uint32_t)src[t] << (8 * t);
                } else if constexpr (NT == 4) {
                    v = *reinterpret_cast<const uint32_t *>(src);
                } else {
                    v = *reinterpret_cast<const uint16_t *>(src);
                }
            }
            w[b] = v ^ 0x80808080u;   // t - 128 as a signed byte
        }
        off += (size_t)64 * M;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            uint32_t m[4] = {w[4 * q], w[4 * q + 1], w[4 * q + 2], w[4 * q + 3]};
            transpose4x4(m);          // m[t]: bytes of column t for codes 4q .. 4q + 3
#pragma unroll
            for (int t = 0; t < NT; ++t) B[t][G][q] = (int)m[t];
        }
        // two codebook groups at a time (32 loads in flight): without this the compiler
        // issues the loads of all groups at once and runs out of registers
        if (G % 2 == 1) asm volatile("" ::: "memory");
    }
}

// Exact sums of 16 rows x (NT * 16) columns.  cw: the packed codes (C / 8 words) of
// the row this lane stands for (row i = lane % 16 of the group); g = lane / 16.
// one_hot: the table fill_one_hot_table wrote (LDS).
template <int KG, int NT, typename Codes>
__device__ __forceinline__ void scan16(const Codes &cw, const v4i (&B)[NT][KG], int g, const v4i *one_hot,
                                       v4i (&acc)[NT])
{
    constexpr int C = 4 * KG;
    const unsigned sh0 = 4u * g, sh1 = 16u + 4u * g;   // nibble of codebook 4 G + g within its word
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = v4i{128 * C, 128 * C, 128 * C, 128 * C};
#pragma unroll
    for (int G = 0; G < KG; ++G) {
        const unsigned word = cw[G >> 1];
        const unsigned code = (word >> ((G & 1) ? sh1 : sh0)) & 15u;
        const v4i oh = one_hot[code];
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(oh, B[t][G], acc[t], 0, 0, 0);
        // at most eight one-hot operands in flight: fetched all at once they take 4 KG registers
        if (G % 8 == 7) __builtin_amdgcn_sched_barrier(0);
    }
}

// Two groups of 16 rows at once: with NT = 2 a single group gives the matrix pipe only two
// independent accumulation chains, which leaves it idle between dependent instructions.
template <int KG, int NT, typename Codes>
__device__ __forceinline__ void scan16x2(const Codes &cw0, const Codes &cw1, const v4i (&B)[NT][KG], int g,
                                         const v4i *one_hot, v4i (&acc0)[NT], v4i (&acc1)[NT])
{
    constexpr int C = 4 * KG;
    const unsigned sh0 = 4u * g, sh1 = 16u + 4u * g;
#pragma unroll
    for (int t = 0; t < NT; ++t) acc0[t] = acc1[t] = v4i{128 * C, 128 * C, 128 * C, 128 * C};
#pragma unroll
    for (int G = 0; G < KG; ++G) {
        const unsigned sh = (G & 1) ? sh1 : sh0;
        const v4i oh0 = one_hot[(cw0[G >> 1] >> sh) & 15u];
        const v4i oh1 = one_hot[(cw1[G >> 1] >> sh) & 15u];
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            acc0[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(oh0, B[t][G], acc0[t], 0, 0, 0);
            acc1[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(oh1, B[t][G], acc1[t], 0, 0, 0);
        }
        if (G % 8 == 7) __builtin_amdgcn_sched_barrier(0);
    }
}

// alpha f + beta (Section 1.1) and the stores: lane (j, g) holds rows 4 g .. 4 g + 3 of
// the group, columns col .. col + NT - 1; row_of(k) is the matrix row of the group's
// k-th row.  A lane's four rows must be consecutive matrix rows (row_of(4 g + r) =
// row_of(4 g) + r): the address of the first is computed once - one 64-bit product per
// lane and group; computed per row, the products were half of the vector instructions of
// the scan phase and held it below the rate of its stores - and the others follow by
// adding the pitch.
template <int NT, typename RowOf>
__device__ __forceinline__ void store16(const ScanOut &o, const v4i (&acc)[NT], RowOf row_of, int64_t N, int g,
                                        int col, const float (&sc)[NT], const float (&of)[NT])
{
    const int64_t first = row_of(4 * g);
    const int rows = N - first >= 4 ? 4 : (int)(N - first);   // <= 0: none of the lane's rows exists
    if (o.out) {
        float *dst = o.out + first * o.ldo + col;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            if (r < rows) {
                if constexpr (NT == 4) {
                    f4 v;
                    v.x = fmaf((float)acc[0][r], sc[0], of[0]);
                    v.y = fmaf((float)acc[1][r], sc[1], of[1]);
                    v.z = fmaf((float)acc[2][r], sc[2], of[2]);
                    v.w = fmaf((float)acc[3][r], sc[3], of[3]);
                    __builtin_nontemporal_store(v, reinterpret_cast<f4 *>(dst));
                } else {
                    typedef float f2 __attribute__((ext_vector_type(2)));
                    f2 v;
                    v.x = fmaf((float)acc[0][r], sc[0], of[0]);
                    v.y = fmaf((float)acc[1][r], sc[1], of[1]);
                    __builtin_nontemporal_store(v, reinterpret_cast<f2 *>(dst));
                }
            }
            dst += o.ldo;
        }
    }
    if (o.acc) {
        uint16_t *dst = o.acc + first * o.M + col;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            if (r < rows) {
                if constexpr (NT == 4) {
                    u2 v = {(unsigned)acc[0][r] | ((unsigned)acc[1][r] << 16),
                            (unsigned)acc[2][r] | ((unsigned)acc[3][r] << 16)};
                    *reinterpret_cast<u2 *>(dst) = v;
                } else {
                    *reinterpret_cast<uint32_t *>(dst) = (unsigned)acc[0][r] | ((unsigned)acc[1][r] << 16);
                }
            }
            dst += o.M;
        }
    }
}

// The same for outputs of any pitch and alignment and for M that is not a multiple of NT: one
// 4-byte (2-byte) store per result, columns >= M left out.
template <int NT, typename RowOf>
__device__ __forceinline__ void store16_any(const ScanOut &o, const v4i (&acc)[NT], RowOf row_of, int64_t N, int g,
                                            int col, const float (&sc)[NT], const float (&of)[NT])
{
    const int64_t first = row_of(4 * g);
    const int rows = N - first >= 4 ? 4 : (int)(N - first);
    float *dst_out = o.out ? o.out + first * o.ldo + col : nullptr;
    uint16_t *dst_acc = o.acc ? o.acc + first * o.M + col : nullptr;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        if (r < rows) {
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                if (col + t >= o.M) continue;
                if (o.out) dst_out[t] = fmaf((float)acc[t][r], sc[t], of[t]);
                if (o.acc) dst_acc[t] = (uint16_t)acc[t][r];
            }
        }
        if (o.out) dst_out += o.ldo;
        if (o.acc) dst_acc += o.M;
    }
}

// Writes `n_rows` consecutive rows of a dense output (pitch = M: the rows form one range of
// n_rows * M floats that begins at `dst`, on any 4-byte boundary) from a tile in LDS (row r of
// the range is tile row `tile_row0 + r`, `tile_ld` floats apart): the aligned 16-byte pieces
// of the range with one store each, up to three floats before the first and after the last
// piece one by one.  Thread t of `nthreads` (at least 6) takes pieces t, t + nthreads, ...
// inv_M = 1 / M; M > 4 and n_rows * M < 2^16 (the row of an element comes from a float product).
// SINGLE (n_rows = 1, inv_M = 0): one row of any pitch as a range of its own; `tile` is 16-byte aligned.
// All stores are nontemporal: with ordinary stores for the lines that also receive single floats
// the whole kernel is slower (N = 2^20, M = 250: scan 0.46 against 0.35 ms).
template <bool SINGLE = false>
__device__ __forceinline__ void store_dense_rows(float *dst, int n_rows, int M, float inv_M, const float *tile,
                                                 int tile_ld, int tile_row0, int t, int nthreads)
{
    const int total = n_rows * M;
    int head = (int)((16u - ((unsigned)reinterpret_cast<uintptr_t>(dst) & 15u)) & 15u) >> 2;
    if (head > total) head = total;
    const int pieces = (total - head) >> 2;
    const int tail = total - head - 4 * pieces;
    if (SINGLE && head == 0 && (tile_ld & 3) == 0) {
        // one row that begins on a 16-byte boundary, as its tile row does: the pieces are read whole
        // (read float by float, the lanes of a wavefront meet in the same LDS banks four at a time: rows of
        // 250 floats with a pitch of 256 take 0.74 ms per 2^20 that way, 0.66 ms stored float by float)
        const f4 *src = reinterpret_cast<const f4 *>(tile + tile_row0 * tile_ld);
        for (int p = t; p < pieces; p += nthreads) __builtin_nontemporal_store(src[p], reinterpret_cast<f4 *>(dst) + p);
        if (t < tail) __builtin_nontemporal_store(tile[tile_row0 * tile_ld + 4 * pieces + t], dst + 4 * pieces + t);
        return;
    }
    for (int p = t; p < pieces; p += nthreads) {
        const int e = head + 4 * p;
        int r = (int)(((float)e + 0.5f) * inv_M);
        int c = e - r * M;
        f4 v;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            v[q] = tile[(tile_row0 + r) * tile_ld + c];
            if (++c == M) { c = 0; ++r; }
        }
        __builtin_nontemporal_store(v, reinterpret_cast<f4 *>(dst + e));
    }
    if (t < head + tail) {
        const int e = t < head ? t : 4 * pieces + t;   // (head + 4 pieces + (t - head))
        const int r = (int)(((float)e + 0.5f) * inv_M);
        __builtin_nontemporal_store(tile[(tile_row0 + r) * tile_ld + (e - r * M)], dst + e);
    }
}

}  // namespace mfma
}  // namespace maddness
