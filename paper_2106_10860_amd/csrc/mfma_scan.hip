// The table scan on the matrix cores.
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
// A wavefront keeps the table entries of its NT * 16 output columns in registers
// for the whole kernel (NT * C registers) and streams over the rows, 16 at a
// time; tile t of the wavefront holds the columns congruent to t modulo NT, so
// that a lane ends up with NT consecutive columns of a row and stores them with
// one instruction.
#include "rows_common.h"

namespace maddness {
namespace {

using namespace rows;

typedef int v4i __attribute__((ext_vector_type(4)));

struct MfmaScanArgs {
    const uint8_t *codes;   // [N][C / 2]
    const uint8_t *luts;    // [C][16][M]
    const float *scale;
    const float *offset;
    float *out;
    int64_t ldo;
    uint16_t *acc;
    int64_t N;
    int C, M;
};

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

// The 16 bytes 0 / 1 with a one at position `code` (0 .. 15), as four registers.
__device__ __forceinline__ v4i one_hot16(unsigned code)
{
    const unsigned long long p = 1ull << ((code & 7u) * 8u);
    const unsigned lo = (unsigned)p, hi = (unsigned)(p >> 32);
    const bool first = code < 8u;
    v4i a;
    a.x = first ? lo : 0u;
    a.y = first ? hi : 0u;
    a.z = first ? 0u : lo;
    a.w = first ? 0u : hi;
    return a;
}

// KG: groups of four codebooks (C = 4 KG); NT: column tiles per wavefront (4 or 2).
template <int KG, int NT>
__global__ __launch_bounds__(256, 2) void mfma_scan_kernel(const MfmaScanArgs a)
{
    static_assert(NT == 4 || NT == 2, "tiles per wavefront");
    static_assert(KG % 2 == 0, "whole words of packed codes");
    constexpr int C = 4 * KG;
    constexpr int CW = C / 8;          // 32-bit words of packed codes per row
    constexpr int SPAN = 16 * NT;      // output columns per wavefront
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int j = lane & 15, g = lane >> 4;
    const int c0 = (blockIdx.y * 4 + wave) * SPAN;   // first column of this wavefront
    if (c0 >= a.M) return;                          // no barriers in this kernel
    const int col = c0 + NT * j;                    // first of this lane's NT columns
    const bool col_on = col < a.M;                  // M is a multiple of NT

    // ---- the tables of this wavefront's columns, once ----
    v4i B[NT][KG];
#pragma unroll
    for (int G = 0; G < KG; ++G) {
        const int cb = 4 * G + g;
        uint32_t w[16];   // w[b]: entries of code b for the lane's NT columns
#pragma unroll
        for (int b = 0; b < 16; ++b) {
            const uint8_t *src = a.luts + (size_t)(cb * 16 + b) * a.M + col;
            uint32_t v = 0;
            if (col_on) {
                if constexpr (NT == 4) v = *reinterpret_cast<const uint32_t *>(src);
                else v = *reinterpret_cast<const uint16_t *>(src);
            }
            w[b] = v ^ 0x80808080u;   // t - 128 as a signed byte
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            uint32_t m[4] = {w[4 * q], w[4 * q + 1], w[4 * q + 2], w[4 * q + 3]};
            transpose4x4(m);          // m[t]: bytes of column t for codes 4q .. 4q + 3
#pragma unroll
            for (int t = 0; t < NT; ++t) B[t][G][q] = (int)m[t];
        }
    }
    float sc[NT], of[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        sc[t] = col_on ? a.scale[col + t] : 0.f;
        of[t] = col_on ? a.offset[col + t] : 0.f;
    }

    // ---- rows, 16 at a time ----
    typedef unsigned cvec __attribute__((ext_vector_type(CW)));
    const int64_t n_groups = (a.N + 15) >> 4;
    const unsigned sh0 = 4u * g, sh1 = 16u + 4u * g;   // nibble of codebook 4 G + g within its word
    auto load_codes = [&](int64_t rg) {
        const int64_t row = rg * 16 + j;
        cvec v = {};
        if (row < a.N) v = *reinterpret_cast<const cvec *>(a.codes + row * (C / 2));
        return v;
    };
    int64_t rg = blockIdx.x;
    cvec next = {};
    if (rg < n_groups) next = load_codes(rg);
    for (; rg < n_groups; rg += gridDim.x) {
        const cvec cw = next;
        if (rg + gridDim.x < n_groups) next = load_codes(rg + gridDim.x);
        v4i acc[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[t] = v4i{128 * C, 128 * C, 128 * C, 128 * C};
#pragma unroll
        for (int G = 0; G < KG; ++G) {
            const unsigned word = cw[G >> 1];
            const unsigned code = (word >> ((G & 1) ? sh1 : sh0)) & 15u;
            const v4i oh = one_hot16(code);
#pragma unroll
            for (int t = 0; t < NT; ++t)
                acc[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(oh, B[t][G], acc[t], 0, 0, 0);
        }
        if (!col_on) continue;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int64_t row = rg * 16 + 4 * g + r;
            if (row >= a.N) break;
            if (a.out) {
                float *dst = a.out + row * a.ldo + col;
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
            if (a.acc) {
                uint16_t *dst = a.acc + row * a.M + col;
                if constexpr (NT == 4) {
                    u2 v = {(unsigned)acc[0][r] | ((unsigned)acc[1][r] << 16),
                            (unsigned)acc[2][r] | ((unsigned)acc[3][r] << 16)};
                    *reinterpret_cast<u2 *>(dst) = v;
                } else {
                    *reinterpret_cast<uint32_t *>(dst) = (unsigned)acc[0][r] | ((unsigned)acc[1][r] << 16);
                }
            }
        }
    }
}

template <int KG, int NT>
int launch_mfma(const MfmaScanArgs &a, hipStream_t stream)
{
    const DeviceInfo &dev = device_info();
    const int span = 16 * NT * 4;                       // columns per workgroup of 4 wavefronts
    const int gy = (a.M + span - 1) / span;
    const int64_t n_groups = (a.N + 15) / 16;
    int64_t gx = (int64_t)dev.cus * 2 / gy;             // two workgroups per CU in all
    if (gx < 1) gx = 1;
    if (gx > n_groups) gx = n_groups;
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
    if (C % 8 != 0 || C > 64 || N < 16384) return 1;
    if (!aligned_to(codes, 16)) return 1;
    const int NT = C <= 32 ? 4 : 2;
    if (M % NT != 0 || !aligned_to(luts, NT)) return 1;
    if (out && (ldo % NT != 0 || !aligned_to(out, 4 * NT))) return 1;
    if (acc && !aligned_to(acc, 2 * NT)) return 1;
    MfmaScanArgs a{codes, luts, scale, offset, out, ldo, acc, N, C, M};
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
