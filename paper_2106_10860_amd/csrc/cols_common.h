// The encoder for an input matrix stored by columns, shared by the column kernels
// (encode_cols.hip) and the fused matrix-core kernel (fused_mfma.hip).
//
// Algorithm 1 (Section 4.1) reads four elements of a row per codebook, so with A
// stored by columns only the 4 C split columns are touched: O(C) elements per
// row instead of O(D) (Section 5.2), each column read as one contiguous run.  A
// lane owns RPL consecutive rows and a wavefront 64 RPL ("a group"), so that
// every load instruction fetches 64 RPL consecutive elements of one column; the
// tree of a codebook is the same for all lanes and sits in scalar registers.  A
// lane packs the codes of each of its rows into C / 8 registers.
#pragma once

#include "rows_common.h"

namespace maddness {
namespace cols {

using rows::RowsArgs;
using rows::u2;

// The tree parameters are read-only for the whole kernel and the same for every
// lane: addressed through the constant address space they are fetched with scalar
// loads into scalar registers (a plain global pointer gives vector loads, because
// the compiler cannot rule out that the kernel's own stores change them).
template <typename T>
using constant_ptr = const T __attribute__((address_space(4))) *;

template <typename T>
__device__ __forceinline__ constant_ptr<T> as_constant(const T *p)
{
    return (constant_ptr<T>)(uintptr_t)p;
}

// RPL consecutive elements of a column, widened to fp32.  idx and the column
// stride are multiples of RPL, so the vector load is aligned.
template <int DT, int RPL>
__device__ __forceinline__ void load_run(const void *A, int64_t idx, float (&x)[RPL])
{
    static_assert(RPL == 1 || RPL == 2 || RPL == 4, "rows per lane");
    if constexpr (RPL == 1) {
        x[0] = widen_at<DT>(A, idx);
    } else if constexpr (DT == kF32) {
        typedef float fv __attribute__((ext_vector_type(RPL)));
        const fv v = *reinterpret_cast<const fv *>(static_cast<const float *>(A) + idx);
#pragma unroll
        for (int r = 0; r < RPL; ++r) x[r] = v[r];
    } else if constexpr (DT == kF16) {
        typedef _Float16 hv __attribute__((ext_vector_type(RPL)));
        const hv v = *reinterpret_cast<const hv *>(static_cast<const _Float16 *>(A) + idx);
#pragma unroll
        for (int r = 0; r < RPL; ++r) x[r] = (float)v[r];
    } else if constexpr (DT == kBF16) {
        const uint32_t *p = reinterpret_cast<const uint32_t *>(static_cast<const uint16_t *>(A) + idx);
        uint32_t w[RPL / 2];
        if constexpr (RPL == 2) {
            w[0] = p[0];
        } else {
            const u2 v = *reinterpret_cast<const u2 *>(p);
            w[0] = v.x; w[1] = v.y;
        }
#pragma unroll
        for (int r = 0; r < RPL; r += 2) {
            x[r] = __uint_as_float(w[r / 2] << 16);
            x[r + 1] = __uint_as_float(w[r / 2] & 0xFFFF0000u);
        }
    } else if constexpr (RPL == 2) {
        const unsigned v = *reinterpret_cast<const uint16_t *>(static_cast<const uint8_t *>(A) + idx);
        x[0] = (float)(v & 255u); x[1] = (float)(v >> 8);
    } else {
        const uint32_t v = *reinterpret_cast<const uint32_t *>(static_cast<const uint8_t *>(A) + idx);
        x[0] = (float)(v & 255u); x[1] = (float)((v >> 8) & 255u);
        x[2] = (float)((v >> 16) & 255u); x[3] = (float)(v >> 24);
    }
}

// The encoder of one group of 64 RPL rows.  CHUNK: codebooks whose loads are issued
// together (4 loads each).  State: where this lane's rows start, the split values and
// trees of the chunk of codebooks being walked (cur) and of the one in flight (nxt), the
// word of eight codes being filled and the words finished.  The number of rows N is a
// multiple of RPL (the launchers hand the last N % 4 rows to the general kernels); a
// lane past the end reads the last run of the matrix instead, and its codes are not used.
template <int C, int DT, int CHUNK, int RPL>
struct ColsEncoder {
    static_assert(C % 8 == 0 && 8 % CHUNK == 0, "a chunk of codebooks lies within one word of codes");
    static constexpr int CW = C / 8;
    static constexpr int NCHUNK = C / CHUNK;
    typedef unsigned cvec __attribute__((ext_vector_type(CW)));

    const RowsArgs &a;
    const constant_ptr<int32_t> split_dims;
    const constant_ptr<float> thresholds;
    float x_cur[CHUNK][4][RPL], x_nxt[CHUNK][4][RPL];
    Tree tr_cur[CHUNK], tr_nxt[CHUNK];   // thresholds only; the same for every lane: scalar registers
    unsigned word[RPL], cwn[RPL][CW];
    int64_t n0 = 0, nq = 0;

    __device__ __forceinline__ explicit ColsEncoder(const RowsArgs &args)
        : a(args), split_dims(as_constant(args.split_dims)), thresholds(as_constant(args.thresholds)) {}

    // loads of chunk k: split values (vector loads, RPL rows per lane) and thresholds
    __device__ __forceinline__ void issue(int k)
    {
#pragma unroll
        for (int u = 0; u < CHUNK; ++u) {
            const int c = k * CHUNK + u;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int j = min(max(split_dims[4 * c + t], 0), a.D - 1);
                load_run<DT, RPL>(a.A, (int64_t)j * a.lda + nq, x_nxt[u][t]);
            }
#pragma unroll
            for (int i = 0; i < 15; ++i) tr_nxt[u].t[i] = thresholds[16 * c + i];
        }
    }
    // first: first row of the group; this lane takes rows first + RPL lane .. + RPL - 1
    __device__ __forceinline__ void begin_group(int64_t first, int lane)
    {
        n0 = first + RPL * lane;
        nq = n0 < a.N ? n0 : a.N - RPL;
#pragma unroll
        for (int r = 0; r < RPL; ++r) word[r] = 0;
        issue(0);
    }
    // Algorithm 1 for the codebooks of chunk k on the values in x, into the code words
    __device__ __forceinline__ void walk(int k, const Tree (&tr)[CHUNK], const float (&x)[CHUNK][4][RPL])
    {
#pragma unroll
        for (int u = 0; u < CHUNK; ++u) {
            const int c = k * CHUNK + u;
#pragma unroll
            for (int r = 0; r < RPL; ++r) {
                const unsigned code = hash_regs(tr[u], x[u][0][r], x[u][1][r], x[u][2][r], x[u][3][r]);
                word[r] |= code << (4 * (c & 7));
            }
        }
        if (((k + 1) * CHUNK & 7) == 0) {
            // a word of eight codes is complete
            const int q_done = (k * CHUNK) >> 3;
#pragma unroll
            for (int r = 0; r < RPL; ++r) {
#pragma unroll
                for (int q = 0; q < CW; ++q) cwn[r][q] = (q == q_done) ? word[r] : cwn[r][q];
                word[r] = 0;
            }
        }
    }
    // One step (k is a run-time value; the loop over k is not unrolled, which also keeps
    // the compiler from moving the loads of later chunks to the front): take over the
    // chunk that was in flight, issue the next one, walk the trees of this one.
    __device__ __forceinline__ void step(int k)
    {
#pragma unroll
        for (int u = 0; u < CHUNK; ++u) {
            tr_cur[u] = tr_nxt[u];
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int r = 0; r < RPL; ++r) x_cur[u][t][r] = x_nxt[u][t][r];
        }
        if (k + 1 < NCHUNK) issue(k + 1);
        walk(k, tr_cur, x_cur);
    }
    // all codebooks of the group, one chunk after the other
    __device__ __forceinline__ void encode_group(int64_t first, int lane)
    {
        begin_group(first, lane);
#pragma unroll 1
        for (int k = 0; k < NCHUNK; ++k) step(k);
    }
    // this lane's finished codes to `codes` ([N][C / 2], the layout of maddness_encode)
    __device__ __forceinline__ void store_codes(uint8_t *codes) const
    {
        if (codes && n0 < a.N) {
#pragma unroll
            for (int r = 0; r < RPL; ++r) {
                cvec v;
#pragma unroll
                for (int q = 0; q < CW; ++q) v[q] = cwn[r][q];
                *reinterpret_cast<cvec *>(codes + (n0 + r) * (C / 2)) = v;
            }
        }
    }
};

}  // namespace cols
}  // namespace maddness
