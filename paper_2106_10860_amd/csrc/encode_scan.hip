// Encode (Algorithm 1, Section 4.1), scan (Section 4.4, exact integer sum, then
// alpha f + beta of Section 1.1) and the fused encode+scan kernel for gfx950.
//
// Mapping of the scan: a wavefront owns a few rows; its 64 lanes are split into
// groups of LPR lanes per row and every lane owns 4 adjacent output columns.
// The uint8 tables of one tile of output columns sit in LDS as [c][k][Mt] bytes,
// so the four entries a lane needs for (codebook c, code k) are one aligned
// 32-bit LDS word and the lanes of a row read consecutive words (no bank
// conflict).  The four bytes are added into two registers that each hold two
// 16-bit sums (even and odd columns): 255 C <= 65535 keeps the fields apart.
#include "common.h"
#include "device_common.h"

// LDS bytes of a column tile when the tables do not fit in LDS at once.
#ifndef MADDNESS_TILE_BYTES
#define MADDNESS_TILE_BYTES (64 * 1024)
#endif

namespace maddness {
namespace {

constexpr int kWave = 64;

struct ScanArgs {
    // inputs of the encode phase (fused kernel only): element (n, d) of A is element
    // n * rs + d * cs of the array, of type dtype
    const void *A;
    int64_t rs, cs;
    int dtype;
    int D;
    const int32_t *split_dims;
    const float *thresholds;
    // codes
    const uint8_t *codes_in;  // scan-only kernel
    uint8_t *codes_out;       // optional output of the fused kernel
    // tables and dequantisation
    const uint8_t *luts;
    const float *scale;
    const float *offset;
    // outputs
    float *out;
    int64_t ldo;
    uint16_t *acc;
    // sizes
    int64_t N;
    int C, Cb, Cp, M;      // Cp: table offsets kept per row in LDS (C rounded up to 4)
    // tiling of the output columns
    int Mt, MtW, T;      // tile width in columns (multiple of 4), in 32-bit words, number of tiles
    int lpr_shift, LPR;  // lanes per row (power of two)
    int col_passes;      // passes of LPR column groups that cover one tile
    int RPP;             // rows a wavefront handles per pass = 64 / LPR
    int RW;              // rows a wavefront handles per iteration (multiple of RPP)
    int n_waves;
    int iters;           // iterations of the persistent loop, the same for every block
    float inv_Cb, inv_MtW;
    int vec_out, vec_acc, vec_lut;
    int averaged;        // aggregation by pairwise averages in blocks of 16 codebooks (Appendix D)
    int seg_shift;       // log2 of 16-byte pieces per table row of a tile, -1: tile not loadable that way
    unsigned lds_codes_off, lds_params_off;
};

// Algorithm 1 on the implicit heap: the threshold v^t_i sits at slot
// s = 2^(t-1) - 1 + (i - 1), whose children are slots 2s+1 and 2s+2, so the walk
// is s <- 2s + 1 + (x >= thr[s]) from s = 0 and the leaf (0-based) is s - 15.
__device__ __forceinline__ unsigned walk_lds(float x0, float x1, float x2, float x3, const float *th)
{
    unsigned s = (x0 >= th[0]) ? 2u : 1u;
    s = 2u * s + 1u + ((x1 >= th[s]) ? 1u : 0u);
    s = 2u * s + 1u + ((x2 >= th[s]) ? 1u : 0u);
    s = 2u * s + 1u + ((x3 >= th[s]) ? 1u : 0u);
    return s - 15u;
}

// GENERIC_A = false: A is fp32 and stored by rows; true: any type and strides.
template <bool GENERIC_A>
__device__ __forceinline__ unsigned hash_lds(const ScanArgs &a, int64_t n, const int *sd, const float *th)
{
    float x0, x1, x2, x3;
    if constexpr (!GENERIC_A) {
        const float *row = static_cast<const float *>(a.A) + n * a.rs;
        x0 = row[sd[0]]; x1 = row[sd[1]]; x2 = row[sd[2]]; x3 = row[sd[3]];
    } else {
        const int64_t base = n * a.rs;
        x0 = widen_at(a.A, a.dtype, base + sd[0] * a.cs);
        x1 = widen_at(a.A, a.dtype, base + sd[1] * a.cs);
        x2 = widen_at(a.A, a.dtype, base + sd[2] * a.cs);
        x3 = widen_at(a.A, a.dtype, base + sd[3] * a.cs);
    }
    return walk_lds(x0, x1, x2, x3, th);
}

template <bool ENCODE, bool GENERIC_A = false>
__global__ __launch_bounds__(1024) void scan_kernel(const ScanArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    uint32_t *lut = reinterpret_cast<uint32_t *>(smem);
    uint32_t *offs_l = reinterpret_cast<uint32_t *>(smem + a.lds_codes_off);
    float *th_l = reinterpret_cast<float *>(smem + a.lds_params_off);
    int *sd_l = reinterpret_cast<int *>(th_l + a.C * 16);

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid >> 6;
    const int MtW = a.MtW;

    auto load_tile = [&](int tile) INLINE_LAMBDA {
        const int m0 = tile * a.Mt;
        if (a.seg_shift >= 0 && m0 + a.Mt <= a.M) {
            // 16-byte pieces, four independent loads per thread in flight
            const int total = (a.C * 16) << a.seg_shift;
            const int nthreads = blockDim.x;
            for (int base = 0; base < total; base += 4 * nthreads) {
                uint4 v[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int idx = base + u * nthreads + tid;
                    if (idx < total) {
                        const int row = idx >> a.seg_shift;
                        const int sg = idx - (row << a.seg_shift);
                        v[u] = *reinterpret_cast<const uint4 *>(a.luts + (size_t)row * a.M + m0 + 16 * sg);
                    }
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int idx = base + u * nthreads + tid;
                    if (idx < total) {
                        const int row = idx >> a.seg_shift;
                        const int sg = idx - (row << a.seg_shift);
                        *reinterpret_cast<uint4 *>(reinterpret_cast<unsigned char *>(lut) + row * a.Mt + 16 * sg) = v[u];
                    }
                }
            }
            return;
        }
        // any width and alignment: one 32-bit LDS word (4 columns) per thread and
        // step, four steps' loads in flight
        const int total = a.C * 16 * MtW;
        const int nthreads = blockDim.x;
        for (int base = 0; base < total; base += 4 * nthreads) {
            uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int idx = base + u * nthreads + tid;
                if (idx < total) {
                    const int row = (int)(((float)idx + 0.5f) * a.inv_MtW);
                    const int gg = idx - row * MtW;
                    const int m = m0 + 4 * gg;
                    const uint8_t *src = a.luts + (size_t)row * a.M + m;
                    if (a.vec_lut && m + 3 < a.M) {
                        w[u] = *reinterpret_cast<const uint32_t *>(src);
                    } else {
#pragma unroll
                        for (int q = 0; q < 4; ++q)
                            if (m + q < a.M) w[u] |= (uint32_t)src[q] << (8 * q);
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int idx = base + u * nthreads + tid;
                if (idx < total) lut[idx] = w[u];
            }
        }
    };

    if (ENCODE) {
        for (int i = tid; i < a.C * 16; i += blockDim.x) th_l[i] = a.thresholds[i];
        for (int i = tid; i < a.C * 4; i += blockDim.x)
            sd_l[i] = min(max(a.split_dims[i], 0), a.D - 1);
    }
    if (a.T == 1) load_tile(0);
    __syncthreads();

    uint32_t *my_offs = offs_l + wave * a.RW * a.Cp;   // [RW][Cp] byte offsets of table rows
    const unsigned row_bytes = 4u * (unsigned)MtW;       // bytes of one table row (c, k) in LDS
    const int rows_per_block = a.n_waves * a.RW;

    for (int it = 0; it < a.iters; ++it) {
        const int64_t row0 =
            ((int64_t)it * gridDim.x + blockIdx.x) * rows_per_block + (int64_t)wave * a.RW;

        // ---- codes of this wavefront's rows -> its private LDS area ----
        for (int p = lane; p < a.RW * a.Cb; p += kWave) {
            const int r = (int)(((float)p + 0.5f) * a.inv_Cb);
            const int b = p - r * a.Cb;
            const int64_t n = row0 + r;
            unsigned byte = 0;
            if (n < a.N) {
                if (ENCODE) {
                    const int c = 2 * b;
                    byte = hash_lds<GENERIC_A>(a, n, sd_l + 4 * c, th_l + 16 * c);
                    if (c + 1 < a.C)
                        byte |= hash_lds<GENERIC_A>(a, n, sd_l + 4 * (c + 1), th_l + 16 * (c + 1)) << 4;
                    if (a.codes_out) a.codes_out[n * a.Cb + b] = (uint8_t)byte;
                } else {
                    byte = a.codes_in[n * a.Cb + b];
                }
            }
            // byte offset in LDS of the table row each code selects
            my_offs[r * a.Cp + 2 * b] = (32u * b + (byte & 15u)) * row_bytes;
            if (2 * b + 1 < a.C) my_offs[r * a.Cp + 2 * b + 1] = (32u * b + 16u + (byte >> 4)) * row_bytes;
        }
        wave_lds_fence();

        for (int tile = 0; tile < a.T; ++tile) {
            if (a.T > 1) {
                __syncthreads();
                load_tile(tile);
                __syncthreads();
            }
            for (int cp = 0; cp < a.col_passes; ++cp) {
                const int g = (lane & (a.LPR - 1)) + cp * a.LPR;
                const bool lane_on = g < MtW;
                const int m = tile * a.Mt + 4 * g;
                float sc[4], of[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const bool ok = lane_on && (m + q < a.M);
                    sc[q] = ok ? a.scale[m + q] : 0.0f;
                    of[q] = ok ? a.offset[m + q] : 0.0f;
                }
                for (int pass = 0; pass < a.RW / a.RPP; ++pass) {
                    const int r = pass * a.RPP + (lane >> a.lpr_shift);
                    const int64_t n = row0 + r;
                    if (!lane_on || n >= a.N) continue;
                    const uint32_t *orow = my_offs + r * a.Cp;
                    const unsigned char *lane_lut = reinterpret_cast<const unsigned char *>(lut) + 4 * g;
                    auto word = [&](uint32_t off) INLINE_LAMBDA { return *reinterpret_cast<const uint32_t *>(lane_lut + off); };
                    uint32_t acc_e = 0, acc_o = 0;
                    auto add4 = [&](const uint4 &o) INLINE_LAMBDA {
                        const uint32_t y0 = word(o.x), y1 = word(o.y), y2 = word(o.z), y3 = word(o.w);
                        acc_e += (y0 & 0x00FF00FFu) + (y1 & 0x00FF00FFu);
                        acc_o += __builtin_amdgcn_perm(y0, y0, 0x0c030c01u) + __builtin_amdgcn_perm(y1, y1, 0x0c030c01u);
                        acc_e += (y2 & 0x00FF00FFu) + (y3 & 0x00FF00FFu);
                        acc_o += __builtin_amdgcn_perm(y2, y2, 0x0c030c01u) + __builtin_amdgcn_perm(y3, y3, 0x0c030c01u);
                    };
                    int c0 = 0;
                    if (a.averaged) {
                        // C is a multiple of 16 here.  floor((a + b + 1) / 2) on four
                        // bytes at once, as a balanced tree over each block of 16
                        for (; c0 < a.C; c0 += 16) {
                            uint32_t y[16];
#pragma unroll
                            for (int q = 0; q < 4; ++q) {
                                const uint4 o = *reinterpret_cast<const uint4 *>(orow + c0 + 4 * q);
                                y[4 * q] = word(o.x); y[4 * q + 1] = word(o.y);
                                y[4 * q + 2] = word(o.z); y[4 * q + 3] = word(o.w);
                            }
#pragma unroll
                            for (int span = 1; span < 16; span *= 2)
#pragma unroll
                                for (int u = 0; u < 16; u += 2 * span)
                                    y[u] = __builtin_amdgcn_lerp(y[u], y[u + span], 0x01010101u);
                            acc_e += y[0] & 0x00FF00FFu;
                            acc_o += __builtin_amdgcn_perm(y[0], y[0], 0x0c030c01u);
                        }
                    } else if (a.C >= 8) {
                        // eight codebooks per step; the offsets of the next step are
                        // fetched before the table words of this one are consumed
                        uint4 oa = *reinterpret_cast<const uint4 *>(orow);
                        uint4 ob = *reinterpret_cast<const uint4 *>(orow + 4);
                        for (; c0 + 16 <= a.C; c0 += 8) {
                            const uint4 na = *reinterpret_cast<const uint4 *>(orow + c0 + 8);
                            const uint4 nb = *reinterpret_cast<const uint4 *>(orow + c0 + 12);
                            add4(oa);
                            add4(ob);
                            oa = na;
                            ob = nb;
                        }
                        add4(oa);
                        add4(ob);
                        c0 += 8;
                    }
                    for (; c0 + 4 <= a.C; c0 += 4) add4(*reinterpret_cast<const uint4 *>(orow + c0));
                    for (; c0 < a.C; ++c0) {
                        const uint32_t y = word(orow[c0]);
                        acc_e += y & 0x00FF00FFu;
                        acc_o += __builtin_amdgcn_perm(y, y, 0x0c030c01u);
                    }
                    uint32_t s[4] = {acc_e & 0xFFFFu, acc_o & 0xFFFFu, acc_e >> 16, acc_o >> 16};
                    // averaged: 16 x (sum of block averages) estimates the sum with an
                    // expected excess of C log2(16) / 4 = C (Theorem D.1)
                    const int excess = a.averaged ? a.C : 0;
                    if (a.averaged) {
#pragma unroll
                        for (int q = 0; q < 4; ++q) s[q] *= 16u;
                    }
                    if (a.out) {
                        float v[4];
#pragma unroll
                        for (int q = 0; q < 4; ++q) v[q] = fmaf((float)((int)s[q] - excess), sc[q], of[q]);
                        float *dst = a.out + n * a.ldo + m;
                        if (a.vec_out && m + 3 < a.M) {
                            *reinterpret_cast<float4 *>(dst) = make_float4(v[0], v[1], v[2], v[3]);
                        } else {
#pragma unroll
                            for (int q = 0; q < 4; ++q)
                                if (m + q < a.M) dst[q] = v[q];
                        }
                    }
                    if (a.acc) {
                        uint16_t *dst = a.acc + n * a.M + m;
                        if (a.vec_acc && m + 3 < a.M) {
                            *reinterpret_cast<uint2 *>(dst) =
                                make_uint2(s[0] | (s[1] << 16), s[2] | (s[3] << 16));
                        } else {
#pragma unroll
                            for (int q = 0; q < 4; ++q)
                                if (m + q < a.M) dst[q] = (uint16_t)s[q];
                        }
                    }
                }
            }
        }
        wave_lds_fence();
    }
}

// ---------------------------------------------------------------------------
// encode only
// ---------------------------------------------------------------------------

struct EncArgs {
    const void *A;       // element (n, d) is element n * rs + d * cs, of type dtype
    int64_t rs, cs;
    int dtype;
    int64_t N;
    int D, C, Cb;
    const int32_t *split_dims;
    const float *thresholds;
    uint8_t *codes;
    int bx_shift;  // log2 of the number of threads that share a row
    int iters;
};

template <bool GENERIC_A>
__global__ __launch_bounds__(256) void encode_kernel(const EncArgs a)
{
    const int tid = threadIdx.x;
    const int b = tid & ((1 << a.bx_shift) - 1);
    const int ty = tid >> a.bx_shift;
    const int rows_per_block = 256 >> a.bx_shift;
    if (b >= a.Cb) return;
    const int c0 = 2 * b;
    const bool two = c0 + 1 < a.C;
    Tree lo, hi;
    load_tree(lo, a.split_dims + 4 * c0, a.thresholds + 16 * c0, a.D);
    load_tree(hi, a.split_dims + 4 * (two ? c0 + 1 : c0), a.thresholds + 16 * (two ? c0 + 1 : c0), a.D);
    for (int it = 0; it < a.iters; ++it) {
        const int64_t n = ((int64_t)it * gridDim.x + blockIdx.x) * rows_per_block + ty;
        if (n >= a.N) break;
        float x0, x1, x2, x3, y0, y1, y2, y3;
        if constexpr (!GENERIC_A) {
            const float *row = static_cast<const float *>(a.A) + n * a.rs;
            x0 = row[lo.j0]; x1 = row[lo.j1]; x2 = row[lo.j2]; x3 = row[lo.j3];
            y0 = row[hi.j0]; y1 = row[hi.j1]; y2 = row[hi.j2]; y3 = row[hi.j3];
        } else {
            const int64_t base = n * a.rs;
            x0 = widen_at(a.A, a.dtype, base + lo.j0 * a.cs); x1 = widen_at(a.A, a.dtype, base + lo.j1 * a.cs);
            x2 = widen_at(a.A, a.dtype, base + lo.j2 * a.cs); x3 = widen_at(a.A, a.dtype, base + lo.j3 * a.cs);
            y0 = widen_at(a.A, a.dtype, base + hi.j0 * a.cs); y1 = widen_at(a.A, a.dtype, base + hi.j1 * a.cs);
            y2 = widen_at(a.A, a.dtype, base + hi.j2 * a.cs); y3 = widen_at(a.A, a.dtype, base + hi.j3 * a.cs);
        }
        unsigned byte = hash_regs(lo, x0, x1, x2, x3);
        if (two) byte |= hash_regs(hi, y0, y1, y2, y3) << 4;
        a.codes[n * a.Cb + b] = (uint8_t)byte;
    }
}

int pow2_ceil_shift(int v)
{
    int s = 0;
    while ((1 << s) < v) ++s;
    return s;
}

}  // namespace

int launch_encode(const maddness_params &p, const MatrixA &A, int64_t N, uint8_t *codes,
                  hipStream_t stream)
{
    EncArgs a{};
    a.A = A.data; a.rs = A.row_stride(); a.cs = A.col_stride(); a.dtype = A.dtype; a.N = N; a.D = p.D; a.C = p.C; a.Cb = (p.C + 1) / 2;
    a.split_dims = p.split_dims; a.thresholds = p.thresholds; a.codes = codes;
    a.bx_shift = pow2_ceil_shift(a.Cb);           // Cb <= 128 < 256
    const int rows_per_block = 256 >> a.bx_shift;
    const int64_t blocks_needed = (N + rows_per_block - 1) / rows_per_block;
    const int64_t max_grid = (int64_t)device_info().cus * 8;
    const int grid = (int)(blocks_needed < max_grid ? blocks_needed : max_grid);
    a.iters = (int)((blocks_needed + grid - 1) / grid);
    note_kernel(A.plain() ? "encode_kernel<false>" : "encode_kernel<true>", nullptr);
    if (A.plain())
        hipLaunchKernelGGL(encode_kernel<false>, dim3(grid), dim3(256), 0, stream, a);
    else
        hipLaunchKernelGGL(encode_kernel<true>, dim3(grid), dim3(256), 0, stream, a);
    return check_hip(hipGetLastError(), "launch encode_kernel");
}

int launch_scan(const maddness_params *p, const MatrixA *A, const uint8_t *codes_in,
                int32_t C, int32_t M, int64_t N, const uint8_t *luts, const float *scale,
                const float *offset, float *out, int64_t ldo, uint16_t *acc, uint8_t *codes_out,
                bool averaged, hipStream_t stream)
{
    const bool fused = A != nullptr;
    const DeviceInfo &dev = device_info();
    ScanArgs a{};
    if (fused) {
        a.A = A->data; a.rs = A->row_stride(); a.cs = A->col_stride(); a.dtype = A->dtype;
        a.D = p->D; a.split_dims = p->split_dims; a.thresholds = p->thresholds;
    }
    a.codes_in = codes_in; a.codes_out = codes_out; a.averaged = averaged ? 1 : 0;
    a.luts = luts; a.scale = scale; a.offset = offset;
    a.out = out; a.ldo = ldo; a.acc = acc;
    a.N = N; a.C = C; a.Cb = (C + 1) / 2; a.Cp = (C + 3) & ~3; a.M = M;
    a.inv_Cb = 1.0f / (float)a.Cb;

    // LDS plan: [table tile | per-row table offsets | tree parameters].  The tile
    // takes what it needs (all of M if that fits), the offsets get the rest.
    const int params_bytes = fused ? C * 80 : 0;
    const int offs_row_bytes = 4 * a.Cp;
    const int min_offs_bytes = 8 * 1024 > 4 * offs_row_bytes ? 8 * 1024 : 4 * offs_row_bytes;
    int lut_budget = dev.lds_per_block - params_bytes - min_offs_bytes - 64;
    // tables that do not fit are tiled over columns and the tile is re-loaded for
    // every block of rows: a smaller tile leaves room for the offsets of more rows
    if ((int64_t)16 * C * ((M + 3) & ~3) > lut_budget && lut_budget > MADDNESS_TILE_BYTES) lut_budget = MADDNESS_TILE_BYTES;
    const int Mpad = (M + 3) & ~3;
    if ((int64_t)16 * C * Mpad <= lut_budget) {
        a.Mt = Mpad;
    } else {
        const int limit = lut_budget / (16 * C);
        if (limit >= 256) {
            a.Mt = 256 * (limit / 256);
        } else {
            a.Mt = 4;
            while (a.Mt * 2 <= limit) a.Mt *= 2;
        }
    }
    a.T = (M + a.Mt - 1) / a.Mt;
    a.MtW = a.Mt / 4;
    a.inv_MtW = 1.0f / (float)a.MtW;
    a.lpr_shift = pow2_ceil_shift(a.MtW < kWave ? a.MtW : kWave);
    a.LPR = 1 << a.lpr_shift;
    a.col_passes = (a.MtW + a.LPR - 1) / a.LPR;
    a.RPP = kWave / a.LPR;
    const int lut_bytes = 16 * C * a.Mt;
    a.lds_codes_off = (unsigned)((lut_bytes + 15) & ~15);
    int offs_avail = dev.lds_per_block - params_bytes - (int)a.lds_codes_off - 64;
    if (a.T == 1 && offs_avail > 48 * 1024) offs_avail = 48 * 1024;
    // wavefronts per block: few when the tables are small (several blocks share a
    // CU), 16 when a tile is re-loaded per row block (more rows per re-load)
    int n_waves = lut_bytes <= 32 * 1024 ? 4 : (a.T > 1 ? 16 : 8);
    while (n_waves > 1 && n_waves * a.RPP * offs_row_bytes > offs_avail) n_waves /= 2;
    if (a.RPP * offs_row_bytes > offs_avail)
        return fail(MADDNESS_E_UNSUPPORTED, "scan: C = %d with M = %d does not fit the LDS plan", C, M);
    // rows per wavefront and iteration: a multiple of RPP; as many as fit when a
    // tile is re-loaded per row block, a few otherwise
    const int max_rw = offs_avail / (n_waves * offs_row_bytes) / a.RPP * a.RPP;
    a.RW = a.RPP > 4 ? a.RPP : 4;
    if (a.T > 1) a.RW = max_rw < 64 ? max_rw : 64 / a.RPP * a.RPP;
    if (a.RW > max_rw) a.RW = max_rw;
    a.n_waves = n_waves;
    const int codes_bytes = n_waves * a.RW * offs_row_bytes;
    a.lds_params_off = (unsigned)((a.lds_codes_off + codes_bytes + 15) & ~15);
    const size_t lds_bytes = a.lds_params_off + params_bytes;
    if ((int)lds_bytes > dev.lds_per_block)
        return fail(MADDNESS_E_UNSUPPORTED, "scan: %zu bytes of LDS needed, %d available", lds_bytes,
                    dev.lds_per_block);

    a.vec_out = out && (ldo % 4 == 0) && (reinterpret_cast<uintptr_t>(out) % 16 == 0);
    a.vec_acc = acc && (M % 4 == 0) && (reinterpret_cast<uintptr_t>(acc) % 8 == 0);
    a.vec_lut = (M % 4 == 0) && (reinterpret_cast<uintptr_t>(luts) % 4 == 0);
    a.seg_shift = -1;
    if (M % 16 == 0 && reinterpret_cast<uintptr_t>(luts) % 16 == 0 && a.Mt % 16 == 0) {
        const int segs = a.Mt / 16;
        if ((segs & (segs - 1)) == 0) a.seg_shift = pow2_ceil_shift(segs);
    }

    const int rows_per_block = n_waves * a.RW;
    const int64_t blocks_needed = (N + rows_per_block - 1) / rows_per_block;
    int per_cu = dev.lds_per_block / (int)lds_bytes;
    if (per_cu > 32 / n_waves) per_cu = 32 / n_waves;
    if (per_cu < 1) per_cu = 1;
    if (per_cu > 8) per_cu = 8;
    const int64_t max_grid = (int64_t)dev.cus * per_cu;
    const int grid = (int)(blocks_needed < max_grid ? blocks_needed : max_grid);
    a.iters = (int)((blocks_needed + grid - 1) / grid);

    int rc;
    note_kernel(fused ? (A->plain() ? "scan_kernel<true>" : "scan_kernel<true, true>") : "scan_kernel<false>", nullptr);
    if (fused && !A->plain()) {
        if ((rc = allow_full_lds<scan_kernel<true, true>>()) != MADDNESS_OK) return rc;
        hipLaunchKernelGGL((scan_kernel<true, true>), dim3(grid), dim3(n_waves * kWave), lds_bytes, stream, a);
    } else if (fused) {
        if ((rc = allow_full_lds<scan_kernel<true>>()) != MADDNESS_OK) return rc;
        hipLaunchKernelGGL(scan_kernel<true>, dim3(grid), dim3(n_waves * kWave), lds_bytes, stream, a);
    } else {
        if ((rc = allow_full_lds<scan_kernel<false>>()) != MADDNESS_OK) return rc;
        hipLaunchKernelGGL(scan_kernel<false>, dim3(grid), dim3(n_waves * kWave), lds_bytes, stream, a);
    }
    return check_hip(hipGetLastError(), fused ? "launch fused encode+scan kernel" : "launch scan kernel");
}

}  // namespace maddness
