// Fused encode + exact scan with the scan on the matrix cores, in phases:
//
// A workgroup of 8 wavefronts (two per SIMD, 256 registers each; one workgroup
// per CU) takes a block of rows through
//   E   every wavefront encodes its share of the rows and leaves the packed codes
//       of the block in LDS (C / 2 bytes per row).  Row-major A (fp32 or a narrow
//       type): as the row kernels do - register prefetch, staging in
//       wavefront-private LDS, Algorithm 1 with the tree in registers.  A stored
//       by columns: as the column kernels do - a lane owns four consecutive rows,
//       only the 4 C split columns are read (cols_common.h);
//   S   wavefront w holds the tables of output columns [SPAN w, SPAN (w + 1)) in
//       registers and goes through all rows of the block, 16 at a time: codes from
//       LDS, one-hot operands, int8 MFMA, dequantise, store (mfma_common.h).  If M
//       exceeds 8 SPAN columns the phase is repeated with the next 8 SPAN columns;
//       if it has at most 4 SPAN, several wavefronts hold the same columns and
//       share out the rows.
//       The tables are re-read from L2 at the start of every S phase (a few hundred
//       bytes per row of the block), which leaves the registers to E meanwhile.
// E is bound by HBM reads, S by HBM writes; they do not overlap within a
// workgroup, and the larger a region, the longer the chip as a whole only reads or
// only writes, which HBM serves faster than a mixture (N = 2^20, D = 512, M = 256,
// C = 32: 0.51 ms with one region, 0.56 ms with four, 0.53 ms for the kernel in which
// every wavefront reads, gathers and writes).  Measured alternatives that overlapped
// the phases within a CU were slower on the stress workload (N = 2^22, D = 1024,
// M = 512, C = 64; this kernel: 4.8 ms): two workgroups of 4 wavefronts per CU
// (6.0 ms; 7.3 ms when started half a period apart), and 4 encoding + 4 scanning
// wavefronts with double-buffered codes (6.2 ms, whatever the encoders' prefetch
// depth; only the by-columns input gained, 0.295 against 0.324 ms at N = 2^20,
// M = 256).  Used for many rows with C = 16, 32 or 64: the metric's shape, tables larger
// than LDS, narrow element types, A stored by columns; and, as its E phase alone, to
// encode fp32 rows.
#include <algorithm>

#include "cols_common.h"
#include "mfma_common.h"

namespace maddness {
namespace {

using namespace rows;
using namespace mfma;

constexpr int kWaves = 8;

// one workgroup per compute unit, or fewer when MADDNESS_OPT_MAX_WORKGROUPS says so (testing aid)
int max_workgroups()
{
    const int cus = device_info().cus, cap = option(MADDNESS_OPT_MAX_WORKGROUPS);
    return cap >= 1 && cap < cus ? cap : cus;
}

// Most rows per wavefront and region.  As many as LDS holds codes for is best: with one
// region the whole chip first only reads, then only writes (N = 2^21, D = 512, M = 256,
// C = 32: 1.02 ms with regions of 2^21 rows, 1.10 ms with 2^20).
#ifndef MADDNESS_PHASED_MAX_ROWS
#define MADDNESS_PHASED_MAX_ROWS 1024
#endif

// the value of x, as far as the compiler knows a new one each time
__device__ __forceinline__ int opaque(int x)
{
    asm volatile("" : "+v"(x));
    return x;
}
enum EncodeMode { kRowMajor = 0, kByColumns = 1 };

// Bytes at the start of LDS that the phases use in turn: E stages RPI rows of DV KiB per wavefront there
// (row-major A); S keeps the one-hot table there (256 bytes) and, when it writes whole rows, two tiles
// of one step's results each (16 rows, or 32 with NT = 2, of 8 blocks of 16 NT columns + 4 floats of padding).
constexpr int tile_bytes(int NT) { return (NT == 2 ? 32 : 16) * (kWaves * 16 * NT + 4) * 4; }
constexpr int shared_bytes(int emode, int RPI, int DV, int NT, bool gather)
{
    const int stage = emode == kRowMajor ? kWaves * RPI * DV * 1024 : 256;
    const int tiles = gather ? 256 + 2 * tile_bytes(NT) : 256;
    return stage > tiles ? stage : tiles;
}

// DV: 16-byte pieces per lane and row (row-major); unused for columns.
// SCAN = false: the E phase only (the codes go to a.codes_out), a kernel of its own name.
// GATHER = true (row-major A, more than 4 blocks of columns): the S phase collects the
// fp32 results of a step in LDS and writes whole rows, for outputs whose rows do not start
// on 128-byte lines.
// PAD = true: a.codebooks < C codebooks exist (a multiple of 8); the kernel runs as for C with
// the others' codes and table entries zero, and writes rows of a.codebooks / 2 bytes to a.codes_out.
// ODD = true (fp32 row-major A, with GATHER and PAD): any shape the tile sizes cover - rows of A that
// start on any 4-byte boundary and end anywhere, any number of codebooks up to C, any M, any pitch
// and alignment of the outputs.  The E phase reads the aligned 16-byte pieces that cover a row,
// the tables are read byte by byte, and the S phase writes through LDS (GATHER) - rows without padding
// between them as ranges of floats in aligned 16-byte pieces, other rows each as a range of its own
// (store_dense_rows) - or, for one or two blocks of columns, with 4-byte stores straight from the registers,
// the wavefronts sharing out the rows (gathered, such narrow outputs would leave the matrix work to one or
// two of the eight wavefronts: N = 2^20, D = 512, M = 10, C = 16 takes 0.37 instead of 0.52 ms).
template <int C, int DV, int NT, int EMODE, int DT, bool SCAN = true, bool GATHER = false, bool PAD = false, bool ODD = false>
__global__ __launch_bounds__(kWaves * 64) void fused_mfma_kernel(const RowsArgs a, const int rw)
{
    static_assert(!ODD || (PAD && EMODE == kRowMajor && DT == kF32), "ODD: fp32 rows, padding codebooks");
    constexpr int KG = C / 4;
    constexpr int RPI = 64 / C;
    constexpr int CB = C / 2;
    constexpr int CW = C / 8;
    constexpr int SPAN = 16 * NT;
    // groups of rows a wavefront of the E phase keeps in flight: one for fp32 (more is slower there: 0.335
    // against 0.310 ms per 2^20 rows of 2 KiB), more for narrow types, whose rows are few bytes each
#ifndef MADDNESS_NARROW_PREFETCH
#define MADDNESS_NARROW_PREFETCH 2
#endif
    constexpr int E_PF = DT == kF32 ? 1 : (DT == kU8 ? 2 * MADDNESS_NARROW_PREFETCH : MADDNESS_NARROW_PREFETCH);
    // row-major: staging of RPI rows per wavefront; by columns: room for the one-hot table only
    constexpr int STAGE_BYTES = shared_bytes(EMODE, RPI, DV, NT, GATHER);
    typedef unsigned cvec __attribute__((ext_vector_type(CW)));

    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    v4i *one_hot = reinterpret_cast<v4i *>(smem);                   // 16 entries of 16 bytes, valid during S
    unsigned char *codes_l = smem + STAGE_BYTES;                   // [kWaves * rw][CB]

    // S: the wavefronts share out blocks of SPAN output columns; when M has at most 4
    // blocks, `share` wavefronts (a power of two) take the same block and every share-th
    // step of the rows each
    const int col_blocks = (a.M + SPAN - 1) / SPAN;
    int share = 1;
    // (with 3 or 4 blocks only beside rows of more than 2 KiB: N = 2^20, C = 32, M = 256 takes
    // 0.510 ms without and 0.516 ms with sharing at D = 512, 0.863 and 0.822 ms at D = 1024)
    // (col_blocks = 0: encode only, nothing to share)
    if (col_blocks > 0 && (col_blocks <= 2 || (col_blocks <= 4 && EMODE == kRowMajor && a.D * elem_size(DT) > 2048)))
        while (share < kWaves && 2 * share * col_blocks <= kWaves) share *= 2;
    const ScanOut o{a.out, a.ldo, a.acc, a.M};

    v4i B[NT][KG];
    float sc[NT], of[NT];
    int col = 0, j = 0, g = 0, lane_in_s = 0;
    bool col_on = false;
    auto take_columns = [&](int block) INLINE_LAMBDA {
        col = block * SPAN + NT * j;
        col_on = col < a.M;
        load_tables<KG, NT, PAD, ODD>(B, a.luts, a.M, col, col_on, g, a.codebooks);
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const bool on = ODD ? col + t < a.M : col_on;    // (else M is a multiple of NT)
            sc[t] = on ? a.scale[col + t] : 0.f;
            of[t] = on ? a.offset[col + t] : 0.f;
        }
    };
    // S for `groups` groups of 16 local rows; row_of(l): matrix row of local row l.
    // `turns` wavefronts hold the same columns, this one takes steps turn, turn + turns, ...
    // (a step: one group, or two for C = 64); the caller passes constants where it can.
    auto scan_rows = [&](int groups, auto row_of, int blocks_per_pass, int my_block, int turns, int turn) INLINE_LAMBDA {
        auto one_group = [&](int rg) INLINE_LAMBDA {
            const cvec cw = *reinterpret_cast<const cvec *>(codes_l + (size_t)(rg * 16 + j) * CB);
            v4i acc[NT];
            scan16<KG, NT>(cw, B, g, one_hot, acc);
            if (col_on) {
                if constexpr (ODD) store16_any<NT>(o, acc, [&](int k) INLINE_LAMBDA { return row_of(16 * rg + k); }, a.N, g, col, sc, of);
                else store16<NT>(o, acc, [&](int k) INLINE_LAMBDA { return row_of(16 * rg + k); }, a.N, g, col, sc, of);
            }
        };
        for (int block = my_block; block < col_blocks; block += blocks_per_pass) {
            take_columns(block);   // re-read every time: the registers are free for E meanwhile
            if constexpr (NT == 2) {
                // two groups per step: four independent accumulation chains for the matrix pipe
#pragma unroll 1
                for (int rg = 2 * turn; rg + 2 <= groups; rg += 2 * turns) {
                    const cvec cw0 = *reinterpret_cast<const cvec *>(codes_l + (size_t)(rg * 16 + j) * CB);
                    const cvec cw1 = *reinterpret_cast<const cvec *>(codes_l + (size_t)(rg * 16 + 16 + j) * CB);
                    v4i acc0[NT], acc1[NT];
                    scan16x2<KG, NT>(cw0, cw1, B, g, one_hot, acc0, acc1);
                    if (col_on) {
                        if constexpr (ODD) {
                            store16_any<NT>(o, acc0, [&](int k) INLINE_LAMBDA { return row_of(16 * rg + k); }, a.N, g, col, sc, of);
                            store16_any<NT>(o, acc1, [&](int k) INLINE_LAMBDA { return row_of(16 * rg + 16 + k); }, a.N, g, col, sc, of);
                        } else {
                            store16<NT>(o, acc0, [&](int k) INLINE_LAMBDA { return row_of(16 * rg + k); }, a.N, g, col, sc, of);
                            store16<NT>(o, acc1, [&](int k) INLINE_LAMBDA { return row_of(16 * rg + 16 + k); }, a.N, g, col, sc, of);
                        }
                    }
                }
                // an odd last group goes to the wavefront whose turn it would be
                if ((groups & 1) && (groups >> 1) % turns == turn) one_group(groups - 1);
            } else {
#pragma unroll 1
                for (int rg = turn; rg < groups; rg += turns) one_group(rg);
            }
        }
    };
    // S with the results of a step (16 rows, or 32 for C = 64, times the up to 8 SPAN columns
    // of a pass) collected in LDS and written out row by row: a wavefront's store then covers
    // 1 KiB of one row instead of 256 (128) bytes of four rows, so that few stores end inside
    // a 128-byte line.  Every wavefront takes every step of every pass (one barrier per step); with at
    // most 4 blocks of columns the four wavefronts without columns do the writing.
    constexpr int GPS = NT == 2 ? 2 : 1;                 // groups of 16 rows per step
    constexpr int TILE_LD = kWaves * SPAN + 4;           // floats per row of the tile (4 of padding)
    auto scan_rows_gathered = [&](int groups, auto row_of) INLINE_LAMBDA {
        typedef float piece __attribute__((ext_vector_type(NT)));
        // two tiles behind the one-hot table, used in turn: a step's results are written out while the
        // next step is computed, with one barrier per step
        float *tiles = reinterpret_cast<float *>(smem + 256);
        constexpr int TILE_FLOATS = tile_bytes(NT) / 4;
        const ScanOut acc_only{nullptr, 0, a.acc, a.M};
        const int n_passes = (col_blocks + kWaves - 1) / kWaves;
        const int n_steps = (groups + GPS - 1) / GPS;
        // rows without padding between them and all columns in one pass: the rows of a unit are one range of floats
        const bool dense = ODD && a.out && a.ldo == a.M && n_passes == 1;
        const float inv_M = 1.0f / (float)a.M;
        // at most 4 blocks of columns: wavefronts 0 - 3 compute, wavefronts 4 - 7 write; else all do both
        const int first_writer = col_blocks <= kWaves / 2 ? kWaves / 2 : 0;
        const int n_writers = kWaves - first_writer;
        int it = 0;
        for (int pass = 0; pass < n_passes; ++pass) {
            const int block = pass * kWaves + wave;
            const bool active = block < col_blocks;
            if (active) take_columns(block);
            const int col0 = pass * kWaves * SPAN;
            const int n_cols = a.M - col0 < kWaves * SPAN ? a.M - col0 : kWaves * SPAN;
#pragma unroll 1
            for (int step = 0; step < n_steps; ++step, ++it) {
                float *tile = tiles + (it & 1) * TILE_FLOATS;
                const int rg = GPS * step;
                if (active) {
                    v4i acc[GPS][NT];
                    const cvec cw0 = *reinterpret_cast<const cvec *>(codes_l + (size_t)(rg * 16 + j) * CB);
                    if constexpr (GPS == 2) {
                        if (rg + 1 < groups) {
                            const cvec cw1 = *reinterpret_cast<const cvec *>(codes_l + (size_t)(rg * 16 + 16 + j) * CB);
                            scan16x2<KG, NT>(cw0, cw1, B, g, one_hot, acc[0], acc[1]);
                        } else {
                            scan16<KG, NT>(cw0, B, g, one_hot, acc[0]);
#pragma unroll
                            for (int t = 0; t < NT; ++t) acc[1][t] = acc[0][t];   // rows that do not exist: never written out
                        }
                    } else {
                        scan16<KG, NT>(cw0, B, g, one_hot, acc[0]);
                    }
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
                            if (a.acc && rg + q < groups) {
                                if constexpr (ODD) {
                                    // rows of acc start anywhere: one 16-bit store per sum
#pragma unroll
                                    for (int r = 0; r < 4; ++r) {
                                        const int64_t row = row_of(16 * (rg + q) + 4 * g + r);
#pragma unroll
                                        for (int t = 0; t < NT; ++t)
                                            if (row < a.N && col + t < a.M) a.acc[row * a.M + col + t] = (uint16_t)acc[q][t][r];
                                    }
                                } else {
                                    store16<NT>(acc_only, acc[q], [&](int k) INLINE_LAMBDA { return row_of(16 * (rg + q) + k); }, a.N, g,
                                                col, sc, of);
                                }
                            }
                        }
                    }
                }
                // (the tile written two steps ago was read before the barrier of the step between)
                __syncthreads();
                if (wave < first_writer) continue;
                const int rows_here = 16 * (groups - rg < GPS ? groups - rg : GPS);
                const int pieces = n_cols / NT;
                if (ODD && dense) {
                    // whole units of 8 consecutive rows = one range of 8 M floats each
                    for (int u = 0; 8 * u < rows_here; ++u) {
                        const int64_t first = row_of(16 * rg + 8 * u);
                        const int64_t left = a.N - first;
                        if (left > 0)
                            store_dense_rows(a.out + first * a.M, left < 8 ? (int)left : 8, a.M, inv_M, tile, TILE_LD, 8 * u,
                                             tid - 64 * first_writer, 64 * n_writers);
                    }
                    continue;
                }
                // row r of the step goes out through one wavefront, a piece of NT columns per lane
                for (int r = wave - first_writer; r < rows_here; r += n_writers) {
                    const int64_t row = row_of(16 * rg + r);
                    if (row >= a.N) continue;
                    float *dst = a.out + row * a.ldo + col0;
                    if constexpr (ODD) {
                        if (!a.out) continue;
                        // a row (its columns of this pass) as a range of its own (N = 2^20, D = 1000, M = 500,
                        // C = 50: 1.64 against 1.82 ms with 4-byte stores)
                        store_dense_rows<true>(dst, 1, n_cols, 0.f, tile, TILE_LD, r, lane_in_s, 64);
                    } else {
                        for (int c = lane_in_s; c < pieces; c += 64)
                            __builtin_nontemporal_store(*reinterpret_cast<const piece *>(tile + r * TILE_LD + NT * c),
                                                        reinterpret_cast<piece *>(dst + NT * c));
                    }
                }
            }
        }
    };
    auto scan_block = [&](int groups, auto row_of) INLINE_LAMBDA {
        // everything S derives from the lane number is derived here, each time: hoisted out
        // of the loop over the regions it would occupy registers during E, and what E keeps
        // in a spilled register it reloads in its inner loop, behind the prefetched rows
        const int lane_s = opaque(lane);
        lane_in_s = lane_s;
        j = lane_s & 15;
        g = lane_s >> 4;
        if constexpr (GATHER) {
            scan_rows_gathered(groups, row_of);
        } else if (share == 1) {
            scan_rows(groups, row_of, kWaves, wave, 1, 0);
        } else {
            const int blocks_per_pass = kWaves / share;
            scan_rows(groups, row_of, blocks_per_pass, wave % blocks_per_pass, share, wave / blocks_per_pass);
        }
    };

    const int64_t G = gridDim.x;
    if constexpr (EMODE == kRowMajor) {
        // Rows are dealt out in units of 8 consecutive rows (one per wavefront), round-robin
        // over the workgroups: in a region of 8 rw gridDim rows, unit u belongs to workgroup
        // u % gridDim and is its local unit u / gridDim.  At any moment the chip as a whole
        // reads one moving window of A (a few DRAM pages) instead of one stream per
        // wavefront, and a last, partly filled region is shared out evenly.
        unsigned char *stage = smem + wave * (RPI * DV * 1024);
        const int64_t region_rows = 8 * (int64_t)rw * G;
        for (int64_t region0 = 0; region0 < a.N; region0 += region_rows) {
            // ---- E: local row 8 k + wave is matrix row region0 + 8 (k G + block) + wave ----
            // (the tree is re-read each time: its 19 registers are better used by S)
            // (and E's own lane-derived values are derived anew, so that S need not keep them)
            const int lane_e = opaque(lane);
            Tree tr;
            {
                int c = lane_e & (C - 1);
                if constexpr (PAD) c = c < a.codebooks ? c : 0;   // a padding lane: any tree, its code is dropped
                load_tree(tr, a.split_dims + 4 * c, a.thresholds + 16 * c, a.D);
            }
            encode_rows_to_lds<C, DV, DT, false, PAD, ODD, E_PF>(a, tr, stage, codes_l + wave * CB, region0 + 8 * (int64_t)blockIdx.x + wave,
                                          rw, lane_e, 8 * G, 8);
            // the one-hot table takes the place of the first wavefront's staging area until the next E
            if (SCAN && wave == 0) {
                wave_lds_fence();
                fill_one_hot_table(one_hot, tid);
            }
            __syncthreads();
            const int64_t units_left = (a.N - region0 + 7) / 8 - (int64_t)blockIdx.x;   // units of this region from ours on
            const int64_t my_units = units_left <= 0 ? 0 : (units_left + G - 1) / G;
            const int units = (int)(my_units < rw ? my_units : rw);
            auto row_of = [&](int l) INLINE_LAMBDA { return region0 + 8 * ((int64_t)(l >> 3) * G + blockIdx.x) + (l & 7); };
            if (ODD && a.codes_out) {
                // rows of (a.codebooks + 1) / 2 bytes that start anywhere: a byte per thread and step
                const int bytes = (a.codebooks + 1) / 2;
                for (int u = tid; u < 8 * units * bytes; u += kWaves * 64) {
                    const int l = u / bytes, b = u - l * bytes;
                    const int64_t row = row_of(l);
                    if (row < a.N) a.codes_out[row * bytes + b] = codes_l[(size_t)l * CB + b];
                }
            } else if (PAD && a.codes_out) {
                // rows of a.codebooks / 2 bytes, a 32-bit word (8 codebooks) per thread and step
                const int words = a.codebooks / 8;
                for (int u = tid; u < 8 * units * words; u += kWaves * 64) {
                    const int l = u / words, w = u - l * words;
                    const int64_t row = row_of(l);
                    if (row < a.N)
                        *reinterpret_cast<uint32_t *>(a.codes_out + row * (a.codebooks / 2) + 4 * w) =
                            *reinterpret_cast<const uint32_t *>(codes_l + (size_t)l * CB + 4 * w);
                }
            } else if (a.codes_out) {
                // The codes of the region's rows, up to 16 bytes per thread and step.  (Stored row by
                // row in the encoder's loop they cost it a tenth of its rate: N = 2^22,
                // D = 1024, C = 64 encodes in 3.07 ms that way.)
                constexpr int PIECE = CB < 16 ? CB : 16;     // C = 16: a row's 8 bytes
                constexpr int PER_ROW = CB / PIECE;
                typedef unsigned piece_t __attribute__((ext_vector_type(PIECE / 4)));
                for (int u = tid; u < 8 * units * PER_ROW; u += kWaves * 64) {
                    const int64_t row = row_of(u / PER_ROW);
                    if (row < a.N)
                        *reinterpret_cast<piece_t *>(a.codes_out + row * CB + PIECE * (u % PER_ROW)) =
                            *reinterpret_cast<const piece_t *>(codes_l + (size_t)u * PIECE);
                }
            }
            // ---- S ----
            if constexpr (SCAN) scan_block((units + 1) / 2, row_of);   // 16 local rows = 2 units
            __syncthreads();   // the codes area is overwritten by the next region's E
        }
    } else {
        // A workgroup takes blocks of 8 rw consecutive rows (rw a multiple of 256), wavefront
        // w the rows [w rw, (w + 1) rw) of the block in groups of 256.  N is a multiple of 4.
        fill_one_hot_table(one_hot, tid);
        const int64_t block_rows = 8 * (int64_t)rw;
        for (int64_t R0 = blockIdx.x * block_rows; R0 < a.N; R0 += G * block_rows) {
            // ---- E ----
            {
                cols::ColsEncoder<C, DT, 2, 4> enc(a);
                for (int grp = 0; grp < rw / 256; ++grp) {
                    const int local = wave * rw + grp * 256;
                    if (R0 + local >= a.N) break;   // the same for the whole wavefront
                    enc.encode_group(R0 + local, lane);
                    enc.store_codes(a.codes_out);
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        cvec v;
#pragma unroll
                        for (int q = 0; q < CW; ++q) v[q] = enc.cwn[r][q];
                        *reinterpret_cast<cvec *>(codes_l + (size_t)(local + 4 * lane + r) * CB) = v;
                    }
                }
            }
            __syncthreads();
            // ---- S ----
            const int64_t left = a.N - R0;
            const int groups = (int)(((left < block_rows ? left : block_rows) + 15) >> 4);
            scan_block(groups, [&](int l) INLINE_LAMBDA { return R0 + l; });
            __syncthreads();   // the codes area is overwritten by the next block's E
        }
    }
}

template <int C, int DV, int NT, int DT, bool SCAN = true, bool GATHER = false, bool PAD = false, bool ODD = false>
int launch_rows(const RowsArgs &a, hipStream_t stream)
{
    constexpr int RPI = 64 / C;
    const DeviceInfo &dev = device_info();
    // (the staging area of E; with GATHER, S puts its two tiles of results there)
    constexpr int stage_bytes = shared_bytes(kRowMajor, RPI, DV, NT, GATHER);
    // rows per wavefront and region: as many as LDS holds codes for (the tables are re-read
    // once per region and pass)
    int rw = (dev.lds_per_block - stage_bytes) / (kWaves * (C / 2));
    if (rw > MADDNESS_PHASED_MAX_ROWS) rw = MADDNESS_PHASED_MAX_ROWS;
    // MADDNESS_OPT_PHASED_ROWS lowers that further (testing aid: several regions and a ragged
    // last one with few rows)
    if (const int v = option(MADDNESS_OPT_PHASED_ROWS); v >= 2 && v < rw) rw = v;
    // whole steps of the encoder (RPI rows) and whole groups of 16 rows for the scan (2 units)
    constexpr int STEP = RPI > 2 ? RPI : 2;
    rw = rw / STEP * STEP;
    if (rw < STEP) return 1;
    // few rows: one region, no more rows per wavefront than it takes
    const int64_t need = (a.N + 8 * (int64_t)dev.cus - 1) / (8 * (int64_t)dev.cus);
    if (need < rw) rw = (int)((need + STEP - 1) / STEP * STEP);
    const size_t lds = (size_t)stage_bytes + (size_t)kWaves * rw * (C / 2);
    if (int rc = allow_full_lds<fused_mfma_kernel<C, DV, NT, kRowMajor, DT, SCAN, GATHER, PAD, ODD>>(); rc != MADDNESS_OK) return rc;
    const int64_t units = (a.N + 7) / 8;
    const int grid = (int)(units < max_workgroups() ? units : max_workgroups());
    note_kernel("fused_mfma_kernel, A by rows", __PRETTY_FUNCTION__);
    hipLaunchKernelGGL((fused_mfma_kernel<C, DV, NT, kRowMajor, DT, SCAN, GATHER, PAD, ODD>), dim3(grid), dim3(kWaves * 64), lds, stream, a, rw);
    return check_hip(hipGetLastError(), "launch fused_mfma_kernel");
}

template <int C, int NT, int DT>
int launch_cols(const RowsArgs &a, hipStream_t stream)
{
    const DeviceInfo &dev = device_info();
    // rows per wavefront and block: a multiple of 256; as few blocks per workgroup as LDS
    // allows, all of the same size
    int rw_max = (dev.lds_per_block - 256) / (kWaves * (C / 2)) / 256 * 256;
    // MADDNESS_OPT_PHASED_ROWS lowers that (testing aid: several blocks per workgroup with few rows)
    if (const int v = option(MADDNESS_OPT_PHASED_ROWS); v >= 2 && (v + 255) / 256 * 256 < rw_max) rw_max = (v + 255) / 256 * 256;
    if (rw_max < 256) return 1;
    const int wgs = max_workgroups();
    const int64_t per_wave = (a.N + (int64_t)kWaves * wgs - 1) / ((int64_t)kWaves * wgs);   // rows per wavefront in all
    const int64_t turns = (per_wave + rw_max - 1) / rw_max;
    int rw = (int)(((per_wave + turns - 1) / turns + 255) / 256 * 256);
    if (rw > rw_max) rw = rw_max;
    const size_t lds = 256 + (size_t)kWaves * rw * (C / 2);
    if (int rc = allow_full_lds<fused_mfma_kernel<C, 1, NT, kByColumns, DT>>(); rc != MADDNESS_OK) return rc;
    const int64_t blocks = (a.N + (int64_t)kWaves * rw - 1) / ((int64_t)kWaves * rw);
    const int grid = (int)(blocks < wgs ? blocks : wgs);
    note_kernel("fused_mfma_kernel, A by columns", __PRETTY_FUNCTION__);
    hipLaunchKernelGGL((fused_mfma_kernel<C, 1, NT, kByColumns, DT>), dim3(grid), dim3(kWaves * 64), lds, stream, a, rw);
    return check_hip(hipGetLastError(), "launch fused_mfma_kernel");
}

template <int C, int DV, int NT>
int launch_rows_typed(const RowsArgs &a, int dtype, hipStream_t stream)
{
    switch (dtype) {
    case MADDNESS_F16: return launch_rows<C, DV, NT, kF16>(a, stream);
    case MADDNESS_BF16: return launch_rows<C, DV, NT, kBF16>(a, stream);
    default: return launch_rows<C, DV, NT, kU8>(a, stream);
    }
}

// fp32 row-major A of any shape the tiles cover (up to 64 codebooks, rows of up to 8 KiB; up to 16
// codebooks: 2 KiB, up to 32: 4 KiB), any M, any pitch and alignment: the ODD form of the kernel.
// Not for short rows: the E phase spends a fixed time per row, and below 512 bytes the general
// kernels, which only fetch the 4 C split values of a row, are faster (D = 27, C = 4, N = 2^20:
// 0.03 against 0.47 ms).
template <bool SCAN, bool GATHER>
int launch_odd_sized(const RowsArgs &a, int codebooks, int need, hipStream_t stream)
{
    if (codebooks <= 16 && need <= 1024) return launch_rows<16, 1, 4, kF32, SCAN, GATHER, true, true>(a, stream);
    if (codebooks <= 16 && need <= 2048) return launch_rows<16, 2, 4, kF32, SCAN, GATHER, true, true>(a, stream);
    if (codebooks <= 32 && need <= 2048) return launch_rows<32, 2, 4, kF32, SCAN, GATHER, true, true>(a, stream);
    if (codebooks <= 32 && need <= 4096) return launch_rows<32, 4, 4, kF32, SCAN, GATHER, true, true>(a, stream);
    if (codebooks <= 64 && need <= 4096) return launch_rows<64, 4, 2, kF32, SCAN, GATHER, true, true>(a, stream);
    if (codebooks <= 64 && need <= 8192) return launch_rows<64, 8, 2, kF32, SCAN, GATHER, true, true>(a, stream);
    return 1;
}

template <bool SCAN>
int launch_odd(const RowsArgs &a, int codebooks, int row_bytes, hipStream_t stream)
{
    if (row_bytes < 512) return 1;
    // a row is staged from the 16-byte boundary at or before its start: row n begins (a0 + n s4) mod 16
    // bytes after one
    const unsigned a0 = (unsigned)reinterpret_cast<uintptr_t>(a.A) & 15u, s4 = (unsigned)(a.lda * 4) & 15u;
    unsigned max_shift = 0;
    for (unsigned n = 0; n < 4; ++n) max_shift = std::max(max_shift, (a0 + n * s4) & 15u);
    const int need = row_bytes + (int)max_shift;
    if constexpr (SCAN) {
        // more than two blocks of columns: whole rows through LDS; else straight from the registers
        const int span = codebooks <= 32 ? 64 : 32;
        if ((a.M + span - 1) / span > 2) return launch_odd_sized<true, true>(a, codebooks, need, stream);
    }
    return launch_odd_sized<SCAN, false>(a, codebooks, need, stream);
}

// Row-major A: rows of 16-byte pieces, at most 8 KiB (fp32) or 4 KiB (narrow types) long.
// SCAN = false (encode only): fp32.
template <bool SCAN>
int launch_row_major(const RowsArgs &a, int C, int D, const MatrixA &A, hipStream_t stream)
{
    const int es = A.elem_bytes();
    if ((D * es) % 16 != 0 || (A.ld * es) % 16 != 0 || !aligned_to(A.data, 16)) return 1;
    if (a.codebooks == C && a.codes_out && !aligned_to(a.codes_out, C == 16 ? 8 : 16)) return 1;
    const int row_bytes = D * es;
    if (a.codebooks != C) {
        // a multiple of 8 codebooks that is not 16, 32 or 64: the next larger kernel, padded (fp32)
        if (A.dtype != MADDNESS_F32 || (a.codes_out && !aligned_to(a.codes_out, 4))) return 1;
        if (C == 16 && D <= 512) return launch_rows<16, 2, 4, kF32, SCAN, false, true>(a, stream);
        if (C == 32 && D <= 512) return launch_rows<32, 2, 4, kF32, SCAN, false, true>(a, stream);
        if (C == 32 && D <= 1024) return launch_rows<32, 4, 4, kF32, SCAN, false, true>(a, stream);
        if (C == 64 && D <= 1024) return launch_rows<64, 4, 2, kF32, SCAN, false, true>(a, stream);
        return 1;
    }
    if constexpr (SCAN) {
        // The S phase that writes whole rows: for fp32 output rows that do not start on 128-byte
        // lines (more than 4 blocks of columns; N = 2^20, C = 32, M = 1000: 1.43 against 2.04 ms),
        // and where one pass of the 8 wavefronts covers the whole row exactly (C <= 32, M in
        // (448, 512]: 0.675 against 0.767 ms at M = 512; no gain elsewhere: at M = 256 0.519 against 0.524 ms
        // beside rows of 2 KiB and 0.864 against 0.834 ms beside rows of 4 KiB, 1.27 against 1.22 ms at
        // M = 1024, 2.89 against 2.39 ms at C = 64, M = 512)
        const int span = C == 64 ? 32 : 64;
        const bool unaligned = a.ldo % 32 != 0 || !aligned_to(a.out, 128);
        const bool one_full_pass = C != 64 && a.M > 7 * span && a.M <= 8 * span;
        if (A.dtype == MADDNESS_F32 && a.out && ((unaligned && a.M > 4 * span) || one_full_pass)) {
            if (C == 16 && D <= 512) return launch_rows<16, 2, 4, kF32, true, true>(a, stream);
            if (C == 32 && D <= 512) return launch_rows<32, 2, 4, kF32, true, true>(a, stream);
            if (C == 32 && D <= 1024) return launch_rows<32, 4, 4, kF32, true, true>(a, stream);
            if (C == 64 && D <= 1024) return launch_rows<64, 4, 2, kF32, true, true>(a, stream);
        }
    }
    if (A.dtype == MADDNESS_F32) {
        if (C == 16 && D <= 256) return launch_rows<16, 1, 4, kF32, SCAN>(a, stream);
        if (C == 16 && D <= 512) return launch_rows<16, 2, 4, kF32, SCAN>(a, stream);
        if (C == 16 && D <= 1024) return launch_rows<16, 4, 4, kF32, SCAN>(a, stream);
        if (C == 64 && D <= 1024) return launch_rows<64, 4, 2, kF32, SCAN>(a, stream);
        if (C == 32 && D <= 512) return launch_rows<32, 2, 4, kF32, SCAN>(a, stream);
        if (C == 32 && D <= 1024) return launch_rows<32, 4, 4, kF32, SCAN>(a, stream);
        if (C == 64 && D <= 2048) return launch_rows<64, 8, 2, kF32, SCAN>(a, stream);
        if (C == 32 && D <= 2048) return launch_rows<32, 8, 4, kF32, SCAN>(a, stream);
        return 1;
    }
    if constexpr (!SCAN) return 1;
    if (row_bytes > 4096 || C == 16) return 1;
    if (C == 32)
        return row_bytes <= 1024   ? launch_rows_typed<32, 1, 4>(a, A.dtype, stream)
               : row_bytes <= 2048 ? launch_rows_typed<32, 2, 4>(a, A.dtype, stream)
                                   : launch_rows_typed<32, 4, 4>(a, A.dtype, stream);
    return row_bytes <= 1024   ? launch_rows_typed<64, 1, 2>(a, A.dtype, stream)
           : row_bytes <= 2048 ? launch_rows_typed<64, 2, 2>(a, A.dtype, stream)
                               : launch_rows_typed<64, 4, 2>(a, A.dtype, stream);
}

}  // namespace

// Returns MADDNESS_OK after a launch, 1 if the shape is not covered.
int launch_fused_mfma(const maddness_params &p, const MatrixA &A, int64_t N, int32_t M, const uint8_t *luts,
                      const float *scale, const float *offset, float *out, int64_t ldo, uint16_t *acc,
                      uint8_t *codes, hipStream_t stream)
{
    const int D = p.D;
    const int es = A.elem_bytes();
    if (N < 16384) return 1;
    RowsArgs a{};
    a.A = A.data; a.lda = A.ld; a.D = D; a.N = N;
    a.split_dims = p.split_dims; a.thresholds = p.thresholds;
    a.luts = luts; a.scale = scale; a.offset = offset; a.M = M;
    a.out = out; a.ldo = ldo; a.acc = acc; a.codes_out = codes;
    a.codebooks = p.C;
    // the kernel's C: 16, 32 or 64; another multiple of 8 takes the next larger one with padding
    const int C = p.C <= 16 ? 16 : (p.C <= 32 ? 32 : 64);
    const int NT = C == 64 ? 2 : 4;
    // shapes the tiled forms do not take as they are (C not a multiple of 8, rows of A or of the outputs that
    // are not whole aligned pieces, M not a multiple of the lane's columns): the form for any shape
    const bool regular = p.C % 8 == 0 && p.C >= 8 && p.C <= 64 && (C == p.C || A.plain()) && M % NT == 0 &&
                         aligned_to(luts, NT) && (!out || (ldo % NT == 0 && aligned_to(out, 4 * NT))) &&
                         (!acc || aligned_to(acc, 2 * NT)) &&
                         (A.col_major || ((D * es) % 16 == 0 && (A.ld * es) % 16 == 0 && aligned_to(A.data, 16) &&
                                          (!codes || aligned_to(codes, C != p.C ? 4 : (C == 16 ? 8 : 16)))));
    if (!regular) {
        if (!A.plain() || p.C > 64) return 1;
        return launch_odd<true>(a, p.C, 4 * D, stream);
    }
    if (A.col_major) {
        if (C == 16) return 1;
        // runs of four rows: column stride and base aligned to four elements, whole quads of rows
        // (the caller takes care of the last N % 4 rows)
        if (N % 4 != 0 || A.ld % 4 != 0 || !aligned_to(A.data, 4 * (size_t)es)) return 1;
        if (codes && !aligned_to(codes, C / 2)) return 1;
        if (C == 32) {
            switch (A.dtype) {
            case MADDNESS_F32: return launch_cols<32, 4, kF32>(a, stream);
            case MADDNESS_F16: return launch_cols<32, 4, kF16>(a, stream);
            case MADDNESS_BF16: return launch_cols<32, 4, kBF16>(a, stream);
            default: return launch_cols<32, 4, kU8>(a, stream);
            }
        }
        switch (A.dtype) {
        case MADDNESS_F32: return launch_cols<64, 2, kF32>(a, stream);
        case MADDNESS_F16: return launch_cols<64, 2, kF16>(a, stream);
        case MADDNESS_BF16: return launch_cols<64, 2, kBF16>(a, stream);
        default: return launch_cols<64, 2, kU8>(a, stream);
        }
    }
    return launch_row_major<true>(a, C, D, A, stream);
}

// Encode only, with the E phase of the same kernel (M = 0: no S phase, the codes are copied
// from LDS to memory after it): the rows of a region are read in one moving window by the
// whole chip.
int launch_encode_phased(const maddness_params &p, const MatrixA &A, int64_t N, uint8_t *codes, hipStream_t stream)
{
    if (p.C > 64 || !A.plain() || N < 16384) return 1;
    const int C = p.C <= 16 ? 16 : (p.C <= 32 ? 32 : 64);   // the kernel's C; the rest is padding
    RowsArgs a{};
    a.A = A.data; a.lda = A.ld; a.D = p.D; a.N = N;
    a.split_dims = p.split_dims; a.thresholds = p.thresholds;
    a.codes_out = codes;
    a.codebooks = p.C;
    if (p.C % 8 == 0) {
        const int rc = launch_row_major<false>(a, C, p.D, A, stream);
        if (rc != 1) return rc;
    }
    return launch_odd<false>(a, p.C, 4 * p.D, stream);
}

}  // namespace maddness
