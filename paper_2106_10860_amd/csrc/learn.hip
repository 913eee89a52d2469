// The learning step on the GPU: the greedy construction of the hashing trees (Section 4.2,
// Algorithm 2; Appendix C, Algorithms 3 and 4) and the prototypes (bucket means; ridge
// regression, Section 4.3).  Set-up work, run once per problem; what matters here is that
// it takes milliseconds instead of seconds and that its decisions can be checked.
//
// Every quantity a decision depends on (bucket losses, cumulative SSEs, level losses) is
// computed in fp64 with the operations in the order Algorithms 2-4 state them - sums over the
// rows of a bucket run sequentially in sorted (or row) order, sums over the columns of the
// subspace in column order - so that the trees are reproducible to the bit and do not depend
// on the launch shape.  The parallelism is ACROSS the independent pieces: codebooks, candidate
// columns, buckets and columns.  This file is compiled without floating-point contraction.
//
// The serial parts are chains of a few instructions per row on a few lanes, and a wavefront issues
// one vector instruction in four cycles whatever the number of its active lanes: each chain is kept
// to the instructions its sum needs, reads operands that all threads have laid side by side in LDS,
// and leaves products, divisions, comparisons and counting to all threads or to wavefront ballots.
//
// Per level t = 1..4 of all C trees at once:
//   order_rows_kernel    the rows of every bucket listed in row order, the bucket sizes
//   bucket_loss_kernel   L(j, B) (Section 4.2) for every column j of every bucket, two passes
//                        over the bucket's own rows
//   select_kernel        heuristic_select_idxs: the four columns with the largest summed loss
//   key_kernel, sort_chunks_kernel, sort_exchange_kernel  the rows ordered by each candidate column (bitonic sort of
//                        (value, row) keys: equal values stay in row order, as a stable sort
//                        of a bucket's rows leaves them)
//   split_ordered_kernel (split_kernel for the widest subspaces)  Algorithm 3 for every bucket of
//                        the level in one forward and one backward sweep over that order
//                        (Algorithm 4's running sums kept per bucket), the best threshold and
//                        loss per bucket
//   choose_kernel        Algorithm 2's choice among the candidates
//   apply_kernel         apply_split: the next level's buckets
// Prototypes: cooccurrence_kernel (G^T G), gta_kernel (G^T A~), cholesky_panel_kernel,
// factor by rows, substitution_kernel; or means_kernel.
#include "common.h"

namespace maddness {
namespace {

constexpr int kSplitBuckets = 8;   // buckets of the deepest level that is split (level 4 splits 8)
constexpr int kCand = 4;           // candidate columns per level (Section 4.2: n = 4)
constexpr int kMaxTile = 256;      // most sorted positions a workgroup of split_ordered_kernel takes at a time (a thread each)
constexpr int kSplitTile = 64;     // sorted positions a workgroup of split_kernel takes at a time
constexpr int kSortChunk = 8192;   // keys sorted in LDS at a time (64 KiB)

// LDS of split_kernel for subspaces of d columns and tiles of T positions (a multiple of 8 bytes)
__host__ __device__ constexpr size_t split_lds_bytes_base(int d, int T)
{
    return sizeof(double) * ((size_t)T * d + 2 * (size_t)kSplitBuckets * d + T) + sizeof(float) * (size_t)T * (d + 2) +
           sizeof(int32_t) * 3 * T + kSplitBuckets * (3 * sizeof(double) + 3 * sizeof(float) + 3 * sizeof(int32_t)) +
           T * (sizeof(double) + sizeof(float)) + sizeof(int32_t) * ((size_t)T + 6 * kSplitBuckets);
}

struct Bounds {
    int32_t v[2 * MADDNESS_MAX_C];
};

struct LearnArgs {
    const float *A;
    int64_t lda, N, Npad;
    int32_t C, dmax;
    int32_t *bounds;      // [C][2] first and one-past-last column of every codebook
    uint8_t *node;        // [C][N] bucket (0-based) of every row in the current level
    double *col_loss;     // [C][8][dmax] L(j, B_i)
    double *bucket_loss;  // [C][8] L(B_i)
    int64_t *bucket_count;  // [C][8]
    int32_t *bucket_start;  // [C][8] where the bucket's rows begin in rows_by_bucket[c]
    int32_t *rows_by_bucket;  // [C][N] the rows of bucket 0 in row order, then those of bucket 1, ...
    int32_t *cand;        // [C][4] candidate columns (within the subspace), best first
    int32_t *n_cand;      // [C]
    uint64_t *keys;       // [C][4][Npad] sorted (value, row) keys
    double *head;         // [C][4][N] Algorithm 4, forward, by sorted position
    double *res_loss;     // [C][4][8] loss of the best split of bucket i along candidate q
    float *res_v;         // [C][4][8] its threshold
    int32_t *chosen;      // [C] the level's column (within the subspace)
    int32_t *split_dims;  // out [C][4]
    float *thresholds;    // out [C][16]
    uint8_t *codes;       // out [N][C] or null
};

__global__ void upload_bounds_kernel(const Bounds b, int32_t n, int32_t *dst)
{
    for (int i = threadIdx.x; i < n; i += blockDim.x) dst[i] = b.v[i];
}

__global__ void fill_bytes_kernel(uint8_t *p, int64_t n, uint8_t v)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

// The rows of every bucket, in row order (a stable counting sort of the rows by bucket): rows_by_bucket[c]
// holds the rows of bucket 0, then those of bucket 1, ...; bucket_start and bucket_count say where.  One
// workgroup per codebook: the counts first, then the rows 256 at a time, a row's place among the rows of its
// bucket from wavefront ballots.
__global__ __launch_bounds__(256) void order_rows_kernel(const LearnArgs a, int n_buckets)
{
    __shared__ int32_t total[kSplitBuckets], first[kSplitBuckets], seen[kSplitBuckets];
    __shared__ int32_t wave_count[2][kSplitBuckets][4];
    const int c = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t N = a.N;
    const uint8_t *node = a.node + (size_t)c * N;
    int32_t *out = a.rows_by_bucket + (size_t)c * N;
    if (tid < kSplitBuckets) total[tid] = 0;
    __syncthreads();
    for (int64_t n0 = 0; n0 < N; n0 += 256) {
        const int my_b = n0 + tid < N ? node[n0 + tid] : -1;
        for (int k = 0; k < n_buckets; ++k) {
            const unsigned long long mask = __ballot(my_b == k);
            if (lane == 0 && mask != 0) atomicAdd(&total[k], __popcll(mask));
        }
    }
    __syncthreads();
    if (tid == 0) {
        int32_t at = 0;
        for (int k = 0; k < kSplitBuckets; ++k) {
            first[k] = at;
            seen[k] = 0;
            a.bucket_start[c * kSplitBuckets + k] = at;
            a.bucket_count[c * kSplitBuckets + k] = k < n_buckets ? total[k] : 0;
            at += k < n_buckets ? total[k] : 0;
        }
    }
    int next_b = tid < N ? node[tid] : -1;
    __syncthreads();
    int parity = 0;
    for (int64_t n0 = 0; n0 < N; n0 += 256, parity ^= 1) {
        const int my_b = next_b;
        next_b = n0 + 256 + tid < N ? node[n0 + 256 + tid] : -1;
        int rank = 0;
        for (int k = 0; k < n_buckets; ++k) {
            const unsigned long long mask = __ballot(my_b == k);
            if (my_b == k) rank = __popcll(mask & ((1ull << lane) - 1ull));
            if (lane == 0) wave_count[parity][k][wave] = __popcll(mask);
        }
        __syncthreads();
        if (my_b >= 0) {
            for (int w = 0; w < wave; ++w) rank += wave_count[parity][my_b][w];
            out[first[my_b] + seen[my_b] + rank] = (int32_t)(n0 + tid);
        }
        __syncthreads();
        if (tid < n_buckets)
            seen[tid] += wave_count[parity][tid][0] + wave_count[parity][tid][1] + wave_count[parity][tid][2] + wave_count[parity][tid][3];
    }
}

// L(j, B_i): a thread per column of the subspace - a chain - takes the bucket's rows in row order, twice (the
// sum, then the squared distances from the mean); one workgroup per (codebook, bucket).  The chains are the
// serial part and a wavefront issues a vector instruction in four cycles, so they are kept short: all threads
// of the workgroup gather the next rows' values into LDS, a column's values side by side, while the chains
// walk the rows gathered before, four rows to an LDS read.  (The list of rows is fetched two tiles ahead, the
// values one tile ahead.)
constexpr int kLossTileFloats = 8192;      // values of a tile (32 KiB), two tiles in LDS
constexpr int kLossTileRows = 512;         // most rows of a tile
constexpr int kLossPer = kLossTileFloats / 256;
constexpr int kLossMaxWidth = 128;         // widest subspace its LDS tiles are laid out for
__host__ __device__ constexpr int loss_tile_rows(int d)
{
    return kLossTileFloats / d >= kLossTileRows ? kLossTileRows : (kLossTileFloats / d) & ~15;
}
constexpr size_t kLossTileStride = kLossTileFloats + 4 * kLossMaxWidth + 8;     // floats between the two tiles
constexpr size_t kLossLdsBytes = sizeof(float) * 2 * kLossTileStride + sizeof(int32_t) * 2 * kLossTileRows;

__global__ __launch_bounds__(256) void bucket_loss_kernel(const LearnArgs a)
{
    extern __shared__ __align__(16) unsigned char lds_raw[];
    float *xt = reinterpret_cast<float *>(lds_raw);                                   // [2][kLossTileStride]
    int32_t *listed = reinterpret_cast<int32_t *>(xt + 2 * kLossTileStride);          // [2][kLossTileRows]
    const int c = blockIdx.y, b = blockIdx.x, tid = threadIdx.x;
    const int lo = a.bounds[2 * c], d = a.bounds[2 * c + 1] - lo;
    const int R = loss_tile_rows(d), Rp = R + 4;       // (columns R + 4 floats apart: 16-byte reads, and the banks spread)
    const int64_t count = a.bucket_count[c * kSplitBuckets + b];
    const int32_t *list = a.rows_by_bucket + (size_t)c * a.N + a.bucket_start[c * kSplitBuckets + b];
    const float *cols = a.A + lo;
    const int64_t n_tiles = (count + R - 1) / R;
    const int jj = tid < d ? tid : 0;
    // what this thread gathers of a tile: elements tid + 256 u of its R x d values; (row, column) of the first,
    // and the step from one to the next
    const int row_first = tid / d, col_first = tid - row_first * d, row_step = 256 / d, col_step = 256 - row_step * d;
    float pre[kLossPer];
    int32_t pre_rows[kLossTileRows / 256];
    auto fetch_list = [&](int64_t tile) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < kLossTileRows / 256; ++u) {
            const int64_t at = tile * R + tid + 256 * u;
            pre_rows[u] = (tid + 256 * u < R && at < count) ? list[at] : 0;
        }
    };
    auto stash_list = [&](int64_t tile) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < kLossTileRows / 256; ++u)
            if (tid + 256 * u < R) listed[(tile & 1) * kLossTileRows + tid + 256 * u] = pre_rows[u];
    };
    auto fetch = [&](int64_t tile) __attribute__((always_inline)) {
        const int32_t *rows = listed + (tile & 1) * kLossTileRows;
        const int64_t left = count - tile * R;
        int row = row_first, col = col_first;
#pragma unroll
        for (int u = 0; u < kLossPer; ++u) {
            pre[u] = (row < R && row < left) ? cols[(int64_t)rows[row] * a.lda + col] : 0.0f;
            row += row_step;
            col += col_step;
            if (col >= d) {
                col -= d;
                ++row;
            }
        }
    };
    auto stash = [&](int64_t tile) __attribute__((always_inline)) {
        float *dst = xt + (tile & 1) * kLossTileStride;
        int row = row_first, col = col_first;
#pragma unroll
        for (int u = 0; u < kLossPer; ++u) {
            if (row < R) dst[col * Rp + row] = pre[u];
            row += row_step;
            col += col_step;
            if (col >= d) {
                col -= d;
                ++row;
            }
        }
    };
    double sum = 0.0, mean = 0.0, loss = 0.0;
    auto walk = [&](auto second) __attribute__((always_inline)) {
        constexpr bool kSecond = decltype(second)::value;
        __syncthreads();
        fetch_list(0);
        stash_list(0);
        fetch_list(1);
        __syncthreads();
        fetch(0);
        stash(0);
        stash_list(1);
        __syncthreads();
        for (int64_t tile = 0; tile < n_tiles; ++tile) {
            if (tile + 2 < n_tiles) fetch_list(tile + 2);
            if (tile + 1 < n_tiles) fetch(tile + 1);
            if (tid < d) {
                const float *xs = xt + (tile & 1) * kLossTileStride + jj * Rp;
                const int64_t left = count - tile * R;
                const int rows_here = (int)(left < R ? left : R);
                // eight rows at a time, the eight after them read from LDS meanwhile (the fences keep the compiler
                // from moving the reads back to where their values are used)
                float x0[8], x1[8];
                auto read = [&](int row, float *x) __attribute__((always_inline)) {
#pragma unroll
                    for (int u = 0; u < 8; ++u) x[u] = xs[row + u];
                };
                auto add = [&](const float *x) __attribute__((always_inline)) {
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        if constexpr (!kSecond) {
                            sum += (double)x[u];
                        } else {
                            const double e = (double)x[u] - mean;
                            loss += e * e;
                        }
                    }
                };
                const int full = rows_here & ~15;
                read(0, x0);
                for (int row = 0; row < full; row += 16) {
                    read(row + 8, x1);
                    __builtin_amdgcn_sched_barrier(0);
                    add(x0);
                    __builtin_amdgcn_sched_barrier(0);
                    read(row + 16, x0);            // (past the tile's last row at the end: read, not used)
                    __builtin_amdgcn_sched_barrier(0);
                    add(x1);
                    __builtin_amdgcn_sched_barrier(0);
                }
                for (int row = full; row < rows_here; ++row) {
                    const double x = (double)xs[row];
                    if constexpr (!kSecond) {
                        sum += x;
                    } else {
                        const double e = x - mean;
                        loss += e * e;
                    }
                }
            }
            if (tile + 1 < n_tiles) stash(tile + 1);
            if (tile + 2 < n_tiles) stash_list(tile + 2);
            __syncthreads();
        }
    };
    walk(std::false_type{});
    mean = count > 0 ? sum / (double)count : 0.0;
    walk(std::true_type{});
    if (tid < d) a.col_loss[((size_t)c * kSplitBuckets + b) * a.dmax + jj] = count > 0 ? loss : 0.0;
}

// heuristic_select_idxs, and L(B_i) = sum over the columns of L(j, B_i).
__global__ __launch_bounds__(64) void select_kernel(const LearnArgs a, int n_buckets)
{
    extern __shared__ double total[];   // [dmax]
    const int c = blockIdx.x;
    const int d = a.bounds[2 * c + 1] - a.bounds[2 * c];
    const double *cl = a.col_loss + (size_t)c * kSplitBuckets * a.dmax;
    for (int jj = threadIdx.x; jj < d; jj += 64) {
        double t = 0.0;
        for (int b = 0; b < n_buckets; ++b) t += cl[(size_t)b * a.dmax + jj];
        total[jj] = t;
    }
    if ((int)threadIdx.x < n_buckets) {
        double l = 0.0;
        for (int jj = 0; jj < d; ++jj) l += cl[(size_t)threadIdx.x * a.dmax + jj];
        a.bucket_loss[c * kSplitBuckets + threadIdx.x] = l;
    }
    __syncthreads();
    if (threadIdx.x != 0) return;
    const int n_cand = d < kCand ? d : kCand;
    int pick[kCand];
    for (int q = 0; q < n_cand; ++q) {
        int best = -1;
        for (int jj = 0; jj < d; ++jj) {
            bool taken = false;
            for (int p = 0; p < q; ++p) taken |= pick[p] == jj;
            if (!taken && (best < 0 || total[jj] > total[best])) best = jj;   // equal losses: the lower column
        }
        pick[q] = best;
        a.cand[c * kCand + q] = best;
    }
    a.n_cand[c] = n_cand;
}

// (bucket, value, row) keys, 3 + 32 + 29 bits: unsigned order = by bucket, then by value, equal values (-0 counts
// as +0) by row.  The rows of a bucket end up side by side, in the order Algorithm 3 wants them.
constexpr int kKeyRowBits = 29;
__device__ __forceinline__ uint64_t make_key(int bucket, float x, uint32_t row)
{
    const uint32_t bits = __float_as_uint(x + 0.0f);
    const uint32_t u = (bits & 0x80000000u) ? ~bits : (bits | 0x80000000u);
    return ((uint64_t)bucket << (32 + kKeyRowBits)) | ((uint64_t)u << kKeyRowBits) | row;
}
__device__ __forceinline__ float key_value(uint64_t key)
{
    const uint32_t u = (uint32_t)(key >> kKeyRowBits);
    return __uint_as_float((u & 0x80000000u) ? (u ^ 0x80000000u) : ~u);
}
__device__ __forceinline__ int32_t key_row(uint64_t key) { return (int32_t)(key & ((1u << kKeyRowBits) - 1u)); }

__global__ __launch_bounds__(256) void key_kernel(const LearnArgs a, int by_bucket)
{
    const int c = blockIdx.z, q = blockIdx.y;
    if (q >= a.n_cand[c]) return;
    const int64_t p = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (p >= a.Npad) return;
    const int j = a.bounds[2 * c] + a.cand[c * kCand + q];
    a.keys[((size_t)c * kCand + q) * a.Npad + p] =
        p < a.N ? make_key(by_bucket ? a.node[(size_t)c * a.N + p] : 0, a.A[p * a.lda + j], (uint32_t)p) : ~0ull;
}

// Bitonic sort of Npad keys (a power of two) per (codebook, candidate).  The exchanges at distances below
// kSortChunk run on chunks of kSortChunk keys in LDS, a workgroup per chunk (sort_chunks_kernel: the stages
// k_first .. k_last whole when j_first is 0, else the distances j_first .. 1 of stage k_first); the exchanges
// at larger distances go through memory, a thread per pair (sort_exchange_kernel: one distance of one stage).
__device__ __forceinline__ void exchange(uint64_t &x, uint64_t &y, bool ascending)
{
    if ((x > y) == ascending) {
        const uint64_t t = x;
        x = y;
        y = t;
    }
}

__global__ __launch_bounds__(1024) void sort_chunks_kernel(const LearnArgs a, int64_t k_first, int64_t k_last, int64_t j_first)
{
    extern __shared__ uint64_t chunk[];   // [min(Npad, kSortChunk)]
    const int c = blockIdx.z, q = blockIdx.y;
    if (q >= a.n_cand[c]) return;
    uint64_t *keys = a.keys + ((size_t)c * kCand + q) * a.Npad;
    const int64_t n = a.Npad;
    const int64_t m = n < kSortChunk ? n : kSortChunk;   // chunk length
    const int64_t base = (int64_t)blockIdx.x * m;
    const int tid = threadIdx.x;
    for (int64_t i = tid; i < m; i += 1024) chunk[i] = keys[base + i];
    __syncthreads();
    for (int64_t k = k_first; k <= k_last; k <<= 1) {
        for (int64_t j = (k == k_first && j_first) ? j_first : k >> 1; j > 0; j >>= 1) {
            for (int64_t t = tid; t < m / 2; t += 1024) {
                const int64_t i = 2 * t - (t & (j - 1));   // the lower index of pair t at distance j
                exchange(chunk[i], chunk[i + j], ((base + i) & k) == 0);
            }
            __syncthreads();
        }
    }
    for (int64_t i = tid; i < m; i += 1024) keys[base + i] = chunk[i];
}

__global__ __launch_bounds__(256) void sort_exchange_kernel(const LearnArgs a, int64_t k, int64_t j)
{
    const int c = blockIdx.z, q = blockIdx.y;
    if (q >= a.n_cand[c]) return;
    uint64_t *keys = a.keys + ((size_t)c * kCand + q) * a.Npad;
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= a.Npad / 2) return;
    const int64_t i = 2 * t - (t & (j - 1));
    const uint64_t x = keys[i], y = keys[i + j];
    if ((x > y) == ((i & k) == 0)) {
        keys[i] = y;
        keys[i + j] = x;
    }
}

// Algorithm 3 for all buckets of the level along candidate q of codebook c.
// Forward sweep over the sorted rows: Algorithm 4's running sums per bucket and column, the
// SSE of the bucket's rows so far (head) stored by position.  Backward sweep: the same from
// the other end (tail); at a row of bucket i the split between it and the bucket's next row
// up is judged by head + tail, if their values differ.  Going down, a loss that is not larger
// replaces the best: the first minimum in ascending order wins.
// kSplitTile positions at a time (a tile): a thread per position fetches its row's bucket and values into LDS, the
// running sums are carried through the tile in order by a thread per column, then summed over the columns (in
// column order) by one thread per position.  This kernel takes the subspaces too wide for split_ordered_kernel.
__global__ __launch_bounds__(256) void split_kernel(const LearnArgs a, int n_buckets)
{
    constexpr int T = kSplitTile;
    extern __shared__ __align__(16) unsigned char lds_raw[];
    const int c = blockIdx.y, q = blockIdx.x;
    if (q >= a.n_cand[c]) return;
    const int lo = a.bounds[2 * c], d = a.bounds[2 * c + 1] - lo;
    const int jsplit = a.cand[c * kCand + q];
    const int tid = threadIdx.x;
    const int64_t N = a.N;
    const uint64_t *keys = a.keys + ((size_t)c * kCand + q) * a.Npad;
    const uint8_t *node = a.node + (size_t)c * N;
    double *head = a.head + ((size_t)c * kCand + q) * N;

    double *term = reinterpret_cast<double *>(lds_raw);            // [T][d]
    double *cumX = term + (size_t)T * d;                       // [8][d]
    double *cumX2 = cumX + (size_t)kSplitBuckets * d;              // [8][d]
    double *sse = cumX2 + (size_t)kSplitBuckets * d;               // [T]
    float *xt = reinterpret_cast<float *>(sse + T);            // [T][d]
    // (rows of xt are xld = d | 1 floats apart: an odd pitch, so that the threads of a wavefront, a slot each,
    // write their rows without meeting in the same LDS banks; the area holds T (d + 2) floats, a whole number
    // of 8 bytes)
    const int xld = d | 1;
    int32_t *rows = reinterpret_cast<int32_t *>(xt + (size_t)T * (d + 2));   // [T]
    int32_t *bkt = rows + T;                                   // [T]
    int32_t *cnt_at = bkt + T;                                 // [T] rows of the bucket up to this one
    // per bucket: rows seen in this sweep; the best split so far; the bucket's row above the current one
    int64_t *count = reinterpret_cast<int64_t *>(cnt_at + T);
    double *best_loss = reinterpret_cast<double *>(count + kSplitBuckets), *up_tail = best_loss + kSplitBuckets;
    float *best_lo = reinterpret_cast<float *>(up_tail + kSplitBuckets), *best_hi = best_lo + kSplitBuckets;
    float *up_value = best_hi + kSplitBuckets;
    int32_t *have_best = reinterpret_cast<int32_t *>(up_value + kSplitBuckets), *have_up = have_best + kSplitBuckets;
    int32_t *first_row = have_up + kSplitBuckets;
    // the backward sweep's copies of a tile's forward sums and values
    double *head_l = reinterpret_cast<double *>(first_row + kSplitBuckets);   // [T]
    float *value_l = reinterpret_cast<float *>(head_l + T);               // [T]

    auto sweep = [&](bool backward, auto per_tile) {
        for (int i = tid; i < kSplitBuckets * d; i += 256) cumX[i] = cumX2[i] = 0.0;
        if (tid < kSplitBuckets) count[tid] = 0;
        __syncthreads();
        const int64_t n_tiles = (N + T - 1) / T;
        for (int64_t tile = 0; tile < n_tiles; ++tile) {
            const int64_t p0 = (backward ? n_tiles - 1 - tile : tile) * T;
            const int len = (int)(N - p0 < T ? N - p0 : T);
            // slot s of the tile: position p0 + s going up, p0 + len - 1 - s going down
            // (a thread per slot fetches its row's bucket and its row's d values: both need only the row number)
            if (tid < len) {
                const int64_t p = backward ? p0 + len - 1 - tid : p0 + tid;
                const int32_t r = key_row(keys[p]);
                rows[tid] = r;
                bkt[tid] = node[r];
                const float *src = a.A + (int64_t)r * a.lda + lo;
                float *dst = xt + tid * xld;
                int jj = 0;
                for (; jj + 8 <= d; jj += 8) {
                    float v[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) v[u] = src[jj + u];
#pragma unroll
                    for (int u = 0; u < 8; ++u) dst[jj + u] = v[u];
                }
                for (; jj < d; ++jj) dst[jj] = src[jj];
            }
            __syncthreads();
            // rows of each bucket up to every slot
            if (tid == 0)
                for (int s = 0; s < len; ++s) cnt_at[s] = (int32_t)++count[bkt[s]];
            __syncthreads();
            {
                for (int jj = tid; jj < d; jj += 256)
                    for (int s = 0; s < len; ++s) {
                        const int b = bkt[s];
                        const double x = (double)xt[s * xld + jj];
                        const double cx = cumX[b * d + jj] + x;
                        const double cx2 = cumX2[b * d + jj] + x * x;
                        cumX[b * d + jj] = cx;
                        cumX2[b * d + jj] = cx2;
                        term[s * d + jj] = cx2 - (cx * cx / (double)cnt_at[s]);
                    }
            }
            __syncthreads();
            if (tid < len) {
                double o = 0.0;
                for (int jj = 0; jj < d; ++jj) o = o + term[tid * d + jj];
                sse[tid] = o;
            }
            __syncthreads();
            per_tile(p0, len);
            __syncthreads();
        }
    };

    sweep(false, [&](int64_t p0, int len) {
        if (tid < len) head[p0 + tid] = sse[tid];
    });
    __syncthreads();

    // Going down: the candidates of a bucket are judged in order, the buckets independently of one another - a
    // thread per bucket walks the tile's slots, its bucket's state in registers, and takes the slots of its bucket
    // (selects, no branches).  The values and the forward sums of the tile's positions are fetched by all threads
    // first, so that the walk reads LDS only, eight slots at a time.
    bool r_have_best = false, r_have_up = false;
    double r_best_loss = 0.0, r_up_tail = 0.0;
    float r_best_lo = 0.0f, r_best_hi = 0.0f, r_up_value = 0.0f;
    int32_t r_first_row = 0;
    sweep(true, [&](int64_t p0, int len) {
        if (tid < len) {
            const int64_t p = p0 + len - 1 - tid;
            head_l[tid] = head[p];
            value_l[tid] = key_value(keys[p]);
        }
        __syncthreads();
        if (tid >= n_buckets) return;
        const int b = tid;
        for (int s0 = 0; s0 < len; s0 += 8) {
            int bk[8], rw[8];
            float val[8];
            double hd[8], ss[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const bool in_tile = s0 + u < len;
                const int s = in_tile ? s0 + u : 0;
                bk[u] = in_tile ? bkt[s] : -1;
                val[u] = value_l[s];
                hd[u] = head_l[s];
                ss[u] = sse[s];
                rw[u] = rows[s];
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const bool mine = bk[u] == b;
                const bool cand = mine && r_have_up && val[u] < r_up_value;
                const double loss = hd[u] + r_up_tail;
                const bool better = cand && (!r_have_best || loss <= r_best_loss);
                r_have_best = r_have_best || better;
                r_best_loss = better ? loss : r_best_loss;
                r_best_lo = better ? val[u] : r_best_lo;
                r_best_hi = better ? r_up_value : r_best_hi;
                r_have_up = r_have_up || mine;
                r_up_value = mine ? val[u] : r_up_value;
                r_up_tail = mine ? ss[u] : r_up_tail;
                r_first_row = mine ? rw[u] : r_first_row;
            }
        }
    });
    if (tid < n_buckets) {
        const int b = tid;
        float v = 0.0f;
        double loss = 0.0;
        if (r_have_best) {
            const float l = r_best_lo, h = r_best_hi;
            v = (float)(((double)l + (double)h) / 2.0);
            if (!(v > l)) v = h;
            loss = r_best_loss;
        } else if (r_have_up) {
            // cannot be split: the value of the bucket's first row in sorted order, the loss L(B)
            v = a.A[(int64_t)r_first_row * a.lda + lo + jsplit];
            loss = a.bucket_loss[c * kSplitBuckets + b];
        }
        a.res_v[(c * kCand + q) * kSplitBuckets + b] = v;
        a.res_loss[(c * kCand + q) * kSplitBuckets + b] = loss;
    }
}

// LDS of split_ordered_kernel for subspaces of d columns and tiles of T positions: two [d][T + kOrderedPad]
// arrays of doubles (the two running sums of every (column, place)), the sums carried from tile to tile, and a
// handful of values per place and per bucket
constexpr int kOrderedPad = 17;    // the batches of 8 read up to 16 places past the last; an odd pitch spreads the columns over the banks
__host__ __device__ constexpr size_t split_ordered_lds_bytes(int d, int T)
{
    return sizeof(double) * (2 * (size_t)d * (T + kOrderedPad) + 2 * (size_t)kSplitBuckets * d + 2 * (size_t)T + 7 * kSplitBuckets) +
           sizeof(int32_t) * (5 * (size_t)T + 16 * kSplitBuckets);
}

// Algorithm 3 as split_kernel does it, for subspaces narrow enough that LDS holds both running sums of a whole
// tile; a workgroup per (candidate, codebook) takes all sorted positions, or (by_bucket) a workgroup per
// (candidate, bucket, codebook) the bucket's stretch of them.  The
// positions of a tile are put in the order of their buckets first (a place each: the places of a
// bucket side by side, in the order of the sweep; wavefront ballots give a position's rank among those of its
// bucket), and their values go to LDS by column, as doubles, beside their squares.  Then
//   - a running sum is a walk over neighbouring doubles, in place: a thread per (bucket, column, which of the two
//     sums) reads a value, adds, writes the sum back (a wavefront issues a vector instruction in four cycles and
//     these chains are the one serial part, so they are kept to those three instructions per position);
//   - the product, the division, the difference and the sum over the columns (in column order) go to a thread
//     per place: the same operations on the same operands as in Algorithm 4;
//   - going down, a place's candidate split (between it and the bucket's place before it) needs no chain at all:
//     its loss is head + the tail of the place before, and "a loss that is not larger replaces the best" is the
//     minimum over the candidates, the last of equal ones - a reduction (comparisons only), by wavefront and
//     then across the four wavefronts and the tiles before.
__global__ __launch_bounds__(256) void split_ordered_kernel(const LearnArgs a, int n_buckets, int T, int by_bucket)
{
    extern __shared__ __align__(16) unsigned char lds_raw[];
    const int c = blockIdx.z, q = blockIdx.x, bucket = blockIdx.y;
    if (q >= a.n_cand[c]) return;
    const int lo = a.bounds[2 * c], d = a.bounds[2 * c + 1] - lo;
    const int jsplit = a.cand[c * kCand + q];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t N = a.N;
    const uint64_t *keys = a.keys + ((size_t)c * kCand + q) * a.Npad;
    const uint8_t *node = a.node + (size_t)c * N;
    double *head = a.head + ((size_t)c * kCand + q) * N;

    const int Tp = T + kOrderedPad;
    double *sumX = reinterpret_cast<double *>(lds_raw);      // [d][Tp] x, then its running sum, then Algorithm 4's term
    double *sumX2 = sumX + (size_t)d * Tp;                   // [d][Tp] x^2, then its running sum
    double *cumX = sumX2 + (size_t)d * Tp;                   // [8][d] the sums at the end of the tile before
    double *cumX2 = cumX + (size_t)kSplitBuckets * d;        // [8][d]
    double *sse = cumX2 + (size_t)kSplitBuckets * d;         // [T] by place
    double *head_l = sse + T;                                // [T] by place (going down)
    double *best_loss = head_l + T;                          // [8]
    double *up_tail = best_loss + kSplitBuckets;             // [8]
    double *wave_loss = up_tail + kSplitBuckets;             // [8][4]
    int64_t *count = reinterpret_cast<int64_t *>(wave_loss + 4 * kSplitBuckets);   // [8] rows seen in this sweep
    float *value_l = reinterpret_cast<float *>(count + kSplitBuckets);             // [T] by place
    int32_t *rows_l = reinterpret_cast<int32_t *>(value_l + T);                    // [T] by place
    int32_t *bucket_l = rows_l + T;                                                // [T] by place
    int32_t *cnt_at = bucket_l + T;                                                // [T] by place: rows of the bucket up to it
    int32_t *slot_of = cnt_at + T;                                                 // [T] by place: its slot in the tile
    int32_t *wave_count = slot_of + T;                                             // [8][4]
    int32_t *wave_place = wave_count + 4 * kSplitBuckets;                          // [8][4]
    int32_t *start = wave_place + 4 * kSplitBuckets;                               // [8]
    int32_t *in_tile = start + kSplitBuckets;                                      // [8]
    int32_t *have_best = in_tile + kSplitBuckets, *have_up = have_best + kSplitBuckets;
    int32_t *first_row = have_up + kSplitBuckets;
    float *best_lo = reinterpret_cast<float *>(first_row + kSplitBuckets), *best_hi = best_lo + kSplitBuckets;
    float *up_value = best_hi + kSplitBuckets;

    if (tid < kSplitBuckets) {
        have_best[tid] = have_up[tid] = 0;
        best_loss[tid] = up_tail[tid] = 0.0;
        best_lo[tid] = best_hi[tid] = up_value[tid] = 0.0f;
        first_row[tid] = 0;
    }
    // the positions this workgroup takes: all of them, or (by_bucket: the keys sort by bucket first) its bucket's
    const int64_t first = by_bucket ? a.bucket_start[c * kSplitBuckets + bucket] : 0;
    const int64_t S = by_bucket ? a.bucket_count[c * kSplitBuckets + bucket] : N;
    const int64_t n_tiles = (S + T - 1) / T;
    for (int sweep = 0; sweep < 2; ++sweep) {
        const bool backward = sweep == 1;
        __syncthreads();
        for (int i = tid; i < kSplitBuckets * d; i += 256) cumX[i] = cumX2[i] = 0.0;
        if (tid < kSplitBuckets) count[tid] = 0;
        __syncthreads();
        for (int64_t tile = 0; tile < n_tiles; ++tile) {
            const int64_t p0 = (backward ? n_tiles - 1 - tile : tile) * T;
            const int len = (int)(S - p0 < T ? S - p0 : T);
            // slot s of the tile: the bucket's position p0 + s going up, p0 + len - 1 - s going down; a thread per slot
            int64_t p = 0;
            int32_t r = 0;
            int my_b = -1;
            float my_value = 0.0f;
            if (tid < len) {
                p = first + (backward ? p0 + len - 1 - tid : p0 + tid);
                const uint64_t key = keys[p];
                r = key_row(key);
                my_value = key_value(key);
                my_b = node[r];
            }
            // the slot's rank among the slots of its bucket: within its wavefront from a ballot, the wavefronts
            // before it from their counts
            int rank = 0;
            for (int b = 0; b < n_buckets; ++b) {
                const unsigned long long mask = __ballot(my_b == b);
                if (my_b == b) rank = __popcll(mask & ((1ull << lane) - 1ull));
                if (lane == 0) wave_count[4 * b + wave] = __popcll(mask);
            }
            __syncthreads();
            if (tid < n_buckets) {
                int before = 0;
                for (int b = 0; b < tid; ++b)
                    before += wave_count[4 * b] + wave_count[4 * b + 1] + wave_count[4 * b + 2] + wave_count[4 * b + 3];
                start[tid] = before;
                in_tile[tid] = wave_count[4 * tid] + wave_count[4 * tid + 1] + wave_count[4 * tid + 2] + wave_count[4 * tid + 3];
            }
            int32_t my_cnt = 0;
            if (my_b >= 0) {
                for (int w = 0; w < wave; ++w) rank += wave_count[4 * my_b + w];
                my_cnt = (int32_t)(count[my_b] + rank + 1);
            }
            __syncthreads();
            if (tid < n_buckets) count[tid] += in_tile[tid];       // (read above, before the barrier)
            if (my_b >= 0) {
                const int place = start[my_b] + rank;
                cnt_at[place] = my_cnt;
                bucket_l[place] = my_b;
                rows_l[place] = r;
                slot_of[place] = tid;
                value_l[place] = my_value;
                if (backward) head_l[place] = head[p];
                const float *src = a.A + (int64_t)r * a.lda + lo;
                double *dx = sumX + place, *dx2 = sumX2 + place;
                int jj = 0;
                for (; jj + 8 <= d; jj += 8) {
                    float v[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) v[u] = src[jj + u];
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const double x = (double)v[u];
                        dx[(size_t)(jj + u) * Tp] = x;
                        dx2[(size_t)(jj + u) * Tp] = x * x;
                    }
                }
                for (; jj < d; ++jj) {
                    const double x = (double)src[jj];
                    dx[(size_t)jj * Tp] = x;
                    dx2[(size_t)jj * Tp] = x * x;
                }
            }
            __syncthreads();
            // the running sums, in place
            const int n_chains = n_buckets * d;
            for (int i = tid; i < 2 * n_chains; i += 256) {
                const int which = i >= n_chains ? 1 : 0;
                const int rem = i - which * n_chains;
                const int b = rem / d, jj = rem - b * d;
                double *cum = (which ? cumX2 : cumX) + rem;
                double *at = (which ? sumX2 : sumX) + (size_t)jj * Tp + start[b];
                const int n_here = in_tile[b];
                double acc = *cum;
                // eight places at a time, the eight after them read from LDS meanwhile (the fences keep the compiler
                // from moving the reads back to where their values are used); a batch past the bucket's last place is
                // read (the arrays end in kOrderedPad spare places) and not used
                double v0[8], v1[8];
                auto read = [&](int k, double *v) __attribute__((always_inline)) {
#pragma unroll
                    for (int u = 0; u < 8; ++u) v[u] = at[k + u];
                };
                auto add = [&](int k, const double *v) __attribute__((always_inline)) {
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        acc = acc + v[u];
                        at[k + u] = acc;
                    }
                };
                const int full = n_here & ~15;
                read(0, v0);
                int k = 0;
                for (; k < full; k += 16) {
                    read(k + 8, v1);
                    __builtin_amdgcn_sched_barrier(0);
                    add(k, v0);
                    __builtin_amdgcn_sched_barrier(0);
                    read(k + 16, v0);
                    __builtin_amdgcn_sched_barrier(0);
                    add(k + 8, v1);
                    __builtin_amdgcn_sched_barrier(0);
                }
                if (k < n_here) {
                    read(k + 8, v1);
#pragma unroll
                    for (int u = 0; u < 8; ++u)
                        if (k + u < n_here) {
                            acc = acc + v0[u];
                            at[k + u] = acc;
                        }
#pragma unroll
                    for (int u = 0; u < 8; ++u)
                        if (k + 8 + u < n_here) {
                            acc = acc + v1[u];
                            at[k + 8 + u] = acc;
                        }
                }
                *cum = acc;
            }
            __syncthreads();
            // Algorithm 4's term of every column and their sum, a thread per place
            double my_sse = 0.0;
            if (tid < len) {
                const double n_rows = (double)cnt_at[tid];
                for (int jj = 0; jj < d; ++jj) {
                    const double cx = sumX[(size_t)jj * Tp + tid];
                    my_sse = my_sse + (sumX2[(size_t)jj * Tp + tid] - (cx * cx / n_rows));
                }
                sse[tid] = my_sse;
                if (!backward) head[first + p0 + slot_of[tid]] = my_sse;
            }
            if (backward) {
                __syncthreads();
                // the candidate of every place, and the best of each bucket's candidates in this wavefront
                bool cand = false;
                double loss = 0.0;
                int b_here = -1;
                if (tid < len) {
                    b_here = bucket_l[tid];
                    const bool first_here = tid == start[b_here];
                    const bool have = first_here ? have_up[b_here] != 0 : true;
                    const float before_value = first_here ? up_value[b_here] : value_l[tid - 1];
                    const double before_tail = first_here ? up_tail[b_here] : sse[tid - 1];
                    cand = have && value_l[tid] < before_value;
                    loss = head_l[tid] + before_tail;
                }
                const int wave_first = 64 * wave, wave_end = min(len, 64 * wave + 64);
                for (int b = 0; b < n_buckets; ++b) {
                    if (lane == 0) wave_place[4 * b + wave] = -1;
                    if (in_tile[b] == 0 || start[b] >= wave_end || start[b] + in_tile[b] <= wave_first) continue;
                    double l = loss;
                    int pl = (cand && b_here == b) ? tid : -1;
#pragma unroll
                    for (int off = 1; off < 64; off <<= 1) {
                        const double l2 = __shfl_xor(l, off);
                        const int pl2 = __shfl_xor(pl, off);
                        const bool take = pl2 >= 0 && (pl < 0 || l2 < l || (l2 == l && pl2 > pl));
                        l = take ? l2 : l;
                        pl = take ? pl2 : pl;
                    }
                    if (lane == 0) {
                        wave_place[4 * b + wave] = pl;
                        wave_loss[4 * b + wave] = l;
                    }
                }
                __syncthreads();
                if (tid < n_buckets && in_tile[tid] > 0) {
                    const int b = tid;
                    int pl = -1;
                    double l = 0.0;
                    for (int w = 0; w < 4; ++w) {
                        const int pl2 = wave_place[4 * b + w];
                        if (pl2 >= 0 && (pl < 0 || wave_loss[4 * b + w] <= l)) {
                            pl = pl2;
                            l = wave_loss[4 * b + w];
                        }
                    }
                    if (pl >= 0 && (!have_best[b] || l <= best_loss[b])) {
                        have_best[b] = 1;
                        best_loss[b] = l;
                        best_lo[b] = value_l[pl];
                        best_hi[b] = pl == start[b] ? up_value[b] : value_l[pl - 1];
                    }
                    const int last = start[b] + in_tile[b] - 1;
                    have_up[b] = 1;
                    up_value[b] = value_l[last];
                    up_tail[b] = sse[last];
                    first_row[b] = rows_l[last];
                }
            }
            __syncthreads();
        }
    }
    if (by_bucket ? tid == bucket : tid < n_buckets) {
        const int b = tid;
        float v = 0.0f;
        double loss = 0.0;
        if (have_best[b]) {
            const float l = best_lo[b], h = best_hi[b];
            v = (float)(((double)l + (double)h) / 2.0);
            if (!(v > l)) v = h;
            loss = best_loss[b];
        } else if (have_up[b]) {
            // cannot be split: the value of the bucket's first row in sorted order, the loss L(B)
            v = a.A[(int64_t)first_row[b] * a.lda + lo + jsplit];
            loss = a.bucket_loss[c * kSplitBuckets + b];
        }
        a.res_v[(c * kCand + q) * kSplitBuckets + b] = v;
        a.res_loss[(c * kCand + q) * kSplitBuckets + b] = loss;
    }
}

// Algorithm 2's choice: the candidate with the smallest loss summed over the buckets (the
// first of equal ones), its thresholds into the tree.
__global__ void choose_kernel(const LearnArgs a, int level, int n_buckets)
{
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= a.C) return;
    int best_q = 0;
    double l_min = 0.0;
    for (int q = 0; q < a.n_cand[c]; ++q) {
        double l = 0.0;
        for (int b = 0; b < n_buckets; ++b) l += a.res_loss[(c * kCand + q) * kSplitBuckets + b];
        if (q == 0 || l < l_min) {
            l_min = l;
            best_q = q;
        }
    }
    const int jj = a.cand[c * kCand + best_q];
    a.chosen[c] = jj;
    a.split_dims[4 * c + level] = a.bounds[2 * c] + jj;
    for (int b = 0; b < n_buckets; ++b)
        a.thresholds[16 * c + n_buckets - 1 + b] = a.res_v[(c * kCand + best_q) * kSplitBuckets + b];
    if (level == 3) a.thresholds[16 * c + 15] = 0.0f;
}

// apply_split: below the threshold stays left (2 i), the rest goes right (2 i + 1).
__global__ __launch_bounds__(256) void apply_kernel(const LearnArgs a, int level, int n_buckets)
{
    const int c = blockIdx.y;
    const int64_t n = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (n >= a.N) return;
    const int j = a.bounds[2 * c] + a.chosen[c];
    const int b = a.node[(size_t)c * a.N + n];
    const float v = a.thresholds[16 * c + n_buckets - 1 + b];
    const int child = 2 * b + (a.A[n * a.lda + j] >= v ? 1 : 0);
    a.node[(size_t)c * a.N + n] = (uint8_t)child;
    if (level == 3 && a.codes) a.codes[n * a.C + c] = (uint8_t)child;
}

// ---------------------------------------------------------------------------------------
// prototypes
// ---------------------------------------------------------------------------------------

struct ProtoArgs {
    const uint8_t *codes;   // [N][C]
    const float *A;
    int64_t lda, N;
    int32_t D, C, Q;        // Q = 16 C
    int32_t *bounds;
    int32_t *counts;        // [Q][Q] G^T G
    double *M;              // [Q][Q]: G^T G + lambda I, then M[k][i] = L[i][k]
    double *Lr;             // [Q][Q]: L by rows
    double *R;              // [Q][D]: G^T A~, then y, then P
    float *P;               // out [C][16][D]
};

// G^T G: entry (q, q') counts the training rows whose one-hot row has ones at q and q'.  A workgroup takes
// codebook c against kCoGroup codebooks c2 and counts in LDS (16 x 16 counters a pair), then stores its
// 16 x (16 kCoGroup) block of the matrix: no two workgroups share an entry.
constexpr int kCoGroup = 8;
__global__ __launch_bounds__(256) void cooccurrence_kernel(const ProtoArgs a)
{
    __shared__ int32_t hist[kCoGroup][256];
    const int c = blockIdx.x, c2_first = blockIdx.y * kCoGroup, tid = threadIdx.x;
    const int n_c2 = min(kCoGroup, a.C - c2_first);
    for (int i = tid; i < kCoGroup * 256; i += 256) (&hist[0][0])[i] = 0;
    __syncthreads();
    for (int64_t n = tid; n < a.N; n += 256) {
        const uint8_t *row = a.codes + n * a.C;
        const int k = row[c] & 15;
        uint8_t k2[kCoGroup];
#pragma unroll
        for (int g = 0; g < kCoGroup; ++g) k2[g] = g < n_c2 ? row[c2_first + g] : 0;
#pragma unroll
        for (int g = 0; g < kCoGroup; ++g)
            if (g < n_c2) atomicAdd(&hist[g][16 * k + (k2[g] & 15)], 1);
    }
    __syncthreads();
    for (int i = tid; i < n_c2 * 256; i += 256) {
        const int g = i >> 8, k = (i >> 4) & 15, k2 = i & 15;
        a.counts[(size_t)(16 * c + k) * a.Q + 16 * (c2_first + g) + k2] = hist[g][16 * k + k2];
    }
}

__global__ __launch_bounds__(256) void ridge_matrix_kernel(const ProtoArgs a, double lambda)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= (int64_t)a.Q * a.Q) return;
    const int r = (int)(i / a.Q), col = (int)(i - (int64_t)r * a.Q);
    a.M[i] = (double)a.counts[i] + (r == col ? lambda : 0.0);
}

// G^T A~: row 16 c + k = the sum, in row order, of the training rows with code k in codebook c.
// A thread per (codebook, column); the four wavefronts of a workgroup take four codebooks over
// the same 64 columns, and the values and codes of kGtaAhead rows are fetched before they are added.
constexpr int kGtaAhead = 16;
__global__ __launch_bounds__(256) void gta_kernel(const ProtoArgs a)
{
    __shared__ double acc[4][16][64];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int c = blockIdx.y * 4 + wave;
    const int col = blockIdx.x * 64 + lane;
    if (c >= a.C || col >= a.D) return;      // no barrier below: every thread works on its own sums
    double(*mine)[64] = acc[wave];
    for (int k = 0; k < 16; ++k) mine[k][lane] = 0.0;
    const float *src = a.A + col;
    const uint8_t *code = a.codes + c;
    int64_t n = 0;
    for (; n + kGtaAhead <= a.N; n += kGtaAhead) {
        float v[kGtaAhead];
        int k[kGtaAhead];
#pragma unroll
        for (int u = 0; u < kGtaAhead; ++u) {
            v[u] = src[(n + u) * a.lda];
            k[u] = code[(n + u) * a.C];
        }
#pragma unroll
        for (int u = 0; u < kGtaAhead; ++u) mine[k[u] & 15][lane] += (double)v[u];
    }
    for (; n < a.N; ++n) mine[code[n * a.C] & 15][lane] += (double)src[n * a.lda];
    for (int k = 0; k < 16; ++k) a.R[((size_t)16 * c + k) * a.D + col] = mine[k][lane];
}

// G^T A~ for problems with few (codebook, column) pairs, where gta_kernel would leave the chip empty and wait
// for its LDS sums row after row: a thread per (codebook, code, column) with its one sum in a register; a row
// with another code adds 0.0, which leaves the sum as it is.
__global__ __launch_bounds__(64) void gta_by_code_kernel(const ProtoArgs a)
{
    const int c = blockIdx.z, k = blockIdx.y;
    const int col = blockIdx.x * 64 + threadIdx.x;
    if (col >= a.D) return;
    const float *src = a.A + col;
    const uint8_t *code = a.codes + c;
    double sum = 0.0;
    int64_t n = 0;
    for (; n + kGtaAhead <= a.N; n += kGtaAhead) {
        float v[kGtaAhead];
        int at[kGtaAhead];
#pragma unroll
        for (int u = 0; u < kGtaAhead; ++u) {
            v[u] = src[(n + u) * a.lda];
            at[u] = code[(n + u) * a.C];
        }
#pragma unroll
        for (int u = 0; u < kGtaAhead; ++u) {
            float x = (at[u] & 15) == k ? v[u] : 0.0f;
            asm volatile("" : "+v"(x));      // (the selection stays one 32-bit move, before the conversion)
            sum += (double)x;
        }
    }
    for (; n < a.N; ++n) sum += (double)((code[n * a.C] & 15) == k ? src[n * a.lda] : 0.0f);
    a.R[((size_t)16 * c + k) * a.D + col] = sum;
}

// Cholesky factorisation M = L L^T: L_jj = sqrt(M_jj - sum_k L_jk^2), L_ij = (M_ij - sum_k L_ik L_jk) / L_jj,
// every sum over k ascending.  M is symmetric, and L_ik is kept at M[k][i] (rows of a column side by side).
// One launch per panel of 16 columns J0 .. J0 + 15; a workgroup takes the 16 rows of the panel's
// diagonal block (every workgroup works them out for itself, the first one stores them) and 48 rows
// below it, four entries of a row per thread.  First the terms of the columns before the panel, in
// chunks of kCholChunk columns staged in LDS, then the panel's own columns one after the other.
constexpr int kCholPanel = 16, kCholRows = 64, kCholChunk = 32;
__global__ __launch_bounds__(256) void cholesky_panel_kernel(const ProtoArgs a, int J0)
{
    __shared__ __align__(16) double Lc[kCholRows][kCholChunk + 2];     // (rows 4 banks apart: 16-byte reads of 16 rows at once)
    __shared__ double T[kCholRows][kCholPanel + 1];
    const int Q = a.Q;
    double *M = a.M;
    const int tid = threadIdx.x;
    auto global_row = [&](int r) {
        return r < kCholPanel ? J0 + r : J0 + kCholPanel + (int)blockIdx.x * (kCholRows - kCholPanel) + (r - kCholPanel);
    };
    const int r = tid >> 2, cg = tid & 3;
    const int gi = global_row(r);
    double s[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) s[e] = gi < Q ? M[(size_t)(J0 + 4 * cg + e) * Q + gi] : 0.0;

    // staging: thread -> row (tid & 63) of the chunk, columns (tid >> 6) + 4 u
    const int srow = tid & 63, sk = tid >> 6;
    const int sgi = global_row(srow);
    constexpr int kPer = kCholChunk / 4;
    double pre[kPer];
    auto fetch = [&](int k0) {
#pragma unroll
        for (int u = 0; u < kPer; ++u) {
            const int k = k0 + sk + 4 * u;
            pre[u] = (sgi < Q && k < J0) ? M[(size_t)k * Q + sgi] : 0.0;
        }
    };
    if (J0 > 0) fetch(0);
    for (int k0 = 0; k0 < J0; k0 += kCholChunk) {
        __syncthreads();                      // the chunk before this one has been used
#pragma unroll
        for (int u = 0; u < kPer; ++u) Lc[srow][sk + 4 * u] = pre[u];
        __syncthreads();
        if (k0 + kCholChunk < J0) fetch(k0 + kCholChunk);
        const int kc = min(kCholChunk, J0 - k0);
        for (int kk = 0; kk < kc; kk += 2) {          // (two columns to an LDS read; kc is a multiple of 16)
            const double2 li = *reinterpret_cast<const double2 *>(&Lc[r][kk]);
            double2 lj[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) lj[e] = *reinterpret_cast<const double2 *>(&Lc[4 * cg + e][kk]);
#pragma unroll
            for (int e = 0; e < 4; ++e) s[e] -= li.x * lj[e].x;
#pragma unroll
            for (int e = 0; e < 4; ++e) s[e] -= li.y * lj[e].y;
        }
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) T[r][4 * cg + e] = s[e];
    __syncthreads();

    // the panel's own columns: a thread per row (the first wavefront), the row's entries in registers
    double t[kCholPanel];
    const int row = tid, grow = global_row(tid < kCholRows ? tid : 0);
    if (tid < kCholRows)
#pragma unroll
        for (int j = 0; j < kCholPanel; ++j) t[j] = T[row][j];
#pragma unroll
    for (int j = 0; j < kCholPanel; ++j) {
        if (tid < kCholRows) {
#pragma unroll
            for (int k = 0; k < j; ++k) t[j] -= t[k] * T[j][k];
            if (row == j) {
                t[j] = sqrt(t[j]);
                T[j][j] = t[j];
            }
        }
        __syncthreads();
        if (tid < kCholRows && row != j) {
            t[j] = t[j] / T[j][j];
            if (row < kCholPanel) T[row][j] = t[j];     // a row of the diagonal block: read by the rows below
        }
        __syncthreads();
    }
    if (tid < kCholRows && grow < Q && (row >= kCholPanel || blockIdx.x == 0))
#pragma unroll
        for (int j = 0; j < kCholPanel; ++j)
            if (row >= kCholPanel || j <= row) M[(size_t)(J0 + j) * Q + grow] = t[j];
}

__global__ __launch_bounds__(256) void transpose_factor_kernel(const ProtoArgs a)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= (int64_t)a.Q * a.Q) return;
    const int r = (int)(i / a.Q), k = (int)(i - (int64_t)r * a.Q);
    a.Lr[i] = k <= r ? a.M[(size_t)k * a.Q + r] : 0.0;
}

// L y = G^T A~ and L^T P = y, sums over k ascending: y_i = (b_i - sum_{k<i} L_ik y_k) / L_ii, then
// P_i = (y_i - sum_{k>i} L_ki P_k) / L_ii.  A workgroup takes NC columns of A~ and keeps them in LDS
// for both sweeps; the first NC threads carry a column each through the sums (in the second sweep the
// sum of a row begins with the value found just before, so a column's subtractions are one chain),
// while all threads fetch the next row of L (first sweep) or of L^T (second sweep, kept at M) through
// registers into the other of two LDS buffers.  A wavefront issues one vector instruction in four
// cycles, so the chain's loop is kept to the two LDS reads, the product and the subtraction of a term:
// NC is a constant (the reads take immediate offsets) and terms go in batches of kSubBatch without a
// bound check.  A batch may run past the row's last term: there the buffer's entry of L is 0 (buffers
// start as zeros, a row's diagonal entry is kept apart, and kSubPad entries and rows follow the last),
// the term is 0 times a finite value, and subtracting 0 changes nothing.
constexpr int kSubMaxPer = MADDNESS_MAX_C * 16 / 256;     // most values of a row a thread fetches
constexpr int kSubBatch = 8;
constexpr int kSubPad = 5 * kSubBatch;                    // the reads run up to five batches past a row's last term
size_t substitution_lds_bytes(int Q, int nc) { return sizeof(double) * ((size_t)(Q + kSubPad) * nc + 2 * (size_t)(Q + kSubPad + 1)); }

template <int NC>
__global__ __launch_bounds__(256) void substitution_kernel(const ProtoArgs a)
{
    extern __shared__ __align__(16) unsigned char lds_raw[];
    const int Q = a.Q, D = a.D, tid = threadIdx.x;
    const int Qp = Q + kSubPad;
    double *X = reinterpret_cast<double *>(lds_raw);      // [Qp][NC]
    double *rows = X + (size_t)Qp * NC;                   // [2][Qp + 1]: a row of the factor, its diagonal entry last
    const int col0 = blockIdx.x * NC;
    const int ncols = min(NC, D - col0);
    for (int idx = tid; idx < Qp * NC; idx += 256) {
        const int i = idx / NC, cc = idx % NC;
        X[idx] = (i < Q && cc < ncols) ? a.R[(size_t)i * D + col0 + cc] : 0.0;
    }
    for (int idx = tid; idx < 2 * (Qp + 1); idx += 256) rows[idx] = 0.0;
    __syncthreads();
    // step s < Q: row i = s of L, entries 0..i; step s >= Q: row i = 2Q - 1 - s of L^T, entries i..Q-1
    const int n_steps = 2 * Q;
    const int per = (Q + 255) / 256;
    double ahead[kSubMaxPer];
    auto fetch = [&](int s) {
        if (s >= n_steps) return;
        const bool fwd = s < Q;
        const int i = fwd ? s : 2 * Q - 1 - s;
        const double *src = (fwd ? a.Lr : a.M) + (size_t)i * Q;
        const int lo = fwd ? 0 : i, hi = fwd ? i + 1 : Q;
#pragma unroll
        for (int u = 0; u < kSubMaxPer; ++u) {
            const int k = lo + tid + 256 * u;
            if (u < per && k < hi) ahead[u] = src[k];
        }
    };
    auto stash = [&](int s) {
        if (s >= n_steps) return;
        const bool fwd = s < Q;
        const int i = fwd ? s : 2 * Q - 1 - s;
        const int lo = fwd ? 0 : i, hi = fwd ? i + 1 : Q;
        double *dst = rows + (size_t)(s & 1) * (Qp + 1);
#pragma unroll
        for (int u = 0; u < kSubMaxPer; ++u) {
            const int k = lo + tid + 256 * u;
            if (u < per && k < hi) {
                dst[k] = k == i ? 0.0 : ahead[u];
                if (k == i) dst[Qp] = ahead[u];
            }
        }
    };
    fetch(0);
    stash(0);
    __syncthreads();
    for (int s = 0; s < n_steps; ++s) {
        fetch(s + 1);
        if (tid < NC) {
            const bool fwd = s < Q;
            const int i = fwd ? s : 2 * Q - 1 - s;
            const double *Li = rows + (size_t)(s & 1) * (Qp + 1);
            const int lo = fwd ? 0 : i + 1, hi = fwd ? i : Q;
            double v = X[(size_t)i * NC + tid];
            const double *pl = Li + lo, *px = X + (size_t)lo * NC + tid;
            double l0[kSubBatch], x0[kSubBatch], l1[kSubBatch], x1[kSubBatch], l2[kSubBatch], x2[kSubBatch];
            auto read = [&](int at, double *l, double *x) {
#pragma unroll
                for (int u = 0; u < kSubBatch; ++u) {
                    l[u] = pl[at + u];
                    x[u] = px[(at + u) * NC];
                }
            };
            auto subtract = [&](const double *l, const double *x) {
#pragma unroll
                for (int u = 0; u < kSubBatch; ++u) v -= l[u] * x[u];
            };
            read(0, l0, x0);
            read(kSubBatch, l1, x1);
            for (int k = lo; k < hi; k += 3 * kSubBatch) {
                // (the fences keep the compiler from gathering the reads of several batches in one place)
                read(2 * kSubBatch, l2, x2);
                __builtin_amdgcn_sched_barrier(0);
                subtract(l0, x0);
                __builtin_amdgcn_sched_barrier(0);
                read(3 * kSubBatch, l0, x0);
                __builtin_amdgcn_sched_barrier(0);
                subtract(l1, x1);
                __builtin_amdgcn_sched_barrier(0);
                read(4 * kSubBatch, l1, x1);
                __builtin_amdgcn_sched_barrier(0);
                subtract(l2, x2);
                __builtin_amdgcn_sched_barrier(0);
                pl += 3 * kSubBatch;
                px += 3 * kSubBatch * NC;
            }
            X[(size_t)i * NC + tid] = v / Li[Qp];
        }
        stash(s + 1);
        __syncthreads();
    }
    for (int idx = tid; idx < Q * NC; idx += 256) {
        const int i = idx / NC, cc = idx % NC;
        if (cc < ncols) a.P[(size_t)i * D + col0 + cc] = (float)X[idx];
    }
}

template <int NC>
int launch_substitution(const ProtoArgs &a, hipStream_t stream)
{
    if (int rc = allow_full_lds<substitution_kernel<NC>>(); rc != MADDNESS_OK) return rc;
    hipLaunchKernelGGL(substitution_kernel<NC>, dim3((a.D + NC - 1) / NC), dim3(256), substitution_lds_bytes(a.Q, NC), stream, a);
    return MADDNESS_OK;
}

// The substitutions with the products taken out of the chain.  While the first wavefront carries its columns
// through the sum of row i, the other three form the products L_i'k x_k of the NEXT row i' for every k whose x_k
// is known by then (all but the one the chain is just working out) and leave them in LDS; the chain of row i'
// then only reads a product and subtracts it, and forms the one missing product itself - the last term going
// forward, the first going back, so that the terms keep their order.  Same products, same subtractions, a chain
// of half the instructions.  LDS holds the columns, two sets of products and three rows of the factor, so a
// workgroup takes fewer columns than substitution_kernel does; factors too large for that stay with it.
constexpr int kSubHelpers = 192;
constexpr int kSubMaxPerHelper = (MADDNESS_MAX_C * 16 + kSubHelpers - 1) / kSubHelpers;
size_t substitution_products_lds_bytes(int Q, int nc)
{
    return sizeof(double) * (3 * (size_t)(Q + kSubPad) * nc + 3 * (size_t)(Q + kSubPad + 1));
}

template <int NC>
__global__ __launch_bounds__(256) void substitution_products_kernel(const ProtoArgs a)
{
    extern __shared__ __align__(16) unsigned char lds_raw[];
    const int Q = a.Q, D = a.D, tid = threadIdx.x;
    const int Qp = Q + kSubPad;
    double *X = reinterpret_cast<double *>(lds_raw);      // [Qp][NC]
    double *P = X + (size_t)Qp * NC;                      // [2][Qp][NC] products of the row of step s in P[s & 1]
    double *rows = P + 2 * (size_t)Qp * NC;               // [3][Qp + 1] the row of step s in rows[s % 3], its diagonal entry last
    const int col0 = blockIdx.x * NC;
    const int ncols = min(NC, D - col0);
    for (int idx = tid; idx < Qp * NC; idx += 256) {
        const int i = idx / NC, cc = idx % NC;
        X[idx] = (i < Q && cc < ncols) ? a.R[(size_t)i * D + col0 + cc] : 0.0;
    }
    for (int idx = tid; idx < 2 * Qp * NC + 3 * (Qp + 1); idx += 256) P[idx] = 0.0;     // (products and rows)
    __syncthreads();
    // step s < Q: row i = s of L, entries 0..i; step s >= Q: row i = 2Q - 1 - s of L^T, entries i..Q-1
    const int n_steps = 2 * Q;
    const int ht = tid - 64;                              // helper number (the threads of the other three wavefronts)
    const int per = (Q + kSubHelpers - 1) / kSubHelpers;
    double ahead[kSubMaxPerHelper];
    auto fetch = [&](int s) __attribute__((always_inline)) {
        if (s >= n_steps || ht < 0) return;
        const bool fwd = s < Q;
        const int i = fwd ? s : 2 * Q - 1 - s;
        const double *src = (fwd ? a.Lr : a.M) + (size_t)i * Q;
        const int lo = fwd ? 0 : i, hi = fwd ? i + 1 : Q;
#pragma unroll
        for (int u = 0; u < kSubMaxPerHelper; ++u) {
            const int k = lo + ht + kSubHelpers * u;
            if (u < per && k < hi) ahead[u] = src[k];
        }
    };
    auto stash = [&](int s) __attribute__((always_inline)) {
        if (s >= n_steps || ht < 0) return;
        const bool fwd = s < Q;
        const int i = fwd ? s : 2 * Q - 1 - s;
        const int lo = fwd ? 0 : i, hi = fwd ? i + 1 : Q;
        double *dst = rows + (size_t)(s % 3) * (Qp + 1);
#pragma unroll
        for (int u = 0; u < kSubMaxPerHelper; ++u) {
            const int k = lo + ht + kSubHelpers * u;
            if (u < per && k < hi) {
                dst[k] = ahead[u];
                if (k == i) dst[Qp] = ahead[u];
            }
        }
    };
    // the products of the row of step s, for every k but the one next to the diagonal; zeros after the last
    // (going forward; going back the places after Q - 1 are never written and stay zero)
    auto products = [&](int s) __attribute__((always_inline)) {
        if (s >= n_steps || ht < 0) return;
        const bool fwd = s < Q;
        const int i = fwd ? s : 2 * Q - 1 - s;
        const double *Li = rows + (size_t)(s % 3) * (Qp + 1);
        double *dst = P + (size_t)(s & 1) * Qp * NC;
        const int k_first = fwd ? 0 : i + 2, k_end = fwd ? max(i - 1, 0) : Q;      // [k_first, k_end)
        int idx = k_first * NC + ht;
        const int idx_end = k_end * NC;
        for (; idx + 3 * kSubHelpers < idx_end; idx += 4 * kSubHelpers) {
            double l[4], x[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                l[u] = Li[(idx + u * kSubHelpers) / NC];
                x[u] = X[idx + u * kSubHelpers];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) dst[idx + u * kSubHelpers] = l[u] * x[u];
        }
        for (; idx < idx_end; idx += kSubHelpers) dst[idx] = Li[idx / NC] * X[idx];
        if (fwd)
            for (int z = k_end * NC + ht; z < (k_end + 2 * kSubBatch) * NC; z += kSubHelpers) dst[z] = 0.0;
    };
    fetch(0);
    stash(0);
    fetch(1);
    stash(1);
    __syncthreads();
    for (int s = 0; s < n_steps; ++s) {
        fetch(s + 2);
        if (tid < NC) {
            const bool fwd = s < Q;
            const int i = fwd ? s : 2 * Q - 1 - s;
            const double *Li = rows + (size_t)(s % 3) * (Qp + 1);
            const int lo = fwd ? 0 : i + 2, hi = fwd ? i - 1 : Q;       // the terms whose products are in P
            double v = X[(size_t)i * NC + tid];
            if (!fwd && i + 1 < Q) v -= Li[i + 1] * X[(size_t)(i + 1) * NC + tid];
            const double *pp = P + (size_t)(s & 1) * Qp * NC + (size_t)lo * NC + tid;
            double p0[kSubBatch], p1[kSubBatch], p2[kSubBatch];
            auto read = [&](int at, double *t) __attribute__((always_inline)) {
#pragma unroll
                for (int u = 0; u < kSubBatch; ++u) t[u] = pp[(at + u) * NC];
            };
            auto subtract = [&](const double *t) __attribute__((always_inline)) {
#pragma unroll
                for (int u = 0; u < kSubBatch; ++u) v -= t[u];
            };
            read(0, p0);
            read(kSubBatch, p1);
            for (int k = lo; k < hi; k += 3 * kSubBatch) {
                // (the fences keep the compiler from gathering the reads of several batches in one place; a batch
                // past the last term subtracts zeros, or is read and not used)
                read(2 * kSubBatch, p2);
                __builtin_amdgcn_sched_barrier(0);
                subtract(p0);
                __builtin_amdgcn_sched_barrier(0);
                read(3 * kSubBatch, p0);
                __builtin_amdgcn_sched_barrier(0);
                if (k + kSubBatch < hi) subtract(p1);
                __builtin_amdgcn_sched_barrier(0);
                read(4 * kSubBatch, p1);
                __builtin_amdgcn_sched_barrier(0);
                if (k + 2 * kSubBatch < hi) subtract(p2);
                __builtin_amdgcn_sched_barrier(0);
                pp += 3 * kSubBatch * NC;
            }
            if (fwd && i >= 1) v -= Li[i - 1] * X[(size_t)(i - 1) * NC + tid];
            X[(size_t)i * NC + tid] = v / Li[Qp];
        } else {
            products(s + 1);
        }
        stash(s + 2);
        __syncthreads();
    }
    for (int idx = tid; idx < Q * NC; idx += 256) {
        const int i = idx / NC, cc = idx % NC;
        if (cc < ncols) a.P[(size_t)i * D + col0 + cc] = (float)X[idx];
    }
}

template <int NC>
int launch_substitution_products(const ProtoArgs &a, hipStream_t stream)
{
    if (int rc = allow_full_lds<substitution_products_kernel<NC>>(); rc != MADDNESS_OK) return rc;
    hipLaunchKernelGGL(substitution_products_kernel<NC>, dim3((a.D + NC - 1) / NC), dim3(256),
                       substitution_products_lds_bytes(a.Q, NC), stream, a);
    return MADDNESS_OK;
}

// Bucket means on the codebook's own columns, 0 elsewhere and for an empty bucket.
__global__ __launch_bounds__(64) void means_kernel(const ProtoArgs a)
{
    const int c = blockIdx.z, k = blockIdx.y;
    const int col = blockIdx.x * 64 + threadIdx.x;
    if (col >= a.D) return;
    float out = 0.0f;
    if (col >= a.bounds[2 * c] && col < a.bounds[2 * c + 1]) {
        double sum = 0.0;
        int64_t count = 0;
        for (int64_t n = 0; n < a.N; ++n)
            if (a.codes[n * a.C + c] == k) {
                sum += (double)a.A[n * a.lda + col];
                ++count;
            }
        if (count > 0) out = (float)(sum / (double)count);
    }
    a.P[((size_t)c * 16 + k) * a.D + col] = out;
}

size_t align_up(size_t v, size_t al) { return (v + al - 1) / al * al; }

int64_t pow2_at_least(int64_t n)
{
    int64_t p = 1;
    while (p < n) p <<= 1;
    return p;
}

// carves `bytes` (rounded up to 256) off the workspace
struct Carver {
    unsigned char *at;
    size_t used = 0;
    template <typename T>
    T *take(size_t count)
    {
        T *p = reinterpret_cast<T *>(at + used);
        used += align_up(count * sizeof(T), 256);
        return p;
    }
};

size_t split_lds_bytes(int d)
{
    return split_lds_bytes_base(d, kSplitTile);
}

void carve_trees(Carver &w, LearnArgs &a)
{
    const size_t C = a.C;
    a.bounds = w.take<int32_t>(2 * C);
    a.node = w.take<uint8_t>(C * a.N);
    a.col_loss = w.take<double>(C * kSplitBuckets * a.dmax);
    a.bucket_loss = w.take<double>(C * kSplitBuckets);
    a.bucket_count = w.take<int64_t>(C * kSplitBuckets);
    a.bucket_start = w.take<int32_t>(C * kSplitBuckets);
    a.rows_by_bucket = w.take<int32_t>(C * a.N);
    a.cand = w.take<int32_t>(C * kCand);
    a.n_cand = w.take<int32_t>(C);
    a.keys = w.take<uint64_t>(C * kCand * a.Npad);
    a.head = w.take<double>(C * kCand * a.N);
    a.res_loss = w.take<double>(C * kCand * kSplitBuckets);
    a.res_v = w.take<float>(C * kCand * kSplitBuckets);
    a.chosen = w.take<int32_t>(C);
}

void carve_prototypes(Carver &w, ProtoArgs &a)
{
    const size_t Q = a.Q;
    a.bounds = w.take<int32_t>(2 * (size_t)a.C);
    a.counts = w.take<int32_t>(Q * Q);
    a.M = w.take<double>(Q * Q);
    a.Lr = w.take<double>(Q * Q);
    a.R = w.take<double>(Q * a.D);
}

}  // namespace

size_t learn_trees_workspace_bytes(int64_t N, int32_t C, int32_t dmax)
{
    LearnArgs a{};
    a.N = N; a.Npad = pow2_at_least(N); a.C = C; a.dmax = dmax;
    Carver w{nullptr};
    carve_trees(w, a);
    return w.used;
}

size_t learn_prototypes_workspace_bytes(int32_t D, int32_t C)
{
    ProtoArgs a{};
    a.D = D; a.C = C; a.Q = 16 * C;
    Carver w{nullptr};
    carve_prototypes(w, a);
    return w.used;
}

int learn_max_subspace_width()
{
    // the running sums of split_kernel (one column per thread slot) must fit in LDS
    int d = 1;
    while (2 * d <= kLossMaxWidth && split_lds_bytes(2 * d) + 1024 <= (size_t)device_info().lds_per_block) d *= 2;
    return d;
}

#define LAUNCH_OK(what)                                                       \
    if (int rc_ = check_hip(hipGetLastError(), what); rc_ != MADDNESS_OK) return rc_

int launch_learn_trees(const float *A, int64_t N, int64_t lda, int32_t C, const int32_t *bounds_host, int32_t dmax,
                       int32_t *split_dims, float *thresholds, uint8_t *codes, void *workspace, hipStream_t stream)
{
    LearnArgs a{};
    a.A = A; a.lda = lda; a.N = N; a.Npad = pow2_at_least(N); a.C = C; a.dmax = dmax;
    a.split_dims = split_dims; a.thresholds = thresholds; a.codes = codes;
    Carver w{static_cast<unsigned char *>(workspace)};
    carve_trees(w, a);
    note_kernel("order_rows_kernel + bucket_loss_kernel + select_kernel + key_kernel + sort_chunks_kernel + sort_exchange_kernel + split_ordered_kernel + choose_kernel + apply_kernel", nullptr);

    Bounds b{};
    for (int i = 0; i < 2 * C; ++i) b.v[i] = bounds_host[i];
    hipLaunchKernelGGL(upload_bounds_kernel, dim3(1), dim3(256), 0, stream, b, 2 * C, a.bounds);
    LAUNCH_OK("launch upload_bounds_kernel");
    const int64_t node_bytes = (int64_t)C * N;
    hipLaunchKernelGGL(fill_bytes_kernel, dim3((unsigned)((node_bytes + 255) / 256)), dim3(256), 0, stream, a.node, node_bytes,
                       (uint8_t)0);
    LAUNCH_OK("launch fill_bytes_kernel");

    const size_t sort_lds = sizeof(uint64_t) * (size_t)(a.Npad < kSortChunk ? a.Npad : kSortChunk);
    // subspaces narrow enough for split_ordered_kernel take it, with the largest tile that fits (a tile costs a
    // fixed chain of barriers and memory latencies, whatever its size); wider ones take split_kernel
    const size_t lds_max = (size_t)device_info().lds_per_block - 1024;
    const bool ordered = split_ordered_lds_bytes(dmax, 64) <= lds_max;
    int tile = 64;
    if (ordered)
        while (2 * tile <= kMaxTile && split_ordered_lds_bytes(dmax, 2 * tile) <= lds_max) tile *= 2;
    const size_t split_lds = ordered ? split_ordered_lds_bytes(dmax, tile) : split_lds_bytes(dmax);
    if (int rc = allow_full_lds<split_ordered_kernel>(); rc != MADDNESS_OK) return rc;
    // With few (candidate, codebook) pairs a workgroup per bucket as well fills more of the chip: the keys then
    // sort by bucket first and every workgroup takes its bucket's stretch.  With many pairs the chip is full
    // anyway, and a tile that mixes the buckets has its running sums on more lanes, each over fewer positions.
    const int by_bucket = ordered && 4 * kCand * C <= device_info().cus ? 1 : 0;
    if (int rc = allow_full_lds<bucket_loss_kernel>(); rc != MADDNESS_OK) return rc;
    if (int rc = allow_full_lds<sort_chunks_kernel>(); rc != MADDNESS_OK) return rc;
    if (int rc = allow_full_lds<split_kernel>(); rc != MADDNESS_OK) return rc;
    for (int level = 0; level < 4; ++level) {
        const int n_buckets = 1 << level;
        hipLaunchKernelGGL(order_rows_kernel, dim3(C), dim3(256), 0, stream, a, n_buckets);
        LAUNCH_OK("launch order_rows_kernel");
        hipLaunchKernelGGL(bucket_loss_kernel, dim3(n_buckets, C), dim3(256), kLossLdsBytes, stream, a);
        LAUNCH_OK("launch bucket_loss_kernel");
        hipLaunchKernelGGL(select_kernel, dim3(C), dim3(64), sizeof(double) * dmax, stream, a, n_buckets);
        LAUNCH_OK("launch select_kernel");
        hipLaunchKernelGGL(key_kernel, dim3((unsigned)((a.Npad + 255) / 256), kCand, C), dim3(256), 0, stream, a, by_bucket);
        LAUNCH_OK("launch key_kernel");
        const int64_t chunk_len = a.Npad < kSortChunk ? a.Npad : kSortChunk;
        const dim3 chunks((unsigned)(a.Npad / chunk_len), kCand, C), pairs((unsigned)((a.Npad / 2 + 255) / 256), kCand, C);
        hipLaunchKernelGGL(sort_chunks_kernel, chunks, dim3(1024), sort_lds, stream, a, (int64_t)2, chunk_len, (int64_t)0);
        LAUNCH_OK("launch sort_chunks_kernel");
        for (int64_t k = 2 * chunk_len; k <= a.Npad; k <<= 1) {
            for (int64_t j = k >> 1; j >= chunk_len; j >>= 1) {
                hipLaunchKernelGGL(sort_exchange_kernel, pairs, dim3(256), 0, stream, a, k, j);
                LAUNCH_OK("launch sort_exchange_kernel");
            }
            hipLaunchKernelGGL(sort_chunks_kernel, chunks, dim3(1024), sort_lds, stream, a, k, k, chunk_len >> 1);
            LAUNCH_OK("launch sort_chunks_kernel");
        }
        if (ordered)
            hipLaunchKernelGGL(split_ordered_kernel, dim3(kCand, by_bucket ? n_buckets : 1, C), dim3(256), split_lds, stream, a,
                               n_buckets, tile, by_bucket);
        else
            hipLaunchKernelGGL(split_kernel, dim3(kCand, C), dim3(256), split_lds, stream, a, n_buckets);
        LAUNCH_OK("launch split_kernel");
        hipLaunchKernelGGL(choose_kernel, dim3((C + 63) / 64), dim3(64), 0, stream, a, level, n_buckets);
        LAUNCH_OK("launch choose_kernel");
        hipLaunchKernelGGL(apply_kernel, dim3((unsigned)((N + 255) / 256), C), dim3(256), 0, stream, a, level, n_buckets);
        LAUNCH_OK("launch apply_kernel");
    }
    return MADDNESS_OK;
}

int launch_learn_prototypes(const uint8_t *codes, const float *A, int64_t N, int64_t lda, int32_t D, int32_t C,
                            const int32_t *bounds_host, bool ridge, double lambda, float *prototypes, void *workspace,
                            hipStream_t stream)
{
    ProtoArgs a{};
    a.codes = codes; a.A = A; a.lda = lda; a.N = N; a.D = D; a.C = C; a.Q = 16 * C; a.P = prototypes;
    Carver w{static_cast<unsigned char *>(workspace)};
    carve_prototypes(w, a);
    Bounds b{};
    for (int i = 0; i < 2 * C; ++i) b.v[i] = bounds_host[i];
    hipLaunchKernelGGL(upload_bounds_kernel, dim3(1), dim3(256), 0, stream, b, 2 * C, a.bounds);
    LAUNCH_OK("launch upload_bounds_kernel");
    if (!ridge) {
        note_kernel("means_kernel", nullptr);
        hipLaunchKernelGGL(means_kernel, dim3((D + 63) / 64, 16, C), dim3(64), 0, stream, a);
        LAUNCH_OK("launch means_kernel");
        return MADDNESS_OK;
    }
    note_kernel("cooccurrence_kernel + gta_kernel + cholesky_panel_kernel + substitution_kernel", nullptr);
    const int64_t QQ = (int64_t)a.Q * a.Q;
    hipLaunchKernelGGL(cooccurrence_kernel, dim3(C, (C + kCoGroup - 1) / kCoGroup), dim3(256), 0, stream, a);
    LAUNCH_OK("launch cooccurrence_kernel");
    hipLaunchKernelGGL(ridge_matrix_kernel, dim3((unsigned)((QQ + 255) / 256)), dim3(256), 0, stream, a, lambda);
    LAUNCH_OK("launch ridge_matrix_kernel");
    // (a thread per (codebook, code, column) while that is at most a wavefront per SIMD of the chip)
    if ((int64_t)C * 16 * D <= (int64_t)device_info().cus * 4 * 64)
        hipLaunchKernelGGL(gta_by_code_kernel, dim3((D + 63) / 64, 16, C), dim3(64), 0, stream, a);
    else
        hipLaunchKernelGGL(gta_kernel, dim3((D + 63) / 64, (C + 3) / 4), dim3(256), 0, stream, a);
    LAUNCH_OK("launch gta_kernel");
    for (int J0 = 0; J0 < a.Q; J0 += kCholPanel) {
        const int below = a.Q - J0 - kCholPanel, per_group = kCholRows - kCholPanel;
        hipLaunchKernelGGL(cholesky_panel_kernel, dim3(std::max(1, (below + per_group - 1) / per_group)), dim3(256), 0,
                           stream, a, J0);
        LAUNCH_OK("launch cholesky_panel_kernel");
    }
    hipLaunchKernelGGL(transpose_factor_kernel, dim3((unsigned)((QQ + 255) / 256)), dim3(256), 0, stream, a);
    LAUNCH_OK("launch transpose_factor_kernel");
    // the kernel that takes the products out of the chain where its LDS layout fits (as many columns of A~ per
    // workgroup as fit, a power of two up to 16); else substitution_kernel (as many columns as LDS holds beside two
    // rows of the factor: a power of two, a wavefront's worth at most)
    const size_t lds_limit = (size_t)device_info().lds_per_block;
    int rc = MADDNESS_OK;
    int npc = 16;
    while (npc > 1 && substitution_products_lds_bytes(a.Q, npc) > lds_limit) npc >>= 1;
    if (substitution_products_lds_bytes(a.Q, npc) <= lds_limit) {
        switch (npc) {
        case 16: rc = launch_substitution_products<16>(a, stream); break;
        case 8: rc = launch_substitution_products<8>(a, stream); break;
        case 4: rc = launch_substitution_products<4>(a, stream); break;
        case 2: rc = launch_substitution_products<2>(a, stream); break;
        default: rc = launch_substitution_products<1>(a, stream); break;
        }
    } else {
        int nc = 64;
        while (nc > 1 && substitution_lds_bytes(a.Q, nc) > lds_limit) nc >>= 1;
        if (substitution_lds_bytes(a.Q, nc) > lds_limit)
            return fail(MADDNESS_E_UNSUPPORTED, "maddness_learn_prototypes: a column of 16 C values does not fit in LDS");
        switch (nc) {
        case 64: rc = launch_substitution<64>(a, stream); break;
        case 32: rc = launch_substitution<32>(a, stream); break;
        case 16: rc = launch_substitution<16>(a, stream); break;
        case 8: rc = launch_substitution<8>(a, stream); break;
        case 4: rc = launch_substitution<4>(a, stream); break;
        case 2: rc = launch_substitution<2>(a, stream); break;
        default: rc = launch_substitution<1>(a, stream); break;
        }
    }
    if (rc != MADDNESS_OK) return rc;
    LAUNCH_OK("launch substitution_kernel");
    return MADDNESS_OK;
}

}  // namespace maddness
