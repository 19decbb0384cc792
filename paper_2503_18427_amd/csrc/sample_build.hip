// aes_sample_build: CSR -> sampled plan on gfx950.
//
// Method: AES-SpMM Sec. 3.2 Algorithm 1 (sampling loop), Sec. 3.3 Table 1
// (strategy selector) and Eq. 3 (start-index hash).  The paper samples inside
// its SpMM kernel into shared memory; here the sampled rows are materialised
// once per (graph, W, seed) so that every later multiply only streams them.
//
// Four launches on the caller's stream, integer work only:
//   1 classify : per 1024-row block, slot total and slot-count-class histogram
//   2 scan     : exclusive scans of the block totals and of the histogram
//   3 offsets  : s_rowptr and the class-ordered row permutation
//   4 sample   : one thread per output slot copies / samples a (col, val) pair
#include "aes_common.hpp"
#include "aes_sampling.hpp"

namespace {

using aes::kBlock;
using aes::kWave;
using aes::row_slot_count;

constexpr int kSubTiles = 4;                          // rows per thread in kernels 1 and 3
constexpr int kRowsPerBlock = kBlock * kSubTiles;     // 1024
constexpr int kClasses = 32;                          // class = bit length of the slot count
constexpr int kScanThreads = 1024;
constexpr int kScanItems = 8;

__device__ inline int slot_class(int64_t slots)
{
    if (slots <= 0) return 0;
    int c = 64 - __builtin_clzll(static_cast<unsigned long long>(slots));
    return c > kClasses - 1 ? kClasses - 1 : c;
}

// Histogram entry of (class, block): classes in DEcreasing order, blocks ascending,
// so that one exclusive scan of the flat array yields the row_perm offsets.
__device__ inline int64_t hist_index(int cls, int64_t blk, int64_t nblk)
{
    return static_cast<int64_t>(kClasses - 1 - cls) * nblk + blk;
}

__device__ inline int64_t wave_inclusive_scan(int64_t v, int lane)
{
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        int64_t o = __shfl_up(v, d, kWave);
        if (lane >= d) v += o;
    }
    return v;
}

// ---- kernel 1 ---------------------------------------------------------------
__global__ void __launch_bounds__(kBlock)
classify_kernel(int64_t n_rows, const int64_t *__restrict__ rowptr, int32_t W, int strategy, int64_t nblk,
                int64_t *__restrict__ blk_slots, int32_t *__restrict__ hist, int want_hist)
{
    __shared__ int32_t sh_hist[kClasses];
    __shared__ int64_t sh_part[aes::kWavesPerBlock];
    const int t = threadIdx.x, lane = t % kWave, wave = t / kWave;
    const int64_t blk = blockIdx.x;
    if (t < kClasses) sh_hist[t] = 0;
    __syncthreads();
    int64_t mine = 0;
    for (int q = 0; q < kSubTiles; ++q) {
        int64_t r = blk * kRowsPerBlock + q * kBlock + t;
        if (r < n_rows) {
            int64_t s = row_slot_count(rowptr[r + 1] - rowptr[r], W, strategy);
            mine += s;
            if (want_hist) atomicAdd(&sh_hist[slot_class(s)], 1);
        }
    }
    int64_t incl = wave_inclusive_scan(mine, lane);
    if (lane == kWave - 1) sh_part[wave] = incl;
    __syncthreads();
    if (t == 0) {
        int64_t tot = 0;
        for (int w = 0; w < aes::kWavesPerBlock; ++w) tot += sh_part[w];
        blk_slots[blk] = tot;
    }
    if (want_hist && t < kClasses) hist[hist_index(t, blk, nblk)] = sh_hist[t];
}

// ---- kernel 2 ---------------------------------------------------------------
// In-place exclusive scan of data[0..n) by one workgroup; returns the total to
// every thread.
template <typename T>
__device__ T block_exclusive_scan_inplace(T *data, int64_t n, T *sh_wave /* kScanThreads/64 + 1 */)
{
    const int t = threadIdx.x, lane = t % kWave, wave = t / kWave;
    constexpr int kWaves = kScanThreads / kWave;
    T carry = 0;
    for (int64_t base = 0; base < n; base += static_cast<int64_t>(kScanThreads) * kScanItems) {
        int64_t first = base + static_cast<int64_t>(t) * kScanItems;
        T item[kScanItems];
        T sum = 0;
#pragma unroll
        for (int i = 0; i < kScanItems; ++i) {
            item[i] = (first + i < n) ? data[first + i] : T(0);
            sum += item[i];
        }
        T incl = sum;
#pragma unroll
        for (int d = 1; d < kWave; d <<= 1) {
            T o = __shfl_up(incl, d, kWave);
            if (lane >= d) incl += o;
        }
        if (lane == kWave - 1) sh_wave[wave] = incl;
        __syncthreads();
        T wave_off = 0, chunk_total = 0;
        for (int w = 0; w < kWaves; ++w) {
            T s = sh_wave[w];
            if (w < wave) wave_off += s;
            chunk_total += s;
        }
        T run = carry + wave_off + (incl - sum);
#pragma unroll
        for (int i = 0; i < kScanItems; ++i) {
            if (first + i < n) data[first + i] = run;
            run += item[i];
        }
        carry += chunk_total;
        __syncthreads();
    }
    return carry;
}

__global__ void __launch_bounds__(kScanThreads)
scan_kernel(int64_t n_rows, int64_t nblk, int64_t *__restrict__ blk_slots,
            int32_t *__restrict__ hist, int n_classes, int64_t *__restrict__ s_rowptr)
{
    __shared__ int64_t sh64[kScanThreads / kWave + 1];
    __shared__ int32_t sh32[kScanThreads / kWave + 1];
    int64_t total = block_exclusive_scan_inplace<int64_t>(blk_slots, nblk, sh64);
    if (threadIdx.x == 0) s_rowptr[n_rows] = total;
    if (hist != nullptr && n_classes > 0) {
        // entries of classes >= n_classes are all zero and never read: skip them
        int64_t skip = static_cast<int64_t>(kClasses - n_classes) * nblk;
        block_exclusive_scan_inplace<int32_t>(hist + skip, static_cast<int64_t>(n_classes) * nblk, sh32);
    }
}

// ---- kernel 3 ---------------------------------------------------------------
__global__ void __launch_bounds__(kBlock)
offsets_kernel(int64_t n_rows, const int64_t *__restrict__ rowptr, int32_t W, int strategy, int64_t nblk,
               const int64_t *__restrict__ blk_slots, const int32_t *__restrict__ hist,
               int n_classes, int64_t *__restrict__ s_rowptr, int32_t *__restrict__ row_perm)
{
    __shared__ int64_t sh_part[aes::kWavesPerBlock];
    __shared__ int32_t sh_wave_cnt[aes::kWavesPerBlock][kClasses];
    __shared__ int32_t sh_running[kClasses];
    const int t = threadIdx.x, lane = t % kWave, wave = t / kWave;
    const int64_t blk = blockIdx.x;
    if (t < kClasses) sh_running[t] = 0;
    int64_t block_prefix = blk_slots[blk];
    for (int q = 0; q < kSubTiles; ++q) {
        const int64_t r = blk * kRowsPerBlock + q * kBlock + t;
        const bool valid = r < n_rows;
        int64_t s = valid ? row_slot_count(rowptr[r + 1] - rowptr[r], W, strategy) : 0;
        int64_t incl = wave_inclusive_scan(s, lane);
        if (lane == kWave - 1) sh_part[wave] = incl;
        const int cls = valid ? slot_class(s) : -1;
        int rank_in_wave = 0;
        if (row_perm != nullptr) {
            for (int c = 0; c < n_classes; ++c) {
                unsigned long long m = __ballot(cls == c);
                if (cls == c) rank_in_wave = __popcll(m & ((1ull << lane) - 1ull));
                if (lane == 0) sh_wave_cnt[wave][c] = __popcll(m);
            }
        }
        __syncthreads();
        int64_t wave_off = 0, tile_total = 0;
        for (int w = 0; w < aes::kWavesPerBlock; ++w) {
            int64_t p = sh_part[w];
            if (w < wave) wave_off += p;
            tile_total += p;
        }
        if (valid) s_rowptr[r] = block_prefix + wave_off + (incl - s);
        block_prefix += tile_total;
        if (row_perm != nullptr && valid) {
            int rank = sh_running[cls] + rank_in_wave;
            for (int w = 0; w < wave; ++w) rank += sh_wave_cnt[w][cls];
            row_perm[hist[hist_index(cls, blk, nblk)] + rank] = static_cast<int32_t>(r);
        }
        __syncthreads();
        if (row_perm != nullptr && t < n_classes) {
            int add = 0;
            for (int w = 0; w < aes::kWavesPerBlock; ++w) add += sh_wave_cnt[w][t];
            sh_running[t] += add;
        }
        __syncthreads();
    }
}

// ---- kernel 4 ---------------------------------------------------------------
// One thread per OUTPUT SLOT.  A workgroup owns kSampleRows consecutive rows:
// their rowptr / s_rowptr segments sit in LDS, every thread finds the row of its
// slot by binary search there, then copies (row fits) or samples: slot k of a
// sampled row is entry j = k / sample_cnt of run i = k % sample_cnt, the run
// starting at Eq. 3's start_i.  Writes are perfectly coalesced and the work per
// thread does not depend on the degree distribution.
constexpr int kSampleRows = 256;

__global__ void __launch_bounds__(kBlock)
sample_slots_kernel(int64_t n_rows, const int64_t *__restrict__ rowptr, const int32_t *__restrict__ colidx,
                    const float *__restrict__ val, int32_t W, uint64_t seed, int strategy,
                    const int64_t *__restrict__ s_rowptr, int32_t *__restrict__ s_col,
                    float *__restrict__ s_val, int64_t *__restrict__ s_eid)
{
    __shared__ int64_t sh_out[kSampleRows + 1];
    __shared__ int64_t sh_in[kSampleRows + 1];
    const int64_t r_lo = static_cast<int64_t>(blockIdx.x) * kSampleRows;
    const int nr = static_cast<int>(n_rows - r_lo < kSampleRows ? n_rows - r_lo : kSampleRows);
    for (int i = threadIdx.x; i <= nr; i += kBlock) {
        sh_out[i] = s_rowptr[r_lo + i];
        sh_in[i] = rowptr[r_lo + i];
    }
    __syncthreads();
    const int64_t base = sh_out[0];
    const int64_t total = sh_out[nr] - base;
    for (int64_t t = threadIdx.x; t < total; t += kBlock) {
        // largest q in [0, nr) with sh_out[q] - base <= t (empty rows are skipped by construction)
        int lo = 0, hi = nr;
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (sh_out[mid] - base <= t) lo = mid; else hi = mid;
        }
        const int64_t r = r_lo + lo;
        const int64_t k = t - (sh_out[lo] - base);
        const int64_t row_begin = sh_in[lo];
        const int64_t row_nnz = sh_in[lo + 1] - row_begin;
        int64_t e;
        if (W == 0 || row_nnz <= W) {
            e = row_begin + k;
        } else {
            int32_t N, cnt;
            aes::sample_strategy(row_nnz, W, strategy, N, cnt);
            e = aes::sampled_entry(row_begin, row_nnz, N, cnt, aes::row_offset(seed, r), static_cast<int32_t>(k));
        }
        s_col[base + t] = colidx[e];
        s_val[base + t] = val[e];
        if (s_eid) s_eid[base + t] = e;
    }
}

int bit_length(int64_t v)
{
    int b = 0;
    while (v > 0) { ++b; v >>= 1; }
    return b;
}

}  // namespace

extern "C" int64_t aes_sample_capacity(int64_t n_rows, int64_t nnz, int32_t W)
{
    if (n_rows < 0 || nnz < 0 || W < 0 || W > AES_MAX_W)
        return aes::fail(AES_ERR_INVALID_ARG, "aes_sample_capacity: n_rows=%lld nnz=%lld W=%d out of range",
                         (long long)n_rows, (long long)nnz, (int)W);
    if (W == 0) return nnz;
    // n_rows * W cannot overflow: n_rows < 2^42 is enforced by aes_sample_build, W <= 2^20
    if (n_rows > (INT64_MAX / AES_MAX_W)) return nnz;
    const int64_t cap = n_rows * static_cast<int64_t>(W);
    return cap < nnz ? cap : nnz;
}

extern "C" size_t aes_sample_workspace_bytes(int64_t n_rows)
{
    if (n_rows < 0) return 0;
    const int64_t nblk = aes::ceil_div(n_rows, kRowsPerBlock);
    return static_cast<size_t>(8 * (nblk + 1) + 4 * static_cast<int64_t>(kClasses) * nblk);
}

extern "C" int aes_sample_build(int64_t n_rows, int64_t n_cols, int64_t nnz,
                                const int64_t *rowptr, const int32_t *colidx, const float *val,
                                int32_t W, uint64_t seed, int32_t strategy,
                                int64_t *s_rowptr, int32_t *s_col, float *s_val, int64_t *s_eid,
                                int32_t *row_perm,
                                void *workspace, size_t workspace_bytes, void *stream_)
{
    if (n_rows < 0 || n_cols < 0 || nnz < 0)
        return aes::fail(AES_ERR_INVALID_ARG, "aes_sample_build: negative size (n_rows=%lld n_cols=%lld nnz=%lld)",
                         (long long)n_rows, (long long)n_cols, (long long)nnz);
    if (n_cols > INT32_MAX)
        return aes::fail(AES_ERR_UNSUPPORTED, "aes_sample_build: n_cols=%lld does not fit int32 column indices",
                         (long long)n_cols);
    if (W < 0 || W > AES_MAX_W)
        return aes::fail(AES_ERR_INVALID_ARG, "aes_sample_build: W=%d outside 0..%d", (int)W, (int)AES_MAX_W);
    if (strategy < AES_STRATEGY_ADAPTIVE || strategy > AES_STRATEGY_SFS)
        return aes::fail(AES_ERR_INVALID_ARG, "aes_sample_build: unknown strategy %d", (int)strategy);
    if (rowptr == nullptr || s_rowptr == nullptr)
        return aes::fail(AES_ERR_INVALID_ARG, "aes_sample_build: rowptr / s_rowptr is NULL");
    if (nnz > 0 && (colidx == nullptr || val == nullptr || s_col == nullptr || s_val == nullptr))
        return aes::fail(AES_ERR_INVALID_ARG, "aes_sample_build: colidx / val / s_col / s_val is NULL with nnz > 0");
    if (row_perm != nullptr && n_rows > INT32_MAX)
        return aes::fail(AES_ERR_UNSUPPORTED, "aes_sample_build: row_perm needs n_rows < 2^31");
    const int64_t nblk = aes::ceil_div(n_rows, kRowsPerBlock);
    if (nblk > INT32_MAX)
        return aes::fail(AES_ERR_UNSUPPORTED, "aes_sample_build: n_rows=%lld too large", (long long)n_rows);
    const size_t need = aes_sample_workspace_bytes(n_rows);
    if (workspace == nullptr || workspace_bytes < need)
        return aes::fail(AES_ERR_WORKSPACE, "aes_sample_build: workspace of %zu bytes needed, %zu given%s", need,
                         workspace_bytes, workspace == nullptr ? " (NULL)" : "");
    if (!aes::aligned(workspace, 8))
        return aes::fail(AES_ERR_WORKSPACE, "aes_sample_build: workspace must be 8-byte aligned");

    hipStream_t stream = static_cast<hipStream_t>(stream_);
    int64_t *blk_slots = static_cast<int64_t *>(workspace);            // nblk + 1
    int32_t *hist = reinterpret_cast<int32_t *>(blk_slots + nblk + 1);  // kClasses * nblk
    const int want_hist = row_perm != nullptr ? 1 : 0;
    const int n_classes = W == 0 ? kClasses : bit_length(W) + 1;        // slot counts are <= W

    if (nblk > 0) {
        classify_kernel<<<dim3(static_cast<unsigned>(nblk)), dim3(kBlock), 0, stream>>>(
            n_rows, rowptr, W, strategy, nblk, blk_slots, hist, want_hist);
        if (int rc = aes::check_launch("aes_sample_build/classify")) return rc;
    }
    scan_kernel<<<dim3(1), dim3(kScanThreads), 0, stream>>>(n_rows, nblk, blk_slots,
                                                            want_hist ? hist : nullptr, n_classes, s_rowptr);
    if (int rc = aes::check_launch("aes_sample_build/scan")) return rc;
    if (nblk == 0) return AES_OK;
    offsets_kernel<<<dim3(static_cast<unsigned>(nblk)), dim3(kBlock), 0, stream>>>(
        n_rows, rowptr, W, strategy, nblk, blk_slots, hist, n_classes, s_rowptr, row_perm);
    if (int rc = aes::check_launch("aes_sample_build/offsets")) return rc;
    if (nnz == 0) return AES_OK;

    const int64_t sample_blocks = aes::ceil_div(n_rows, kSampleRows);
    if (sample_blocks > INT32_MAX)
        return aes::fail(AES_ERR_UNSUPPORTED, "aes_sample_build: n_rows=%lld too large", (long long)n_rows);
    sample_slots_kernel<<<dim3(static_cast<unsigned>(sample_blocks)), dim3(kBlock), 0, stream>>>(
        n_rows, rowptr, colidx, val, W, seed, strategy, s_rowptr, s_col, s_val, s_eid);
    return aes::check_launch("aes_sample_build/sample");
}
