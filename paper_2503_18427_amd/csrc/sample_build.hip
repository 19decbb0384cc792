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
#include <mutex>

#include "aes_common.hpp"
#include "aes_sampling.hpp"

// Scratch of aes_sample_build_noalloc: the workspace of a build of up to AES_NOALLOC_MAX_ROWS rows,
// part of the code object, so every GPU the library runs on holds its own copy until the process
// ends.  In host code this name is only a handle for hipGetSymbolAddress; the device address that
// call yields (one per device) is what kernels receive.  No attribute may keep the symbol local to
// the code object: the runtime finds it by name.
constexpr size_t kScratchBytes = 2228232;   // the workspace of AES_NOALLOC_MAX_ROWS rows (asserted where it is used)
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {

using aes::kBlock;
using aes::kWave;
using aes::row_slot_count;

constexpr int kSubTiles = 4;                          // rows per thread in kernels 1 and 3
constexpr int kRowsPerBlock = kBlock * kSubTiles;     // 1024
constexpr int kClasses = 32;                          // class = bit length of the slot count
constexpr int kScanThreads = 1024;
constexpr int kScanItems = 8;

// Workspace layout of one build: block slot totals (nblk + 1 int64), then the class histogram
// (kClasses * nblk int32), nblk = ceil(n_rows / kRowsPerBlock).
constexpr size_t workspace_bytes_for(int64_t n_rows)
{
    return static_cast<size_t>(8 * ((n_rows + kRowsPerBlock - 1) / kRowsPerBlock + 1) +
                               4 * static_cast<int64_t>(kClasses) * ((n_rows + kRowsPerBlock - 1) / kRowsPerBlock));
}

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
// One thread per OUTPUT SLOT.  A workgroup owns kSampleRows consecutive rows, whose
// rowptr / s_rowptr segments sit in LDS, and walks its slots in chunks of kChunkSlots:
//   1 every non-empty row that starts inside the chunk writes its index at its first slot
//   2 an inclusive prefix maximum over the chunk turns these head marks into the row of
//     every slot (slots before the first mark belong to the row carried over from the
//     previous chunk)
//   3 thread t takes slots t, t + 256, ... of the chunk: entry k of a row that fits, or
//     entry j = k / sample_cnt of run i = k % sample_cnt (the run starting at Eq. 3's
//     start_i) of a sampled row; the loads of all its slots are issued before the first
//     store.
// Reads of whole rows and all writes are coalesced, and the work per slot does not depend
// on the degree distribution: a hub row of millions of entries (W = 0) costs what the same
// number of short rows costs.
constexpr int kSampleRows = 256;
constexpr int kSlotsPerThread = 8;
constexpr int kChunkSlots = kBlock * kSlotsPerThread;

__global__ void __launch_bounds__(kBlock)
sample_slots_kernel(int64_t n_rows, const int64_t *__restrict__ rowptr, const int32_t *__restrict__ colidx,
                    const float *__restrict__ val, int32_t W, uint64_t seed, int strategy,
                    const int64_t *__restrict__ s_rowptr, int32_t *__restrict__ s_col,
                    float *__restrict__ s_val, int64_t *__restrict__ s_eid)
{
    static_assert(kSampleRows == kBlock, "one thread marks one row");
    __shared__ int64_t sh_out[kSampleRows + 1];
    __shared__ int64_t sh_in[kSampleRows + 1];
    __shared__ __attribute__((aligned(16))) int32_t sh_row[kChunkSlots];   // head marks, then the row of every slot
    __shared__ int32_t sh_wave_max[aes::kWavesPerBlock];
    const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    const int64_t r_lo = static_cast<int64_t>(blockIdx.x) * kSampleRows;
    const int nr = static_cast<int>(n_rows - r_lo < kSampleRows ? n_rows - r_lo : kSampleRows);
    for (int i = tid; i <= nr; i += kBlock) {
        sh_out[i] = s_rowptr[r_lo + i];
        sh_in[i] = rowptr[r_lo + i];
    }
#pragma unroll
    for (int u = 0; u < kSlotsPerThread; ++u) sh_row[u * kBlock + tid] = -1;
    __syncthreads();
    const int64_t base = sh_out[0];
    const int64_t total = sh_out[nr] - base;
    if (total == 0) return;                                   // uniform
    const int64_t e_any = sh_in[0];                           // a valid entry index: some row here is non-empty
    int64_t my_head = -1;                                     // first slot of this thread's row, block-relative
    if (tid < nr && sh_out[tid + 1] > sh_out[tid]) my_head = sh_out[tid] - base;
    int carry = 0;
    for (int64_t c0 = 0; c0 < total; c0 += kChunkSlots) {
        if (my_head >= c0 && my_head < c0 + kChunkSlots) sh_row[my_head - c0] = tid;
        __syncthreads();
        // inclusive prefix maximum: 8 consecutive marks per thread, then across the wave, then across waves
        int m[kSlotsPerThread];
        {
            const int4 a = reinterpret_cast<const int4 *>(sh_row)[2 * tid];
            const int4 b = reinterpret_cast<const int4 *>(sh_row)[2 * tid + 1];
            m[0] = a.x; m[1] = a.y; m[2] = a.z; m[3] = a.w; m[4] = b.x; m[5] = b.y; m[6] = b.z; m[7] = b.w;
        }
#pragma unroll
        for (int u = 1; u < kSlotsPerThread; ++u) m[u] = m[u] > m[u - 1] ? m[u] : m[u - 1];
        int incl = m[kSlotsPerThread - 1];
#pragma unroll
        for (int d = 1; d < kWave; d <<= 1) {
            const int o = __shfl_up(incl, d, kWave);
            if (lane >= d && o > incl) incl = o;
        }
        int before = __shfl_up(incl, 1, kWave);               // maximum over the earlier lanes of this wave
        if (lane == 0) before = -1;
        if (lane == kWave - 1) sh_wave_max[wave] = incl;
        __syncthreads();
        int next_carry = carry;
        if (carry > before) before = carry;
#pragma unroll
        for (int w = 0; w < aes::kWavesPerBlock; ++w) {
            const int wm = sh_wave_max[w];
            if (w < wave && wm > before) before = wm;
            if (wm > next_carry) next_carry = wm;
        }
        carry = next_carry;
#pragma unroll
        for (int u = 0; u < kSlotsPerThread; ++u) m[u] = m[u] > before ? m[u] : before;
        reinterpret_cast<int4 *>(sh_row)[2 * tid] = make_int4(m[0], m[1], m[2], m[3]);
        reinterpret_cast<int4 *>(sh_row)[2 * tid + 1] = make_int4(m[4], m[5], m[6], m[7]);
        __syncthreads();

        int64_t e[kSlotsPerThread];
#pragma unroll
        for (int u = 0; u < kSlotsPerThread; ++u) {
            const int idx = u * kBlock + tid;
            const int64_t t = c0 + idx;
            const int q = sh_row[idx];
            sh_row[idx] = -1;                                 // this thread's own entries: ready for the next chunk
            e[u] = e_any;                                     // slots past the end read a valid entry and store nothing
            if (t < total) {
                const int64_t k = t - (sh_out[q] - base);
                const int64_t row_begin = sh_in[q];
                const int64_t row_nnz = sh_in[q + 1] - row_begin;
                if (W == 0 || row_nnz <= W) {
                    e[u] = row_begin + k;
                } else {
                    int32_t N, cnt;
                    aes::sample_strategy(row_nnz, W, strategy, N, cnt);
                    e[u] = aes::sampled_entry(row_begin, row_nnz, N, cnt, aes::row_offset(seed, r_lo + q),
                                              static_cast<int32_t>(k));
                }
            }
        }
        int32_t c[kSlotsPerThread];
        float v[kSlotsPerThread];
#pragma unroll
        for (int u = 0; u < kSlotsPerThread; ++u) {
            c[u] = colidx[e[u]];
            v[u] = val[e[u]];
        }
#pragma unroll
        for (int u = 0; u < kSlotsPerThread; ++u) {
            const int64_t t = c0 + u * kBlock + tid;
            if (t < total) {
                s_col[base + t] = c[u];
                s_val[base + t] = v[u];
                if (s_eid) s_eid[base + t] = e[u];
            }
        }
        __syncthreads();                                      // marks reset before the next chunk's heads are written
    }
}

int bit_length(int64_t v)
{
    int b = 0;
    while (v > 0) { ++b; v >>= 1; }
    return b;
}

// Argument checks of both entry points (everything but the workspace).
int check_build_args(const char *what, int64_t n_rows, int64_t n_cols, int64_t nnz, const int64_t *rowptr,
                     const int32_t *colidx, const float *val, int32_t W, int32_t strategy, const int64_t *s_rowptr,
                     const int32_t *s_col, const float *s_val, const int32_t *row_perm)
{
    if (n_rows < 0 || n_cols < 0 || nnz < 0)
        return aes::fail(AES_ERR_INVALID_ARG, "%s: negative size (n_rows=%lld n_cols=%lld nnz=%lld)", what,
                         (long long)n_rows, (long long)n_cols, (long long)nnz);
    if (n_cols > INT32_MAX)
        return aes::fail(AES_ERR_UNSUPPORTED, "%s: n_cols=%lld does not fit int32 column indices", what,
                         (long long)n_cols);
    if (W < 0 || W > AES_MAX_W) return aes::fail(AES_ERR_INVALID_ARG, "%s: W=%d outside 0..%d", what, (int)W, (int)AES_MAX_W);
    if (strategy < AES_STRATEGY_ADAPTIVE || strategy > AES_STRATEGY_SFS)
        return aes::fail(AES_ERR_INVALID_ARG, "%s: unknown strategy %d", what, (int)strategy);
    if (rowptr == nullptr || s_rowptr == nullptr) return aes::fail(AES_ERR_INVALID_ARG, "%s: rowptr / s_rowptr is NULL", what);
    if (nnz > 0 && (colidx == nullptr || val == nullptr || s_col == nullptr || s_val == nullptr))
        return aes::fail(AES_ERR_INVALID_ARG, "%s: colidx / val / s_col / s_val is NULL with nnz > 0", what);
    if (row_perm != nullptr && n_rows > INT32_MAX) return aes::fail(AES_ERR_UNSUPPORTED, "%s: row_perm needs n_rows < 2^31", what);
    if (aes::ceil_div(n_rows, kRowsPerBlock) > INT32_MAX || aes::ceil_div(n_rows, kSampleRows) > INT32_MAX)
        return aes::fail(AES_ERR_UNSUPPORTED, "%s: n_rows=%lld too large", what, (long long)n_rows);
    return AES_OK;
}

// The four launches; `workspace` holds aes_sample_workspace_bytes(n_rows) bytes, 8-byte aligned.
// Every workspace element a kernel reads has been written by an earlier kernel of the same call
// (block totals by classify, the histogram by classify when a permutation is wanted), so the
// workspace needs no clearing, whatever an earlier call left in it.
int enqueue_build(const char *what, int64_t n_rows, int64_t nnz, const int64_t *rowptr, const int32_t *colidx,
                  const float *val, int32_t W, uint64_t seed, int32_t strategy, int64_t *s_rowptr, int32_t *s_col,
                  float *s_val, int64_t *s_eid, int32_t *row_perm, void *workspace, hipStream_t stream)
{
    const int64_t nblk = aes::ceil_div(n_rows, kRowsPerBlock);
    int64_t *blk_slots = static_cast<int64_t *>(workspace);            // nblk + 1
    int32_t *hist = reinterpret_cast<int32_t *>(blk_slots + nblk + 1);  // kClasses * nblk
    const int want_hist = row_perm != nullptr ? 1 : 0;
    const int n_classes = W == 0 ? kClasses : bit_length(W) + 1;        // slot counts are <= W
    char stage[96];

    if (nblk > 0) {
        classify_kernel<<<dim3(static_cast<unsigned>(nblk)), dim3(kBlock), 0, stream>>>(
            n_rows, rowptr, W, strategy, nblk, blk_slots, hist, want_hist);
        snprintf(stage, sizeof stage, "%s/classify", what);
        if (int rc = aes::check_launch(stage)) return rc;
    }
    scan_kernel<<<dim3(1), dim3(kScanThreads), 0, stream>>>(n_rows, nblk, blk_slots,
                                                            want_hist ? hist : nullptr, n_classes, s_rowptr);
    snprintf(stage, sizeof stage, "%s/scan", what);
    if (int rc = aes::check_launch(stage)) return rc;
    if (nblk == 0) return AES_OK;
    offsets_kernel<<<dim3(static_cast<unsigned>(nblk)), dim3(kBlock), 0, stream>>>(
        n_rows, rowptr, W, strategy, nblk, blk_slots, hist, n_classes, s_rowptr, row_perm);
    snprintf(stage, sizeof stage, "%s/offsets", what);
    if (int rc = aes::check_launch(stage)) return rc;
    if (nnz == 0) return AES_OK;

    const int64_t sample_blocks = aes::ceil_div(n_rows, kSampleRows);
    sample_slots_kernel<<<dim3(static_cast<unsigned>(sample_blocks)), dim3(kBlock), 0, stream>>>(
        n_rows, rowptr, colidx, val, W, seed, strategy, s_rowptr, s_col, s_val, s_eid);
    snprintf(stage, sizeof stage, "%s/sample", what);
    return aes::check_launch(stage);
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
    return workspace_bytes_for(n_rows);
}

extern "C" int aes_sample_build(int64_t n_rows, int64_t n_cols, int64_t nnz,
                                const int64_t *rowptr, const int32_t *colidx, const float *val,
                                int32_t W, uint64_t seed, int32_t strategy,
                                int64_t *s_rowptr, int32_t *s_col, float *s_val, int64_t *s_eid,
                                int32_t *row_perm,
                                void *workspace, size_t workspace_bytes, void *stream_)
{
    const char *what = "aes_sample_build";
    if (int rc = check_build_args(what, n_rows, n_cols, nnz, rowptr, colidx, val, W, strategy, s_rowptr, s_col, s_val,
                                  row_perm))
        return rc;
    const size_t need = aes_sample_workspace_bytes(n_rows);
    if (workspace == nullptr || workspace_bytes < need)
        return aes::fail(AES_ERR_WORKSPACE, "aes_sample_build: workspace of %zu bytes needed, %zu given%s", need,
                         workspace_bytes, workspace == nullptr ? " (NULL)" : "");
    if (!aes::aligned(workspace, 8))
        return aes::fail(AES_ERR_WORKSPACE, "aes_sample_build: workspace must be 8-byte aligned");
    return enqueue_build(what, n_rows, nnz, rowptr, colidx, val, W, seed, strategy, s_rowptr, s_col, s_val, s_eid,
                         row_perm, workspace, static_cast<hipStream_t>(stream_));
}

// ---- the variant that allocates nothing and takes no workspace -----------------------------
namespace {

constexpr int kMaxDevices = 64;
std::mutex scratch_mutex;
void *scratch_address[kMaxDevices];          // device address of `scratch` on each device, once resolved

// Device address of this device's copy of `scratch`; resolved on the first call per device, with
// that device current.  NULL (and the error message set) on failure.
void *scratch_on_current_device(const char *what)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        aes::fail(AES_ERR_HIP, "%s: hipGetDevice: %s (device %d)", what, hipGetErrorString(e), dev);
        return nullptr;
    }
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (scratch_address[dev] == nullptr) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || ptr == nullptr) {
            aes::fail(AES_ERR_HIP, "%s: hipGetSymbolAddress(scratch): %s", what, hipGetErrorString(e));
            return nullptr;
        }
        scratch_address[dev] = ptr;
    }
    return scratch_address[dev];
}

}  // namespace

extern "C" int aes_sample_build_noalloc(int64_t n_rows, int64_t n_cols, int64_t nnz,
                                        const int64_t *rowptr, const int32_t *colidx, const float *val,
                                        int32_t W, uint64_t seed, int32_t strategy,
                                        int64_t *s_rowptr, int32_t *s_col, float *s_val, int64_t *s_eid,
                                        int32_t *row_perm, void *stream_)
{
    const char *what = "aes_sample_build_noalloc";
    if (int rc = check_build_args(what, n_rows, n_cols, nnz, rowptr, colidx, val, W, strategy, s_rowptr, s_col, s_val,
                                  row_perm))
        return rc;
    if (n_rows > AES_NOALLOC_MAX_ROWS)
        return aes::fail(AES_ERR_UNSUPPORTED,
                         "%s: n_rows=%lld exceeds the built-in scratch (at most %lld rows); use aes_sample_build with a "
                         "workspace", what, (long long)n_rows, (long long)AES_NOALLOC_MAX_ROWS);
    static_assert(workspace_bytes_for(AES_NOALLOC_MAX_ROWS) == kScratchBytes, "scratch covers the largest build");
    void *ws = scratch_on_current_device(what);
    if (ws == nullptr) return AES_ERR_HIP;
    return enqueue_build(what, n_rows, nnz, rowptr, colidx, val, W, seed, strategy, s_rowptr, s_col, s_val, s_eid,
                         row_perm, ws, static_cast<hipStream_t>(stream_));
}
