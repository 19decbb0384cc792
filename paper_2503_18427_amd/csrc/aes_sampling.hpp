// Device-side pieces of the adaptive edge sampling strategy, shared by the plan
// builder and the fused SpMM kernels.
//
// Method: AES-SpMM Sec. 3.3 - Table 1 (strategy selector), Eq. 3 (start-index
// hash) - and the slot layout of Sec. 3.2 Algorithm 1's sampling loop.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

#include "aes_spmm.h"

namespace aes {

// (N, sample_cnt) of a row with row_nnz > W >= 1.
//   ADAPTIVE: Table 1 with R = row_nnz / W as a real ratio (integer
//             cross-multiplication), N >= 1 and sample_cnt <= W.
//   AFS     : N = 1, sample_cnt = W  (fine-grained; the paper's description of
//             ES-SpMM's accuracy-first strategy)
//   SFS     : N = W, sample_cnt = 1  (coarse-grained; speed-first)
__device__ inline void sample_strategy(int64_t row_nnz, int64_t W, int strategy, int32_t &N, int32_t &sample_cnt)
{
    if (strategy == AES_STRATEGY_AFS) {
        N = 1;
        sample_cnt = static_cast<int32_t>(W);
        return;
    }
    if (strategy == AES_STRATEGY_SFS) {
        N = static_cast<int32_t>(W);
        sample_cnt = 1;
        return;
    }
    int32_t c;
    if (row_nnz <= 2 * W)
        c = 4;
    else if (row_nnz <= 36 * W)
        c = 8;
    else if (row_nnz <= 54 * W)
        c = 16;
    else
        c = 32;
    const int32_t n = static_cast<int32_t>(W) / c;
    N = n < 1 ? 1 : n;
    sample_cnt = c > W ? static_cast<int32_t>(W) : c;
}

// Slots owned by a row: the whole row if it fits (or W == 0), else N * sample_cnt.
__device__ inline int64_t row_slot_count(int64_t row_nnz, int32_t W, int strategy)
{
    if (W == 0 || row_nnz <= W) return row_nnz;
    int32_t N, cnt;
    sample_strategy(row_nnz, W, strategy, N, cnt);
    return static_cast<int64_t>(N) * cnt;
}

// Per-row offset added to the sample index; 0 when seed == 0 (then Eq. 3 as printed).
__device__ inline uint32_t row_offset(uint64_t seed, int64_t r)
{
    return static_cast<uint32_t>(seed * (2ull * static_cast<uint64_t>(r) + 1ull) * 2654435761ull);
}

// Eq. 3: start_ind = (current_ind * 1429) mod (row_nnz - N + 1).
__device__ inline int64_t hash_start(uint64_t current_ind, int64_t row_nnz, int32_t N)
{
    const uint64_t modulus = static_cast<uint64_t>(row_nnz - N + 1);
    const uint64_t prod = current_ind * 1429ull;
    if (prod < modulus) return static_cast<int64_t>(prod);
    if (((prod | modulus) >> 32) == 0)
        return static_cast<int64_t>(static_cast<uint32_t>(prod) % static_cast<uint32_t>(modulus));
    return static_cast<int64_t>(prod % modulus);
}

// Index into colidx/val of slot k of a SAMPLED row (row_nnz > W): entry
// j = k / sample_cnt of run i = k % sample_cnt (Algorithm 1: slot i + j*sample_cnt).
__device__ inline int64_t sampled_entry(int64_t row_begin, int64_t row_nnz, int32_t N, int32_t sample_cnt,
                                        uint32_t s_r, int32_t k)
{
    const int32_t i = k % sample_cnt;
    const int32_t j = k / sample_cnt;
    return row_begin + hash_start(static_cast<uint64_t>(i) + s_r, row_nnz, N) + j;
}

}  // namespace aes
