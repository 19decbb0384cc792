// The SpMM kernel of the multiply stage (aes_spmm_f32 / aes_spmm_q8 and their single-kernel
// forms) on gfx950, with its launch helpers; instantiated by spmm_f32.hip and spmm_q8.hip.
//
// Method: Sec. 3.2 Algorithm 1, accumulation loop: result += sh_val[k] *
// B[sh_col[k], cid] over the row's sampled slots; the quantised variant applies
// Sec. 2.3 Eq. 2 to each gathered feature.  The paper maps one thread to one
// output element and one thread block to a row; here the mapping follows the
// 64-wide wavefront and the 512 B - 1 KB feature rows instead:
//
//   - a GROUP of LPR lanes owns one output row; each lane owns 4 consecutive
//     features, so one wavefront load instruction fetches 64/LPR whole feature
//     rows, each as one contiguous, 16 B-per-lane coalesced segment;
//   - a wavefront therefore works on 64/LPR rows at once (2 rows at F = 128, 1
//     at F = 256); rows are taken in natural order, or in the slot-count-class
//     order of an optional row_perm (natural order measured faster: the kernel is
//     bound by the memory system, and a sorted order unbalances the 8 XCDs);
//   - the row's (col, val) slots are staged through a wavefront-private LDS tile
//     (coalesced load, broadcast read), no workgroup barrier anywhere;
//   - UNROLL independent feature-row gathers are in flight per lane before the
//     first fused multiply-add consumes one, which is what keeps HBM busy;
//   - no cross-lane reduction is needed: a lane sees every slot of its row.
//
// The kernel is bound by the gather traffic (about 2 flop per 4 bytes), not by
// arithmetic, so there is no MFMA here.
#pragma once

#include "spmm_core.hpp"

namespace aes {

// Rows with more slots than this are not left to one lane group: all groups of the
// workgroup share such a row (LONG variant, used when the caller's width allows them).
constexpr int kLongRow = 2048;

// LPR   lanes per output row (8, 16, 32 or 64); a wavefront holds 64/LPR rows
// Feat  feature loader: Feat::VEC features per lane per chunk (4 on the aligned
//       fast paths, 1 otherwise)
// QMODE how the constants of the 8-bit path are applied (kQNone: float32 features); FUSED: sample
//       from the CSR on the fly
// NV    vectors per lane and pass: 1 for rows of up to LPR * VEC features; 2, 3 or 4 (with LPR = 64) for
//       wider rows, so that the slots are staged once and a gathered row is read in one piece (which
//       widths take which NV: dispatch_lanes)
// LONG  rows above kLongRow slots are processed by the whole workgroup: its lane groups
//       take the row's tiles round-robin and their partial sums (carried in float64,
//       since such sums run over up to millions of terms) are added in a fixed order
//       through LDS, so the result stays bit-reproducible.  Without LONG the kernel
//       has no workgroup barrier at all.
// Second launch bound: the 8-bit kernels that read a materialised plan are held to 8 wavefronts per SIMD.  Left
// alone, the unsigned-code variants come out at 66-71 vector registers (7 wavefronts) and the narrow-group
// variants that take a node's constants from the gather at 73-88 (6); held to 64 they spill nothing, and the
// latency-bound ragged rows gain from the extra wavefronts: -9 % on the products- and arxiv-shaped graphs with the
// affine scheme, -13 % with constants from the gather, nothing slower.  The sample-on-the-fly variants (77-110
// registers, some would spill) and the long-row variants are left to the compiler, except the 32-lane form that
// takes constants from the gather.
template <typename Feat, int QMODE, int LPR, bool FUSED, bool LONG>
constexpr int min_waves_per_simd()
{
    constexpr bool kCodes = sizeof(typename Feat::elem_t) == 1;
    if (kCodes && !FUSED && !LONG) return 8;
    if (QMODE == kQRowInGather && LPR == 32 && FUSED && !LONG) return 8;
    return 1;
}

template <int LPR, int UNROLL, typename Feat, int QMODE, bool FUSED, bool LONG, int NV = 1>
__global__ void __launch_bounds__(kBlock, (min_waves_per_simd<Feat, QMODE, LPR, FUSED, LONG>()))
spmm_rows_kernel(int64_t n_rows, SlotSource src, const int32_t *__restrict__ row_perm,
                 const typename Feat::elem_t *__restrict__ X, int64_t ldx, int32_t F, QParams qp,
                 float *__restrict__ Y, int64_t ldy)
{
    constexpr int VEC = Feat::VEC;
    constexpr int kGroups = kWave / LPR;                 // rows per wavefront
    constexpr int kRowsPerBlock = kGroups * aes::kWavesPerBlock;
    constexpr int kStride = kTile + 1;                   // +1 slot: groups start in different LDS banks
    // Where a row's per-column constants are requested: before its gathers, so that their latency passes
    // behind the gathers, where the four registers that hold them meanwhile fit under 64 (8 wavefronts
    // per SIMD: signed codes, wide lane groups); after the gathers otherwise.  Measured: 2-7 % on the
    // short-row workloads where it applies, 10-15 % slower where it costs a wavefront of occupancy.
    constexpr bool kEarlyConstants = QMODE == kQColumn && Feat::kSigned && LPR >= 32;
    __shared__ int2 stage[aes::kWavesPerBlock][kGroups][kStride];

    const int wave = threadIdx.x / kWave;
    const int group = (threadIdx.x % kWave) / LPR;
    const int lane = threadIdx.x % LPR;
    // Lanes whose features lie below this gather: the F features, and with kQRowInGather also the words
    // behind them that hold the node's constants (the host has checked that one pass of the group reaches them).
    const int32_t f_gather = QMODE == kQRowInGather ? qp.inline_off + (QTraits<Feat, QMODE>::kAffine ? 8 : 4) : F;
    const int64_t slot_in_order = static_cast<int64_t>(blockIdx.x) * kRowsPerBlock + wave * kGroups + group;
    const bool valid = slot_in_order < n_rows;
    if (!LONG && !valid) return;                         // whole group leaves together
    int2 *my_stage = stage[wave][group];
    int64_t r = 0;
    RowInfo ri = {};
    if (valid) {
        r = row_perm ? static_cast<int64_t>(row_perm[slot_in_order]) : slot_in_order;
        ri = row_info<FUSED>(src, r);
    }
    const bool is_long = LONG && valid && ri.n_slots > kLongRow;

    if (valid && !is_long) {
        if constexpr (NV == 1) {
            for (int32_t f0 = 0; f0 < F; f0 += LPR * VEC) {
                const int32_t f = f0 + lane * VEC;
                const bool lane_on = f < F;
                float acc[VEC];
#pragma unroll
                for (int i = 0; i < VEC; ++i) acc[i] = 0.0f;
                float side = 0.0f;      // this lane's share of sum(val * zero-point weight)
                LaneConstants<Feat, QMODE> k;
                if constexpr (kEarlyConstants) load_lane_constants<Feat, QMODE>(qp, f, lane_on, r, k);
                accumulate_tiles<LPR, UNROLL, Feat, QMODE, FUSED, float>(src, ri, my_stage, lane, f < f_gather, X, ldx, f, qp,
                                                                         0, 1, acc, side);
                if constexpr (!kEarlyConstants) load_lane_constants<Feat, QMODE>(qp, f, lane_on, r, k);
                if constexpr (QTraits<Feat, QMODE>::kSideOverLanes) side = group_sum<LPR, float>(side);
                finish_chunk<Feat, QMODE, float>(acc, side, lane_on, k, Y + r * ldy + f);
            }
        } else {
            for (int32_t f0 = 0; f0 < F; f0 += NV * LPR * VEC) {
                const int32_t f = f0 + lane * VEC;
                bool on[NV], gather[NV];
                float acc[NV][VEC];
#pragma unroll
                for (int j = 0; j < NV; ++j) {
                    on[j] = f + j * LPR * VEC < F;
                    gather[j] = f + j * LPR * VEC < f_gather;
#pragma unroll
                    for (int i = 0; i < VEC; ++i) acc[j][i] = 0.0f;
                }
                float side = 0.0f;
                accumulate_tiles_wide<LPR, UNROLL, Feat, QMODE, FUSED, float, NV>(src, ri, my_stage, lane, gather, X, ldx, f,
                                                                                  qp, 0, 1, acc, side);
                if constexpr (QTraits<Feat, QMODE>::kSideOverLanes) side = group_sum<LPR, float>(side);
#pragma unroll
                for (int j = 0; j < NV; ++j) {
                    const int32_t fj = f + j * LPR * VEC;
                    LaneConstants<Feat, QMODE> k;
                    load_lane_constants<Feat, QMODE>(qp, fj, on[j], r, k);
                    finish_chunk<Feat, QMODE, float>(acc[j], side, on[j], k, Y + r * ldy + fj);
                }
            }
        }
    }

    if constexpr (LONG) {
        __shared__ int sh_n_long;
        __shared__ int64_t sh_long_row[kRowsPerBlock];
        __shared__ double sh_part[kRowsPerBlock][LPR][NV * VEC + 1];
        if (threadIdx.x == 0) sh_n_long = 0;
        __syncthreads();
        if (is_long && lane == 0) sh_long_row[atomicAdd(&sh_n_long, 1)] = r;   // order affects no sum
        __syncthreads();
        const int n_long = sh_n_long;
        const int gib = wave * kGroups + group;          // this group's index in the workgroup
        for (int i = 0; i < n_long; ++i) {
            const int64_t lr = sh_long_row[i];
            const RowInfo lri = row_info<FUSED>(src, lr);
            for (int32_t f0 = 0; f0 < F; f0 += NV * LPR * VEC) {
                const int32_t f = f0 + lane * VEC;
                bool on[NV], gather[NV];
                double acc[NV][VEC];                     // long sums are carried in float64
#pragma unroll
                for (int j = 0; j < NV; ++j) {
                    on[j] = f + j * LPR * VEC < F;
                    gather[j] = f + j * LPR * VEC < f_gather;
#pragma unroll
                    for (int q = 0; q < VEC; ++q) acc[j][q] = 0.0;
                }
                double side = 0.0;
                if constexpr (NV == 1)
                    accumulate_tiles<LPR, UNROLL, Feat, QMODE, FUSED, double>(src, lri, my_stage, lane, gather[0], X, ldx, f,
                                                                              qp, gib, kRowsPerBlock, acc[0], side);
                else
                    accumulate_tiles_wide<LPR, UNROLL, Feat, QMODE, FUSED, double, NV>(src, lri, my_stage, lane, gather, X,
                                                                                       ldx, f, qp, gib, kRowsPerBlock, acc,
                                                                                       side);
                if constexpr (QTraits<Feat, QMODE>::kSideOverLanes) side = group_sum<LPR, double>(side);
#pragma unroll
                for (int j = 0; j < NV; ++j)
#pragma unroll
                    for (int q = 0; q < VEC; ++q) sh_part[gib][lane][j * VEC + q] = acc[j][q];
                sh_part[gib][lane][NV * VEC] = side;
                __syncthreads();
                if (gib == 0) {
                    for (int g = 1; g < kRowsPerBlock; ++g) {   // fixed order: bit-reproducible
#pragma unroll
                        for (int j = 0; j < NV; ++j)
#pragma unroll
                            for (int q = 0; q < VEC; ++q) acc[j][q] += sh_part[g][lane][j * VEC + q];
                        side += sh_part[g][lane][NV * VEC];
                    }
#pragma unroll
                    for (int j = 0; j < NV; ++j) {
                        const int32_t fj = f + j * LPR * VEC;
                        LaneConstants<Feat, QMODE> k;
                        load_lane_constants<Feat, QMODE>(qp, fj, on[j], lr, k);
                        finish_chunk<Feat, QMODE, double>(acc[j], side, on[j], k, Y + lr * ldy + fj);
                    }
                }
                __syncthreads();
            }
        }
    }
}

template <int LPR, int UNROLL, typename Feat, int QMODE, bool FUSED, int NV = 1>
inline int launch_rows(bool long_rows, int64_t n_rows, const SlotSource &src,
                const int32_t *row_perm, const typename Feat::elem_t *X, int64_t ldx, int32_t F, QParams qp,
                float *Y, int64_t ldy, hipStream_t stream, const char *what)
{
    constexpr int kRowsPerBlock = (kWave / LPR) * aes::kWavesPerBlock;
    const int64_t grid = aes::ceil_div(n_rows, kRowsPerBlock);
    if (grid > INT32_MAX) return aes::fail(AES_ERR_UNSUPPORTED, "%s: n_rows=%lld too large", what, (long long)n_rows);
    const dim3 g(static_cast<unsigned>(grid)), b(kBlock);
    if (long_rows)
        spmm_rows_kernel<LPR, UNROLL, Feat, QMODE, FUSED, true, NV>
            <<<g, b, 0, stream>>>(n_rows, src, row_perm, X, ldx, F, qp, Y, ldy);
    else
        spmm_rows_kernel<LPR, UNROLL, Feat, QMODE, FUSED, false, NV>
            <<<g, b, 0, stream>>>(n_rows, src, row_perm, X, ldx, F, qp, Y, ldy);
    return aes::check_launch(what);
}

// Lanes per row when every lane owns `vec` consecutive features.
inline int lanes_per_row(int32_t F, int vec)
{
    int l = aes::pow2_ceil(aes::ceil_div(F, vec));
    return l < 8 ? 8 : l > 64 ? 64 : l;
}

// Codes one pass of a lane group reaches on the 8-bit vector path (the shape dispatch_lanes picks for F).
inline int32_t codes_per_pass(int32_t F)
{
    constexpr int kPass = kWave * 4;
    if (F > 2 * kPass) return 4 * kPass;
    if (F > kPass) return 2 * kPass;
    return lanes_per_row(F, 4) * 4;
}

// Rows can exceed kLongRow slots only without sampling (W == 0) or with a very wide W.
inline bool long_rows_possible(int32_t W) { return W == 0 || W > kLongRow; }

// Vector path: pick the lane-group width from F.
template <typename Feat, int QMODE, bool FUSED>
int dispatch_lanes(bool lr, int64_t n_rows, const SlotSource &src, const int32_t *row_perm,
                   const typename Feat::elem_t *X, int64_t ldx, int32_t F, QParams qp, float *Y, int64_t ldy,
                   hipStream_t stream, const char *what)
{
    // Rows wider than one pass of 64 lanes (256 features): several vectors per lane, so that the slots are
    // staged once and a gathered row is read in one piece.  8-bit codes (one register per gather): two
    // vectors with sixteen gathers in flight, four vectors beyond 512 features (-22 % at F = 300 and 602).
    // float32: only where the last of the 256-feature passes would be less than half full (-7 % at
    // F = 300, -10 % at F = 602) - two vectors, three for 513..768 features, passes of 512 beyond; at
    // whole multiples of 256 the plain passes are as fast or 3 % faster.
    constexpr bool kCodes = sizeof(typename Feat::elem_t) == 1;
    constexpr int kPass = kWave * Feat::VEC;
    if constexpr (kCodes) {
        if (F > 2 * kPass)
            return launch_rows<64, 4, Feat, QMODE, FUSED, 4>(lr, n_rows, src, row_perm, X, ldx, F, qp, Y, ldy, stream, what);
        if (F > kPass)
            return launch_rows<64, 8, Feat, QMODE, FUSED, 2>(lr, n_rows, src, row_perm, X, ldx, F, qp, Y, ldy, stream, what);
    } else if (F > kPass && 2 * (F - kPass * ((F - 1) / kPass)) <= kPass) {
        if (F > 2 * kPass && F <= 3 * kPass)
            return launch_rows<64, 3, Feat, QMODE, FUSED, 3>(lr, n_rows, src, row_perm, X, ldx, F, qp, Y, ldy, stream, what);
        return launch_rows<64, 4, Feat, QMODE, FUSED, 2>(lr, n_rows, src, row_perm, X, ldx, F, qp, Y, ldy, stream, what);
    }
    switch (lanes_per_row(F, Feat::VEC)) {
        case 8: return launch_rows<8, 8, Feat, QMODE, FUSED>(lr, n_rows, src, row_perm, X, ldx, F, qp, Y, ldy, stream, what);
        case 16: return launch_rows<16, 8, Feat, QMODE, FUSED>(lr, n_rows, src, row_perm, X, ldx, F, qp, Y, ldy, stream, what);
        case 32: return launch_rows<32, 8, Feat, QMODE, FUSED>(lr, n_rows, src, row_perm, X, ldx, F, qp, Y, ldy, stream, what);
        default: return launch_rows<64, 8, Feat, QMODE, FUSED>(lr, n_rows, src, row_perm, X, ldx, F, qp, Y, ldy, stream, what);
    }
}

inline int check_sampling(const char *what, int32_t W, int32_t strategy)
{
    if (W < 0 || W > AES_MAX_W) return aes::fail(AES_ERR_INVALID_ARG, "%s: W=%d outside 0..%d", what, (int)W, (int)AES_MAX_W);
    if (strategy < AES_STRATEGY_ADAPTIVE || strategy > AES_STRATEGY_SFS)
        return aes::fail(AES_ERR_INVALID_ARG, "%s: unknown strategy %d", what, (int)strategy);
    return AES_OK;
}

// s_col / s_val are not examined: they may be NULL for a plan without slots, which the host cannot see.
inline int check_common(const char *what, int64_t n_rows, int64_t n_cols, const int64_t *s_rowptr, const void *X,
                        int64_t ldx, int32_t F, const float *Y, int64_t ldy)
{
    if (n_rows < 0 || n_cols < 0)
        return aes::fail(AES_ERR_INVALID_ARG, "%s: negative size (n_rows=%lld n_cols=%lld)", what, (long long)n_rows,
                         (long long)n_cols);
    if (n_cols > INT32_MAX) return aes::fail(AES_ERR_UNSUPPORTED, "%s: n_cols=%lld does not fit int32", what, (long long)n_cols);
    if (F < 1 || F >= (1 << 24)) return aes::fail(AES_ERR_INVALID_ARG, "%s: F=%d outside 1..2^24-1", what, (int)F);
    if (ldx < F || ldy < F)
        return aes::fail(AES_ERR_INVALID_ARG, "%s: leading dimension smaller than F (ldx=%lld ldy=%lld F=%d)", what,
                         (long long)ldx, (long long)ldy, (int)F);
    if (ldx > UINT32_MAX)
        return aes::fail(AES_ERR_UNSUPPORTED, "%s: feature leading dimension %lld does not fit 32 bits", what, (long long)ldx);
    if (s_rowptr == nullptr) return aes::fail(AES_ERR_INVALID_ARG, "%s: s_rowptr is NULL", what);
    if (n_rows > 0 && Y == nullptr) return aes::fail(AES_ERR_INVALID_ARG, "%s: Y is NULL", what);
    if (n_rows > 0 && n_cols > 0 && X == nullptr) return aes::fail(AES_ERR_INVALID_ARG, "%s: X is NULL", what);
    return AES_OK;
}

}  // namespace aes
