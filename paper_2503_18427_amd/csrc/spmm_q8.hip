// aes_spmm_q8 / aes_spmm_fused_q8: 8-bit features, Sec. 2.3 Eq. 2 applied inside the
// gather of the SpMM kernel (Sec. 3.2 Algorithm 1, accumulation loop).
#include "spmm_kernel.hpp"

namespace {

using namespace aes;

// 8-bit features: four codes per lane (any alignment) for columns 0 .. 4*floor(F/4) - 1, then a second
// launch of the element-wise kernel on the same plan for the last F % 4 columns, if any.
template <bool SIGNED, int QMODE, bool FUSED>
int dispatch_q8(int64_t n_rows, const SlotSource &src, const int32_t *row_perm, const int8_t *Xq,
                int64_t ldq, int32_t F, QParams qp, float *Y, int64_t ldy, hipStream_t stream, const char *what)
{
    const bool lr = long_rows_possible(src.W);
    const int32_t F4 = F & ~3;
    if (F4 > 0)
        if (int rc = dispatch_lanes<FeatQ8<4, SIGNED>, QMODE, FUSED>(lr, n_rows, src, row_perm, Xq, ldq, F4, qp, Y, ldy, stream, what))
            return rc;
    if (F4 < F) {
        if (QMODE == kQColumn) {                         // the columns' own constants
            qp.scale += F4;
            if (qp.zero) qp.zero += F4;
        }
        // (constants that the vector launch takes from its own gather are read with a load of their own here)
        constexpr int kTailMode = QMODE == kQRowInGather ? kQRowScale : QMODE;
        return launch_rows<8, 8, FeatQ8<1, SIGNED>, kTailMode, FUSED>(lr, n_rows, src, row_perm, Xq + F4, ldq, F - F4, qp,
                                                                     Y + F4, ldy, stream, what);
    }
    return AES_OK;
}

template <bool SIGNED, bool FUSED>
int dispatch_granularity(int32_t granularity, int64_t n_rows, const SlotSource &src, const int32_t *row_perm,
                         const int8_t *Xq, int64_t ldq, int32_t F, QParams qp, float *Y, int64_t ldy,
                         hipStream_t stream, const char *what)
{
    switch (granularity) {
        case AES_Q_PER_TENSOR: return dispatch_q8<SIGNED, kQTensor, FUSED>(n_rows, src, row_perm, Xq, ldq, F, qp, Y, ldy, stream, what);
        case AES_Q_PER_COLUMN: return dispatch_q8<SIGNED, kQColumn, FUSED>(n_rows, src, row_perm, Xq, ldq, F, qp, Y, ldy, stream, what);
        case AES_Q_PER_ROW: {
            // Constants inside the rows: where one pass of the lane group that gathers a row's codes also reaches
            // the words behind them, the group takes them from that gather; otherwise (and for constants in arrays
            // of their own) each slot's constants are loaded when the slot is staged.
            const int32_t F4 = F & ~3;
            const int32_t end = qp.inline_off + (SIGNED ? 4 : 8);
            if (qp.inline_off >= 0 && F4 > 0 && F4 <= codes_per_pass(F4) && end <= codes_per_pass(F4))
                return dispatch_q8<SIGNED, kQRowInGather, FUSED>(n_rows, src, row_perm, Xq, ldq, F, qp, Y, ldy, stream, what);
            return dispatch_q8<SIGNED, kQRowScale, FUSED>(n_rows, src, row_perm, Xq, ldq, F, qp, Y, ldy, stream, what);
        }
        default:
            if constexpr (FUSED) return aes::fail(AES_ERR_INVALID_ARG, "%s: folded constants need a materialised plan", what);
            else return dispatch_q8<SIGNED, kQFolded, false>(n_rows, src, row_perm, Xq, ldq, F, qp, Y, ldy, stream, what);
    }
}

template <bool FUSED>
int run_q8(const char *what, int64_t n_rows, const SlotSource &src, const int32_t *row_perm, const int8_t *Xq,
           int64_t ldq, int32_t F, int32_t scheme, int32_t granularity, const float *scale, const float *zero,
           float *Y, int64_t ldy, hipStream_t stream)
{
    QParams qp;
    if (int rc = resolve_q8(what, FUSED, Xq, ldq, F, scheme, granularity, scale, zero, qp)) return rc;
    if (n_rows == 0) return AES_OK;
    const bool affine = scheme == AES_Q_AFFINE_FLOOR_U8;
    if (affine) return dispatch_granularity<false, FUSED>(granularity, n_rows, src, row_perm, Xq, ldq, F, qp, Y, ldy, stream, what);
    return dispatch_granularity<true, FUSED>(granularity, n_rows, src, row_perm, Xq, ldq, F, qp, Y, ldy, stream, what);
}

// One group of 16 lanes per row: s_val_folded = s_val * scale[col], row_bias = sum s_val * zero[col].
__global__ void __launch_bounds__(kBlock)
fold_row_constants_kernel(int64_t n_rows, const int64_t *__restrict__ s_rowptr, const int32_t *__restrict__ s_col,
                          const float *s_val, const float *__restrict__ scale, const float *__restrict__ zero,
                          float *s_val_folded, float *__restrict__ row_bias)
{
    constexpr int kLanes = 16;
    const int lane = threadIdx.x % kLanes;
    const int64_t r = static_cast<int64_t>(blockIdx.x) * (kBlock / kLanes) + threadIdx.x / kLanes;
    if (r >= n_rows) return;
    const int64_t k_end = s_rowptr[r + 1];
    float bias = 0.0f;
    for (int64_t k = s_rowptr[r] + lane; k < k_end; k += kLanes) {
        const int32_t c = s_col[k];
        const float v = s_val[k];
        if (zero) bias = __builtin_fmaf(v, zero[c], bias);
        s_val_folded[k] = v * scale[c];
    }
    if (row_bias) {
        bias = group_sum<kLanes, float>(bias);
        if (lane == 0) row_bias[r] = bias;
    }
}

// Symmetric scheme: no row sums are needed, so the fold is element-wise over the S = s_rowptr[n_rows]
// slots (read on the device); four slots per thread and round, their scale gathers in flight together.
__global__ void __launch_bounds__(kBlock)
fold_scales_flat_kernel(int64_t n_rows, const int64_t *__restrict__ s_rowptr, const int32_t *__restrict__ s_col,
                        const float *s_val, const float *__restrict__ scale, float *s_val_folded)
{
    constexpr int kPerThread = 4;
    const int64_t S = s_rowptr[n_rows];
    const int64_t step = static_cast<int64_t>(gridDim.x) * kBlock * kPerThread;
    for (int64_t k0 = static_cast<int64_t>(blockIdx.x) * kBlock * kPerThread + threadIdx.x; k0 < S; k0 += step) {
        float v[kPerThread], sc[kPerThread];
#pragma unroll
        for (int u = 0; u < kPerThread; ++u) {
            const int64_t k = k0 + u * kBlock;
            const int64_t kc = k < S ? k : S - 1;      // clamped: a valid slot, read twice, stored once
            v[u] = s_val[kc];
            sc[u] = scale[s_col[kc]];
        }
#pragma unroll
        for (int u = 0; u < kPerThread; ++u) {
            const int64_t k = k0 + u * kBlock;
            if (k < S) s_val_folded[k] = v[u] * sc[u];
        }
    }
}

}  // namespace

extern "C" int aes_plan_fold_row_constants(int64_t n_rows,
                                           const int64_t *s_rowptr, const int32_t *s_col, const float *s_val,
                                           int32_t scheme, const float *scale, const float *zero,
                                           float *s_val_folded, float *row_bias, void *stream)
{
    const char *what = "aes_plan_fold_row_constants";
    if (n_rows < 0) return aes::fail(AES_ERR_INVALID_ARG, "%s: n_rows=%lld is negative", what, (long long)n_rows);
    if (scheme != AES_Q_AFFINE_FLOOR_U8 && scheme != AES_Q_SYMMETRIC_RNE_I8)
        return aes::fail(AES_ERR_INVALID_ARG, "%s: unknown scheme %d", what, (int)scheme);
    const bool affine = scheme == AES_Q_AFFINE_FLOOR_U8;
    if (s_rowptr == nullptr || scale == nullptr) return aes::fail(AES_ERR_INVALID_ARG, "%s: s_rowptr / scale is NULL", what);
    if (affine && (zero == nullptr || row_bias == nullptr))
        return aes::fail(AES_ERR_INVALID_ARG, "%s: zero / row_bias is NULL for the affine scheme", what);
    if (n_rows == 0) return AES_OK;
    if (!affine) {
        fold_scales_flat_kernel<<<dim3(256 * 16), dim3(kBlock), 0, static_cast<hipStream_t>(stream)>>>(
            n_rows, s_rowptr, s_col, s_val, scale, s_val_folded);
        return aes::check_launch(what);
    }
    const int64_t grid = aes::ceil_div(n_rows, kBlock / 16);
    if (grid > INT32_MAX) return aes::fail(AES_ERR_UNSUPPORTED, "%s: n_rows=%lld too large", what, (long long)n_rows);
    fold_row_constants_kernel<<<dim3(static_cast<unsigned>(grid)), dim3(kBlock), 0, static_cast<hipStream_t>(stream)>>>(
        n_rows, s_rowptr, s_col, s_val, scale, affine ? zero : nullptr, s_val_folded, affine ? row_bias : nullptr);
    return aes::check_launch(what);
}

extern "C" int aes_spmm_q8(int64_t n_rows, int64_t n_cols, int32_t W,
                           const int64_t *s_rowptr, const int32_t *s_col, const float *s_val,
                           const int32_t *row_perm,
                           const int8_t *Xq, int64_t ldq, int32_t F,
                           int32_t scheme, int32_t granularity,
                           const float *scale, const float *zero,
                           float *Y, int64_t ldy, void *stream)
{
    const char *what = "aes_spmm_q8";
    if (int rc = check_common(what, n_rows, n_cols, s_rowptr, Xq, ldq, F, Y, ldy)) return rc;
    if (int rc = check_sampling(what, W, AES_STRATEGY_ADAPTIVE)) return rc;
    const SlotSource src = {s_rowptr, s_col, s_val, W, 0, 0};   // W: only the bound on slots per row
    return run_q8<false>(what, n_rows, src, row_perm, Xq, ldq, F, scheme, granularity, scale, zero, Y, ldy,
                         static_cast<hipStream_t>(stream));
}

extern "C" int aes_spmm_fused_q8(int64_t n_rows, int64_t n_cols,
                                 const int64_t *rowptr, const int32_t *colidx, const float *val,
                                 int32_t W, uint64_t seed, int32_t strategy,
                                 const int8_t *Xq, int64_t ldq, int32_t F,
                                 int32_t scheme, int32_t granularity,
                                 const float *scale, const float *zero,
                                 float *Y, int64_t ldy, void *stream)
{
    const char *what = "aes_spmm_fused_q8";
    if (int rc = check_common(what, n_rows, n_cols, rowptr, Xq, ldq, F, Y, ldy)) return rc;
    if (int rc = check_sampling(what, W, strategy)) return rc;
    const SlotSource src = {rowptr, colidx, val, W, strategy, seed};
    return run_q8<true>(what, n_rows, src, nullptr, Xq, ldq, F, scheme, granularity, scale, zero, Y, ldy,
                        static_cast<hipStream_t>(stream));
}
