// aes_spmm_q8 / aes_spmm_fused_q8: 8-bit features, Sec. 2.3 Eq. 2 applied inside the
// gather of the SpMM kernel (Sec. 3.2 Algorithm 1, accumulation loop).
#include "spmm_kernel.hpp"

namespace {

using namespace aes;

// 8-bit features: 4 codes per lane when rows are 4-byte aligned, else element-wise.
template <bool SIGNED, int QMODE, bool FUSED>
int dispatch_q8(bool fast, int64_t n_rows, const SlotSource &src, const int32_t *row_perm, const int8_t *Xq,
                int64_t ldq, int32_t F, QParams qp, float *Y, int64_t ldy, hipStream_t stream, const char *what)
{
    const bool lr = long_rows_possible(src.W);
    if (fast)
        return dispatch_lanes<FeatQ8<4, SIGNED>, QMODE, true, FUSED>(lr, n_rows, src, row_perm, Xq, ldq, F, qp, Y, ldy, stream, what);
    return launch_rows<64, 4, FeatQ8<1, SIGNED>, QMODE, true, FUSED>(lr, n_rows, src, row_perm, Xq, ldq, F, qp, Y, ldy, stream, what);
}

template <bool FUSED>
int run_q8(const char *what, int64_t n_rows, const SlotSource &src, const int32_t *row_perm, const int8_t *Xq,
           int64_t ldq, int32_t F, int32_t scheme, int32_t granularity, const float *scale, const float *zero,
           float *Y, int64_t ldy, hipStream_t stream)
{
    if (scheme != AES_Q_AFFINE_FLOOR_U8 && scheme != AES_Q_SYMMETRIC_RNE_I8)
        return aes::fail(AES_ERR_INVALID_ARG, "%s: unknown scheme %d", what, (int)scheme);
    if (granularity < AES_Q_PER_TENSOR || granularity > AES_Q_PER_ROW)
        return aes::fail(AES_ERR_INVALID_ARG, "%s: unknown granularity %d", what, (int)granularity);
    if (scale == nullptr) return aes::fail(AES_ERR_INVALID_ARG, "%s: scale is NULL", what);
    const bool affine = scheme == AES_Q_AFFINE_FLOOR_U8;
    if (affine && zero == nullptr) return aes::fail(AES_ERR_INVALID_ARG, "%s: zero is NULL for the affine scheme", what);
    if (n_rows == 0) return AES_OK;
    const bool fast = aes::aligned(Y, 16) && ldy % 4 == 0 && aes::aligned(Xq, 4) && F % 4 == 0 && ldq % 4 == 0;
    QParams qp = {scale, zero, granularity, affine ? 1 : 0};
    const bool per_row = granularity == AES_Q_PER_ROW;
    if (affine) {
        if (per_row) return dispatch_q8<false, kQRowScale, FUSED>(fast, n_rows, src, row_perm, Xq, ldq, F, qp, Y, ldy, stream, what);
        return dispatch_q8<false, kQNone, FUSED>(fast, n_rows, src, row_perm, Xq, ldq, F, qp, Y, ldy, stream, what);
    }
    if (per_row) return dispatch_q8<true, kQRowScale, FUSED>(fast, n_rows, src, row_perm, Xq, ldq, F, qp, Y, ldy, stream, what);
    return dispatch_q8<true, kQNone, FUSED>(fast, n_rows, src, row_perm, Xq, ldq, F, qp, Y, ldy, stream, what);
}

}  // namespace

extern "C" int aes_spmm_q8(int64_t n_rows, int64_t n_cols, int32_t W,
                           const int64_t *s_rowptr, const int32_t *s_col, const float *s_val,
                           const int32_t *row_perm,
                           const int8_t *Xq, int64_t ldq, int32_t F,
                           int32_t scheme, int32_t granularity,
                           const float *scale, const float *zero,
                           float *Y, int64_t ldy, void *stream)
{
    const char *what = "aes_spmm_q8";
    if (int rc = check_common(what, n_rows, n_cols, s_rowptr, s_col, s_val, Xq, ldq, F, Y, ldy)) return rc;
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
    if (int rc = check_common(what, n_rows, n_cols, rowptr, colidx, val, Xq, ldq, F, Y, ldy)) return rc;
    if (int rc = check_sampling(what, W, strategy)) return rc;
    const SlotSource src = {rowptr, colidx, val, W, strategy, seed};
    return run_q8<true>(what, n_rows, src, nullptr, Xq, ldq, F, scheme, granularity, scale, zero, Y, ldy,
                        static_cast<hipStream_t>(stream));
}
