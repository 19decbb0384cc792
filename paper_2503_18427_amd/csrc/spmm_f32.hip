// aes_spmm_f32 / aes_spmm_fused_f32: float32 features through the SpMM kernel
// (Sec. 3.2 Algorithm 1, accumulation loop; the fused form samples on the fly).
#include "spmm_kernel.hpp"

namespace {

using namespace aes;

// Features 0 .. 4*floor(F/4) - 1 go through the vector kernel (four per lane, any alignment); the
// last F % 4 columns, if any, through a second launch of the element-wise kernel on the same plan.
// Every output element sees its slots in the same order either way.
template <bool FUSED>
int run_f32(const char *what, int64_t n_rows, const SlotSource &src, const int32_t *row_perm, const float *X,
            int64_t ldx, int32_t F, float *Y, int64_t ldy, hipStream_t stream)
{
    const bool lr = long_rows_possible(src.W);
    const QParams qp = {nullptr, nullptr, 1, -1};
    const int32_t F4 = F & ~3;
    if (F4 > 0)
        if (int rc = dispatch_lanes<FeatF32<4>, kQNone, FUSED>(lr, n_rows, src, row_perm, X, ldx, F4, qp, Y, ldy, stream, what))
            return rc;
    if (F4 < F)
        return launch_rows<8, 8, FeatF32<1>, kQNone, FUSED>(lr, n_rows, src, row_perm, X + F4, ldx, F - F4, qp,
                                                                  Y + F4, ldy, stream, what);
    return AES_OK;
}

}  // namespace

extern "C" int aes_spmm_f32(int64_t n_rows, int64_t n_cols, int32_t W,
                            const int64_t *s_rowptr, const int32_t *s_col, const float *s_val,
                            const int32_t *row_perm,
                            const float *X, int64_t ldx, int32_t F,
                            float *Y, int64_t ldy, void *stream)
{
    const char *what = "aes_spmm_f32";
    if (int rc = check_common(what, n_rows, n_cols, s_rowptr, X, ldx, F, Y, ldy)) return rc;
    if (int rc = check_sampling(what, W, AES_STRATEGY_ADAPTIVE)) return rc;
    if (n_rows == 0) return AES_OK;
    const SlotSource src = {s_rowptr, s_col, s_val, W, 0, 0};   // W: only the bound on slots per row
    return run_f32<false>(what, n_rows, src, row_perm, X, ldx, F, Y, ldy, static_cast<hipStream_t>(stream));
}

extern "C" int aes_spmm_fused_f32(int64_t n_rows, int64_t n_cols,
                                  const int64_t *rowptr, const int32_t *colidx, const float *val,
                                  int32_t W, uint64_t seed, int32_t strategy,
                                  const float *X, int64_t ldx, int32_t F,
                                  float *Y, int64_t ldy, void *stream)
{
    const char *what = "aes_spmm_fused_f32";
    if (int rc = check_common(what, n_rows, n_cols, rowptr, X, ldx, F, Y, ldy)) return rc;
    if (int rc = check_sampling(what, W, strategy)) return rc;
    if (n_rows == 0) return AES_OK;
    const SlotSource src = {rowptr, colidx, val, W, strategy, seed};
    return run_f32<true>(what, n_rows, src, nullptr, X, ldx, F, Y, ldy, static_cast<hipStream_t>(stream));
}

