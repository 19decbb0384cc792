// aes_gcn_layer_f32: aggregation and combination of one GNN layer in one kernel,
//     H = (A_s X) Theta
// on gfx950.
//
// Method: Sec. 2.1 of the AES-SpMM paper splits a layer into the aggregation
// phase (the sampled SpMM of Sec. 3.2 Algorithm 1) and the combination phase (a
// dense GEMM with the layer's weight matrix).  Here a workgroup aggregates a tile
// of 32 output rows into LDS with the same lane-group gather loop as the SpMM
// kernels and multiplies the tile by Theta on the matrix cores
// (v_mfma_f32_32x32x2_f32, float32 in, float32 accumulate) before anything is
// written: the aggregated features never travel to HBM and back.  The gather
// phase is bound by memory, the MFMA phase by the matrix cores, and workgroups in
// different phases overlap on a CU, so the GEMM is mostly hidden.
#include "spmm_core.hpp"

namespace {

using namespace aes;

constexpr int kTileRows = 32;        // rows per workgroup = M of the MFMA block
constexpr int kMaxFeatures = 256;    // one chunk of four features per lane, at most 64 lanes

typedef float floatx16 __attribute__((ext_vector_type(16)));

template <int LPR>
__global__ void __launch_bounds__(kBlock)
gcn_layer_kernel(int64_t n_rows, SlotSource src, const float *__restrict__ X, int64_t ldx, int32_t F,
                 const float *__restrict__ Theta, int64_t ldt, int32_t Fo, float *__restrict__ H, int64_t ldh)
{
    constexpr int kGroups = kWave / LPR;
    constexpr int kGroupsPerBlock = kGroups * kWavesPerBlock;
    constexpr int kStride = kTile + 1;
    __shared__ int2 stage[kWavesPerBlock][kGroups][kStride];
    extern __shared__ float ys[];        // kTileRows x (F + 1): the aggregated tile, padded against bank conflicts
    const int y_stride = F + 1;

    const int wave = threadIdx.x / kWave;
    const int wl = threadIdx.x % kWave;
    const int group = wl / LPR;
    const int lane = wl % LPR;
    const int64_t row0 = static_cast<int64_t>(blockIdx.x) * kTileRows;

    // ---- aggregation: Algorithm 1's accumulation loop, one lane group per row ----
    const int32_t f = lane * 4;
    const bool lane_on = f < F;
    const QParams no_q = {nullptr, nullptr, 0, 0};
    for (int rr = wave * kGroups + group; rr < kTileRows; rr += kGroupsPerBlock) {
        const int64_t r = row0 + rr;
        float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        float side = 0.0f, vsum = 0.0f;
        if (r < n_rows) {
            const RowInfo ri = row_info<false>(src, r);
            accumulate_tiles<LPR, 8, FeatF32<4>, kQNone, false, false, float>(src, ri, stage[wave][group], lane, lane_on, X, ldx,
                                                                       f, no_q, 0, 1, acc, side, vsum);
        }
        if (lane_on) {
#pragma unroll
            for (int i = 0; i < 4; ++i) ys[rr * y_stride + f + i] = acc[i];
        }
    }
    __syncthreads();

    // ---- combination: H_tile (32 x Fo) = ys (32 x F) * Theta (F x Fo) on the matrix cores ----
    // v_mfma_f32_32x32x2_f32: lane l supplies A[l % 32][l / 32] and B[l / 32][l % 32];
    // it receives D[8 * (v / 4) + 4 * (l / 32) + v % 4][l % 32] in result register v.
    const int i = wl % 32, h = wl / 32;
    for (int nb = wave; nb * 32 < Fo; nb += kWavesPerBlock) {
        const int col = nb * 32 + i;
        const bool col_on = col < Fo;
        const float *theta_col = Theta + (col_on ? col : 0);
        floatx16 c;
#pragma unroll
        for (int v = 0; v < 16; ++v) c[v] = 0.0f;
        // Operands are fetched kBatch MFMAs ahead: the loads of the next batch are issued
        // before the current batch's MFMA chain, so Theta's L2 latency hides behind it.
        constexpr int kBatch = 8;
        float a_cur[kBatch], b_cur[kBatch], a_nxt[kBatch], b_nxt[kBatch];
        auto fetch = [&](int k_base, float (&a)[kBatch], float (&b)[kBatch]) {
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                const int k = k_base + 2 * u + h;
                const bool on = k < F;
                a[u] = on ? ys[i * y_stride + k] : 0.0f;
                b[u] = (on && col_on) ? theta_col[static_cast<int64_t>(k) * ldt] : 0.0f;
            }
        };
        fetch(0, a_cur, b_cur);
        for (int k0 = 0; k0 < F; k0 += 2 * kBatch) {
            if (k0 + 2 * kBatch < F) fetch(k0 + 2 * kBatch, a_nxt, b_nxt);
#pragma unroll
            for (int u = 0; u < kBatch; ++u) c = __builtin_amdgcn_mfma_f32_32x32x2f32(a_cur[u], b_cur[u], c, 0, 0, 0);
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                a_cur[u] = a_nxt[u];
                b_cur[u] = b_nxt[u];
            }
        }
        if (col_on) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t r = row0 + 8 * (v / 4) + 4 * h + (v % 4);
                if (r < n_rows) H[r * ldh + col] = c[v];
            }
        }
    }
}

template <int LPR>
int launch_gcn(int64_t n_rows, const SlotSource &src, const float *X, int64_t ldx, int32_t F, const float *Theta,
               int64_t ldt, int32_t Fo, float *H, int64_t ldh, hipStream_t stream)
{
    const int64_t grid = ceil_div(n_rows, kTileRows);
    if (grid > INT32_MAX) return fail(AES_ERR_UNSUPPORTED, "aes_gcn_layer_f32: n_rows=%lld too large", (long long)n_rows);
    const size_t shmem = static_cast<size_t>(kTileRows) * (F + 1) * sizeof(float);
    gcn_layer_kernel<LPR><<<dim3(static_cast<unsigned>(grid)), dim3(kBlock), shmem, stream>>>(n_rows, src, X, ldx, F, Theta,
                                                                                             ldt, Fo, H, ldh);
    return check_launch("aes_gcn_layer_f32");
}

}  // namespace

extern "C" int aes_gcn_layer_f32(int64_t n_rows, int64_t n_cols, int32_t W,
                                 const int64_t *s_rowptr, const int32_t *s_col, const float *s_val,
                                 const float *X, int64_t ldx, int32_t F,
                                 const float *Theta, int64_t ldt, int32_t Fo,
                                 float *H, int64_t ldh, void *stream)
{
    const char *what = "aes_gcn_layer_f32";
    if (n_rows < 0 || n_cols < 0)
        return aes::fail(AES_ERR_INVALID_ARG, "%s: negative size (n_rows=%lld n_cols=%lld)", what, (long long)n_rows,
                         (long long)n_cols);
    if (n_cols > INT32_MAX) return aes::fail(AES_ERR_UNSUPPORTED, "%s: n_cols=%lld does not fit int32", what, (long long)n_cols);
    if (W < 0 || W > AES_MAX_W) return aes::fail(AES_ERR_INVALID_ARG, "%s: W=%d outside 0..%d", what, (int)W, (int)AES_MAX_W);
    if (F < 1 || Fo < 1 || Fo >= (1 << 24))
        return aes::fail(AES_ERR_INVALID_ARG, "%s: F=%d / Fo=%d out of range", what, (int)F, (int)Fo);
    if (ldx < F || ldt < Fo || ldh < Fo)
        return aes::fail(AES_ERR_INVALID_ARG, "%s: leading dimension too small (ldx=%lld ldt=%lld ldh=%lld)", what,
                         (long long)ldx, (long long)ldt, (long long)ldh);
    if (s_rowptr == nullptr || Theta == nullptr) return aes::fail(AES_ERR_INVALID_ARG, "%s: s_rowptr / Theta is NULL", what);
    if (n_rows > 0 && H == nullptr) return aes::fail(AES_ERR_INVALID_ARG, "%s: H is NULL", what);
    if (n_rows > 0 && n_cols > 0 && X == nullptr) return aes::fail(AES_ERR_INVALID_ARG, "%s: X is NULL", what);
    if (F > kMaxFeatures || F % 4 != 0 || ldx % 4 != 0 || !aes::aligned(X, 16))
        return aes::fail(AES_ERR_UNSUPPORTED,
                         "%s: needs F <= %d, F and ldx multiples of 4 and X 16-byte aligned (F=%d ldx=%lld); "
                         "use aes_spmm_f32 and a GEMM instead", what, kMaxFeatures, (int)F, (long long)ldx);
    if (n_rows == 0) return AES_OK;
    hipStream_t stream_ = static_cast<hipStream_t>(stream);
    const SlotSource src = {s_rowptr, s_col, s_val, W, 0, 0};
    int l = aes::pow2_ceil(aes::ceil_div(F, 4));
    l = l < 8 ? 8 : l;
    switch (l) {
        case 8: return launch_gcn<8>(n_rows, src, X, ldx, F, Theta, ldt, Fo, H, ldh, stream_);
        case 16: return launch_gcn<16>(n_rows, src, X, ldx, F, Theta, ldt, Fo, H, ldh, stream_);
        case 32: return launch_gcn<32>(n_rows, src, X, ldx, F, Theta, ldt, Fo, H, ldh, stream_);
        default: return launch_gcn<64>(n_rows, src, X, ldx, F, Theta, ldt, Fo, H, ldh, stream_);
    }
}
