// aes_quantize_features: float32 features -> 8-bit codes + (scale, zero) on gfx950.
//
// Method: Sec. 2.3 Eq. 1 (b = 8) for the affine scheme; the symmetric scheme is
// the round-to-nearest variant the benchmark configurations use.  The paper
// runs this step offline on the CPU; it is on the GPU here so that a feature
// matrix already resident in HBM can be compressed in place of a host round
// trip.  Every floating-point step is a single IEEE binary32 operation
// (subtract, divide, multiply, floor / divide, round-half-even): the file is
// compiled without contraction and with correctly rounded division, so the
// codes do not depend on the hardware.
//
//   per row            : one kernel, a lane group per row (min/max by cross-lane
//                        shuffles, then encode; the row stays in registers
//                        when it fits one chunk)
//   per column / tensor: column-wise partial min/max over row slabs, a small
//                        finalise kernel (plus a one-workgroup fold for per
//                        tensor), then an element-wise encode kernel
#include <cmath>

#include "aes_common.hpp"

namespace {

using aes::kBlock;
using aes::kWave;

constexpr int kColsPerBlock = 64;                  // partial kernel: 64 columns x 4 row lanes
constexpr int kRowLanes = kBlock / kColsPerBlock;  // 4
constexpr int kMaxSlabs = 512;

__device__ inline uint32_t encode(float x, float lo, float d, float scale, bool affine)
{
    if (affine) {
        int q = 0;
        if (d != 0.0f) {
            float t = (x - lo) / d;
            t = t * 255.0f;
            q = static_cast<int>(floorf(t));
            q = q < 0 ? 0 : q > 255 ? 255 : q;
        }
        return static_cast<uint32_t>(q);
    }
    int q = static_cast<int>(rintf(x / scale));
    q = q < -127 ? -127 : q > 127 ? 127 : q;
    return static_cast<uint32_t>(q) & 0xffu;
}

__device__ inline void group_constants(float lo, float hi, bool affine, float &d, float &scale, float &zero)
{
    if (affine) {
        d = hi - lo;
        scale = d / 255.0f;
        zero = lo;
    } else {
        d = 0.0f;
        scale = hi == 0.0f ? 1.0f : hi / 127.0f;   // hi holds max |x|
        zero = 0.0f;
    }
}

// ---- per row ----------------------------------------------------------------
template <int LPR, int VEC, bool SINGLE>
__global__ void __launch_bounds__(kBlock)
quantize_rows_kernel(int64_t n, int32_t F, const float *__restrict__ X, int64_t ldx, int affine_,
                     int8_t *__restrict__ Xq, int64_t ldq, float *scale_out, float *zero_out, int64_t cstride)
{
    constexpr int kGroups = kBlock / LPR;
    const bool affine = affine_ != 0;
    const int lane = threadIdx.x % LPR;
    const int64_t r = static_cast<int64_t>(blockIdx.x) * kGroups + threadIdx.x / LPR;
    if (r >= n) return;
    const float *x_row = X + r * ldx;
    float lo = INFINITY, hi = -INFINITY;
    float keep[VEC];
    for (int32_t f0 = 0; f0 < F; f0 += LPR * VEC) {
        const int32_t f = f0 + lane * VEC;
        if (f < F) {
            float x[VEC];
            if constexpr (VEC == 4) {
                const aes::Float4U v = *reinterpret_cast<const aes::Float4U *>(x_row + f);
                x[0] = v.x; x[1] = v.y; x[2] = v.z; x[3] = v.w;
            } else {
                x[0] = x_row[f];
            }
#pragma unroll
            for (int i = 0; i < VEC; ++i) {
                if (SINGLE) keep[i] = x[i];
                const float a = affine ? x[i] : fabsf(x[i]);
                lo = fminf(lo, a);
                hi = fmaxf(hi, a);
            }
        }
    }
#pragma unroll
    for (int s = LPR / 2; s >= 1; s >>= 1) {
        lo = fminf(lo, __shfl_xor(lo, s, LPR));
        hi = fmaxf(hi, __shfl_xor(hi, s, LPR));
    }
    float d, scale, zero;
    group_constants(lo, hi, affine, d, scale, zero);
    if (lane == 0) {
        scale_out[r * cstride] = scale;
        if (zero_out) zero_out[r * cstride] = zero;
    }
    int8_t *q_row = Xq + r * ldq;
    for (int32_t f0 = 0; f0 < F; f0 += LPR * VEC) {
        const int32_t f = f0 + lane * VEC;
        if (f < F) {
            float x[VEC];
            if (SINGLE) {
#pragma unroll
                for (int i = 0; i < VEC; ++i) x[i] = keep[i];
            } else if constexpr (VEC == 4) {
                const aes::Float4U v = *reinterpret_cast<const aes::Float4U *>(x_row + f);
                x[0] = v.x; x[1] = v.y; x[2] = v.z; x[3] = v.w;
            } else {
                x[0] = x_row[f];
            }
            if constexpr (VEC == 4) {
                uint32_t w = encode(x[0], lo, d, scale, affine) | (encode(x[1], lo, d, scale, affine) << 8) |
                             (encode(x[2], lo, d, scale, affine) << 16) | (encode(x[3], lo, d, scale, affine) << 24);
                reinterpret_cast<aes::Word1U *>(q_row + f)->v = w;
            } else {
                q_row[f] = static_cast<int8_t>(encode(x[0], lo, d, scale, affine));
            }
        }
    }
}

// Rows that fit one chunk (F <= 4 * LPR, aligned): every lane group takes RPG rows and
// issues all their loads before the first reduction, so several 16-byte loads per lane
// are in flight; the rows stay in registers until they are encoded.
template <int LPR, int RPG>
__global__ void __launch_bounds__(kBlock)
quantize_rows_batched_kernel(int64_t n, int32_t F, const float *__restrict__ X, int64_t ldx, int affine_,
                             int8_t *__restrict__ Xq, int64_t ldq, float *scale_out, float *zero_out,
                             int64_t cstride)
{
    constexpr int kGroups = kBlock / LPR;
    const bool affine = affine_ != 0;
    const int lane = threadIdx.x % LPR;
    const int64_t r0 = (static_cast<int64_t>(blockIdx.x) * kGroups + threadIdx.x / LPR) * RPG;
    const int32_t f = lane * 4;
    const bool lane_on = f < F;
    aes::Float4U v[RPG];
#pragma unroll
    for (int j = 0; j < RPG; ++j) {
        v[j] = aes::Float4U{0.f, 0.f, 0.f, 0.f};
        if (lane_on && r0 + j < n) v[j] = *reinterpret_cast<const aes::Float4U *>(X + (r0 + j) * ldx + f);
    }
#pragma unroll
    for (int j = 0; j < RPG; ++j) {
        const int64_t r = r0 + j;
        if (r >= n) break;                                    // uniform within the group
        const float x[4] = {v[j].x, v[j].y, v[j].z, v[j].w};
        float lo = INFINITY, hi = -INFINITY;
        if (lane_on) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float a = affine ? x[i] : fabsf(x[i]);
                lo = fminf(lo, a);
                hi = fmaxf(hi, a);
            }
        }
#pragma unroll
        for (int s = LPR / 2; s >= 1; s >>= 1) {
            lo = fminf(lo, __shfl_xor(lo, s, LPR));
            hi = fmaxf(hi, __shfl_xor(hi, s, LPR));
        }
        float d, scale, zero;
        group_constants(lo, hi, affine, d, scale, zero);
        if (lane == 0) {
            scale_out[r * cstride] = scale;
            if (zero_out) zero_out[r * cstride] = zero;
        }
        if (lane_on) {
            const uint32_t w = encode(x[0], lo, d, scale, affine) | (encode(x[1], lo, d, scale, affine) << 8) |
                               (encode(x[2], lo, d, scale, affine) << 16) | (encode(x[3], lo, d, scale, affine) << 24);
            reinterpret_cast<aes::Word1U *>(Xq + r * ldq + f)->v = w;
        }
    }
}

// ---- per column / per tensor --------------------------------------------------
// partial[(slab*2 + 0) * F + c] = min, [(slab*2 + 1) * F + c] = max over the slab's rows
__global__ void __launch_bounds__(kBlock)
column_partials_kernel(int64_t n, int32_t F, const float *__restrict__ X, int64_t ldx, int affine_,
                       float *__restrict__ partial)
{
    __shared__ float sh_lo[kRowLanes][kColsPerBlock];
    __shared__ float sh_hi[kRowLanes][kColsPerBlock];
    const bool affine = affine_ != 0;
    const int tx = threadIdx.x % kColsPerBlock, ty = threadIdx.x / kColsPerBlock;
    const int32_t c = blockIdx.y * kColsPerBlock + tx;
    float lo = INFINITY, hi = -INFINITY;
    if (c < F) {
        const int64_t step = static_cast<int64_t>(gridDim.x) * kRowLanes;
        int64_t r = static_cast<int64_t>(blockIdx.x) * kRowLanes + ty;
        for (; r + 3 * step < n; r += 4 * step) {     // four independent loads in flight
            const float x0 = X[r * ldx + c], x1 = X[(r + step) * ldx + c];
            const float x2 = X[(r + 2 * step) * ldx + c], x3 = X[(r + 3 * step) * ldx + c];
            const float a0 = affine ? x0 : fabsf(x0), a1 = affine ? x1 : fabsf(x1);
            const float a2 = affine ? x2 : fabsf(x2), a3 = affine ? x3 : fabsf(x3);
            lo = fminf(fminf(lo, a0), fminf(a1, fminf(a2, a3)));
            hi = fmaxf(fmaxf(hi, a0), fmaxf(a1, fmaxf(a2, a3)));
        }
        for (; r < n; r += step) {
            const float x = X[r * ldx + c];
            const float a = affine ? x : fabsf(x);
            lo = fminf(lo, a);
            hi = fmaxf(hi, a);
        }
    }
    sh_lo[ty][tx] = lo;
    sh_hi[ty][tx] = hi;
    __syncthreads();
    if (ty == 0 && c < F) {
        for (int j = 1; j < kRowLanes; ++j) {
            lo = fminf(lo, sh_lo[j][tx]);
            hi = fmaxf(hi, sh_hi[j][tx]);
        }
        partial[(static_cast<int64_t>(blockIdx.x) * 2 + 0) * F + c] = lo;
        partial[(static_cast<int64_t>(blockIdx.x) * 2 + 1) * F + c] = hi;
    }
}

// Folds the slab partials of kFoldCols columns per workgroup (kFoldLanes lanes per column, four
// independent loads in flight per lane).
// Per column: writes (scale, zero) and keeps x_min and d = x_max - x_min for the
// encode kernel, which must divide by exactly the d that Eq. 1 names (scale * 255
// would have been rounded twice).  Per tensor: leaves the column's (min, max) in
// lo_out / d_out for tensor_fold_kernel.
constexpr int kFoldCols = 16;
constexpr int kFoldLanes = kBlock / kFoldCols;

__global__ void __launch_bounds__(kBlock)
finalise_kernel(int32_t F, int n_slabs, int empty, const float *__restrict__ partial, int affine_, int per_tensor,
                float *__restrict__ scale_out, float *__restrict__ zero_out, float *__restrict__ lo_out,
                float *__restrict__ d_out)
{
    __shared__ float sh_lo[kFoldLanes][kFoldCols];
    __shared__ float sh_hi[kFoldLanes][kFoldCols];
    const bool affine = affine_ != 0;
    const int tx = threadIdx.x % kFoldCols, ty = threadIdx.x / kFoldCols;
    const int32_t c = blockIdx.x * kFoldCols + tx;
    float lo = INFINITY, hi = -INFINITY;
    if (c < F) {
        const float *p = partial + c;
        const int64_t slab_stride = 2 * static_cast<int64_t>(F);
        int s = ty;
        for (; s + 3 * kFoldLanes < n_slabs; s += 4 * kFoldLanes) {
            float l[4], h[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                l[u] = p[(s + u * kFoldLanes) * slab_stride];
                h[u] = p[(s + u * kFoldLanes) * slab_stride + F];
            }
            lo = fminf(fminf(lo, l[0]), fminf(l[1], fminf(l[2], l[3])));
            hi = fmaxf(fmaxf(hi, h[0]), fmaxf(h[1], fmaxf(h[2], h[3])));
        }
        for (; s < n_slabs; s += kFoldLanes) {
            lo = fminf(lo, p[s * slab_stride]);
            hi = fmaxf(hi, p[s * slab_stride + F]);
        }
    }
    sh_lo[ty][tx] = lo;
    sh_hi[ty][tx] = hi;
    __syncthreads();
    if (ty != 0 || c >= F) return;
    for (int j = 1; j < kFoldLanes; ++j) {
        lo = fminf(lo, sh_lo[j][tx]);
        hi = fmaxf(hi, sh_hi[j][tx]);
    }
    if (empty) { lo = 0.0f; hi = 0.0f; }
    if (per_tensor) {
        lo_out[c] = lo;
        d_out[c] = hi;
        return;
    }
    float d, scale, zero;
    group_constants(lo, hi, affine, d, scale, zero);
    scale_out[c] = scale;
    if (zero_out) zero_out[c] = zero;
    lo_out[c] = lo;
    d_out[c] = d;
}

// Per tensor: one workgroup folds the F per-column (min, max) pairs left in
// lo_io / hi_io and replaces entry 0 by the tensor's x_min and d.
__global__ void __launch_bounds__(kBlock)
tensor_fold_kernel(int32_t F, int affine_, float *__restrict__ lo_io, float *__restrict__ hi_io,
                   float *__restrict__ scale_out, float *__restrict__ zero_out)
{
    __shared__ float sh_lo[kBlock];
    __shared__ float sh_hi[kBlock];
    float lo = INFINITY, hi = -INFINITY;
    for (int32_t c = threadIdx.x; c < F; c += kBlock) {
        lo = fminf(lo, lo_io[c]);
        hi = fmaxf(hi, hi_io[c]);
    }
    sh_lo[threadIdx.x] = lo;
    sh_hi[threadIdx.x] = hi;
    __syncthreads();
    for (unsigned s = kBlock / 2; s >= 1; s >>= 1) {
        if (threadIdx.x < s) {
            sh_lo[threadIdx.x] = fminf(sh_lo[threadIdx.x], sh_lo[threadIdx.x + s]);
            sh_hi[threadIdx.x] = fmaxf(sh_hi[threadIdx.x], sh_hi[threadIdx.x + s]);
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        float d, scale, zero;
        group_constants(sh_lo[0], sh_hi[0], affine_ != 0, d, scale, zero);
        scale_out[0] = scale;
        if (zero_out) zero_out[0] = zero;
        lo_io[0] = sh_lo[0];
        hi_io[0] = d;
    }
}

// Position of a grid-stride walk over the n x per_row items of a matrix (an item = VEC consecutive
// features of one row): one 64-bit division per thread, then an add-with-carry per step.
struct ItemWalk {
    int64_t r, dr;
    int32_t i, di, per_row;      // item within the row, its step, items per row
    __device__ ItemWalk(int32_t per_row_) : per_row(per_row_)
    {
        const int64_t first = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
        const int64_t stride = static_cast<int64_t>(gridDim.x) * kBlock;
        r = first / per_row;
        i = static_cast<int32_t>(first - r * per_row);
        dr = stride / per_row;
        di = static_cast<int32_t>(stride - dr * per_row);
    }
    __device__ void next()
    {
        r += dr;
        i += di;
        if (i >= per_row) { i -= per_row; ++r; }
    }
};

// Element-wise encode with the finished group constants.  The vector form walks over groups of
// kEncodeRows consecutive rows: a thread encodes the same four columns of each of them, so their
// loads are in flight together and the columns' constants are fetched once per group.
constexpr int kEncodeRows = 4;

__global__ void __launch_bounds__(kBlock)
encode_vec_kernel(int64_t n, int32_t F, const float *__restrict__ X, int64_t ldx, int affine_, int per_tensor,
                  const float *__restrict__ scale_in, const float *__restrict__ lo_in, const float *__restrict__ d_in,
                  int8_t *__restrict__ Xq, int64_t ldq)
{
    const bool affine = affine_ != 0;
    const int64_t n_groups = (n + kEncodeRows - 1) / kEncodeRows;
    for (ItemWalk w(F / 4); w.r < n_groups; w.next()) {
        const int64_t r0 = w.r * kEncodeRows;
        const int32_t f = w.i * 4;
        aes::Float4U v[kEncodeRows];
#pragma unroll
        for (int b = 0; b < kEncodeRows; ++b)
            if (r0 + b < n) v[b] = *reinterpret_cast<const aes::Float4U *>(X + (r0 + b) * ldx + f);
        float sc[4], lo[4], d[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int g = per_tensor ? 0 : f + i;
            sc[i] = scale_in[g];
            lo[i] = affine ? lo_in[g] : 0.0f;
            d[i] = affine ? d_in[g] : 0.0f;
        }
#pragma unroll
        for (int b = 0; b < kEncodeRows; ++b) {
            if (r0 + b >= n) break;
            const float x[4] = {v[b].x, v[b].y, v[b].z, v[b].w};
            uint32_t q = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) q |= encode(x[i], lo[i], d[i], sc[i], affine) << (8 * i);
            reinterpret_cast<aes::Word1U *>(Xq + (r0 + b) * ldq + f)->v = q;
        }
    }
}

__global__ void __launch_bounds__(kBlock)
encode_scalar_kernel(int64_t n, int32_t F, const float *__restrict__ X, int64_t ldx, int affine_, int per_tensor,
                     const float *__restrict__ scale_in, const float *__restrict__ lo_in,
                     const float *__restrict__ d_in, int8_t *__restrict__ Xq, int64_t ldq)
{
    const bool affine = affine_ != 0;
    for (ItemWalk w(F); w.r < n; w.next()) {
        const int g = per_tensor ? 0 : w.i;
        Xq[w.r * ldq + w.i] = static_cast<int8_t>(
            encode(X[w.r * ldx + w.i], affine ? lo_in[g] : 0.0f, affine ? d_in[g] : 0.0f, scale_in[g], affine));
    }
}

// Eq. 2 as a stand-alone pass (the paper's placement: dequantise after loading,
// before the SpMM): x_hat = q * scale_g + zero_g, multiply then add, binary32.
__device__ inline float dequantize_one(uint32_t byte, bool affine, float scale, float zero)
{
    const float q = affine ? static_cast<float>(byte) : static_cast<float>(static_cast<int8_t>(byte));
    float t = q * scale;
    if (affine) t = t + zero;
    return t;
}

// Vector form: groups of kEncodeRows consecutive rows per thread, as in encode_vec_kernel.
__global__ void __launch_bounds__(kBlock)
dequantize_vec_kernel(int64_t n, int32_t F, const int8_t *__restrict__ Xq, int64_t ldq, int affine_, int granularity,
                      const float *__restrict__ scale, const float *__restrict__ zero, int64_t cstride,
                      float *__restrict__ X, int64_t ldx)
{
    const bool affine = affine_ != 0;
    const int64_t n_groups = (n + kEncodeRows - 1) / kEncodeRows;
    for (ItemWalk w(F / 4); w.r < n_groups; w.next()) {
        const int64_t r0 = w.r * kEncodeRows;
        const int32_t f = w.i * 4;
        uint32_t word[kEncodeRows];
#pragma unroll
        for (int b = 0; b < kEncodeRows; ++b)
            if (r0 + b < n) word[b] = reinterpret_cast<const aes::Word1U *>(Xq + (r0 + b) * ldq + f)->v;
#pragma unroll
        for (int b = 0; b < kEncodeRows; ++b) {
            const int64_t r = r0 + b;
            if (r >= n) break;
            float out[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int64_t g = granularity == AES_Q_PER_TENSOR ? 0 : granularity == AES_Q_PER_COLUMN ? f + i : r * cstride;
                out[i] = dequantize_one((word[b] >> (8 * i)) & 0xffu, affine, scale[g], affine ? zero[g] : 0.0f);
            }
            *reinterpret_cast<aes::Float4U *>(X + r * ldx + f) = aes::Float4U{out[0], out[1], out[2], out[3]};
        }
    }
}

__global__ void __launch_bounds__(kBlock)
dequantize_scalar_kernel(int64_t n, int32_t F, const int8_t *__restrict__ Xq, int64_t ldq, int affine_,
                         int granularity, const float *__restrict__ scale, const float *__restrict__ zero,
                         int64_t cstride, float *__restrict__ X, int64_t ldx)
{
    const bool affine = affine_ != 0;
    for (ItemWalk w(F); w.r < n; w.next()) {
        const int64_t g = granularity == AES_Q_PER_TENSOR ? 0 : granularity == AES_Q_PER_COLUMN ? w.i : w.r * cstride;
        X[w.r * ldx + w.i] = dequantize_one(static_cast<uint8_t>(Xq[w.r * ldq + w.i]), affine, scale[g],
                                            affine ? zero[g] : 0.0f);
    }
}

int slabs_for(int64_t n)
{
    int64_t s = aes::ceil_div(n, static_cast<int64_t>(kRowLanes) * 16);
    return static_cast<int>(s < 1 ? 1 : s > kMaxSlabs ? kMaxSlabs : s);
}

constexpr int kRowsPerGroup = 4;
constexpr int64_t kMaxElementwiseBlocks = 256 * 64;   // grid-stride beyond: measured faster than one item per thread

template <int LPR, int VEC>
void launch_rows(int64_t n, int32_t F, const float *X, int64_t ldx, int affine, int8_t *Xq, int64_t ldq,
                 float *scale, float *zero, int64_t cstride, hipStream_t stream)
{
    const unsigned grid = static_cast<unsigned>(aes::ceil_div(n, kBlock / LPR));
    if (VEC == 4 && F <= LPR * VEC) {
        const unsigned bgrid = static_cast<unsigned>(aes::ceil_div(n, static_cast<int64_t>(kBlock / LPR) * kRowsPerGroup));
        quantize_rows_batched_kernel<LPR, kRowsPerGroup><<<dim3(bgrid), dim3(kBlock), 0, stream>>>(n, F, X, ldx, affine, Xq,
                                                                                                   ldq, scale, zero, cstride);
    } else if (F <= LPR * VEC)
        quantize_rows_kernel<LPR, VEC, true><<<dim3(grid), dim3(kBlock), 0, stream>>>(n, F, X, ldx, affine, Xq, ldq, scale, zero, cstride);
    else
        quantize_rows_kernel<LPR, VEC, false><<<dim3(grid), dim3(kBlock), 0, stream>>>(n, F, X, ldx, affine, Xq, ldq, scale, zero, cstride);
}

}  // namespace

extern "C" size_t aes_quantize_workspace_bytes(int64_t n, int32_t F, int32_t granularity)
{
    if (n < 0 || F < 1 || granularity == AES_Q_PER_ROW || granularity == AES_Q_PER_ROW_INLINE) return 0;
    // slab partials (min and max per column) + per-group x_min and range
    return (static_cast<size_t>(slabs_for(n)) * 2 + 2) * static_cast<size_t>(F) * sizeof(float);
}

extern "C" int64_t aes_quantize_inline_ld(int32_t F, int32_t scheme)
{
    if (F < 1 || F >= (1 << 24) || (scheme != AES_Q_AFFINE_FLOOR_U8 && scheme != AES_Q_SYMMETRIC_RNE_I8))
        return aes::fail(AES_ERR_INVALID_ARG, "aes_quantize_inline_ld: F=%d / scheme=%d out of range", (int)F, (int)scheme);
    const int64_t need = aes::q_inline_offset(F) + (scheme == AES_Q_AFFINE_FLOOR_U8 ? 8 : 4);
    return (need + 127) / 128 * 128;
}

extern "C" int aes_quantize_features(int64_t n, int32_t F, const float *X, int64_t ldx,
                                     int32_t scheme, int32_t granularity,
                                     int8_t *Xq, int64_t ldq, float *scale, float *zero,
                                     void *workspace, size_t workspace_bytes, void *stream_)
{
    const char *what = "aes_quantize_features";
    if (n < 0) return aes::fail(AES_ERR_INVALID_ARG, "%s: n=%lld is negative", what, (long long)n);
    if (F < 1 || F >= (1 << 24)) return aes::fail(AES_ERR_INVALID_ARG, "%s: F=%d outside 1..2^24-1", what, (int)F);
    if (ldx < F || ldq < F)
        return aes::fail(AES_ERR_INVALID_ARG, "%s: leading dimension smaller than F (ldx=%lld ldq=%lld F=%d)", what,
                         (long long)ldx, (long long)ldq, (int)F);
    if (scheme != AES_Q_AFFINE_FLOOR_U8 && scheme != AES_Q_SYMMETRIC_RNE_I8)
        return aes::fail(AES_ERR_INVALID_ARG, "%s: unknown scheme %d", what, (int)scheme);
    if (granularity == AES_Q_PER_ROW_FOLDED || granularity < AES_Q_PER_TENSOR || granularity > AES_Q_PER_ROW_INLINE)
        return aes::fail(AES_ERR_INVALID_ARG, "%s: unknown granularity %d", what, (int)granularity);
    const int affine = scheme == AES_Q_AFFINE_FLOOR_U8 ? 1 : 0;
    if (n > 0 && (X == nullptr || Xq == nullptr)) return aes::fail(AES_ERR_INVALID_ARG, "%s: X / Xq is NULL", what);
    int64_t cstride = 1;
    if (granularity == AES_Q_PER_ROW_INLINE) {       // the constants go into the rows of codes
        const float *s = nullptr, *z = nullptr;
        if (int rc = aes::q_inline_constants(what, Xq, ldq, F, affine != 0, s, z, cstride)) return rc;
        scale = const_cast<float *>(s);
        zero = const_cast<float *>(z);
        granularity = AES_Q_PER_ROW;
    }
    if (scale == nullptr && (n > 0 || granularity != AES_Q_PER_ROW))
        return aes::fail(AES_ERR_INVALID_ARG, "%s: scale is NULL", what);
    if (affine && zero == nullptr && (n > 0 || granularity != AES_Q_PER_ROW))
        return aes::fail(AES_ERR_INVALID_ARG, "%s: zero is NULL for the affine scheme", what);
    const size_t need = aes_quantize_workspace_bytes(n, F, granularity);
    if (need > 0 && (workspace == nullptr || workspace_bytes < need))
        return aes::fail(AES_ERR_WORKSPACE, "%s: workspace of %zu bytes needed, %zu given%s", what, need,
                         workspace_bytes, workspace == nullptr ? " (NULL)" : "");
    if (need > 0 && !aes::aligned(workspace, 4))
        return aes::fail(AES_ERR_WORKSPACE, "%s: workspace must be 4-byte aligned", what);
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    const bool vec = F % 4 == 0;      // four features per lane; no alignment needed beyond an element's

    if (granularity == AES_Q_PER_ROW) {
        if (n == 0) return AES_OK;
        if (aes::ceil_div(n, kBlock / 64) > INT32_MAX) return aes::fail(AES_ERR_UNSUPPORTED, "%s: n=%lld too large", what, (long long)n);
        if (!vec) {
            launch_rows<64, 1>(n, F, X, ldx, affine, Xq, ldq, scale, zero, cstride, stream);
        } else {
            int l = aes::pow2_ceil(aes::ceil_div(F, 4));
            l = l < 8 ? 8 : l > 64 ? 64 : l;
            switch (l) {
                case 8: launch_rows<8, 4>(n, F, X, ldx, affine, Xq, ldq, scale, zero, cstride, stream); break;
                case 16: launch_rows<16, 4>(n, F, X, ldx, affine, Xq, ldq, scale, zero, cstride, stream); break;
                case 32: launch_rows<32, 4>(n, F, X, ldx, affine, Xq, ldq, scale, zero, cstride, stream); break;
                default: launch_rows<64, 4>(n, F, X, ldx, affine, Xq, ldq, scale, zero, cstride, stream); break;
            }
        }
        return aes::check_launch("aes_quantize_features/rows");
    }

    const int per_tensor = granularity == AES_Q_PER_TENSOR ? 1 : 0;
    const int n_slabs = slabs_for(n);
    float *partial = static_cast<float *>(workspace);
    float *group_lo = partial + static_cast<size_t>(n_slabs) * 2 * F;
    float *group_d = group_lo + F;
    const unsigned col_blocks = static_cast<unsigned>(aes::ceil_div(F, kColsPerBlock));
    if (col_blocks > 65535u)
        return aes::fail(AES_ERR_UNSUPPORTED, "%s: F=%d too wide for per-column / per-tensor groups", what, (int)F);
    if (n > 0) {
        column_partials_kernel<<<dim3(n_slabs, col_blocks), dim3(kBlock), 0, stream>>>(n, F, X, ldx, affine, partial);
        if (int rc = aes::check_launch("aes_quantize_features/partials")) return rc;
    }
    const int empty = n == 0 ? 1 : 0;
    finalise_kernel<<<dim3(static_cast<unsigned>(aes::ceil_div(F, kFoldCols))), dim3(kBlock), 0, stream>>>(F, empty ? 0 : n_slabs, empty, partial, affine,
                                                                   per_tensor, scale, zero, group_lo, group_d);
    if (int rc = aes::check_launch("aes_quantize_features/finalise")) return rc;
    if (per_tensor) {
        tensor_fold_kernel<<<dim3(1), dim3(kBlock), 0, stream>>>(F, affine, group_lo, group_d, scale, zero);
        if (int rc = aes::check_launch("aes_quantize_features/tensor_fold")) return rc;
    }
    if (n == 0) return AES_OK;
    const int64_t items = vec ? aes::ceil_div(n, kEncodeRows) * (F / 4) : n * F;
    int64_t blocks = aes::ceil_div(items, kBlock);
    if (blocks > kMaxElementwiseBlocks) blocks = kMaxElementwiseBlocks;
    if (vec)
        encode_vec_kernel<<<dim3(static_cast<unsigned>(blocks)), dim3(kBlock), 0, stream>>>(
            n, F, X, ldx, affine, per_tensor, scale, group_lo, group_d, Xq, ldq);
    else
        encode_scalar_kernel<<<dim3(static_cast<unsigned>(blocks)), dim3(kBlock), 0, stream>>>(
            n, F, X, ldx, affine, per_tensor, scale, group_lo, group_d, Xq, ldq);
    return aes::check_launch("aes_quantize_features/encode");
}

extern "C" int aes_dequantize_features(int64_t n, int32_t F, const int8_t *Xq, int64_t ldq,
                                       int32_t scheme, int32_t granularity,
                                       const float *scale, const float *zero,
                                       float *X, int64_t ldx, void *stream_)
{
    const char *what = "aes_dequantize_features";
    if (n < 0) return aes::fail(AES_ERR_INVALID_ARG, "%s: n=%lld is negative", what, (long long)n);
    if (F < 1 || F >= (1 << 24)) return aes::fail(AES_ERR_INVALID_ARG, "%s: F=%d outside 1..2^24-1", what, (int)F);
    if (ldx < F || ldq < F)
        return aes::fail(AES_ERR_INVALID_ARG, "%s: leading dimension smaller than F (ldx=%lld ldq=%lld F=%d)", what,
                         (long long)ldx, (long long)ldq, (int)F);
    if (scheme != AES_Q_AFFINE_FLOOR_U8 && scheme != AES_Q_SYMMETRIC_RNE_I8)
        return aes::fail(AES_ERR_INVALID_ARG, "%s: unknown scheme %d", what, (int)scheme);
    if (granularity == AES_Q_PER_ROW_FOLDED || granularity < AES_Q_PER_TENSOR || granularity > AES_Q_PER_ROW_INLINE)
        return aes::fail(AES_ERR_INVALID_ARG, "%s: unknown granularity %d", what, (int)granularity);
    const int affine = scheme == AES_Q_AFFINE_FLOOR_U8 ? 1 : 0;
    int64_t cstride = 1;
    if (granularity == AES_Q_PER_ROW_INLINE) {
        if (int rc = aes::q_inline_constants(what, Xq, ldq, F, affine != 0, scale, zero, cstride)) return rc;
        granularity = AES_Q_PER_ROW;
    }
    if (scale == nullptr || (affine && zero == nullptr))
        return aes::fail(AES_ERR_INVALID_ARG, "%s: scale (or zero, affine scheme) is NULL", what);
    if (n == 0) return AES_OK;
    if (Xq == nullptr || X == nullptr) return aes::fail(AES_ERR_INVALID_ARG, "%s: Xq / X is NULL", what);
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    const bool vec = F % 4 == 0;
    const int64_t items = vec ? aes::ceil_div(n, kEncodeRows) * (F / 4) : n * F;
    int64_t blocks = aes::ceil_div(items, kBlock);
    if (blocks > kMaxElementwiseBlocks) blocks = kMaxElementwiseBlocks;
    if (vec)
        dequantize_vec_kernel<<<dim3(static_cast<unsigned>(blocks)), dim3(kBlock), 0, stream>>>(
            n, F, Xq, ldq, affine, granularity, scale, zero, cstride, X, ldx);
    else
        dequantize_scalar_kernel<<<dim3(static_cast<unsigned>(blocks)), dim3(kBlock), 0, stream>>>(
            n, F, Xq, ldq, affine, granularity, scale, zero, cstride, X, ldx);
    return aes::check_launch(what);
}
