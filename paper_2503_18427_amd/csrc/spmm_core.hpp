// Device-side core of the multiply stage, shared by the SpMM kernels and the fused
// GCN-layer kernel: slot sources, feature loaders, the tile accumulation loop.
//
// Method: AES-SpMM Sec. 3.2 Algorithm 1 (accumulation loop), Sec. 2.3 Eq. 2
// (dequantisation inside the gather).
#pragma once

#include "aes_common.hpp"
#include "aes_sampling.hpp"

namespace aes {

constexpr int kTile = 64;          // slots staged in LDS per group per round

// How the constants of Eq. 2 reach an output of the 8-bit path.  Known at compile time, so that the
// epilogue of a row is straight-line code: one vector load of constants per lane at most.
enum QMode {
    kQNone = 0,      // float32 features: no constants
    kQRowScale = 1,  // one pair per node (= per gathered row): folded into the staged edge value
    kQTensor = 2,    // one pair for the whole matrix: applied once per output
    kQColumn = 3,    // one pair per feature column: applied once per output
    kQFolded = 4,    // per-node pairs already multiplied into the plan's values; zero = row bias or NULL
    kQRowInGather = 5  // one pair per node, stored behind the node's codes inside the row the lane group gathers
                       // anyway: the lane that holds those words hands them to the group by a cross-lane read,
                       // so the constants cost neither a memory request nor a step in the chain of dependent loads
};

// Where a row's (col, val) slots come from: a materialised plan (FUSED = false: the
// three arrays are s_rowptr / s_col / s_val) or the CSR matrix itself, sampled on
// the fly by Table 1 and Eq. 3 (FUSED = true).
struct SlotSource {
    const int64_t *rowptr;
    const int32_t *col;
    const float *val;
    int32_t W;
    int32_t strategy;
    uint64_t seed;
};

struct QParams {
    const float *scale;   // kQRowScale: indexed by column of A (= row of X); kQFolded: unused
    const float *zero;    // NULL for signed codes; kQFolded: the row bias, or NULL
    int64_t node_stride;  // kQRowScale: floats between two nodes' constants (1: plain arrays; ldq / 4: constants
                          // kept inside the rows of codes)
    int32_t inline_off;   // constants inside the rows: byte offset of the scale in a row (the zero point follows); else -1
};

// Unsigned codes carry a zero point (x_hat = q*scale + zero), signed codes do not (x_hat = q*scale).
// With folded constants the zero points already sit in the row bias: no per-slot sums are needed.
template <typename Feat, int QMODE>
struct QTraits {
    static constexpr bool kQuant = QMODE != kQNone;
    static constexpr bool kAffine = kQuant && QMODE != kQFolded && !Feat::kSigned;
    // The zero-point sum is collected by the lanes that stage the slots (one share each, added over the group
    // before the epilogue), except where every lane sees every slot's constants itself.
    static constexpr bool kSideOverLanes = kAffine && QMODE != kQRowInGather;
};

// The scheme / granularity / scale / zero arguments of an 8-bit entry point, checked and turned into
// the kernels' QParams; `granularity` comes back as the one that selects the kernel (constants inside
// the rows are per-node constants read with a stride).
inline int resolve_q8(const char *what, bool fused, const int8_t *Xq, int64_t ldq, int32_t F, int32_t scheme,
                      int32_t &granularity, const float *scale, const float *zero, QParams &qp)
{
    if (scheme != AES_Q_AFFINE_FLOOR_U8 && scheme != AES_Q_SYMMETRIC_RNE_I8)
        return fail(AES_ERR_INVALID_ARG, "%s: unknown scheme %d", what, (int)scheme);
    if (granularity < AES_Q_PER_TENSOR || granularity > AES_Q_PER_ROW_INLINE)
        return fail(AES_ERR_INVALID_ARG, "%s: unknown granularity %d", what, (int)granularity);
    const bool affine = scheme == AES_Q_AFFINE_FLOOR_U8;
    const bool folded = granularity == AES_Q_PER_ROW_FOLDED;
    if (fused && folded) return fail(AES_ERR_INVALID_ARG, "%s: folded constants need a materialised plan", what);
    int64_t stride = 1;
    if (granularity == AES_Q_PER_ROW_INLINE) {
        if (int rc = q_inline_constants(what, Xq, ldq, F, affine, scale, zero, stride)) return rc;
        granularity = AES_Q_PER_ROW;
    }
    if (!folded && scale == nullptr) return fail(AES_ERR_INVALID_ARG, "%s: scale is NULL", what);
    if (affine && zero == nullptr)
        return fail(AES_ERR_INVALID_ARG, "%s: zero (the row bias, for folded constants) is NULL for the affine scheme", what);
    // Unsigned codes (the affine scheme) use zero; signed codes ignore it.  Folded: zero is the row
    // bias the fold pass wrote for the affine scheme, and nothing otherwise.
    qp = QParams{scale, affine ? zero : nullptr, stride,
                 stride == 1 ? -1 : static_cast<int32_t>(q_inline_offset(F))};
    return AES_OK;
}

// acc + a * b in the accumulator's precision: one fused multiply-add in float32 for
// ordinary rows, in float64 for the long-row variant (whose sums run over up to
// millions of terms and would otherwise outgrow float32's relative error target).
__device__ inline float fma_acc(float a, float b, float acc) { return __builtin_fmaf(a, b, acc); }
__device__ inline double fma_acc(float a, float b, double acc)
{
    return __builtin_fma(static_cast<double>(a), static_cast<double>(b), acc);
}

// ---- feature loaders: VEC consecutive features of one row of X --------------
// fma(acc, v, x) adds v * feature to acc for each of the VEC features.
//
// The vector loads and stores only assume the alignment of one element (Float4U / Word1U),
// so any leading dimension takes the vector path.
template <int VEC_> struct FeatF32;
template <> struct FeatF32<4> {
    static constexpr int VEC = 4;
    static constexpr bool kSigned = true;
    using elem_t = float;
    using raw_t = Float4U;
    static __device__ inline raw_t load(const elem_t *p) { return *reinterpret_cast<const Float4U *>(p); }
    // The first nv (1..3) features only, zeros for the rest: the last lane of a row whose length is not
    // a multiple of four.
    static __device__ inline raw_t load_n(const elem_t *p, int nv)
    {
        raw_t x = {p[0], 0.0f, 0.0f, 0.0f};
        if (nv > 1) x.y = p[1];
        if (nv > 2) x.z = p[2];
        return x;
    }
    template <typename AccT>
    static __device__ inline void fma(AccT (&acc)[4], float v, const raw_t &x)
    {
        acc[0] = fma_acc(v, x.x, acc[0]);
        acc[1] = fma_acc(v, x.y, acc[1]);
        acc[2] = fma_acc(v, x.z, acc[2]);
        acc[3] = fma_acc(v, x.w, acc[3]);
    }
};
template <> struct FeatF32<1> {
    static constexpr int VEC = 1;
    static constexpr bool kSigned = true;
    using elem_t = float;
    using raw_t = float;
    static __device__ inline raw_t load(const elem_t *p) { return *p; }
    static __device__ inline raw_t load_n(const elem_t *p, int) { return *p; }
    template <typename AccT>
    static __device__ inline void fma(AccT (&acc)[1], float v, const raw_t &x) { acc[0] = fma_acc(v, x, acc[0]); }
};

// Four packed bytes -> four floats: one conversion instruction per byte, which selects its byte and, for
// signed codes, sign-extends it (v_cvt_f32_ubyteN / v_cvt_f32_i32 with a byte selector).
template <bool SIGNED, typename AccT>
__device__ inline void fma_bytes(AccT *acc, float v, uint32_t w)
{
    if (SIGNED) {
        acc[0] = fma_acc(v, static_cast<float>(static_cast<int8_t>(w & 0xffu)), acc[0]);
        acc[1] = fma_acc(v, static_cast<float>(static_cast<int8_t>((w >> 8) & 0xffu)), acc[1]);
        acc[2] = fma_acc(v, static_cast<float>(static_cast<int8_t>((w >> 16) & 0xffu)), acc[2]);
        acc[3] = fma_acc(v, static_cast<float>(static_cast<int8_t>(w >> 24)), acc[3]);
    } else {
        acc[0] = fma_acc(v, static_cast<float>(w & 0xffu), acc[0]);
        acc[1] = fma_acc(v, static_cast<float>((w >> 8) & 0xffu), acc[1]);
        acc[2] = fma_acc(v, static_cast<float>((w >> 16) & 0xffu), acc[2]);
        acc[3] = fma_acc(v, static_cast<float>(w >> 24), acc[3]);
    }
}

template <int VEC_, bool SIGNED> struct FeatQ8;
template <bool SIGNED> struct FeatQ8<4, SIGNED> {
    static constexpr int VEC = 4;
    static constexpr bool kSigned = SIGNED;
    using elem_t = int8_t;
    using raw_t = uint32_t;
    static __device__ inline raw_t load(const elem_t *p) { return reinterpret_cast<const Word1U *>(p)->v; }
    static __device__ inline raw_t load_n(const elem_t *p, int nv)     // missing codes read as 0
    {
        uint32_t w = static_cast<uint8_t>(p[0]);
        if (nv > 1) w |= static_cast<uint32_t>(static_cast<uint8_t>(p[1])) << 8;
        if (nv > 2) w |= static_cast<uint32_t>(static_cast<uint8_t>(p[2])) << 16;
        return w;
    }
    template <typename AccT>
    static __device__ inline void fma(AccT (&acc)[4], float v, const raw_t &x) { fma_bytes<SIGNED>(acc, v, x); }
};
template <bool SIGNED> struct FeatQ8<1, SIGNED> {
    static constexpr int VEC = 1;
    static constexpr bool kSigned = SIGNED;
    using elem_t = int8_t;
    using raw_t = int8_t;
    static __device__ inline raw_t load(const elem_t *p) { return *p; }
    static __device__ inline raw_t load_n(const elem_t *p, int) { return *p; }
    template <typename AccT>
    static __device__ inline void fma(AccT (&acc)[1], float v, const raw_t &x)
    {
        float q = SIGNED ? static_cast<float>(x) : static_cast<float>(static_cast<uint8_t>(x));
        acc[0] = fma_acc(v, q, acc[0]);
    }
};

// Orders this wavefront's LDS traffic: earlier LDS accesses of any lane are
// complete (and not moved by the compiler) before later ones start.
__device__ inline void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// ---- the kernel ---------------------------------------------------------------
// What a lane group needs to know about its row.
struct RowInfo {
    int64_t k_begin;     // first slot (plan) or first CSR entry (fused)
    int64_t n_slots;
    int64_t row_nnz;     // fused only: entries of the CSR row
    int32_t samp_n;      // fused, sampled row: N and sample_cnt of Table 1, per-row offset
    int32_t samp_cnt;
    uint32_t s_r;
    bool sampled;
};

template <bool FUSED>
__device__ inline RowInfo row_info(const SlotSource &src, int64_t r)
{
    RowInfo ri;
    ri.k_begin = src.rowptr[r];
    ri.n_slots = src.rowptr[r + 1] - ri.k_begin;
    ri.row_nnz = ri.n_slots;
    ri.sampled = false;
    ri.samp_n = 0;
    ri.samp_cnt = 1;
    ri.s_r = 0;
    if (FUSED && src.W != 0 && ri.row_nnz > src.W) {
        ri.sampled = true;
        aes::sample_strategy(ri.row_nnz, src.W, src.strategy, ri.samp_n, ri.samp_cnt);
        ri.n_slots = static_cast<int64_t>(ri.samp_n) * ri.samp_cnt;
        ri.s_r = aes::row_offset(src.seed, r);
    }
    return ri;
}

// Stages slots t0 .. t0 + m - 1 of the row in the group's LDS tile: a coalesced load of the (col, val)
// pairs (from the plan, or sampled on the fly from the CSR row), per-node 8-bit constants folded into
// the value, then the fences that make the tile visible to the whole group.
template <int LPR, typename Feat, int QMODE, bool FUSED, typename AccT>
__device__ __forceinline__ void stage_tile(const SlotSource &src, const RowInfo &ri, int2 *my_stage, int lane,
                                           const QParams &qp, int64_t t0, int m, AccT &side)
{
    wave_lds_sync();                                 // previous tile fully consumed
#pragma unroll
    for (int s = lane; s < kTile; s += LPR) {
        if (s < m) {
            int64_t e = ri.k_begin + t0 + s;
            if (FUSED && ri.sampled)
                e = aes::sampled_entry(ri.k_begin, ri.row_nnz, ri.samp_n, ri.samp_cnt, ri.s_r,
                                       static_cast<int32_t>(t0) + s);
            const int32_t c = src.col[e];
            float v = src.val[e];
            if constexpr (QMODE == kQRowScale) {
                const uint64_t g = static_cast<uint64_t>(static_cast<uint32_t>(c)) * static_cast<uint64_t>(qp.node_stride);
                if constexpr (QTraits<Feat, QMODE>::kAffine) side = fma_acc(v, qp.zero[g], side);
                v *= qp.scale[g];
            } else if constexpr (QTraits<Feat, QMODE>::kSideOverLanes) {
                side += v;
            }
            my_stage[s] = make_int2(c, __float_as_int(v));
        }
    }
    wave_lds_sync();                                 // tile visible to the whole group
}

// Adds the row's tiles first_tile, first_tile + tile_step, ... into acc (one chunk of
// features).  side collects the zero-point sum the affine 8-bit epilogue needs.
// PARTIAL: a lane may own fewer than VEC valid features (nv of them: the end of a row whose length is
// not a multiple of VEC); such a lane loads them one by one.
template <int LPR, int UNROLL, typename Feat, int QMODE, bool FUSED, typename AccT, bool PARTIAL = false>
__device__ __forceinline__ void accumulate_tiles(const SlotSource &src, const RowInfo &ri, int2 *my_stage, int lane,
                                                 bool lane_on, const typename Feat::elem_t *__restrict__ X,
                                                 int64_t ldx, int32_t f, const QParams &qp, int64_t first_tile,
                                                 int64_t tile_step, AccT (&acc)[Feat::VEC], AccT &side,
                                                 int nv = Feat::VEC)
{
    auto load_feat = [&](const typename Feat::elem_t *p) {
        if constexpr (PARTIAL) {
            if (nv != Feat::VEC) return Feat::load_n(p, nv);
        }
        return Feat::load(p);
    };
    // Column indices are non-negative and the host has checked ldx < 2^32: the row offset is one
    // 32 x 32 -> 64-bit multiply-add per gather instead of a sign-extended 64 x 64-bit product.
    const uint32_t ld = static_cast<uint32_t>(ldx);
    const typename Feat::elem_t *const x_lane = X + f;
    auto row_of = [&](int32_t c) { return x_lane + static_cast<uint64_t>(static_cast<uint32_t>(c)) * ld; };
    // kQRowInGather: lane_on covers the lanes up to the constants, which the lanes k_lane (scale) and
    // k_lane + 1 (zero point) of the group hold as their gathered word.
    const int k_lane = QMODE == kQRowInGather ? qp.inline_off / Feat::VEC : 0;
    auto consume = [&](const int2 &slot, const typename Feat::raw_t &x) {
        float v = __int_as_float(slot.y);
        if constexpr (QMODE == kQRowInGather) {
            static_assert(QMODE != kQRowInGather || (sizeof(typename Feat::raw_t) == 4 && !PARTIAL), "four codes per lane");
            const float word = __uint_as_float(static_cast<uint32_t>(x));
            if constexpr (QTraits<Feat, QMODE>::kAffine) side = fma_acc(v, __shfl(word, k_lane + 1, LPR), side);
            v *= __shfl(word, k_lane, LPR);
        }
        Feat::fma(acc, v, x);
    };
    for (int64_t t0 = first_tile * kTile; t0 < ri.n_slots; t0 += tile_step * kTile) {
        const int m = static_cast<int>(ri.n_slots - t0 < kTile ? ri.n_slots - t0 : kTile);
        stage_tile<LPR, Feat, QMODE, FUSED, AccT>(src, ri, my_stage, lane, qp, t0, m, side);
        if (lane_on) {
            // UNROLL gathers are issued back to back before the first one is consumed.
            int k = 0;
            for (; k + UNROLL <= m; k += UNROLL) {
                int2 cv[UNROLL];
                typename Feat::raw_t x[UNROLL];
#pragma unroll
                for (int u = 0; u < UNROLL; ++u) cv[u] = my_stage[k + u];
#pragma unroll
                for (int u = 0; u < UNROLL; ++u) x[u] = load_feat(row_of(cv[u].x));
#pragma unroll
                for (int u = 0; u < UNROLL; ++u) consume(cv[u], x[u]);
            }
            // Ragged last round: the missing slots are predicated off (value 0, no load), so
            // short rows and row tails keep their gathers in flight together as well.
            if (k < m) {
                int2 cv[UNROLL];
                typename Feat::raw_t x[UNROLL];
#pragma unroll
                for (int u = 0; u < UNROLL; ++u) cv[u] = (k + u < m) ? my_stage[k + u] : make_int2(-1, 0);
#pragma unroll
                for (int u = 0; u < UNROLL; ++u) {
                    x[u] = typename Feat::raw_t{};
                    if (cv[u].x >= 0) x[u] = load_feat(row_of(cv[u].x));
                }
#pragma unroll
                for (int u = 0; u < UNROLL; ++u) consume(cv[u], x[u]);
            }
        }
    }
}

// The same for feature rows wider than one pass of the lane group: a lane owns NV vectors, LPR * VEC
// features apart (f, f + LPR*VEC, ...; on[j] says which of them exist), and gathers all of them for a
// slot together.  The slots are staged once for the NV * LPR * VEC features, and a gathered row is
// read as one contiguous piece instead of once per pass.
template <int LPR, int UNROLL, typename Feat, int QMODE, bool FUSED, typename AccT, int NV>
__device__ __forceinline__ void accumulate_tiles_wide(const SlotSource &src, const RowInfo &ri, int2 *my_stage, int lane,
                                                      const bool (&on)[NV], const typename Feat::elem_t *__restrict__ X,
                                                      int64_t ldx, int32_t f, const QParams &qp, int64_t first_tile,
                                                      int64_t tile_step, AccT (&acc)[NV][Feat::VEC], AccT &side)
{
    constexpr int kApart = LPR * Feat::VEC;
    const uint32_t ld = static_cast<uint32_t>(ldx);
    const typename Feat::elem_t *const x_lane = X + f;
    auto row_of = [&](int32_t c) { return x_lane + static_cast<uint64_t>(static_cast<uint32_t>(c)) * ld; };
    // kQRowInGather: which of a lane's NV words, in which lane, is the node's scale / zero point
    const int k_off = QMODE == kQRowInGather ? qp.inline_off : 0;
    const int ks_vec = k_off / kApart, ks_lane = (k_off % kApart) / Feat::VEC;
    const int kz_vec = (k_off + 4) / kApart, kz_lane = ((k_off + 4) % kApart) / Feat::VEC;
    for (int64_t t0 = first_tile * kTile; t0 < ri.n_slots; t0 += tile_step * kTile) {
        const int m = static_cast<int>(ri.n_slots - t0 < kTile ? ri.n_slots - t0 : kTile);
        stage_tile<LPR, Feat, QMODE, FUSED, AccT>(src, ri, my_stage, lane, qp, t0, m, side);
        if (on[0]) {
            for (int k = 0; k < m; k += UNROLL) {
                int2 cv[UNROLL];
                typename Feat::raw_t x[UNROLL][NV];
#pragma unroll
                for (int u = 0; u < UNROLL; ++u) cv[u] = (k + u < m) ? my_stage[k + u] : make_int2(-1, 0);
#pragma unroll
                for (int u = 0; u < UNROLL; ++u)
#pragma unroll
                    for (int j = 0; j < NV; ++j) {
                        x[u][j] = typename Feat::raw_t{};
                        if (cv[u].x >= 0 && on[j]) x[u][j] = Feat::load(row_of(cv[u].x) + j * kApart);
                    }
#pragma unroll
                for (int u = 0; u < UNROLL; ++u) {
                    float v = __int_as_float(cv[u].y);
                    if constexpr (QMODE == kQRowInGather) {
                        static_assert(QMODE != kQRowInGather || sizeof(typename Feat::raw_t) == 4, "four codes per lane");
                        uint32_t ws = static_cast<uint32_t>(x[u][0]), wz = ws;
#pragma unroll
                        for (int j = 1; j < NV; ++j) {
                            ws = j == ks_vec ? static_cast<uint32_t>(x[u][j]) : ws;
                            wz = j == kz_vec ? static_cast<uint32_t>(x[u][j]) : wz;
                        }
                        if constexpr (QTraits<Feat, QMODE>::kAffine)
                            side = fma_acc(v, __shfl(__uint_as_float(wz), kz_lane, LPR), side);
                        v *= __shfl(__uint_as_float(ws), ks_lane, LPR);
                    }
#pragma unroll
                    for (int j = 0; j < NV; ++j) Feat::fma(acc[j], v, x[u][j]);
                }
            }
        }
    }
}

// The constants one lane needs for the epilogue of its VEC features: fetched by one (vector) load per
// array, not one dependent load per feature - on short rows the epilogue's memory round trips are a
// large part of a row's life.
template <typename Feat, int QMODE>
struct LaneConstants {
    float scale[Feat::VEC];
    float zero[Feat::VEC];
    bool bias;            // kQFolded: the plan comes with a row bias (held in zero[])
};

template <typename Feat, int QMODE>
__device__ __forceinline__ void load_lane_constants(const QParams &qp, int32_t f, bool lane_on, int64_t r,
                                                    LaneConstants<Feat, QMODE> &k, int nv = Feat::VEC)
{
    constexpr int VEC = Feat::VEC;
    constexpr bool AFFINE = QTraits<Feat, QMODE>::kAffine;
#pragma unroll
    for (int i = 0; i < VEC; ++i) {
        k.scale[i] = 1.0f;
        k.zero[i] = 0.0f;
    }
    k.bias = false;
    if constexpr (QMODE == kQTensor) {
        const float s = qp.scale[0];                 // uniform address: a scalar load
        float z = 0.0f;
        if constexpr (AFFINE) z = qp.zero[0];
#pragma unroll
        for (int i = 0; i < VEC; ++i) {
            k.scale[i] = s;
            k.zero[i] = z;
        }
    } else if constexpr (QMODE == kQColumn) {
        if (lane_on) {
            bool fetched = false;
            if constexpr (VEC == 4) {
                if (nv == VEC) {
                    const Float4U s = *reinterpret_cast<const Float4U *>(qp.scale + f);
                    k.scale[0] = s.x; k.scale[1] = s.y; k.scale[2] = s.z; k.scale[3] = s.w;
                    if constexpr (AFFINE) {
                        const Float4U z = *reinterpret_cast<const Float4U *>(qp.zero + f);
                        k.zero[0] = z.x; k.zero[1] = z.y; k.zero[2] = z.z; k.zero[3] = z.w;
                    }
                    fetched = true;
                }
            }
            if (!fetched) {                           // one column per lane, or the ragged end of a row
#pragma unroll
                for (int i = 0; i < VEC; ++i) {
                    if (i < nv) {
                        k.scale[i] = qp.scale[f + i];
                        if constexpr (AFFINE) k.zero[i] = qp.zero[f + i];
                    }
                }
            }
        }
    } else if constexpr (QMODE == kQFolded) {
        if (qp.zero != nullptr) {                    // uniform: the plan carries a row bias or it does not
            const float b = qp.zero[r];
            k.bias = true;
#pragma unroll
            for (int i = 0; i < VEC; ++i) k.zero[i] = b;
        }
    }
}

// Applies the 8-bit group constants to one chunk of a row:
// out[] holds the finished float32 values of features f .. f + VEC - 1 of row r.
// `side` must already be summed over the lanes of the group.
//   per tensor / column: Y = scale_c * sum(v*q) + zero_c * sum(v)
//   per row            : Y = sum((v*scale_col)*q) + sum(v*zero_col)
//   folded             : Y = sum(v'*q) + bias_r
template <typename Feat, int QMODE, typename AccT>
__device__ __forceinline__ void finish_values(const AccT (&acc_in)[Feat::VEC], AccT side_in,
                                              const LaneConstants<Feat, QMODE> &k, float (&out)[Feat::VEC])
{
    constexpr int VEC = Feat::VEC;
    constexpr bool AFFINE = QTraits<Feat, QMODE>::kAffine;
    const float side = static_cast<float>(side_in);
#pragma unroll
    for (int i = 0; i < VEC; ++i) {
        out[i] = static_cast<float>(acc_in[i]);
        if constexpr (QMODE == kQRowScale || QMODE == kQRowInGather) {
            if constexpr (AFFINE) out[i] += side;
        } else if constexpr (QMODE == kQFolded) {
            if (k.bias) out[i] += k.zero[i];
        } else if constexpr (QMODE == kQTensor || QMODE == kQColumn) {
            out[i] *= k.scale[i];
            if constexpr (AFFINE) out[i] = __builtin_fmaf(side, k.zero[i], out[i]);
        }
    }
}

// finish_values, then the store of the chunk to Y[r, f ...] (16-byte streaming stores, 4-byte aligned, on the vector paths).
template <typename Feat, int QMODE, typename AccT>
__device__ __forceinline__ void finish_chunk(const AccT (&acc_in)[Feat::VEC], AccT side_in, bool lane_on,
                                             const LaneConstants<Feat, QMODE> &k, float *__restrict__ y)
{
    constexpr int VEC = Feat::VEC;
    if (!lane_on) return;
    float acc[VEC];
    finish_values<Feat, QMODE, AccT>(acc_in, side_in, k, acc);
    if constexpr (VEC % 4 == 0) {
        // Streaming (non-temporal) stores: Y is written once and never read here, and as ordinary stores its
        // lines take L2 and Infinity Cache space from the feature rows the gathers re-use (-17 % on the
        // 8-bit multiply of rmat20 W = 16, where Y is 40 % of the traffic; -2 % on products_like).
        typedef float f4 __attribute__((ext_vector_type(4), aligned(4)));
#pragma unroll
        for (int i = 0; i < VEC; i += 4) {
            const f4 v = {acc[i], acc[i + 1], acc[i + 2], acc[i + 3]};
            __builtin_nontemporal_store(v, reinterpret_cast<f4 *>(y + i));
        }
    } else {
#pragma unroll
        for (int i = 0; i < VEC; ++i) y[i] = acc[i];
    }
}

template <int LPR, typename AccT>
__device__ __forceinline__ AccT group_sum(AccT v)
{
#pragma unroll
    for (int d = LPR / 2; d >= 1; d >>= 1) v += __shfl_xor(v, d, LPR);
    return v;
}

}  // namespace aes
