// aes_gcn_layer_f32 / aes_gcn_layer_q8: aggregation and combination of one GNN layer in one
// kernel, H = (A_s X) Theta (X float32, or 8-bit codes dequantised inside the gather), on gfx950.
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
constexpr int kMaxFeatures = 256;    // the specialised kernel: one chunk of four features per lane, at most 64 lanes

typedef float floatx16 __attribute__((ext_vector_type(16)));

// Feat / QMODE as in the SpMM kernel: float32 features, or 8-bit codes dequantised in the gather.
// The register budget is set per variant.  float32: at least four waves per SIMD (the gather phase needs
// the occupancy, and the register allocator would otherwise spend the whole file on the unrolled MFMA
// phase).  8-bit: its gather phase is short and bound by latency, so it wants six to seven waves per SIMD
// more than it wants a deep Theta prefetch (kChunk below): 65-75 registers, no spills.
template <int LPR, typename Feat, int QMODE>
__global__ void __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(QMODE != kQNone ? 6 : 4)))
gcn_layer_kernel(int64_t n_rows, SlotSource src, const typename Feat::elem_t *__restrict__ X, int64_t ldx, int32_t F,
                 QParams qp, const float *__restrict__ Theta, int64_t ldt, int32_t Fo, float *__restrict__ H,
                 int64_t ldh)
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
    // With a node's constants taken from the gather itself, the lanes up to those words gather too.
    const bool gather_on = QMODE == kQRowInGather ? f < qp.inline_off + (QTraits<Feat, QMODE>::kAffine ? 8 : 4) : lane_on;
    for (int rr = wave * kGroups + group; rr < kTileRows; rr += kGroupsPerBlock) {
        const int64_t r = row0 + rr;
        float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        float side = 0.0f;
        LaneConstants<Feat, QMODE> k;
        if (r < n_rows) {
            const RowInfo ri = row_info<false>(src, r);
            accumulate_tiles<LPR, 8, Feat, QMODE, false, float>(src, ri, stage[wave][group], lane, gather_on, X, ldx, f, qp,
                                                                0, 1, acc, side);
            load_lane_constants<Feat, QMODE>(qp, f, lane_on, r, k);
        }
        if constexpr (QTraits<Feat, QMODE>::kSideOverLanes) side = group_sum<LPR, float>(side);
        if (lane_on) {
            float y[4] = {0.0f, 0.0f, 0.0f, 0.0f};
            if (r < n_rows) finish_values<Feat, QMODE, float>(acc, side, k, y);
#pragma unroll
            for (int i = 0; i < 4; ++i) ys[rr * y_stride + f + i] = y[i];
        }
    }
    // ---- combination: H_tile (32 x Fo) = ys (32 x F) * Theta (F x Fo) on the matrix cores ----
    // v_mfma_f32_32x32x2_f32: lane l supplies A[l % 32][l / 32] and B[l / 32][l % 32];
    // it receives D[8 * (v / 4) + 4 * (l / 32) + v % 4][l % 32] in result register v.
    //
    // A wave owns the 32-column blocks nb = wave, wave + 4, ...  Its Theta operands are held in
    // registers in chunks of kChunk MFMAs (2 * kChunk rows of Theta): the first two chunks are requested
    // BEFORE the workgroup barrier, right after the wave's last gather, so their latency - long,
    // because the vector memory path is saturated by the gathers of the other workgroups - passes
    // while the wave waits for the rest of the tile; a chunk's registers are refilled as soon as it
    // has been consumed.  The gather loop's registers are dead by then, so this costs no occupancy.
    constexpr int kChunk = QMODE != kQNone ? 8 : 32;
    const int i = wl % 32, h = wl / 32;
    const int n_chunks = (F + 2 * kChunk - 1) / (2 * kChunk);
    float b0[kChunk], b1[kChunk];
    // Address = wave-uniform row base (scalar registers) + one 32-bit per-lane offset, so the
    // 32 loads of a chunk share a single address register.
    auto load_b = [&](int nb, int chunk, float (&b)[kChunk]) {
        const int col = nb * 32 + i;
        const bool col_on = col < Fo;
        const uint32_t lane_off = static_cast<uint32_t>(h) * static_cast<uint32_t>(ldt) + (col_on ? col : 0);
#pragma unroll
        for (int u = 0; u < kChunk; ++u) {
            const int k_even = chunk * 2 * kChunk + 2 * u;              // uniform; this lane reads row k_even + h
            const float *row_base = Theta + static_cast<int64_t>(k_even) * ldt;
            b[u] = (k_even + h < F && col_on) ? row_base[lane_off] : 0.0f;
        }
    };
    if (wave * 32 < Fo) {
        load_b(wave, 0, b0);
        if (n_chunks > 1) load_b(wave, 1, b1);
    }
    __syncthreads();

    floatx16 c;
    auto run_chunk = [&](int chunk, const float (&b)[kChunk]) {
        constexpr int kBatch = 8;                    // A operands come from LDS, eight reads ahead
        float a_cur[kBatch], a_nxt[kBatch];
        auto load_a = [&](int u0, float (&a)[kBatch]) {
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                const int k = chunk * 2 * kChunk + 2 * (u0 + u) + h;
                a[u] = k < F ? ys[i * y_stride + k] : 0.0f;
            }
        };
        load_a(0, a_cur);
#pragma unroll
        for (int u0 = 0; u0 < kChunk; u0 += kBatch) {
            const bool more = u0 + kBatch < kChunk;  // known at compile time: the loop is unrolled
            if (more) load_a(u0 + kBatch, a_nxt);
            __builtin_amdgcn_sched_barrier(0);       // keep the read-ahead at one batch: registers
#pragma unroll
            for (int u = 0; u < kBatch; ++u) c = __builtin_amdgcn_mfma_f32_32x32x2f32(a_cur[u], b[u0 + u], c, 0, 0, 0);
            if (more) {
#pragma unroll
                for (int u = 0; u < kBatch; ++u) a_cur[u] = a_nxt[u];
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    for (int nb = wave; nb * 32 < Fo; nb += kWavesPerBlock) {
#pragma unroll
        for (int v = 0; v < 16; ++v) c[v] = 0.0f;
        for (int chunk = 0; chunk < n_chunks; chunk += 2) {
            run_chunk(chunk, b0);
            if (chunk + 2 < n_chunks) load_b(nb, chunk + 2, b0);
            __builtin_amdgcn_sched_barrier(0);
            if (chunk + 1 < n_chunks) {
                run_chunk(chunk + 1, b1);
                if (chunk + 3 < n_chunks) load_b(nb, chunk + 3, b1);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        const int col = nb * 32 + i;
        if (col < Fo) {
            const uint32_t out_off = static_cast<uint32_t>(4 * h) * static_cast<uint32_t>(ldh) + col;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t r_base = row0 + 8 * (v / 4) + (v % 4);     // uniform; this lane's row is r_base + 4h
                // streaming store: H is written once and must not take cache space from the gathered rows
                if (r_base + 4 * h < n_rows) __builtin_nontemporal_store(c[v], &(H + r_base * ldh)[out_off]);
            }
        }
        const int next = nb + kWavesPerBlock;        // a further column block of this wave: its first chunks
        if (next * 32 < Fo) {
            load_b(next, 0, b0);
            if (n_chunks > 1) load_b(next, 1, b1);
        }
    }
}

template <int LPR, typename Feat, int QMODE>
int launch_gcn(const char *what, int64_t n_rows, const SlotSource &src, const typename Feat::elem_t *X, int64_t ldx,
               int32_t F, QParams qp, const float *Theta, int64_t ldt, int32_t Fo, float *H, int64_t ldh,
               hipStream_t stream)
{
    const int64_t grid = ceil_div(n_rows, kTileRows);
    if (grid > INT32_MAX) return fail(AES_ERR_UNSUPPORTED, "%s: n_rows=%lld too large", what, (long long)n_rows);
    const size_t shmem = static_cast<size_t>(kTileRows) * (F + 1) * sizeof(float);
    gcn_layer_kernel<LPR, Feat, QMODE><<<dim3(static_cast<unsigned>(grid)), dim3(kBlock), shmem, stream>>>(
        n_rows, src, X, ldx, F, qp, Theta, ldt, Fo, H, ldh);
    return check_launch(what);
}

template <typename Feat, int QMODE>
int dispatch_gcn(const char *what, int64_t n_rows, const SlotSource &src, const typename Feat::elem_t *X, int64_t ldx,
                 int32_t F, QParams qp, const float *Theta, int64_t ldt, int32_t Fo, float *H, int64_t ldh,
                 hipStream_t stream)
{
    int l = pow2_ceil(ceil_div(F, 4));
    l = l < 8 ? 8 : l;
    switch (l) {
        case 8: return launch_gcn<8, Feat, QMODE>(what, n_rows, src, X, ldx, F, qp, Theta, ldt, Fo, H, ldh, stream);
        case 16: return launch_gcn<16, Feat, QMODE>(what, n_rows, src, X, ldx, F, qp, Theta, ldt, Fo, H, ldh, stream);
        case 32: return launch_gcn<32, Feat, QMODE>(what, n_rows, src, X, ldx, F, qp, Theta, ldt, Fo, H, ldh, stream);
        default: return launch_gcn<64, Feat, QMODE>(what, n_rows, src, X, ldx, F, qp, Theta, ldt, Fo, H, ldh, stream);
    }
}

// Lane groups of 32 or 64 only (F > 64).
template <typename Feat, int QMODE>
int dispatch_gcn_lanes(const char *what, int64_t n_rows, const SlotSource &src, const typename Feat::elem_t *X, int64_t ldx,
                       int32_t F, QParams qp, const float *Theta, int64_t ldt, int32_t Fo, float *H, int64_t ldh,
                       hipStream_t stream)
{
    if (F <= 128) return launch_gcn<32, Feat, QMODE>(what, n_rows, src, X, ldx, F, qp, Theta, ldt, Fo, H, ldh, stream);
    return launch_gcn<64, Feat, QMODE>(what, n_rows, src, X, ldx, F, qp, Theta, ldt, Fo, H, ldh, stream);
}

// ---- the general form: any F, any row length --------------------------------------------------
// The kernel above keeps a whole aggregated row (F <= 256 features, F % 4 == 0) in LDS and leaves
// every row to one lane group.  This one walks the features in chunks of kChunkF:
//   for each chunk: aggregate the chunk of the 32 rows into LDS, then add tile_chunk * Theta_chunk
//   to the wavefront's MFMA accumulators, which live in registers across the chunks
// so F is unbounded and the LDS tile is 33 KB whatever F is.  One lane group is a whole wavefront
// (64 lanes x 4 features = one chunk); the last lane of a row whose length is not a multiple of
// four loads its 1-3 features one by one.  LONG (plans whose width allows rows above kLongRowLayer
// slots: W == 0 or W > 2048): such a row is shared by the four wavefronts, partial sums carried in
// float64 and added in a fixed order through LDS, exactly as in the SpMM kernel.
// NB = 32-column blocks of H per wavefront (1: Fo <= 128, 4: Fo <= 512).
constexpr int kChunkF = 256;
constexpr int kLongRowLayer = 2048;

template <typename Feat, int QMODE, int NB, bool LONG>
__global__ void __launch_bounds__(kBlock)
gcn_layer_wide_kernel(int64_t n_rows, SlotSource src, const typename Feat::elem_t *__restrict__ X, int64_t ldx,
                      int32_t F, QParams qp, const float *__restrict__ Theta, int64_t ldt, int32_t Fo,
                      float *__restrict__ H, int64_t ldh)
{
    constexpr int LPR = kWave;
    constexpr int kStride = kTile + 1;
    constexpr int kYStride = kChunkF + 1;             // 32 rows of an A operand fall in 32 different banks
    __shared__ int2 stage[kWavesPerBlock][kStride];
    __shared__ float ys[kTileRows * kYStride];
    __shared__ double sh_part[LONG ? kWavesPerBlock : 1][LONG ? LPR : 1][5];

    const int wave = threadIdx.x / kWave;
    const int lane = threadIdx.x % kWave;
    const int64_t row0 = static_cast<int64_t>(blockIdx.x) * kTileRows;
    const int i = lane % 32, h = lane / 32;           // MFMA operand coordinates of this lane

    floatx16 c[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) c[j][v] = 0.0f;

    for (int32_t f0 = 0; f0 < F; f0 += kChunkF) {
        const int32_t chunk_len = F - f0 < kChunkF ? F - f0 : kChunkF;
        const int32_t f = f0 + lane * 4;
        const bool lane_on = f < F;
        const int nv = lane_on ? (F - f < 4 ? F - f : 4) : 0;

        // ---- aggregation of the chunk: Algorithm 1's accumulation loop, one wavefront per row ----
        for (int rr = wave; rr < kTileRows; rr += kWavesPerBlock) {
            const int64_t r = row0 + rr;
            float y[4] = {0.0f, 0.0f, 0.0f, 0.0f};
            if (r < n_rows) {
                const RowInfo ri = row_info<false>(src, r);
                if (!(LONG && ri.n_slots > kLongRowLayer)) {
                    float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
                    float side = 0.0f;
                    LaneConstants<Feat, QMODE> k;
                    accumulate_tiles<LPR, 8, Feat, QMODE, false, float, true>(src, ri, stage[wave], lane, lane_on, X, ldx, f,
                                                                              qp, 0, 1, acc, side, nv);
                    load_lane_constants<Feat, QMODE>(qp, f, lane_on, r, k, nv);
                    if constexpr (QTraits<Feat, QMODE>::kAffine) side = group_sum<LPR, float>(side);
                    if (lane_on) finish_values<Feat, QMODE, float>(acc, side, k, y);
                }
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) ys[rr * kYStride + lane * 4 + q] = (lane_on && q < nv) ? y[q] : 0.0f;
        }
        if constexpr (LONG) {
            // Long rows of the tile, one after another, by all four wavefronts (uniform control flow:
            // every thread reads the same row pointers).
            for (int rr = 0; rr < kTileRows; ++rr) {
                const int64_t r = row0 + rr;
                if (r >= n_rows) break;
                const RowInfo ri = row_info<false>(src, r);
                if (ri.n_slots <= kLongRowLayer) continue;
                double acc[4] = {0.0, 0.0, 0.0, 0.0};
                double side = 0.0;
                accumulate_tiles<LPR, 8, Feat, QMODE, false, double, true>(src, ri, stage[wave], lane, lane_on, X, ldx, f,
                                                                           qp, wave, kWavesPerBlock, acc, side, nv);
                if constexpr (QTraits<Feat, QMODE>::kAffine) side = group_sum<LPR, double>(side);
#pragma unroll
                for (int q = 0; q < 4; ++q) sh_part[wave][lane][q] = acc[q];
                sh_part[wave][lane][4] = side;
                __syncthreads();
                if (wave == 0) {
                    for (int g = 1; g < kWavesPerBlock; ++g) {     // fixed order: bit-reproducible
#pragma unroll
                        for (int q = 0; q < 4; ++q) acc[q] += sh_part[g][lane][q];
                        side += sh_part[g][lane][4];
                    }
                    float y[4] = {0.0f, 0.0f, 0.0f, 0.0f};
                    LaneConstants<Feat, QMODE> k;
                    load_lane_constants<Feat, QMODE>(qp, f, lane_on, r, k, nv);
                    if (lane_on) finish_values<Feat, QMODE, double>(acc, side, k, y);
#pragma unroll
                    for (int q = 0; q < 4; ++q) ys[rr * kYStride + lane * 4 + q] = (lane_on && q < nv) ? y[q] : 0.0f;
                }
                __syncthreads();
            }
        }
        __syncthreads();

        // ---- combination of the chunk: c[j] += ys (32 x chunk_len) * Theta[f0 .. f0 + chunk_len, block] ----
        // v_mfma_f32_32x32x2_f32: lane l supplies A[l % 32][l / 32] and B[l / 32][l % 32].
        const int32_t k_end = (chunk_len + 1) & ~1;
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            const int nb = wave + j * kWavesPerBlock;
            if (nb * 32 < Fo) {
                const int col = nb * 32 + i;
                const bool col_on = col < Fo;
                const float *t_col = Theta + (col_on ? col : 0);
                for (int32_t k0 = 0; k0 < k_end; k0 += 16) {
                    float a[8], b[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const int32_t kk = k0 + 2 * u + h;             // feature within the chunk
                        a[u] = kk < chunk_len ? ys[i * kYStride + kk] : 0.0f;
                        b[u] = (kk < chunk_len && col_on) ? t_col[static_cast<int64_t>(f0 + kk) * ldt] : 0.0f;
                    }
#pragma unroll
                    for (int u = 0; u < 8; ++u)
                        if (k0 + 2 * u < k_end) c[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u], b[u], c[j], 0, 0, 0);
                }
            }
        }
        __syncthreads();                               // the tile is overwritten by the next chunk
    }

    // result register v of lane l holds D[8 * (v / 4) + 4 * (l / 32) + v % 4][l % 32]
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        const int col = (wave + j * kWavesPerBlock) * 32 + i;
        if (col < Fo) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t r = row0 + 8 * (v / 4) + 4 * h + (v % 4);
                if (r < n_rows) __builtin_nontemporal_store(c[j][v], &H[r * ldh + col]);
            }
        }
    }
}

template <typename Feat, int QMODE, int NB>
int launch_gcn_wide(const char *what, bool long_rows, int64_t n_rows, const SlotSource &src,
                    const typename Feat::elem_t *X, int64_t ldx, int32_t F, QParams qp, const float *Theta,
                    int64_t ldt, int32_t Fo, float *H, int64_t ldh, hipStream_t stream)
{
    const int64_t grid = ceil_div(n_rows, kTileRows);
    if (grid > INT32_MAX) return fail(AES_ERR_UNSUPPORTED, "%s: n_rows=%lld too large", what, (long long)n_rows);
    const dim3 g(static_cast<unsigned>(grid)), b(kBlock);
    if (long_rows)
        gcn_layer_wide_kernel<Feat, QMODE, NB, true><<<g, b, 0, stream>>>(n_rows, src, X, ldx, F, qp, Theta, ldt, Fo, H, ldh);
    else
        gcn_layer_wide_kernel<Feat, QMODE, NB, false><<<g, b, 0, stream>>>(n_rows, src, X, ldx, F, qp, Theta, ldt, Fo, H, ldh);
    return check_launch(what);
}

// Output columns in groups of at most 512 (four 32-column blocks per wavefront); a wider Theta takes
// one launch per group, each of which aggregates again.
template <typename Feat, int QMODE>
int dispatch_gcn_wide(const char *what, bool long_rows, int64_t n_rows, const SlotSource &src,
                      const typename Feat::elem_t *X, int64_t ldx, int32_t F, QParams qp, const float *Theta,
                      int64_t ldt, int32_t Fo, float *H, int64_t ldh, hipStream_t stream)
{
    constexpr int kGroupCols = 4 * kWavesPerBlock * 32;
    for (int32_t o = 0; o < Fo; o += kGroupCols) {
        const int32_t fo = Fo - o < kGroupCols ? Fo - o : kGroupCols;
        int rc;
        if (fo <= kWavesPerBlock * 32)
            rc = launch_gcn_wide<Feat, QMODE, 1>(what, long_rows, n_rows, src, X, ldx, F, qp, Theta + o, ldt, fo, H + o, ldh, stream);
        else
            rc = launch_gcn_wide<Feat, QMODE, 4>(what, long_rows, n_rows, src, X, ldx, F, qp, Theta + o, ldt, fo, H + o, ldh, stream);
        if (rc) return rc;
    }
    return AES_OK;
}

// The specialised kernel where it applies, the general one otherwise.
template <typename Feat, int QMODE>
int run_gcn(const char *what, int32_t W, int64_t n_rows, const SlotSource &src, const typename Feat::elem_t *X,
            int64_t ldx, int32_t F, QParams qp, const float *Theta, int64_t ldt, int32_t Fo, float *H, int64_t ldh,
            hipStream_t stream)
{
    const bool long_rows = W == 0 || W > kLongRowLayer;
    if (F <= kMaxFeatures && F % 4 == 0 && !long_rows) {
        if constexpr (QMODE == kQRowScale && sizeof(typename Feat::elem_t) == 1) {
            // Constants inside the rows of codes, within reach of the lane group that gathers the row: taken
            // from that gather (as in the SpMM; lane groups of 32 and 64, the narrower ones would spill a register);
            // otherwise loaded when a slot is staged.
            int lanes = pow2_ceil(ceil_div(F, 4));
            lanes = lanes < 8 ? 8 : lanes;
            if (qp.inline_off >= 0 && lanes >= 32 && qp.inline_off + (Feat::kSigned ? 4 : 8) <= lanes * 4)
                return dispatch_gcn_lanes<Feat, kQRowInGather>(what, n_rows, src, X, ldx, F, qp, Theta, ldt, Fo, H, ldh, stream);
        }
        return dispatch_gcn<Feat, QMODE>(what, n_rows, src, X, ldx, F, qp, Theta, ldt, Fo, H, ldh, stream);
    }
    return dispatch_gcn_wide<Feat, QMODE>(what, long_rows, n_rows, src, X, ldx, F, qp, Theta, ldt, Fo, H, ldh, stream);
}

// Argument checks shared by the float32 and the 8-bit entry point.
int check_layer(const char *what, int64_t n_rows, int64_t n_cols, int32_t W, const int64_t *s_rowptr, const void *X,
                int64_t ldx, int32_t F, const float *Theta, int64_t ldt, int32_t Fo, const float *H,
                int64_t ldh)
{
    if (n_rows < 0 || n_cols < 0)
        return fail(AES_ERR_INVALID_ARG, "%s: negative size (n_rows=%lld n_cols=%lld)", what, (long long)n_rows,
                    (long long)n_cols);
    if (n_cols > INT32_MAX) return fail(AES_ERR_UNSUPPORTED, "%s: n_cols=%lld does not fit int32", what, (long long)n_cols);
    if (W < 0 || W > AES_MAX_W) return fail(AES_ERR_INVALID_ARG, "%s: W=%d outside 0..%d", what, (int)W, (int)AES_MAX_W);
    if (F < 1 || Fo < 1 || Fo >= (1 << 24)) return fail(AES_ERR_INVALID_ARG, "%s: F=%d / Fo=%d out of range", what, (int)F, (int)Fo);
    if (ldx < F || ldt < Fo || ldh < Fo)
        return fail(AES_ERR_INVALID_ARG, "%s: leading dimension too small (ldx=%lld ldt=%lld ldh=%lld)", what,
                    (long long)ldx, (long long)ldt, (long long)ldh);
    if (s_rowptr == nullptr || Theta == nullptr) return fail(AES_ERR_INVALID_ARG, "%s: s_rowptr / Theta is NULL", what);
    if (n_rows > 0 && H == nullptr) return fail(AES_ERR_INVALID_ARG, "%s: H is NULL", what);
    if (n_rows > 0 && n_cols > 0 && X == nullptr) return fail(AES_ERR_INVALID_ARG, "%s: X is NULL", what);
    if (ldx > UINT32_MAX)
        return fail(AES_ERR_UNSUPPORTED, "%s: feature leading dimension %lld does not fit 32 bits", what, (long long)ldx);
    if (ldt >= (1 << 28) || ldh >= (1 << 28))
        return fail(AES_ERR_UNSUPPORTED, "%s: ldt / ldh must stay below 2^28 (32-bit lane offsets)", what);
    if (F >= (1 << 24)) return fail(AES_ERR_INVALID_ARG, "%s: F=%d outside 1..2^24-1", what, (int)F);
    return AES_OK;
}

}  // namespace

extern "C" int aes_gcn_layer_f32(int64_t n_rows, int64_t n_cols, int32_t W,
                                 const int64_t *s_rowptr, const int32_t *s_col, const float *s_val,
                                 const float *X, int64_t ldx, int32_t F,
                                 const float *Theta, int64_t ldt, int32_t Fo,
                                 float *H, int64_t ldh, void *stream)
{
    const char *what = "aes_gcn_layer_f32";
    if (int rc = check_layer(what, n_rows, n_cols, W, s_rowptr, X, ldx, F, Theta, ldt, Fo, H, ldh)) return rc;
    if (n_rows == 0) return AES_OK;
    const SlotSource src = {s_rowptr, s_col, s_val, W, 0, 0};
    const QParams qp = {nullptr, nullptr, 1, -1};
    return run_gcn<FeatF32<4>, kQNone>(what, W, n_rows, src, X, ldx, F, qp, Theta, ldt, Fo, H, ldh,
                                       static_cast<hipStream_t>(stream));
}

extern "C" int aes_gcn_layer_q8(int64_t n_rows, int64_t n_cols, int32_t W,
                                const int64_t *s_rowptr, const int32_t *s_col, const float *s_val,
                                const int8_t *Xq, int64_t ldq, int32_t F,
                                int32_t scheme, int32_t granularity, const float *scale, const float *zero,
                                const float *Theta, int64_t ldt, int32_t Fo,
                                float *H, int64_t ldh, void *stream_)
{
    const char *what = "aes_gcn_layer_q8";
    if (int rc = check_layer(what, n_rows, n_cols, W, s_rowptr, Xq, ldq, F, Theta, ldt, Fo, H, ldh)) return rc;
    QParams qp;
    if (int rc = resolve_q8(what, false, Xq, ldq, F, scheme, granularity, scale, zero, qp)) return rc;
    if (n_rows == 0) return AES_OK;
    const bool affine = scheme == AES_Q_AFFINE_FLOOR_U8;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    const SlotSource src = {s_rowptr, s_col, s_val, W, 0, 0};
#define AES_GCN_Q8(SIGNED, MODE) \
    run_gcn<FeatQ8<4, SIGNED>, MODE>(what, W, n_rows, src, Xq, ldq, F, qp, Theta, ldt, Fo, H, ldh, stream)
    switch (granularity) {
        case AES_Q_PER_TENSOR: return affine ? AES_GCN_Q8(false, kQTensor) : AES_GCN_Q8(true, kQTensor);
        case AES_Q_PER_COLUMN: return affine ? AES_GCN_Q8(false, kQColumn) : AES_GCN_Q8(true, kQColumn);
        case AES_Q_PER_ROW: return affine ? AES_GCN_Q8(false, kQRowScale) : AES_GCN_Q8(true, kQRowScale);
        default: return affine ? AES_GCN_Q8(false, kQFolded) : AES_GCN_Q8(true, kQFolded);
    }
#undef AES_GCN_Q8
}
