// Score-tile kernel of the tiled schedule (Algorithm 2's inner statement for one
// (c_S x c_T) tile): the key sweep of score_sweep.h over keys [t0, t0 + width) for the queries
// [s0, s0 + rows) of every batch, either storing the dense fp32 tile or appending the
// entries that pass the mask and the row's threshold to the row buffers.

#include "score_sweep.h"

namespace si {

template <int D, int HB, bool FILTER>
__global__ __launch_bounds__(kScoreThreads) __attribute__((amdgpu_waves_per_eu(2, 2)))
void score_tile_kernel(const __bf16* __restrict__ q, const __bf16* __restrict__ K,
                       const float* __restrict__ w, int S, int H, int T, int m, int mask_mode,
                       int s0, int t0, int rows, int width, int tile_rows, int tile_cols,
                       float* __restrict__ tile, RowBuffers rb) {
    __shared__ __attribute__((aligned(1024))) unsigned char lds[sweep_lds_bytes<D>()];

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int b = blockIdx.y;
    const int r_first = blockIdx.x * kQB;
    const int r = r_first + wave;  // row inside the tile
    const bool live = r < rows;
    const int64_t ws_row = static_cast<int64_t>(b) * tile_rows + r;

    // Keys of this tile that the last query of the workgroup may see (causal block mask,
    // Section 4.2).  Uniform over the workgroup, so the early return is safe.
    const int r_last = min(rows, r_first + kQB) - 1;
    const int n_keys = min(width, legal_count(s0 + r_last, T, m, mask_mode) - t0);
    if (n_keys <= 0) return;

    // Addresses are clamped into the problem instead of predicated: a wave whose row is past
    // the tile edge recomputes the last row (never stored).
    bf16x8 a[HB][D / 16];
    float wr[HB][16];
    const int64_t qrow = static_cast<int64_t>(b) * S + s0 + (live ? r : rows - 1);
    load_query<D, HB>(q, w, qrow, H, lane, a, wr);

    SweepOut o;
    o.row_keys = 0;
    o.theta = 0.0f;
    o.cand = nullptr;
    o.cap = 0;
    o.n_cand = 0;
    o.overflow = false;
    o.index0 = static_cast<uint32_t>(t0);
    o.live = live;
    o.out_row = tile + ws_row * tile_cols;
    if (FILTER && live) {  // this row's legal keys inside the tile, its threshold, its buffer
        o.row_keys = min(width, legal_count(s0 + r, T, m, mask_mode) - t0);
        o.theta = rb.theta[ws_row];
        o.n_cand = rb.count[ws_row];
        o.cand = rb.keys + ws_row * rb.cap;
        o.cap = rb.cap;
        if (o.n_cand < 0) {  // overflowed in an earlier key tile: stays marked, appends nothing
            o.overflow = true;
            o.n_cand = 0;
            o.row_keys = 0;
        }
    }
    const __bf16* Kb = K + (static_cast<int64_t>(b) * T + t0) * D;
    score_sweep<D, HB, FILTER, false>(lds, a, wr, Kb, width, n_keys, o, nullptr, 0);
    if (FILTER && live && lane == 0) rb.count[ws_row] = o.overflow ? -1 : o.n_cand;  // -1: see finalize
}

namespace {
template <bool FILTER>
hipError_t launch(const void* q, const void* K, const float* w, const si_dims& d, int32_t m,
                  int32_t mask_mode, int32_t s0, int32_t t0, int32_t rows, int32_t width,
                  int32_t tile_rows, int32_t tile_cols, float* tile, const RowBuffers& rb,
                  hipStream_t stream) {
    const dim3 grid((rows + kQB - 1) / kQB, d.B);
    const dim3 block(kScoreThreads);
    const __bf16* qp = static_cast<const __bf16*>(q);
    const __bf16* Kp = static_cast<const __bf16*>(K);
    const int HB = (d.H_I + 31) / 32;
#define SI_LAUNCH(DD, HH)                                                                        \
    hipLaunchKernelGGL((score_tile_kernel<DD, HH, FILTER>), grid, block, 0, stream, qp, Kp, w,  \
                       d.S, d.H_I, d.T, m, mask_mode, s0, t0, rows, width, tile_rows, tile_cols, \
                       tile, rb)
    if (d.D == 128 && HB == 2) SI_LAUNCH(128, 2);
    else if (d.D == 128 && HB == 1) SI_LAUNCH(128, 1);
    else if (d.D == 64 && HB == 2) SI_LAUNCH(64, 2);
    else if (d.D == 64 && HB == 1) SI_LAUNCH(64, 1);
    else if (d.D == 32 && HB == 2) SI_LAUNCH(32, 2);
    else if (d.D == 32 && HB == 1) SI_LAUNCH(32, 1);
    else return hipErrorInvalidValue;
#undef SI_LAUNCH
    return hipGetLastError();
}
}  // namespace

hipError_t launch_score_tile(const void* q, const void* K, const float* w, const si_dims& d,
                             int32_t m, int32_t mask_mode, int32_t s0, int32_t t0, int32_t rows,
                             int32_t width, int32_t tile_rows, int32_t tile_cols, float* tile,
                             hipStream_t stream) {
    return launch<false>(q, K, w, d, m, mask_mode, s0, t0, rows, width, tile_rows, tile_cols, tile,
                         RowBuffers{}, stream);
}

hipError_t launch_score_filter(const void* q, const void* K, const float* w, const si_dims& d,
                               int32_t m, int32_t mask_mode, int32_t k, int32_t s0, int32_t t0, int32_t rows,
                               int32_t width, int32_t tile_rows, const RowBuffers& rb,
                               hipStream_t stream) {
    // a row enters the tile with at most 2k - 1 keys and must have room for the whole tile
    if (k < 1 || width < 1 || static_cast<int64_t>(rb.cap) < 2 * static_cast<int64_t>(k) + width)
        return hipErrorInvalidValue;
    return launch<true>(q, K, w, d, m, mask_mode, s0, t0, rows, width, tile_rows, 0, nullptr, rb,
                        stream);
}

}  // namespace si
