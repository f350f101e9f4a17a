// Fused score-tile kernel (Section 5, "fused score kernel"; Section 1 for the formula):
//   tile[t, s] = sum_h w[t,h] * max(0, sum_d q[t,h,d] * K[s,d])
// for one (c_S x c_T) tile.  bf16 operands, fp32 MFMA accumulation, ReLU and the weighted
// head sum done on the MFMA result registers; the per-head values never leave the wave.
//
// Mapping (gfx950, wave64, v_mfma_f32_32x32x16_bf16):
//   - one wave owns one query for the whole key sweep.  The query's heads are the M side of
//     the MFMA (32 heads per block, HB blocks), kept in registers: HB * D/16 operands of
//     8 bf16.  Keys are the N side, 32 per MFMA, read from LDS.
//   - the 32x32 result puts one key per lane column (lane & 31) and 16 heads per lane, so the
//     head sum is 16 in-lane FMAs per head block plus one exchange between lane and lane^32.
//   - a workgroup is 8 waves = 8 consecutive queries sharing each staged block of keys.
// Every (query, key) score is produced by the same instruction sequence wherever the pair
// falls in a tile, which is what makes results independent of the tiling.

#include "si_internal.h"

namespace si {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kKeyChunk = 128;  // keys staged in LDS per step
constexpr int kScoreThreads = 64 * kQueriesPerBlock;

template <int D, int HB>
__global__ __launch_bounds__(kScoreThreads) void score_tile_kernel(
    const __bf16* __restrict__ q, const __bf16* __restrict__ K, const float* __restrict__ w,
    int S, int H, int T, int m, int mask_mode, int s0, int t0, int rows, int width,
    int tile_rows, int tile_cols, float* __restrict__ tile) {
    constexpr int KS = D / 16;           // MFMA steps along d
    constexpr int kRowBytes = D * 2 + 16;  // LDS key row, padded by 16 B against bank conflicts
    constexpr int kPieces = D / 8;       // 16-byte pieces per key row
    __shared__ __attribute__((aligned(16))) unsigned char lds[kKeyChunk * kRowBytes];

    const int wave = threadIdx.x >> 6;
    const int lane = threadIdx.x & 63;
    const int col = lane & 31;
    const int half = lane >> 5;
    const int b = blockIdx.y;
    const int r_first = blockIdx.x * kQueriesPerBlock;
    const int r = r_first + wave;  // row inside the tile
    const bool live = r < rows;
    const int t = s0 + r;

    // Keys of this tile that the last query of the workgroup may see (causal block mask,
    // Section 4.2).  Uniform over the workgroup, so the early return is safe.
    const int r_last = min(rows, r_first + kQueriesPerBlock) - 1;
    const int n_keys = min(width, legal_count(s0 + r_last, T, m, mask_mode) - t0);
    if (n_keys <= 0) return;

    // Query operand: head h = hb*32 + col, d = ks*16 + half*8 .. +8.
    bf16x8 a[HB][KS];
    float wr[HB][16];
    const int64_t qrow = static_cast<int64_t>(b) * S + t;
#pragma unroll
    for (int hb = 0; hb < HB; ++hb) {
        const int h = hb * 32 + col;
        const bool ok = live && h < H;
        const __bf16* src = q + (qrow * H + h) * D + half * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            bf16x8 v = {0, 0, 0, 0, 0, 0, 0, 0};
            if (ok) v = *reinterpret_cast<const bf16x8*>(src + ks * 16);
            a[hb][ks] = v;
        }
        // Result register j of this lane holds head hb*32 + 8*(j/4) + 4*half + j%4.
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int hh = hb * 32 + 8 * (j >> 2) + 4 * half + (j & 3);
            wr[hb][j] = (live && hh < H) ? w[qrow * H + hh] : 0.0f;
        }
    }

    const __bf16* Kb = K + (static_cast<int64_t>(b) * T + t0) * D;
    float* out_row = tile + (static_cast<int64_t>(b) * tile_rows + r) * tile_cols;

    for (int kc0 = 0; kc0 < n_keys; kc0 += kKeyChunk) {
        // Stage keys [kc0, kc0 + kKeyChunk) of the tile; rows past the tile edge are zero.
        for (int p = threadIdx.x; p < kKeyChunk * kPieces; p += kScoreThreads) {
            const int row = p / kPieces;
            const int c = p % kPieces;
            const int key = kc0 + row;
            uint4 v = make_uint4(0u, 0u, 0u, 0u);
            if (key < width) v = *reinterpret_cast<const uint4*>(Kb + static_cast<int64_t>(key) * D + c * 8);
            *reinterpret_cast<uint4*>(lds + row * kRowBytes + c * 16) = v;
        }
        __syncthreads();

        const int chunk_keys = min(kKeyChunk, n_keys - kc0);
        for (int sb = 0; sb * 32 < chunk_keys; ++sb) {
            floatx16 acc[HB];
#pragma unroll
            for (int hb = 0; hb < HB; ++hb)
#pragma unroll
                for (int j = 0; j < 16; ++j) acc[hb][j] = 0.0f;
            const unsigned char* krow = lds + (sb * 32 + col) * kRowBytes + half * 16;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const bf16x8 kv = *reinterpret_cast<const bf16x8*>(krow + ks * 32);
#pragma unroll
                for (int hb = 0; hb < HB; ++hb)
                    acc[hb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[hb][ks], kv, acc[hb], 0, 0, 0);
            }
            // ReLU, weight, head sum: fixed order hb, j; then the two lane halves.
            float s = 0.0f;
#pragma unroll
            for (int hb = 0; hb < HB; ++hb)
#pragma unroll
                for (int j = 0; j < 16; ++j) s = fmaf(wr[hb][j], fmaxf(acc[hb][j], 0.0f), s);
            s += __shfl_xor(s, 32);
            const int key = kc0 + sb * 32 + col;
            if (live && half == 0 && key < n_keys) out_row[key] = s;
        }
        __syncthreads();
    }
}

hipError_t launch_score_tile(const void* q, const void* K, const float* w, const si_dims& d,
                             int32_t m, int32_t mask_mode, int32_t s0, int32_t t0, int32_t rows,
                             int32_t width, int32_t tile_rows, int32_t tile_cols, float* tile,
                             hipStream_t stream) {
    const dim3 grid((rows + kQueriesPerBlock - 1) / kQueriesPerBlock, d.B);
    const dim3 block(kScoreThreads);
    const __bf16* qp = static_cast<const __bf16*>(q);
    const __bf16* Kp = static_cast<const __bf16*>(K);
    const int HB = (d.H_I + 31) / 32;
#define SI_LAUNCH(DD, HH)                                                                      \
    hipLaunchKernelGGL((score_tile_kernel<DD, HH>), grid, block, 0, stream, qp, Kp, w, d.S,   \
                       d.H_I, d.T, m, mask_mode, s0, t0, rows, width, tile_rows, tile_cols,    \
                       tile)
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

}  // namespace si
