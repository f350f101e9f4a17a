// Fused score-tile kernel (Section 5, "fused score kernel"; Section 1 for the formula):
//   score[t, s] = sum_h w[t,h] * max(0, sum_d q[t,h,d] * K[s,d])
// for one (c_S x c_T) tile.  bf16 operands, fp32 MFMA accumulation, ReLU and the weighted
// head sum done on the MFMA result registers; the per-head values never leave the wave.
//
// Mapping (gfx950, wave64, v_mfma_f32_32x32x16_bf16):
//   - one wave owns one query for the whole key sweep.  The query's heads are the M side of
//     the MFMA (32 heads per block, HB blocks), kept in registers: HB * D/16 operands of
//     8 bf16.  Keys are the N side, 32 per MFMA, read from LDS.
//   - the 32x32 result puts one key per lane column (lane & 31) and 16 heads per lane, so the
//     head sum is 16 in-lane FMAs per head block plus one exchange between lane and lane^32.
//   - a workgroup is 8 waves = 8 consecutive queries sharing each staged block of keys; the
//     next block is prefetched into registers while the current one is being used.
// Every (query, key) score is produced by the same instruction sequence wherever the pair
// falls in a tile, which is what makes results independent of the tiling.
//
// Two outputs, chosen at compile time:
//   dense  : the fp32 tile itself (entry point si_score_tile);
//   filter : the per-tile mask (Section 5) and the first half of the per-tile select are
//            applied in registers: only legal entries that beat the row's threshold (the k-th
//            best score of an earlier prefix of the key axis) are appended, as 64-bit
//            (score, ~index) keys, to the row's buffer.  An entry that does not beat it can
//            never enter the final top-k: key tiles are visited in ascending index order, so
//            on equal score the entry already held has the smaller index and wins
//            (Section 4.1).  One wave owns one row, so the append needs no atomics.

#include "si_internal.h"

namespace si {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kKeyChunk = 128;  // keys staged in LDS per step
constexpr int kScoreThreads = 64 * kQueriesPerBlock;

// max(x, 0) on the bit pattern: negative floats (and -0) are negative integers.
__device__ inline float relu(float x) { return __int_as_float(max(__float_as_int(x), 0)); }

template <int D, int HB, bool FILTER>
__global__ __launch_bounds__(kScoreThreads) __attribute__((amdgpu_waves_per_eu(2, 2)))
void score_tile_kernel(const __bf16* __restrict__ q, const __bf16* __restrict__ K,
                       const float* __restrict__ w, int S, int H, int T, int m, int mask_mode,
                       int s0, int t0, int rows, int width, int tile_rows, int tile_cols,
                       float* __restrict__ tile, RowBuffers rb) {
    constexpr int KS = D / 16;             // MFMA steps along d
    constexpr int kRowBytes = D * 2 + 16;  // LDS key row, padded by 16 B against bank conflicts
    constexpr int kPieces = D / 8;         // 16-byte pieces per key row
    constexpr int kBufBytes = kKeyChunk * kRowBytes;
    constexpr int kLoads = kKeyChunk * kPieces / kScoreThreads;  // 16-byte loads per thread per chunk
    static_assert(kKeyChunk * kPieces % kScoreThreads == 0, "chunk must split evenly over the threads");
    __shared__ __attribute__((aligned(16))) unsigned char lds[2 * kBufBytes];

    const int wave = threadIdx.x >> 6;
    const int lane = threadIdx.x & 63;
    const int col = lane & 31;
    const int half = lane >> 5;
    const int b = blockIdx.y;
    const int r_first = blockIdx.x * kQueriesPerBlock;
    const int r = r_first + wave;  // row inside the tile
    const bool live = r < rows;
    const int64_t ws_row = static_cast<int64_t>(b) * tile_rows + r;

    // Keys of this tile that the last query of the workgroup may see (causal block mask,
    // Section 4.2).  Uniform over the workgroup, so the early return is safe.
    const int r_last = min(rows, r_first + kQueriesPerBlock) - 1;
    const int n_keys = min(width, legal_count(s0 + r_last, T, m, mask_mode) - t0);
    if (n_keys <= 0) return;

    // Query operand: head h = hb*32 + col, d = ks*16 + half*8 .. +8.  Addresses are clamped into
    // the problem instead of predicated: a wave whose row is past the tile edge recomputes the
    // last row (never stored); a head slot past H_I reuses head H_I-1 with weight 0, which
    // adds exactly +0.
    bf16x8 a[HB][KS];
    float wr[HB][16];
    const int64_t qrow = static_cast<int64_t>(b) * S + s0 + (live ? r : rows - 1);
#pragma unroll
    for (int hb = 0; hb < HB; ++hb) {
        const int h = min(hb * 32 + col, H - 1);
        const __bf16* src = q + (qrow * H + h) * D + half * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) a[hb][ks] = *reinterpret_cast<const bf16x8*>(src + ks * 16);
        // Result register j of this lane holds head hb*32 + 8*(j/4) + 4*half + j%4.
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int hh = hb * 32 + 8 * (j >> 2) + 4 * half + (j & 3);
            const float wv = w[qrow * H + min(hh, H - 1)];
            wr[hb][j] = hh < H ? wv : 0.0f;
        }
    }

    // filter mode: this row's legal keys inside the tile, its threshold score, its buffer
    int row_keys = 0;
    float theta = 0.0f;
    key64_t* cand = nullptr;
    int n_cand = 0;
    if (FILTER && live) {
        row_keys = min(width, legal_count(s0 + r, T, m, mask_mode) - t0);
        theta = rb.theta[ws_row];
        n_cand = rb.count[ws_row];
        cand = rb.keys + ws_row * rb.cap;
    }

    const __bf16* Kb = K + (static_cast<int64_t>(b) * T + t0) * D;
    float* out_row = tile + ws_row * tile_cols;

    u32x4 pre[kLoads];
#define SI_FETCH(KC0)                                                                              \
    _Pragma("unroll") for (int i = 0; i < kLoads; ++i) {                                            \
        const int p = threadIdx.x + i * kScoreThreads;                                              \
        const int row = p / kPieces, c = p % kPieces;                                               \
        const int key = min((KC0) + row, width - 1); /* rows past the edge repeat the last key */   \
        pre[i] = *reinterpret_cast<const u32x4*>(Kb + static_cast<int64_t>(key) * D + c * 8);       \
    }
#define SI_STASH(BUF)                                                                              \
    _Pragma("unroll") for (int i = 0; i < kLoads; ++i) {                                            \
        const int p = threadIdx.x + i * kScoreThreads;                                              \
        const int row = p / kPieces, c = p % kPieces;                                               \
        *reinterpret_cast<u32x4*>(lds + (BUF) * kBufBytes + row * kRowBytes + c * 16) = pre[i];     \
    }

    SI_FETCH(0)
    SI_STASH(0)
    // every prologue load has landed before the loop, so no wait on them is needed inside it
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
    __syncthreads();

    int buf = 0;
    for (int kc0 = 0; kc0 < n_keys; kc0 += kKeyChunk, buf ^= 1) {
        const bool more = kc0 + kKeyChunk < n_keys;
        if (more) { SI_FETCH(kc0 + kKeyChunk) }
        const unsigned char* base = lds + buf * kBufBytes + col * kRowBytes + half * 16;
        float res[kKeyChunk / 64];  // lane l: score of key kc0 + i*64 + l
#pragma unroll
        for (int sb = 0; sb < kKeyChunk / 32; ++sb) {
            floatx16 acc[HB];
#pragma unroll
            for (int hb = 0; hb < HB; ++hb)
#pragma unroll
                for (int j = 0; j < 16; ++j) acc[hb][j] = 0.0f;
            const unsigned char* krow = base + sb * 32 * kRowBytes;
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
                for (int j = 0; j < 16; ++j) s = fmaf(wr[hb][j], relu(acc[hb][j]), s);
            s += __shfl_xor(s, 32);
            // even sub-blocks stay in the low half-wave, odd ones in the high half
            if ((sb & 1) == 0) res[sb >> 1] = s;
            else res[sb >> 1] = half ? s : res[sb >> 1];
        }
        if (more) { SI_STASH(buf ^ 1) }
        if (FILTER) {
#pragma unroll
            for (int i = 0; i < kKeyChunk / 64; ++i) {
                const int key = kc0 + i * 64 + lane;
                const bool keep = key < row_keys && res[i] > theta;
                const unsigned long long mask = __ballot(keep);
                if (mask != 0ull) {
                    const int below = __builtin_amdgcn_mbcnt_hi(static_cast<unsigned>(mask >> 32),
                                      __builtin_amdgcn_mbcnt_lo(static_cast<unsigned>(mask), 0u));
                    if (keep) cand[n_cand + below] = make_key(res[i], static_cast<uint32_t>(t0 + key));
                    n_cand += __popcll(mask);
                }
            }
        } else if (live) {
#pragma unroll
            for (int i = 0; i < kKeyChunk / 64; ++i) {
                const int key = kc0 + i * 64 + lane;
                if (key < n_keys) out_row[key] = res[i];
            }
        }
        __syncthreads();
    }
#undef SI_FETCH
#undef SI_STASH
    if (FILTER && live && lane == 0) rb.count[ws_row] = n_cand;
}

namespace {
template <bool FILTER>
hipError_t launch(const void* q, const void* K, const float* w, const si_dims& d, int32_t m,
                  int32_t mask_mode, int32_t s0, int32_t t0, int32_t rows, int32_t width,
                  int32_t tile_rows, int32_t tile_cols, float* tile, const RowBuffers& rb,
                  hipStream_t stream) {
    const dim3 grid((rows + kQueriesPerBlock - 1) / kQueriesPerBlock, d.B);
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
                               int32_t m, int32_t mask_mode, int32_t s0, int32_t t0, int32_t rows,
                               int32_t width, int32_t tile_rows, const RowBuffers& rb,
                               hipStream_t stream) {
    return launch<true>(q, K, w, d, m, mask_mode, s0, t0, rows, width, tile_rows, 0, nullptr, rb,
                        stream);
}

}  // namespace si
