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
//   - a workgroup is 8 waves = 8 consecutive queries sharing each staged block of 128 keys.
//     Key blocks travel HBM/L2 -> LDS directly (global_load_lds, no register round trip) into
//     a ring of three buffers, two blocks ahead of the one being multiplied.
//   - the loop is a software pipeline over 32-key sub-blocks: MFMAs of sub-block g, epilogue
//     of sub-block g-1 and LDS reads for sub-block g+1 are interleaved instruction by
//     instruction, so the matrix pipe, the vector ALU and the LDS work at the same time.
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

constexpr int kWaves = 8;            // waves per workgroup, one query each
constexpr int kQB = kWaves;          // queries per workgroup
constexpr int kKeyChunk = 128;       // keys per LDS buffer
constexpr int kScoreThreads = 64 * kWaves;
constexpr int kLdsBuffers = 3;

// max(x, 0) on the bit pattern: negative floats (and -0) are negative integers.
__device__ inline float relu(float x) { return __int_as_float(max(__float_as_int(x), 0)); }

template <int D, int HB, bool FILTER>
__global__ __launch_bounds__(kScoreThreads) __attribute__((amdgpu_waves_per_eu(2, 2)))
void score_tile_kernel(const __bf16* __restrict__ q, const __bf16* __restrict__ K,
                       const float* __restrict__ w, int S, int H, int T, int m, int mask_mode,
                       int s0, int t0, int rows, int width, int tile_rows, int tile_cols,
                       float* __restrict__ tile, RowBuffers rb) {
    constexpr int KS = D / 16;             // MFMA steps along d
    constexpr int EPM = 16 / KS;           // epilogue elements handled next to one MFMA
    static_assert(16 * HB % KS == 0, "epilogue elements must split evenly over the MFMA steps");
    // LDS key rows are unpadded (2*D bytes); the 16-byte pieces of a row are XOR-swizzled so
    // that the 16 lanes served together by one ds_read_b128 hit 16 different bank groups:
    // piece p of row r sits in slot p ^ swz(r), swz(r) = (r / rows per 256 B) mod pieces per row.
    constexpr int kRowBytes = D * 2;
    constexpr int kPieces = D / 8;         // 16-byte pieces per key row
    constexpr int kRowsPer256 = 256 / kRowBytes;
    constexpr int kBufBytes = kKeyChunk * kRowBytes;
    constexpr int kRowsPerLoad = 64 / kPieces;  // key rows covered by one wave-wide 1 KiB load
    constexpr int kLoads = kKeyChunk / kRowsPerLoad / kWaves;  // loads per wave per chunk
    static_assert(kKeyChunk % (kRowsPerLoad * kWaves) == 0, "chunk must split evenly over the waves");
    static_assert(kKeyChunk == 128, "the pipelined loop is written for 4 sub-blocks per chunk");
    __shared__ __attribute__((aligned(1024))) unsigned char lds[kLdsBuffers * kBufBytes];

    // wave-uniform values (row, threshold, counters, pointers) live in scalar registers
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int col = lane & 31;
    const int half = lane >> 5;
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
            float wv = w[qrow * H + min(hh, H - 1)];
            wv = hh < H ? wv : 0.0f;
            asm volatile("" : "+v"(wv));  // keep the masked weight in a register for the whole sweep
            wr[hb][j] = wv;
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
    float* out_row = tile + ws_row * tile_cols;
    const __bf16* Kb = K + (static_cast<int64_t>(b) * T + t0) * D;

    // Global -> LDS without a register round trip: each wave-wide load writes 1 KiB of LDS
    // (lane l to byte l*16 of the block); the lane picks the global piece that belongs there.
    typedef __attribute__((address_space(3))) void lds_void;
    typedef __attribute__((address_space(1))) const void gbl_void;
#define SI_FETCH(KC0, BUFOFF)                                                                      \
    _Pragma("unroll") for (int i = 0; i < kLoads; ++i) {                                            \
        const int blk = wave * kLoads + i;                   /* 1 KiB block inside the chunk */     \
        const int row = blk * kRowsPerLoad + lane / kPieces; /* key row inside the chunk */         \
        const int piece = (lane % kPieces) ^ ((row / kRowsPer256) % kPieces);                       \
        const int key = min((KC0) + row, width - 1); /* rows past the edge repeat the last key */   \
        const __bf16* src = Kb + static_cast<int64_t>(key) * D + piece * 8;                         \
        __builtin_amdgcn_global_load_lds((gbl_void*)(src),                                          \
            (lds_void*)(lds + (BUFOFF) + blk * 1024), 16, 0, 0);                                    \
    }

    // This lane's byte offset, inside a 32-key sub-block, of the operand for MFMA step ks.
    const int swz = (col / kRowsPer256) % kPieces;
    int koff[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) koff[ks] = col * kRowBytes + (((ks * 2 + half) ^ swz) * 16);
#define SI_KREAD(BYTEOFF, KSTEP) \
    (*reinterpret_cast<const bf16x8*>(lds + (BYTEOFF) + koff[KSTEP]))

    // Chunks 0 and 1 in flight; chunk 0 must have landed before its first read.
    int off_cur = 0, off_next = kBufBytes, off_nn = 2 * kBufBytes;  // LDS buffers: being read, next, filling
    SI_FETCH(0, off_cur)
    SI_FETCH(kKeyChunk, off_next)
    __builtin_amdgcn_s_waitcnt(0x0F70 | kLoads);  // vmcnt(kLoads): everything but chunk 1 has landed
    __syncthreads();

    bf16x8 bq[KS];  // key operand of the sub-block about to be multiplied
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) bq[ks] = SI_KREAD(off_cur, ks);

    // Software pipeline, one step per 32-key sub-block: the MFMAs of sub-block g fill one
    // accumulator set while the ReLU / weight / head-sum epilogue drains the other one (sub-block
    // g-1), and the key operand of sub-block g+1 is read from LDS into the registers the MFMAs
    // have just consumed.  The scheduling barriers pin this interleaving: per MFMA, 16/KS epilogue
    // elements and (in the last head block) one LDS read.  Each head block's KS MFMAs are issued
    // back to back as one dependent accumulator chain, which measured slightly faster than
    // alternating the head blocks.
    floatx16 accA[HB], accB[HB];
    const floatx16 zero16 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int hb = 0; hb < HB; ++hb) accB[hb] = zero16;
#define SI_STEP(CUR, PREV, OUT, NEXT_BYTEOFF)                                                      \
    {                                                                                               \
        float s_ = 0.0f;                                                                            \
        _Pragma("unroll") for (int hb = 0; hb < HB; ++hb)                                           \
            _Pragma("unroll") for (int ks = 0; ks < KS; ++ks) {                                     \
                CUR[hb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[hb][ks], bq[ks],                \
                                                                  ks == 0 ? zero16 : CUR[hb], 0, 0, 0); \
                _Pragma("unroll") for (int e = (hb * KS + ks) * EPM; e < (hb * KS + ks + 1) * EPM; ++e)   \
                    s_ = fmaf(wr[e / 16][e % 16], relu(PREV[e / 16][e % 16]), s_);                  \
                if (hb == HB - 1) bq[ks] = SI_KREAD(NEXT_BYTEOFF, ks);                              \
                __builtin_amdgcn_sched_barrier(0);                                                  \
            }                                                                                       \
        OUT = s_ + __shfl_xor(s_, 32);                                                              \
    }
    // 64 finished scores (lane l holds key KEY0 + l): append the kept ones / store the tile row.
#define SI_EMIT(VAL, KEY0)                                                                         \
    {                                                                                               \
        const int key = (KEY0) + lane;                                                              \
        if (FILTER) {                                                                               \
            const bool keep = key >= 0 && key < row_keys && (VAL) > theta;                          \
            const unsigned long long mask = __ballot(keep);                                         \
            if (mask != 0ull) {                                                                     \
                const int below = __builtin_amdgcn_mbcnt_hi(static_cast<unsigned>(mask >> 32),      \
                                  __builtin_amdgcn_mbcnt_lo(static_cast<unsigned>(mask), 0u));      \
                if (keep) cand[n_cand + below] = make_key((VAL), static_cast<uint32_t>(t0 + key));  \
                n_cand += __popcll(mask);                                                           \
            }                                                                                       \
        } else if (live && key >= 0 && key < n_keys) {                                              \
            out_row[key] = (VAL);                                                                   \
        }                                                                                           \
    }

    float r_even = 0.0f;  // epilogue result of the last even sub-block, waiting for its odd partner
    int kc0 = 0;
    for (; kc0 < n_keys; kc0 += kKeyChunk) {
        // Chunk kc0/128 + 2 starts its trip to LDS.  Issued unconditionally (addresses are clamped,
        // the buffer is unused if the chunk does not exist) so that the vmcnt arithmetic below holds.
        SI_FETCH(kc0 + 2 * kKeyChunk, off_nn)
        float sp, s0v, s1v, s2v;
        SI_STEP(accA, accB, sp, off_cur + 1 * 32 * kRowBytes)
        SI_STEP(accB, accA, s0v, off_cur + 2 * 32 * kRowBytes)
        SI_STEP(accA, accB, s1v, off_cur + 3 * 32 * kRowBytes)
        // The next chunk must be in LDS, and visible to every wave, before its first read below.
        __builtin_amdgcn_s_waitcnt(0x0F70 | kLoads);  // vmcnt(kLoads): only the newest chunk may be in flight
        __syncthreads();
        SI_STEP(accB, accA, s2v, off_next)
        // even sub-blocks stay in the low half-wave, odd ones in the high half
        const float res_prev = half ? sp : r_even;   // keys kc0 - 64 + lane (previous chunk)
        const float res_cur = half ? s1v : s0v;      // keys kc0 + lane
        r_even = s2v;
        if (!FILTER || __ballot((res_prev > theta) | (res_cur > theta)) != 0ull) {
            SI_EMIT(res_prev, kc0 - 64)
            SI_EMIT(res_cur, kc0)
        }
        const int t_ = off_cur; off_cur = off_next; off_next = off_nn; off_nn = t_;
    }
    {   // drain: the last sub-block's epilogue and the last 64 scores
        float s_ = 0.0f;
#pragma unroll
        for (int e = 0; e < 16 * HB; ++e) s_ = fmaf(wr[e / 16][e % 16], relu(accB[e / 16][e % 16]), s_);
        const float sp = s_ + __shfl_xor(s_, 32);
        const float res_prev = half ? sp : r_even;
        SI_EMIT(res_prev, kc0 - 64)
    }
#undef SI_STEP
#undef SI_EMIT
#undef SI_FETCH
#undef SI_KREAD
    if (FILTER && live && lane == 0) rb.count[ws_row] = n_cand;
    // loads of chunks past the end may still be in flight: let them land before the LDS is released
    __builtin_amdgcn_s_waitcnt(0x0F70);
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
                               int32_t m, int32_t mask_mode, int32_t s0, int32_t t0, int32_t rows,
                               int32_t width, int32_t tile_rows, const RowBuffers& rb,
                               hipStream_t stream) {
    return launch<true>(q, K, w, d, m, mask_mode, s0, t0, rows, width, tile_rows, 0, nullptr, rb,
                        stream);
}

}  // namespace si
