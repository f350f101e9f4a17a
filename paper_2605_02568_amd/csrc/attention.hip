// The consumer of the index lists (Section 3, step 4): sparse attention of every query over
// U(t) = TopK(t) U Window(t), where the keys and the values are the rows of the compressed cache K_C
// (Section 3, step 1), TopK(t) is the query's index list as si_indexer_topk writes it (pads = -1)
// and Window(t) is the last min(n_win, legal(t)) legal keys (Section 4.2 for legal(t)):
//
//   out[t,h,:] = sum_{s in U(t)} p_s K_C[s,:],   p = softmax_{s in U(t)}( scale * <qa[t,h,:], K_C[s,:]> )
//
// and out = 0 where U(t) is empty.  The paper names this step and gives no formula; the reading is
// spelled out in the public header.
//
// Mapping (gfx950, wave64).  One workgroup = one query; its waves split the heads, 32 per wave, and
// share the gathered key rows.  The rows of U(t) are gathered 32 at a time (a tile) straight from
// global memory into LDS (global_load ... lds, no register round trip), row-major and XOR-swizzled
// like the indexer's key chunks, two tiles in flight.  Per tile and wave:
//   S^T[32 keys x 32 heads] = Ktile . q^T     v_mfma_f32_32x32x16_bf16, keys on the M side: each lane
//                                             then holds 16 keys of ONE head, so the softmax
//                                             statistics of a head are in-lane (+ one lane^32 exchange)
//   p = exp2(x - m_ref)                       running reference maximum per head, raised (and the
//                                             accumulators rescaled) only when a tile exceeds it by
//                                             more than 2^8; fp32
//   O^T[D x 32 heads] += Vtile^T . P^T        P^T is the B operand straight from the S^T registers
//                                             (the contraction order over the tile's keys is permuted
//                                             the same way on both operands); Vtile^T, a column access
//                                             of the row-major tile, comes from the transposing LDS
//                                             read ds_read_b64_tr_b16.  p is split into two bf16
//                                             (high part + remainder) and multiplied twice, so the
//                                             weights carry 16 mantissa bits, not 8.
// The denominator is accumulated in fp32 from the unsplit p and divides O^T at the end.

#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <type_traits>

#include "si_internal.h"
#include "streamindex_attention.h"

namespace si {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kTileKeys = 32;        // keys per gathered tile
constexpr float kRescaleSlack = 8.0f;  // log2 units a tile may exceed the reference maximum

// LDS slot (16-byte unit inside the tile) of piece `piece` (8 elements) of tile row `row`.
// Rows are unpadded (2*D bytes); the pieces of a row are XOR-swizzled with the row number so that
// the 16 lanes served together by one LDS read hit different bank groups, for the row reads of the
// first product and for the transposing reads of the second one alike.
template <int D>
__device__ __forceinline__ int tile_slot(int row, int piece) {
    constexpr int kPieces = D / 8;              // 16-byte pieces per key row
    constexpr int kRowsPer256 = 256 / (D * 2);  // rows per 256 bytes of LDS
    return row * kPieces + (piece ^ ((row / kRowsPer256) % kPieces));
}

// The value lane (l ^ 32) holds, by v_permlane32_swap instead of an LDS round trip: of the swap's two
// results one carries the low half-wave's values in both halves, the other the high half-wave's;
// each lane picks the one that is not its own.
__device__ __forceinline__ float other_half(float v) {
    const unsigned bits = __builtin_bit_cast(unsigned, v);
    const auto both = __builtin_amdgcn_permlane32_swap(bits, bits, false, false);
    return __builtin_bit_cast(float, (threadIdx.x & 32) ? both[0] : both[1]);
}

// One workgroup per query; HW waves of 64 lanes, wave w owns heads [32 w, 32 w + 32).
// Dynamic LDS: 2 tiles of 32 x D bf16, then the query's key list (k + n_win ints, padded to a tile).
// Two waves per SIMD are asked for explicitly: with a register budget of 256 the compiler keeps the
// accumulators in ordinary VGPRs; left to a budget of 512 it parks them in AGPRs and copies all 64
// of them out and back around the rescale test of every tile.
template <int D, int HW>
__global__ __launch_bounds__(64 * HW) __attribute__((amdgpu_waves_per_eu(2)))
void sparse_attention_kernel(const __bf16* __restrict__ qa, const __bf16* __restrict__ Kc,
                             const int32_t* __restrict__ idx, int S, int H, int T, int m, int mask_mode,
                             int k, int n_win, float scale_log2e, float* __restrict__ out) {
    constexpr int KS = D / 16;                 // MFMA steps along d in the first product
    constexpr int DB = D / 32;                 // 32-row blocks of O^T
    constexpr int kRowBytes = D * 2;
    constexpr int kPieces = D / 8;
    constexpr int kTileBytes = kTileKeys * kRowBytes;
    constexpr int kLoadsPerWave = kTileBytes / 1024 / HW;  // wave-wide 1 KiB gathers per wave and tile
    static_assert(kTileBytes % (1024 * HW) == 0 && kLoadsPerWave >= 1, "a tile must split over the waves");
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    int* const s_list = reinterpret_cast<int*>(lds + 2 * kTileBytes);
    __shared__ int s_count;

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int col = lane & 31;
    const int half = lane >> 5;
    const int64_t row_q = blockIdx.x;          // b * S + t
    const int b = static_cast<int>(row_q / S);
    const int t = static_cast<int>(row_q % S);
    const int legal = legal_count(t, T, m, mask_mode);
    const int w0 = max(0, legal - n_win);      // Window(t) = [w0, legal)

    // ---- U(t): the list's entries outside the window (they are valid and distinct by contract),
    // in list order, then the window.  Built by wave 0, padded to whole tiles with key 0.
    if (wave == 0) {
        const int32_t* row = idx + row_q * k;
        int n = 0;
        for (int j0 = 0; j0 < k; j0 += 64) {
            const int j = j0 + lane;
            const int s = j < k ? row[j] : -1;
            const bool keep = s >= 0 && !(s >= w0 && s < legal);
            const unsigned long long mask = __ballot(keep);
            const int below = __builtin_amdgcn_mbcnt_hi(static_cast<unsigned>(mask >> 32),
                              __builtin_amdgcn_mbcnt_lo(static_cast<unsigned>(mask), 0u));
            if (keep) s_list[n + below] = s;
            n += __popcll(mask);
        }
        for (int s = w0 + lane; s < legal; s += 64) s_list[n + (s - w0)] = s;
        n += legal - w0;
        const int padded = (n + kTileKeys - 1) / kTileKeys * kTileKeys;
        for (int j = n + lane; j < padded; j += 64) s_list[j] = 0;
        if (lane == 0) s_count = n;
    }
    __syncthreads();
    const int n_u = s_count;
    const int64_t out_base = (row_q * H) * D;
    if (n_u == 0) {  // empty set: zeros (uniform over the workgroup)
        for (int i = threadIdx.x; i < H * D; i += 64 * HW) out[out_base + i] = 0.0f;
        return;
    }
    const int n_tiles = (n_u + kTileKeys - 1) / kTileKeys;
    const __bf16* Kb = Kc + static_cast<int64_t>(b) * T * D;

    // ---- gather of one tile: wave w brings rows [rows_per_wave * w, ...) of the tile
    typedef __attribute__((address_space(3))) void lds_void;
    typedef __attribute__((address_space(1))) const void gbl_void;
    auto gather = [&](int tile, int buf) {
        int key[kLoadsPerWave];  // all of this lane's list entries first: one LDS round trip, not one per load
#pragma unroll
        for (int i = 0; i < kLoadsPerWave; ++i) {
            const int unit = (wave * kLoadsPerWave + i) * 64 + lane;  // 16-byte LDS slot this lane fills
            key[i] = s_list[tile * kTileKeys + unit / kPieces];
        }
#pragma unroll
        for (int i = 0; i < kLoadsPerWave; ++i) {
            const int blk = wave * kLoadsPerWave + i;         // 1 KiB block of the tile
            const int unit = blk * 64 + lane;
            const int r = unit / kPieces;                      // tile row
            const int slot = unit % kPieces;
            constexpr int kRowsPer256 = 256 / kRowBytes;
            const int piece = slot ^ ((r / kRowsPer256) % kPieces);
            const char* src = reinterpret_cast<const char*>(Kb) + static_cast<int64_t>(key[i]) * kRowBytes + piece * 16;
            __builtin_amdgcn_global_load_lds((gbl_void*)src, (lds_void*)(lds + buf * kTileBytes + blk * 1024), 16, 0, 0);
        }
    };
    gather(0, 0);

    // ---- this wave's query operand: head = 32*wave + col, 8 consecutive d at 16*ks + 8*half
    bf16x8 qf[KS];
    {
        const int h = min(32 * wave + col, H - 1);
        const __bf16* src = qa + (row_q * H + h) * D + half * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qf[ks] = *reinterpret_cast<const bf16x8*>(src + ks * 16);
    }

    // A negative scale goes into the query operand: flipping the sign bit of a bf16 is exact, every
    // product and partial sum changes sign and nothing else, so the scores are those of (-q, -scale).
    if (scale_log2e < 0.0f) {
        typedef unsigned uintx4 __attribute__((ext_vector_type(4)));
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            qf[ks] = __builtin_bit_cast(bf16x8, __builtin_bit_cast(uintx4, qf[ks]) ^ 0x80008000u);
        scale_log2e = -scale_log2e;
    }
    // LDS byte offsets that do not depend on the tile: first product, row = col, piece 2 ks + half
    int ka[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) ka[ks] = tile_slot<D>(col, 2 * ks + half) * 16;
    // second product: this lane is source lane s = lane % 16 of its 16-lane group G = lane / 16 for the
    // transposing read; the group serves d rows [32 db + 16 (G % 2), +16) and the keys of half G / 2.
    // Source lane s points at 4 consecutive d (8 bytes) of key row 4 (G / 2) + s / 4 (+ 8 for the
    // second read, + 16 u), at d = 32 db + 16 (G % 2) + 4 (s % 4).
    int va[DB][2];
    {
        const int G = lane >> 4, s = lane & 15;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int w = 0; w < 2; ++w) {
                const int r = 8 * w + 4 * (G >> 1) + (s >> 2);
                const int d = 32 * db + 16 * (G & 1) + 4 * (s & 3);
                va[db][w] = tile_slot<D>(r, d / 8) * 16 + ((d % 8) / 4) * 8;
            }
    }

    floatx16 acc[DB];
    const floatx16 zero16 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int db = 0; db < DB; ++db) acc[db] = zero16;
    float m_ref = -__builtin_huge_valf();  // reference maximum of this lane's head (log2 domain)
    float l_sum = 0.0f;                    // sum of p over this half-wave's keys

    // One tile; the buffer index is a compile-time constant so that every LDS address of the tile is
    // a loop-invariant register plus an immediate offset.
    auto step = [&](int tile, auto buf_tag) {
        constexpr int buf = decltype(buf_tag)::value;
        // tile `tile` has landed for every wave; everyone is done with tile - 1, whose buffer the next
        // gather overwrites
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
        __syncthreads();
        if (tile + 1 < n_tiles) gather(tile + 1, buf ^ 1);
        const unsigned char* tb = lds + buf * kTileBytes;

        // S^T = Ktile . q^T : register j of a lane = key row 8 (j / 4) + 4 half + j % 4, head = col
        floatx16 sacc = zero16;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const bf16x8 kf = *reinterpret_cast<const bf16x8*>(tb + ka[ks]);
            sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], sacc, 0, 0, 0);
        }
        // The scale is >= 0 here (a negative one was moved into the query operand), so the largest scaled
        // score is the largest raw one times the scale, and scale and reference go into one fma per key.
        const bool ragged = tile == n_tiles - 1 && n_u < n_tiles * kTileKeys;  // rows past the end of U(t): rare
        if (ragged) {
            float low = -3.0e38f;
            asm volatile("" : "+v"(low));  // keeps this block a branch instead of 16 selects per tile
            const int live = n_u - tile * kTileKeys;
#pragma unroll
            for (int j = 0; j < 16; ++j)
                if (8 * (j >> 2) + 4 * half + (j & 3) >= live) sacc[j] = low;  // out of the maximum; weight zeroed below
        }
        float smax = sacc[0];
#pragma unroll
        for (int j = 1; j < 16; ++j) smax = fmaxf(smax, sacc[j]);
        float tmax = smax * scale_log2e;
        tmax = fmaxf(tmax, other_half(tmax));  // the tile's maximum for this head (finite: row 0 of a tile is live)
        const bool raise = tmax > m_ref + kRescaleSlack;
        if (__ballot(raise) != 0ull) {  // rare after the first tiles
            const float m_new = raise ? tmax : m_ref;
            const float alpha = __builtin_amdgcn_exp2f(m_ref - m_new);  // 1 where nothing changes, 0 on the first tile
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int j = 0; j < 16; ++j) acc[db][j] *= alpha;
            l_sum *= alpha;
            m_ref = m_new;
        }
        float p[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) p[j] = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[j], scale_log2e, -m_ref));
        if (ragged) {
            float none = 0.0f;
            asm volatile("" : "+v"(none));
            const int live = n_u - tile * kTileKeys;
#pragma unroll
            for (int j = 0; j < 16; ++j)
                if (8 * (j >> 2) + 4 * half + (j & 3) >= live) p[j] = none;
        }
        // weights as two bf16 parts, two keys per conversion: hi = bf16(p), lo = bf16(p - hi)
        typedef float floatx2 __attribute__((ext_vector_type(2)));
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
        typedef unsigned uintx4 __attribute__((ext_vector_type(4)));
        uintx4 hi_bits[2], lo_bits[2];
#pragma unroll
        for (int jj = 0; jj < 8; ++jj) {
            const float p0 = p[2 * jj], p1 = p[2 * jj + 1];
            l_sum += p0 + p1;
            const unsigned hb = __builtin_bit_cast(unsigned, __builtin_convertvector(floatx2{p0, p1}, bf16x2));
            const float r0 = p0 - __builtin_bit_cast(float, hb << 16);
            const float r1 = p1 - __builtin_bit_cast(float, hb & 0xFFFF0000u);
            hi_bits[jj >> 2][jj & 3] = hb;
            lo_bits[jj >> 2][jj & 3] = __builtin_bit_cast(unsigned, __builtin_convertvector(floatx2{r0, r1}, bf16x2));
        }
        bf16x8 p_hi[2], p_lo[2];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            p_hi[u] = __builtin_bit_cast(bf16x8, hi_bits[u]);
            p_lo[u] = __builtin_bit_cast(bf16x8, lo_bits[u]);
        }
        // O^T += Vtile^T . P^T : contraction index e of step u <-> tile row 16 u + 8 (e / 4) + 4 half + e % 4
        // on both operands
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;
                const bf16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
                    (lds_bf16x4*)(tb + va[db][0] + u * 16 * kRowBytes));
                const bf16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
                    (lds_bf16x4*)(tb + va[db][1] + u * 16 * kRowBytes));
                const bf16x8 vf = {v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
                acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, p_hi[u], acc[db], 0, 0, 0);
                acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, p_lo[u], acc[db], 0, 0, 0);
            }
    };
    for (int tile = 0; tile < n_tiles; tile += 2) {
        step(tile, std::integral_constant<int, 0>{});
        if (tile + 1 < n_tiles) step(tile + 1, std::integral_constant<int, 1>{});
    }

    // ---- out[t, head, d] = O^T[d, head] / l : register j of block db = d row 32 db + 8 (j / 4) + 4 half + j % 4
    const float l_all = l_sum + other_half(l_sum);
    const float inv = 1.0f / l_all;
    const int h = 32 * wave + col;
    if (h < H) {
        float* o = out + out_base + static_cast<int64_t>(h) * D;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                const floatx4 v = {acc[db][4 * a] * inv, acc[db][4 * a + 1] * inv, acc[db][4 * a + 2] * inv,
                                   acc[db][4 * a + 3] * inv};
                *reinterpret_cast<floatx4*>(o + 32 * db + 8 * a + 4 * half) = v;
            }
    }
}

// LDS a workgroup needs: two tiles and the key list padded to a whole tile.
size_t attention_lds_bytes(int D, int k, int n_win) {
    const size_t list = static_cast<size_t>((k + n_win + kTileKeys - 1) / kTileKeys * kTileKeys) * sizeof(int);
    return 2 * static_cast<size_t>(kTileKeys) * D * 2 + list;
}

// Raises the dynamic LDS limit of a kernel once per device and size (as in the write-out kernel).
template <typename Kernel>
hipError_t allow_lds(Kernel kernel, size_t bytes, std::atomic<size_t>* allowed) {
    if (bytes <= 48 * 1024) return hipSuccess;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const bool tracked = dev >= 0 && dev < 64;
    if (tracked && allowed[dev].load(std::memory_order_acquire) >= bytes) return hipSuccess;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                            static_cast<int>(bytes));
    if (e == hipSuccess && tracked) {
        size_t seen = allowed[dev].load(std::memory_order_relaxed);
        while (seen < bytes && !allowed[dev].compare_exchange_weak(seen, bytes, std::memory_order_release)) {}
    }
    return e;
}

template <int D, int HW>
hipError_t launch(const __bf16* qa, const __bf16* Kc, const int32_t* idx, const si_dims& d, int32_t m,
                  int32_t mask_mode, int32_t k, int32_t n_win, float scale, float* out, hipStream_t stream) {
    static std::atomic<size_t> allowed[64];
    const size_t lds = attention_lds_bytes(D, k, n_win);
    hipError_t e = allow_lds(sparse_attention_kernel<D, HW>, lds, allowed);
    if (e != hipSuccess) return e;
    const int64_t rows = static_cast<int64_t>(d.B) * d.S;
    hipLaunchKernelGGL((sparse_attention_kernel<D, HW>), dim3(static_cast<unsigned>(rows)), dim3(64 * HW), lds,
                       stream, qa, Kc, idx, d.S, d.H_I, d.T, m, mask_mode, k, n_win,
                       scale * 1.4426950408889634f, out);
    return hipGetLastError();
}

}  // namespace

}  // namespace si

using namespace si;

extern "C" {

si_status si_sparse_attention(const void* qa, const void* Kc, const int32_t* idx, const si_dims* dims,
                              int32_t m, int32_t k, si_mask_mode mask_mode, int32_t n_win, float scale,
                              float* out, void* stream) {
    if (!dims || !qa || !Kc || !idx || !out) return SI_ERR_INVALID_ARG;
    const si_dims d = *dims;
    if (d.B < 1 || d.S < 1 || d.H_I < 1 || d.D < 1 || d.T < 1 || m < 1 || k < 1 || n_win < 0) return SI_ERR_INVALID_ARG;
    if (mask_mode != SI_MASK_NONE && mask_mode != SI_MASK_CAUSAL_BLOCK) return SI_ERR_INVALID_ARG;
    if (!(scale == scale) || scale - scale != 0.0f) return SI_ERR_INVALID_ARG;  // NaN or infinite
    if (d.D != 64 && d.D != 128) return SI_ERR_UNSUPPORTED_SHAPE;
    if (d.H_I > kMaxHeads || k > kMaxK || n_win > kMaxK) return SI_ERR_UNSUPPORTED_SHAPE;
    if (static_cast<int64_t>(d.B) * d.S >= (int64_t{1} << 31)) return SI_ERR_UNSUPPORTED_SHAPE;
    if (attention_lds_bytes(d.D, k, n_win) > 160 * 1024) return SI_ERR_UNSUPPORTED_SHAPE;
    const __bf16* q = static_cast<const __bf16*>(qa);
    const __bf16* K = static_cast<const __bf16*>(Kc);
    hipStream_t hs = static_cast<hipStream_t>(stream);
    const bool two = d.H_I > 32;
    hipError_t e;
    if (d.D == 128) e = two ? launch<128, 2>(q, K, idx, d, m, mask_mode, k, n_win, scale, out, hs)
                            : launch<128, 1>(q, K, idx, d, m, mask_mode, k, n_win, scale, out, hs);
    else e = two ? launch<64, 2>(q, K, idx, d, m, mask_mode, k, n_win, scale, out, hs)
                 : launch<64, 1>(q, K, idx, d, m, mask_mode, k, n_win, scale, out, hs);
    return e == hipSuccess ? SI_OK : SI_ERR_HIP;
}

}  // extern "C"
