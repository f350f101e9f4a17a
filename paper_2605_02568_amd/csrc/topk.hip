// Per-tile select, cross-tile merge and write-out (Algorithm 2: the topk, merge_topk and
// out[...] <- run steps; Section 4.3 corollary for why per-partition top-k then merge is exact).
//
// Everything works on 64-bit keys whose unsigned order is the total order of Section 4.1
// (see make_key), so a tie on score is always resolved towards the smaller key index and
// the final top-k set is unique: whatever the tiling, the same keys come out.
//
// Each query row of the current query tile owns a buffer of keys, a count and a threshold
// score.  The buffer holds the k best keys of some prefix of the key axis plus every later
// entry that beat the threshold (the k-th best score of that prefix).  An entry that does not
// beat the threshold can never be in the final top-k, so dropping it early is exact.
//   filter  : done where the scores are produced (score kernel, or filter_scores_kernel for
//             caller-supplied scores): legal entries with score > threshold are appended.
//   compact : the merge.  When a row holds at least 2k keys it is cut back to its k best by an
//             MSB-first radix descent over the 64-bit keys (8 bits per pass, LDS histogram),
//             and the threshold is raised.  Tiles narrower than k simply accumulate until
//             then (the "saturated tile" case of Section 6.6 keeps every entry).
//   finalize: last cut to k, bitonic sort (LDS + registers), decode to (index, score), pad
//             (Section 4.2).

#include <atomic>

#include "si_internal.h"

namespace si {

constexpr int kTopkThreads = 256;

constexpr int kRowWaves = kTopkThreads / 64;  // compaction / finalize: one wave per query row
constexpr int kKeysInFlight = 16;             // global loads a lane issues before it uses them

// ---- wave-level selection -----------------------------------------------------------------
// One wave works on one row without workgroup barriers: its 64 lanes stream the row's keys from
// global memory (the row buffer is L2 resident), build a 256-bin histogram in the wave's own
// slice of LDS, and walk the bins with a wave prefix sum.

// A row's keys as seen by one wave.  Lane l is responsible for keys l, l+64, l+128, ...
// RegKeys holds them in registers (rows of up to 64*R keys: read from memory once);
// StreamKeys re-reads them from global memory on every sweep (any length).
template <int R>
struct RegKeys {
    key64_t kb[R];
    int n;
    __device__ inline void load(const key64_t* buf, int n_) {
        n = n_;
        const int lane = threadIdx.x & 63;
#pragma unroll
        for (int i = 0; i < R; ++i) {
            const int j = lane + 64 * i;
            kb[i] = j < n ? buf[j] : 0ull;
        }
    }
    // f(key, valid, first_lane_index): called for successive blocks of 64 keys, in key order
    template <typename F>
    __device__ inline void sweep(F&& f) const {
        const int lane = threadIdx.x & 63;
#pragma unroll
        for (int i = 0; i < R; ++i) f(kb[i], lane + 64 * i < n);
    }
};

struct StreamKeys {
    const key64_t* buf;
    int n;
    template <typename F>
    __device__ inline void sweep(F&& f) const {
        const int lane = threadIdx.x & 63;
        // several keys per lane in flight at a time: latency is what matters
        for (int base = 0; base < n; base += 64 * kKeysInFlight) {
            key64_t kb[kKeysInFlight];
#pragma unroll
            for (int i = 0; i < kKeysInFlight; ++i) {
                const int j = base + 64 * i + lane;
                kb[i] = j < n ? buf[j] : 0ull;
            }
#pragma unroll
            for (int i = 0; i < kKeysInFlight; ++i) f(kb[i], base + 64 * i + lane < n);
        }
    }
};

// Threshold key `thr` and count `kept` such that exactly `kept` of the row's n distinct keys
// are >= thr, with k <= kept <= max(k, limit).  MSB-first radix descent, 8 bits per pass; it
// stops as soon as the bin holding the k-th largest key is small enough for `kept` to respect
// the limit (limit == k: exact selection).  Requires n > k.  Wave-uniform arguments.
template <typename Keys>
__device__ inline key64_t wave_radix_kth(const Keys& keys, int k, int limit, int* hist, int* kept) {
    const int lane = threadIdx.x & 63;
    key64_t prefix = 0ull;
    int need = k;
    int bin = 0;
    for (int shift = 56; shift >= 0; shift -= 8) {
#pragma unroll
        for (int i = 0; i < 4; ++i) hist[lane + 64 * i] = 0;
        __builtin_amdgcn_wave_barrier();
        if (shift >= 32) {
            // digits of the score word: 32-bit arithmetic on the high half of the key
            const int sh = shift - 32;
            const uint32_t want = sh == 24 ? 0u : static_cast<uint32_t>(prefix >> 32) >> (sh + 8);
            keys.sweep([&](key64_t key, bool valid) {
                const uint32_t hi = static_cast<uint32_t>(key >> 32);
                const bool in_prefix = (sh == 24) || ((hi >> (sh + 8)) == want);
                if (valid && in_prefix) atomicAdd(&hist[(hi >> sh) & 255u], 1);
            });
        } else {
            // equal scores: digits of the index word
            const key64_t want = prefix >> (shift + 8);
            keys.sweep([&](key64_t key, bool valid) {
                const bool in_prefix = (key >> (shift + 8)) == want;
                if (valid && in_prefix) atomicAdd(&hist[(key >> shift) & 255ull], 1);
            });
        }
        __builtin_amdgcn_wave_barrier();
        // Lane l owns bins 255-4l .. 252-4l (walking down from the top bin).
        int h[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) h[j] = hist[255 - 4 * lane - j];
        __builtin_amdgcn_wave_barrier();
        const int local = h[0] + h[1] + h[2] + h[3];
        int incl = local;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int up = __shfl_up(incl, off);
            if (lane >= off) incl += up;
        }
        int cum = incl - local;  // keys in bins above this lane's
        const bool crossing = cum < need && need <= incl;  // true in exactly one lane
        int digit = 0, new_need = 0, new_bin = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (crossing && cum < need && need <= cum + h[j]) {
                digit = 255 - 4 * lane - j;
                new_need = need - cum;
                new_bin = h[j];
            }
            cum += h[j];
        }
        const int src = __builtin_ctzll(__ballot(crossing));
        digit = __shfl(digit, src);
        need = __shfl(new_need, src);
        bin = __shfl(new_bin, src);
        prefix |= static_cast<key64_t>(digit) << shift;
        // keys >= prefix: the (k - need) in higher bins plus this whole bin
        if (k - need + bin <= limit) break;
    }
    *kept = k - need + bin;
    return prefix;
}

struct IdentitySlot {
    __device__ inline int operator()(int i) const { return i; }
};

// Writes the row's keys >= thr to dst[slot(0)], dst[slot(1)], ... in key order (dst may be the
// row buffer itself when slot is the identity: a block of keys is always read before anything
// at or behind it is written).  `cap` bounds the logical positions written.  Returns how many
// keys qualified.
template <typename Keys, typename Slot = IdentitySlot>
__device__ inline int wave_keep(const Keys& keys, key64_t thr, key64_t* dst, int cap, Slot slot = Slot()) {
    int pos = 0;
    keys.sweep([&](key64_t key, bool valid) {
        const bool keep = valid && key >= thr;
        const unsigned long long mask = __ballot(keep);
        const int below = __builtin_amdgcn_mbcnt_hi(static_cast<unsigned>(mask >> 32),
                          __builtin_amdgcn_mbcnt_lo(static_cast<unsigned>(mask), 0u));
        if (keep && pos + below < cap) dst[slot(pos + below)] = key;
        pos += __popcll(mask);
    });
    return pos;
}

// ---- wave-level sort ------------------------------------------------------------------------
// Bitonic network over P keys (a power of two >= 16) in one wave's slice of LDS, best (largest)
// key first.  A compare-exchange at stride 2^j only pairs keys whose positions differ in bit j,
// so a lane that holds the 2^NB keys spanning bits [b, b+NB) of the position can run NB
// consecutive strides of the network in registers: one LDS round trip per group of up to four
// strides instead of one per stride (15 instead of 55 for P = 1024).
// Sixteen keys (128 B) are followed by two slots of padding, so that lanes reading their own
// 16-key block with 128-bit loads start in different banks.
struct SortSlot {
    __device__ inline int operator()(int i) const { return i + ((i >> 4) << 1); }
};
__host__ __device__ inline int sort_slots(int P) { return P + P / 8; }

__device__ inline void compare_exchange(key64_t& x, key64_t& y, bool descending) {
    const bool swap = (x < y) == descending;
    const key64_t a = swap ? y : x;
    const key64_t b = swap ? x : y;
    x = a;
    y = b;
}

// Strides 2^(b+NB-1) .. 2^b of the merge phase that builds sorted runs of `size` (> 2^(b+NB-1)).
template <int NB>
__device__ inline void sort_pass(key64_t* s, int P, int b, int size) {
    constexpr int E = 1 << NB;
    const SortSlot slot;
    const int lane = threadIdx.x & 63;
    for (int u = lane; u < (P >> NB); u += 64) {
        const int base = (u & ((1 << b) - 1)) | ((u >> b) << (b + NB));
        const bool descending = (base & size) == 0;
        key64_t v[E];
#pragma unroll
        for (int j = 0; j < E; ++j) v[j] = s[slot(base | (j << b))];
#pragma unroll
        for (int d = E >> 1; d > 0; d >>= 1)
#pragma unroll
            for (int i = 0; i < (E >> 1); ++i) {
                const int lo = 2 * i - (i & (d - 1));
                compare_exchange(v[lo], v[lo + d], descending);
            }
#pragma unroll
        for (int j = 0; j < E; ++j) s[slot(base | (j << b))] = v[j];
    }
    __builtin_amdgcn_wave_barrier();
}

// The four lowest strides (8, 4, 2, 1) on a lane's own block of 16 consecutive keys; with
// FIRST, the whole network up to runs of 16 (sizes 2, 4, 8, 16) instead.
template <bool FIRST>
__device__ inline void sort_block16(key64_t* s, int P, int size) {
    typedef key64_t key64x2 __attribute__((ext_vector_type(2)));
    const SortSlot slot;
    const int lane = threadIdx.x & 63;
    for (int base = 16 * lane; base < P; base += 16 * 64) {
        key64x2* blk = reinterpret_cast<key64x2*>(s + slot(base));  // 16-byte aligned
        key64_t v[16];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const key64x2 t = blk[j];
            v[2 * j] = t.x;
            v[2 * j + 1] = t.y;
        }
        if (FIRST) {
#pragma unroll
            for (int sz = 2; sz <= 16; sz <<= 1)
#pragma unroll
                for (int d = sz >> 1; d > 0; d >>= 1)
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        const int lo = 2 * i - (i & (d - 1));
                        compare_exchange(v[lo], v[lo + d], ((base + lo) & sz) == 0);
                    }
        } else {
            const bool descending = (base & size) == 0;
#pragma unroll
            for (int d = 8; d > 0; d >>= 1)
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const int lo = 2 * i - (i & (d - 1));
                    compare_exchange(v[lo], v[lo + d], descending);
                }
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            key64x2 t;
            t.x = v[2 * j];
            t.y = v[2 * j + 1];
            blk[j] = t;
        }
    }
    __builtin_amdgcn_wave_barrier();
}

// s: sort_slots(P) keys of LDS owned by this wave, key i at s[SortSlot()(i)].
__device__ inline void wave_sort_descending(key64_t* s, int P) {
    sort_block16<true>(s, P, 0);
    for (int lg = 5; (1 << lg) <= P; ++lg) {
        const int size = 1 << lg;
        for (int top = lg; top > 4;) {  // stride bits [4, lg), four at a time from the top
            const int nb = min(4, top - 4);
            const int b = top - nb;
            if (nb == 4) sort_pass<4>(s, P, b, size);
            else if (nb == 3) sort_pass<3>(s, P, b, size);
            else if (nb == 2) sort_pass<2>(s, P, b, size);
            else sort_pass<1>(s, P, b, size);
            top = b;
        }
        sort_block16<false>(s, P, size);
    }
}

// Dense-score front end (entry point si_topk_from_scores): appends the legal entries of one
// column tile that beat the row's threshold to the row's buffer.  Same contract as the filter
// mode of the score kernel.
__global__ __launch_bounds__(kTopkThreads) void filter_scores_kernel(
    const float* __restrict__ scores, int n_cols, int t0, int width,
    const int32_t* __restrict__ legal_rows, RowBuffers rb) {
    __shared__ int s_cnt;
    const int tid = threadIdx.x;
    const int64_t row = blockIdx.x;
    const int L = legal_rows ? legal_rows[row] : n_cols;
    const int n = min(width, L - t0);  // legal entries of this row inside the tile
    if (n <= 0) return;
    const float* sc = scores + row * n_cols + t0;
    const float theta = rb.theta[row];
    const int c0 = rb.count[row];
    key64_t* buf = rb.keys + row * rb.cap;
    if (tid == 0) s_cnt = 0;
    __syncthreads();
    for (int j = tid; j < n; j += kTopkThreads) {
        const float v = sc[j];
        if (v > theta) buf[c0 + atomicAdd(&s_cnt, 1)] = make_key(v, static_cast<uint32_t>(t0 + j));
    }
    __syncthreads();
    if (tid == 0) rb.count[row] = c0 + s_cnt;
}


__host__ __device__ inline int compact_limit(int k) { return k + k / 16; }
constexpr int kCompactRegKeys = 48;   // compaction keeps rows of up to 3072 keys in registers
constexpr int kFinalizeRegKeys = 32;  // finalize: rows of up to 2048 keys

// Merge step, done lazily: a row's buffer holds the k best keys of an earlier prefix plus
// everything appended since.  Once it holds at least `trigger` keys it is cut back to its best
// k .. k + k/16 keys (an exact cut is only needed at the very end) and the row's threshold is
// raised to the score below which everything was dropped.  One wave per row.
__global__ __launch_bounds__(kTopkThreads) void compact_kernel(RowBuffers rb, int rows, int tile_rows,
                                                               int k, int trigger) {
    __shared__ int s_hist[kRowWaves][256];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    {
        const int r = blockIdx.x * kRowWaves + wave;
        if (r >= rows) return;
        const int64_t row = static_cast<int64_t>(blockIdx.y) * tile_rows + r;
        const int c = rb.count[row];
        if (c < trigger) return;  // most rows need nothing on most calls
        key64_t* buf = rb.keys + row * rb.cap;
        int kept = 0;
        key64_t thr;
        if (c <= 64 * kCompactRegKeys) {  // the usual case: one read of the row
            RegKeys<kCompactRegKeys> keys;
            keys.load(buf, c);
            thr = wave_radix_kth(keys, k, compact_limit(k), s_hist[wave], &kept);
            wave_keep(keys, thr, buf, rb.cap);
        } else {
            const StreamKeys keys{buf, c};
            thr = wave_radix_kth(keys, k, compact_limit(k), s_hist[wave], &kept);
            wave_keep(keys, thr, buf, rb.cap);
        }
        if ((threadIdx.x & 63) == 0) {
            rb.count[row] = kept;
            rb.theta[row] = fmaxf(rb.theta[row], key_score(thr));  // the cut may be coarser than the old threshold
        }
    }
}

// After the last key tile: final exact cut to k, sort best first, decode, pad (Section 4.2).
// One wave per row; the sort runs in the wave's own slice of LDS.
__global__ __launch_bounds__(kTopkThreads) void finalize_kernel(
    RowBuffers rb, int rows, int tile_rows, int k, int pow2_k, int64_t out_batch_stride,
    int64_t out_row0, int32_t* __restrict__ out_idx, float* __restrict__ out_score) {
    extern __shared__ __attribute__((aligned(16))) key64_t s_sort_all[];  // [kRowWaves][sort_slots(pow2_k)]
    __shared__ int s_hist[kRowWaves][256];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int r = blockIdx.x * kRowWaves + wave;
    if (r >= rows) return;
    const int64_t row = static_cast<int64_t>(blockIdx.y) * tile_rows + r;
    const key64_t* buf = rb.keys + row * rb.cap;
    key64_t* s_sort = s_sort_all + static_cast<size_t>(wave) * sort_slots(pow2_k);
    const SortSlot slot;
    const int n = rb.count[row];
    int c = min(n, k);
    if (n <= 64 * kFinalizeRegKeys) {
        RegKeys<kFinalizeRegKeys> keys;
        keys.load(buf, n);
        key64_t thr = 0ull;
        int kept = 0;
        if (n > k) thr = wave_radix_kth(keys, k, k, s_hist[wave], &kept);  // limit k: exact
        wave_keep(keys, thr, s_sort, pow2_k, slot);
    } else {
        const StreamKeys keys{buf, n};
        key64_t thr = 0ull;
        int kept = 0;
        if (n > k) thr = wave_radix_kth(keys, k, k, s_hist[wave], &kept);
        wave_keep(keys, thr, s_sort, pow2_k, slot);
    }
    int P = 16;
    while (P < c) P <<= 1;
    for (int i = c + lane; i < P; i += 64) s_sort[slot(i)] = 0ull;  // empty keys sort last
    __builtin_amdgcn_wave_barrier();
    wave_sort_descending(s_sort, P);
    const int64_t o = (static_cast<int64_t>(blockIdx.y) * out_batch_stride + out_row0 + r) * k;
    for (int j = lane; j < k; j += 64) {
        if (j < c) {
            const key64_t key = s_sort[slot(j)];
            out_idx[o + j] = key_index(key);
            out_score[o + j] = key_score(key);
        } else {  // Section 4.2: pad
            out_idx[o + j] = -1;
            out_score[o + j] = -__builtin_huge_valf();
        }
    }
}

__global__ void init_rows_kernel(int32_t* count, float* theta, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) {
        count[i] = 0;
        theta[i] = -__builtin_huge_valf();
    }
}

namespace {
// Large k: raises finalize_kernel's dynamic LDS limit (gfx950 has 160 KB per CU).  Done once per
// device and size, so that later calls (possibly under stream capture) launch only.
hipError_t allow_finalize_lds(size_t bytes) {
    if (bytes <= 32 * 1024) return hipSuccess;
    const void* fn = reinterpret_cast<const void*>(finalize_kernel);
    constexpr int kMaxDevices = 64;
    static std::atomic<size_t> allowed[kMaxDevices];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const bool tracked = dev >= 0 && dev < kMaxDevices;
    if (tracked && allowed[dev].load(std::memory_order_acquire) >= bytes) return hipSuccess;
    e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(bytes));
    if (e == hipSuccess && tracked) {
        size_t seen = allowed[dev].load(std::memory_order_relaxed);
        while (seen < bytes && !allowed[dev].compare_exchange_weak(seen, bytes, std::memory_order_release)) {}
    }
    return e;
}
}  // namespace

hipError_t launch_init_rows(const RowBuffers& rb, int32_t n, hipStream_t stream) {
    hipLaunchKernelGGL(init_rows_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, rb.count, rb.theta, n);
    return hipGetLastError();
}

hipError_t launch_filter_scores(const float* scores, int32_t R, int32_t n_cols, int32_t t0,
                                int32_t width, const int32_t* legal_rows, const RowBuffers& rb,
                                hipStream_t stream) {
    hipLaunchKernelGGL(filter_scores_kernel, dim3(R), dim3(kTopkThreads), 0, stream, scores, n_cols, t0,
                       width, legal_rows, rb);
    return hipGetLastError();
}

hipError_t launch_compact(const RowBuffers& rb, int32_t B, int32_t rows, int32_t tile_rows, int32_t k,
                          int32_t trigger, hipStream_t stream) {
    hipLaunchKernelGGL(compact_kernel, dim3((rows + kRowWaves - 1) / kRowWaves, B), dim3(kTopkThreads), 0, stream, rb, rows, tile_rows, k,
                       trigger);
    return hipGetLastError();
}

hipError_t launch_finalize(const RowBuffers& rb, int32_t B, int32_t rows, int32_t tile_rows, int32_t k,
                           int64_t out_batch_stride, int64_t out_row0, int32_t* out_idx,
                           float* out_score, hipStream_t stream) {
    int pow2_k = 16;
    while (pow2_k < k) pow2_k <<= 1;
    const size_t lds = static_cast<size_t>(kRowWaves) * sort_slots(pow2_k) * sizeof(key64_t);
    hipError_t e = allow_finalize_lds(lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(finalize_kernel, dim3((rows + kRowWaves - 1) / kRowWaves, B), dim3(kTopkThreads), lds,
                       stream, rb, rows, tile_rows, k, pow2_k, out_batch_stride, out_row0, out_idx, out_score);
    return hipGetLastError();
}

}  // namespace si
