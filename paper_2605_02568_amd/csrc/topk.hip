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
#include "topk_wave.h"

namespace si {

constexpr int kTopkThreads = 256;

constexpr int kRowWaves = kTopkThreads / 64;  // compaction / finalize: one wave per query row

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
    const int64_t o = (static_cast<int64_t>(blockIdx.y) * out_batch_stride + out_row0 + r) * k;
    if (n < 0) {  // the score kernel marked the row: its buffer overflowed
        poison_row(out_idx, out_score, o, k);
        return;
    }
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

hipError_t launch_filter_scores(const float* scores, int32_t R, int32_t n_cols, int32_t k, int32_t t0,
                                int32_t width, const int32_t* legal_rows, const RowBuffers& rb,
                                hipStream_t stream) {
    // same room rule as the score kernel's filter: fewer than 2k keys held, at most `width` more
    if (k < 1 || width < 1 || static_cast<int64_t>(rb.cap) < 2 * static_cast<int64_t>(k) + width)
        return hipErrorInvalidValue;
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
