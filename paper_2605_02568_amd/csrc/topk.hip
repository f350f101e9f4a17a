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
//   finalize: last cut to k, bitonic sort in LDS, decode to (index, score), pad (Section 4.2).

#include "si_internal.h"

namespace si {

constexpr int kTopkThreads = 256;

constexpr int kHistCopies = kTopkThreads / 64;  // one histogram per wave: less atomic contention

struct SelectShared {
    int hist[kHistCopies][256];
    int tmp;
    int digit, need, bin;
};

__device__ inline int block_sum(int v, int* s_scratch) {
    // wave reduce, then one LDS atomic per wave
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    if (threadIdx.x == 0) *s_scratch = 0;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) atomicAdd(s_scratch, v);
    __syncthreads();
    const int total = *s_scratch;
    __syncthreads();
    return total;
}

// Threshold key `thr` such that exactly k of the n keys produced by fetch(j), j in [0,n),
// that are > floor satisfy key >= thr.  Requires more than k such keys.  All threads of the
// workgroup call it with the same arguments.
template <typename Fetch>
__device__ inline key64_t radix_kth(Fetch fetch, int n, key64_t floor_key, int k, SelectShared& sh) {
    const int tid = threadIdx.x;
    key64_t prefix = 0ull;
    int need = k;
    for (int shift = 56; shift >= 0; shift -= 8) {
#pragma unroll
        for (int cpy = 0; cpy < kHistCopies; ++cpy) sh.hist[cpy][tid] = 0;
        __syncthreads();
        for (int j = tid; j < n; j += kTopkThreads) {
            const key64_t key = fetch(j);
            const bool in_prefix = (shift == 56) || ((key >> (shift + 8)) == (prefix >> (shift + 8)));
            if (key > floor_key && in_prefix) atomicAdd(&sh.hist[tid >> 6][(key >> shift) & 255ull], 1);
        }
        __syncthreads();
        if (tid < 64) {
            // Wave 0 walks the bins from the top: lane l owns bins 255-4l .. 252-4l.  A wave
            // prefix sum locates the lane, then the bin, where the running count reaches `need`.
            int h[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                h[j] = 0;
#pragma unroll
                for (int cpy = 0; cpy < kHistCopies; ++cpy) h[j] += sh.hist[cpy][255 - 4 * tid - j];
            }
            const int local = h[0] + h[1] + h[2] + h[3];
            int incl = local;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const int up = __shfl_up(incl, off);
                if (tid >= off) incl += up;
            }
            int cum = incl - local;  // keys in bins above this lane's
            if (cum < need && need <= incl) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (cum < need && need <= cum + h[j]) {
                        sh.digit = 255 - 4 * tid - j;
                        sh.need = need - cum;
                        sh.bin = h[j];
                    }
                    cum += h[j];
                }
            }
        }
        __syncthreads();
        prefix |= static_cast<key64_t>(sh.digit) << shift;
        need = sh.need;
        const bool whole_bin = (sh.bin == need);
        __syncthreads();
        if (whole_bin) break;  // every key of this bin is kept: prefix is the threshold
    }
    return prefix;
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

constexpr int kStageKeys = 4096;  // buffers up to this long are staged in LDS for the selection

// Keeps exactly the k best of a row's n > k buffered keys in s_keep[0,k) (any order) and
// returns the smallest kept key.  s_stage: kStageKeys slots of LDS; the radix passes read the
// keys from there when they fit, else from global memory.  All threads of the workgroup call it.
__device__ inline key64_t keep_top_k(const key64_t* buf, int n, int k, key64_t* s_keep,
                                     key64_t* s_stage, SelectShared& sh, key64_t* s_min) {
    const key64_t* src = buf;
    if (n <= kStageKeys) {
        for (int j = threadIdx.x; j < n; j += kTopkThreads) s_stage[j] = buf[j];
        __syncthreads();
        src = s_stage;
    }
    auto fetch = [&](int j) { return src[j]; };
    const key64_t thr = radix_kth(fetch, n, 0ull, k, sh);
    if (threadIdx.x == 0) {
        sh.tmp = 0;
        *s_min = ~0ull;
    }
    __syncthreads();
    for (int j = threadIdx.x; j < n; j += kTopkThreads) {
        const key64_t key = src[j];
        if (key >= thr) {
            const int pos = atomicAdd(&sh.tmp, 1);
            if (pos < k) s_keep[pos] = key;  // pos < k always holds; the guard keeps a slip in bounds
            atomicMin(s_min, key);
        }
    }
    __syncthreads();
    return *s_min;
}

// Merge step, done lazily: a row's buffer holds the k best keys of an earlier prefix plus
// everything appended since.  Once it holds at least `trigger` keys it is cut back to its k
// best and the row's threshold becomes the score of the k-th of them.
__global__ __launch_bounds__(kTopkThreads) void compact_kernel(RowBuffers rb, int rows, int tile_rows,
                                                               int k, int trigger) {
    extern __shared__ key64_t s_keep[];  // [k] kept keys, then [kStageKeys] staging
    __shared__ SelectShared sh;
    __shared__ key64_t s_min;
    const int64_t row = static_cast<int64_t>(blockIdx.y) * tile_rows + blockIdx.x;
    (void)rows;
    const int c = rb.count[row];
    if (c < trigger) return;
    key64_t* buf = rb.keys + row * rb.cap;
    const key64_t kth = keep_top_k(buf, c, k, s_keep, s_keep + k, sh, &s_min);
    for (int i = threadIdx.x; i < k; i += kTopkThreads) buf[i] = s_keep[i];
    if (threadIdx.x == 0) {
        rb.count[row] = k;
        rb.theta[row] = key_score(kth);
    }
}

// After the last key tile: final cut to k, sort best first, decode, pad (Section 4.2).
__global__ __launch_bounds__(kTopkThreads) void finalize_kernel(
    RowBuffers rb, int tile_rows, int k, int pow2_k, int64_t out_batch_stride, int64_t out_row0,
    int32_t* __restrict__ out_idx, float* __restrict__ out_score) {
    extern __shared__ key64_t s_keep[];  // [pow2_k] kept keys, then [kStageKeys] staging
    __shared__ SelectShared sh;
    __shared__ key64_t s_min;
    const int tid = threadIdx.x;
    const int64_t row = static_cast<int64_t>(blockIdx.y) * tile_rows + blockIdx.x;
    const key64_t* buf = rb.keys + row * rb.cap;
    int c = rb.count[row];
    if (c > k) {
        keep_top_k(buf, c, k, s_keep, s_keep + pow2_k, sh, &s_min);
        c = k;
    } else {
        for (int i = tid; i < c; i += kTopkThreads) s_keep[i] = buf[i];
    }
    int P = 1;
    while (P < c) P <<= 1;
    for (int i = c + tid; i < P; i += kTopkThreads) s_keep[i] = 0ull;
    __syncthreads();
    // bitonic sort, best (largest key) first
    for (int size = 2; size <= P; size <<= 1) {
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            for (int i = tid; i < (P >> 1); i += kTopkThreads) {
                const int lo = 2 * i - (i & (stride - 1));
                const int hi = lo + stride;
                const bool descending = (lo & size) == 0;
                const key64_t x = s_keep[lo], y = s_keep[hi];
                if ((x < y) == descending) {
                    s_keep[lo] = y;
                    s_keep[hi] = x;
                }
            }
            __syncthreads();
        }
    }
    const int64_t o = (static_cast<int64_t>(blockIdx.y) * out_batch_stride + out_row0 + blockIdx.x) * k;
    for (int j = tid; j < k; j += kTopkThreads) {
        if (j < c) {
            const key64_t key = s_keep[j];
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
hipError_t allow_lds(const void* fn, size_t bytes) {
    if (bytes <= 32 * 1024) return hipSuccess;
    // large k: raise the kernel's dynamic LDS limit (gfx950 has 160 KB per CU)
    return hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(bytes));
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
    const size_t lds = (static_cast<size_t>(k) + kStageKeys) * sizeof(key64_t);
    hipError_t e = allow_lds(reinterpret_cast<const void*>(compact_kernel), lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(compact_kernel, dim3(rows, B), dim3(kTopkThreads), lds, stream, rb, rows, tile_rows,
                       k, trigger);
    return hipGetLastError();
}

hipError_t launch_finalize(const RowBuffers& rb, int32_t B, int32_t rows, int32_t tile_rows, int32_t k,
                           int64_t out_batch_stride, int64_t out_row0, int32_t* out_idx,
                           float* out_score, hipStream_t stream) {
    int pow2_k = 1;
    while (pow2_k < k) pow2_k <<= 1;
    const size_t lds = (static_cast<size_t>(pow2_k) + kStageKeys) * sizeof(key64_t);
    hipError_t e = allow_lds(reinterpret_cast<const void*>(finalize_kernel), lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(finalize_kernel, dim3(rows, B), dim3(kTopkThreads), lds, stream, rb, tile_rows, k,
                       pow2_k, out_batch_stride, out_row0, out_idx, out_score);
    return hipGetLastError();
}

}  // namespace si
