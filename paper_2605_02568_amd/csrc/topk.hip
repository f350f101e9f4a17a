// Per-tile select, cross-tile merge and write-out (Algorithm 2: the topk, merge_topk and
// out[...] <- run steps; Section 4.3 corollary for why per-tile top-k then merge is exact).
//
// All three work on 64-bit keys whose unsigned order is the total order of Section 4.1
// (see make_key), so a tie on score is always resolved towards the smaller key index and
// the final top-k set is unique: whatever the tiling, the same keys come out.
//
// select : exact top-min(k, n) of one row's candidates.  If at most k candidates exist all
//          are kept (this is also the "saturated tile" branch of Section 6.6: a tile narrower
//          than k keeps every entry); otherwise an MSB-first radix descent over the 64-bit
//          keys (8 bits per pass, LDS histogram) finds the k-th largest and exactly k are kept.
//          Two front ends share it: select_kernel reads a dense fp32 score tile (and first
//          drops entries that do not beat the row's current k-th best); merge_kernel applies
//          it to a candidate list that the fused score kernel has already filtered.
// merge  : one workgroup per row.  Candidates are sorted in LDS (bitonic), then each element
//          of the two sorted lists finds its rank in the union by binary search in the other
//          list; ranks below k are written back as the new running buffer.
// write-out: decode keys to (index, score) and pad (Section 4.2).

#include "si_internal.h"

namespace si {

constexpr int kTopkThreads = 256;

struct SelectShared {
    int hist[256];
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
        sh.hist[tid] = 0;
        __syncthreads();
        for (int j = tid; j < n; j += kTopkThreads) {
            const key64_t key = fetch(j);
            const bool in_prefix = (shift == 56) || ((key >> (shift + 8)) == (prefix >> (shift + 8)));
            if (key > floor_key && in_prefix) atomicAdd(&sh.hist[(key >> shift) & 255ull], 1);
        }
        __syncthreads();
        if (tid == 0) {
            int cum = 0, d = 255;
            for (; d > 0; --d) {
                if (cum + sh.hist[d] >= need) break;
                cum += sh.hist[d];
            }
            sh.digit = d;
            sh.need = need - cum;
            sh.bin = sh.hist[d];
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

__global__ __launch_bounds__(kTopkThreads) void select_kernel(TopkTileArgs a) {
    __shared__ SelectShared sh;
    const int tid = threadIdx.x;
    const int64_t row = static_cast<int64_t>(blockIdx.y) * a.tile_rows + blockIdx.x;
    const int L = a.legal_rows ? a.legal_rows[row]
                               : legal_count(a.s0 + blockIdx.x, a.T, a.m, a.mask_mode);
    const int n = min(a.width, L - a.t0);  // legal entries of this row inside the tile
    if (n <= 0) {
        if (tid == 0) a.cand_count[row] = 0;
        return;
    }
    const float* sc = a.scores + row * a.tile_cols + a.col0;
    const int k = a.k;
    const key64_t theta = (a.run_count[row] == k) ? a.run_keys[row * k + k - 1] : 0ull;
    key64_t* cand = a.cand_keys + row * a.cand_stride;
    const uint32_t idx0 = static_cast<uint32_t>(a.t0);
    auto fetch = [&](int j) { return make_key(sc[j], idx0 + j); };

    // survivors: entries strictly better than the current k-th best
    int mine = 0;
    for (int j = tid; j < n; j += kTopkThreads) mine += fetch(j) > theta;
    const int c = block_sum(mine, &sh.tmp);

    key64_t thr = theta + 1ull;  // keep key >= thr
    if (c > k) thr = radix_kth(fetch, n, theta, k, sh);

    if (tid == 0) sh.tmp = 0;
    __syncthreads();
    for (int j = tid; j < n; j += kTopkThreads) {
        const key64_t key = fetch(j);
        if (key >= thr) {
            const int pos = atomicAdd(&sh.tmp, 1);
            if (pos < k) cand[pos] = key;  // pos < k always holds; the guard keeps a logic slip in bounds
        }
    }
    if (tid == 0) a.cand_count[row] = min(c, k);
}

__global__ __launch_bounds__(kTopkThreads) void merge_kernel(TopkTileArgs a, int pow2_k) {
    extern __shared__ key64_t smem[];
    __shared__ SelectShared sh;
    key64_t* s_cand = smem;           // [pow2_k]
    key64_t* s_run = smem + pow2_k;   // [k]

    const int tid = threadIdx.x;
    const int64_t row = static_cast<int64_t>(blockIdx.y) * a.tile_rows + blockIdx.x;
    int c = a.cand_count[row];
    if (c == 0) return;
    const int k = a.k;
    const int rc = a.run_count[row];
    key64_t* run = a.run_keys + row * k;
    const key64_t* cand = a.cand_keys + row * a.cand_stride;

    if (c > k) {
        // more candidates than slots: keep exactly the k best of them
        auto fetch = [&](int j) { return cand[j]; };
        const key64_t thr = radix_kth(fetch, c, 0ull, k, sh);
        if (tid == 0) sh.tmp = 0;
        __syncthreads();
        for (int j = tid; j < c; j += kTopkThreads) {
            const key64_t key = cand[j];
            if (key >= thr) {
                const int pos = atomicAdd(&sh.tmp, 1);
                if (pos < k) s_cand[pos] = key;
            }
        }
        c = k;
        for (int i = k + tid; i < pow2_k; i += kTopkThreads) s_cand[i] = 0ull;
    } else {
        int P = 1;
        while (P < c) P <<= 1;
        for (int i = tid; i < P; i += kTopkThreads) s_cand[i] = (i < c) ? cand[i] : 0ull;
    }
    for (int i = tid; i < rc; i += kTopkThreads) s_run[i] = run[i];
    __syncthreads();

    int P = 1;
    while (P < c) P <<= 1;
    // bitonic sort of the candidates, best (largest key) first
    for (int size = 2; size <= P; size <<= 1) {
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            for (int i = tid; i < (P >> 1); i += kTopkThreads) {
                const int lo = 2 * i - (i & (stride - 1));
                const int hi = lo + stride;
                const bool descending = (lo & size) == 0;
                const key64_t x = s_cand[lo], y = s_cand[hi];
                if ((x < y) == descending) {
                    s_cand[lo] = y;
                    s_cand[hi] = x;
                }
            }
            __syncthreads();
        }
    }

    // rank of each element in the union = own position + number of better elements in the
    // other list (all keys are distinct: a key index appears once)
    for (int i = tid; i < rc; i += kTopkThreads) {
        const key64_t x = s_run[i];
        int lo = 0, hi = c;  // first position in s_cand[0,c) holding a key < x
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (s_cand[mid] > x) lo = mid + 1; else hi = mid;
        }
        const int rank = i + lo;
        if (rank < k) run[rank] = x;
    }
    for (int j = tid; j < c; j += kTopkThreads) {
        const key64_t y = s_cand[j];
        int lo = 0, hi = rc;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (s_run[mid] > y) lo = mid + 1; else hi = mid;
        }
        const int rank = j + lo;
        if (rank < k) run[rank] = y;
    }
    if (tid == 0) a.run_count[row] = min(k, rc + c);
}

__global__ __launch_bounds__(kTopkThreads) void writeout_kernel(
    const key64_t* __restrict__ run_keys, const int32_t* __restrict__ run_count, int rows,
    int tile_rows, int k, int64_t out_batch_stride, int64_t out_row0,
    int32_t* __restrict__ out_idx, float* __restrict__ out_score) {
    const int64_t e = static_cast<int64_t>(blockIdx.x) * kTopkThreads + threadIdx.x;
    if (e >= static_cast<int64_t>(rows) * k) return;
    const int r = static_cast<int>(e / k);
    const int j = static_cast<int>(e % k);
    const int64_t row = static_cast<int64_t>(blockIdx.y) * tile_rows + r;
    const int64_t o = (static_cast<int64_t>(blockIdx.y) * out_batch_stride + out_row0 + r) * k + j;
    if (j < run_count[row]) {
        const key64_t key = run_keys[row * k + j];
        out_idx[o] = key_index(key);
        out_score[o] = key_score(key);
    } else {  // Section 4.2: pad
        out_idx[o] = -1;
        out_score[o] = -__builtin_huge_valf();
    }
}

__global__ void init_rows_kernel(int32_t* run_count, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) run_count[i] = 0;
}

hipError_t launch_init_rows(int32_t* run_count, int32_t n, hipStream_t stream) {
    hipLaunchKernelGGL(init_rows_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, run_count, n);
    return hipGetLastError();
}

hipError_t launch_select(const TopkTileArgs& a, hipStream_t stream) {
    hipLaunchKernelGGL(select_kernel, dim3(a.rows, a.B), dim3(kTopkThreads), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_merge(const TopkTileArgs& a, hipStream_t stream) {
    int pow2_k = 1;
    while (pow2_k < a.k) pow2_k <<= 1;
    const size_t lds = (static_cast<size_t>(pow2_k) + a.k) * sizeof(key64_t);
    if (lds > 32 * 1024) {  // large k: raise the kernel's dynamic LDS limit (gfx950 has 160 KB per CU)
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(merge_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(merge_kernel, dim3(a.rows, a.B), dim3(kTopkThreads), lds, stream, a, pow2_k);
    return hipGetLastError();
}

hipError_t launch_writeout(const key64_t* run_keys, const int32_t* run_count, int32_t B,
                           int32_t rows, int32_t tile_rows, int32_t k, int64_t out_batch_stride,
                           int64_t out_row0, int32_t* out_idx, float* out_score,
                           hipStream_t stream) {
    const int64_t elems = static_cast<int64_t>(rows) * k;
    const dim3 grid(static_cast<unsigned>((elems + kTopkThreads - 1) / kTopkThreads), B);
    hipLaunchKernelGGL(writeout_kernel, grid, dim3(kTopkThreads), 0, stream, run_keys, run_count,
                       rows, tile_rows, k, out_batch_stride, out_row0, out_idx, out_score);
    return hipGetLastError();
}

}  // namespace si
