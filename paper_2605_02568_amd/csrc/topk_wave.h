// Wave-level building blocks of the per-tile select, the merge and the write-out (Algorithm 2):
// radix selection of the k-th largest key, order-preserving compaction, and a bitonic sort, each
// run by one 64-lane wave on one query row without workgroup barriers.  Keys are the 64-bit
// (score, ~index) words of si_internal.h, whose unsigned order is the total order of Section 4.1.
#pragma once

#include "si_internal.h"

namespace si {

constexpr int kKeysInFlight = 16;  // global loads a lane issues before it uses them

// A mid-stream cut keeps the best k .. compact_limit(k) keys of a row (only the last cut has to
// be exact).
__host__ __device__ inline int compact_limit(int k) { return k + k / 16; }

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
        n = min(n_, 64 * R);
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
// are >= thr, with k <= kept <= max(k, limit).  MSB-first radix descent, up to 8 bits per pass; it
// stops as soon as the bin holding the k-th largest key is small enough for `kept` to respect
// the limit (limit == k: exact selection).  Requires n > k.  Wave-uniform arguments.
//
// The descent starts at the highest bit in which two score words of the row differ (one OR / AND
// scan of the keys): the candidates of a row are the upper tail of its score distribution, so their
// sign and exponent bits agree, and a first pass over those bits would put every key into one or
// two bins -- no information, and 64 lanes adding to the same LDS word serialise.  Windows never
// straddle the boundary between the score word and the index word, so each pass works on one
// 32-bit half of the keys.
template <typename Keys>
__device__ inline key64_t wave_radix_kth(const Keys& keys, int k, int limit, int* hist, int* kept) {
    const int lane = threadIdx.x & 63;
    uint32_t any_hi = 0u, all_hi = 0xFFFFFFFFu;
    keys.sweep([&](key64_t key, bool valid) {
        const uint32_t hi = static_cast<uint32_t>(key >> 32);
        any_hi |= valid ? hi : 0u;
        all_hi &= valid ? hi : 0xFFFFFFFFu;
    });
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        any_hi |= __shfl_xor(any_hi, off);
        all_hi &= __shfl_xor(all_hi, off);
    }
    const uint32_t diff_hi = __builtin_amdgcn_readfirstlane(any_hi ^ all_hi);
    // highest undecided bit of the 64-bit key; equal scores everywhere: the index word decides
    int top = diff_hi != 0u ? 63 - __builtin_clz(diff_hi) : 31;
    key64_t prefix = top >= 32
        ? static_cast<key64_t>(__builtin_amdgcn_readfirstlane(all_hi) & ~((2u << (top - 32)) - 1u)) << 32
        : static_cast<key64_t>(__builtin_amdgcn_readfirstlane(all_hi)) << 32;
    int need = k;
    int bin = 0;
    for (;;) {
        const int shift = max(top - 7, top >= 32 ? 32 : 0);  // this pass decides bits [shift, top]
        const int nbits = top - shift + 1;
        const uint32_t dmask = (1u << nbits) - 1u;
#pragma unroll
        for (int i = 0; i < 4; ++i) hist[lane + 64 * i] = 0;
        __builtin_amdgcn_wave_barrier();
        if (shift >= 32) {
            // digits of the score word: 32-bit arithmetic on the high half of the key
            const int sh = shift - 32;
            const bool whole = top == 63;  // nothing above the window
            const uint32_t want = whole ? 0u : static_cast<uint32_t>(prefix >> 32) >> (top - 31);
            keys.sweep([&](key64_t key, bool valid) {
                const uint32_t hi = static_cast<uint32_t>(key >> 32);
                const bool in_prefix = whole || ((hi >> (top - 31)) == want);
                if (valid && in_prefix) atomicAdd(&hist[(hi >> sh) & dmask], 1);
            });
        } else {
            // equal scores: digits of the index word
            const key64_t want = prefix >> (top + 1);
            keys.sweep([&](key64_t key, bool valid) {
                const bool in_prefix = (key >> (top + 1)) == want;
                if (valid && in_prefix) atomicAdd(&hist[static_cast<uint32_t>(key >> shift) & dmask], 1);
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
        if (k - need + bin <= limit || shift == 0) break;
        top = shift - 1;
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

// The LG lowest strides (2^(LG-1) .. 1) on a lane's own block of E = 2^LG consecutive keys (LG = 3
// or 4, so that a block never straddles a padding gap); with FIRST, the whole network up to runs
// of E (sizes 2 .. E) instead.
template <int LG, bool FIRST>
__device__ inline void sort_block(key64_t* s, int P, int size) {
    constexpr int E = 1 << LG;
    typedef key64_t key64x2 __attribute__((ext_vector_type(2)));
    const SortSlot slot;
    const int lane = threadIdx.x & 63;
    for (int base = E * lane; base < P; base += E * 64) {
        key64x2* blk = reinterpret_cast<key64x2*>(s + slot(base));  // 16-byte aligned
        key64_t v[E];
#pragma unroll
        for (int j = 0; j < E / 2; ++j) {
            const key64x2 t = blk[j];
            v[2 * j] = t.x;
            v[2 * j + 1] = t.y;
        }
        if (FIRST) {
#pragma unroll
            for (int sz = 2; sz <= E; sz <<= 1)
#pragma unroll
                for (int d = sz >> 1; d > 0; d >>= 1)
#pragma unroll
                    for (int i = 0; i < E / 2; ++i) {
                        const int lo = 2 * i - (i & (d - 1));
                        compare_exchange(v[lo], v[lo + d], ((base + lo) & sz) == 0);
                    }
        } else {
            const bool descending = (base & size) == 0;
#pragma unroll
            for (int d = E / 2; d > 0; d >>= 1)
#pragma unroll
                for (int i = 0; i < E / 2; ++i) {
                    const int lo = 2 * i - (i & (d - 1));
                    compare_exchange(v[lo], v[lo + d], descending);
                }
        }
#pragma unroll
        for (int j = 0; j < E / 2; ++j) {
            key64x2 t;
            t.x = v[2 * j];
            t.y = v[2 * j + 1];
            blk[j] = t;
        }
    }
    __builtin_amdgcn_wave_barrier();
}

// LG = keys per lane and pass (as a power of two): 4 keeps all 64 lanes busy from P = 1024 on,
// 3 does so for P = 512.
template <int LG>
__device__ inline void wave_sort_descending_by(key64_t* s, int P) {
    sort_block<LG, true>(s, P, 0);
    for (int lg = LG + 1; (1 << lg) <= P; ++lg) {
        const int size = 1 << lg;
        for (int top = lg; top > LG;) {  // stride bits [LG, lg), up to LG at a time from the top
            const int nb = min(LG, top - LG);
            const int b = top - nb;
            if (nb == 4) sort_pass<4>(s, P, b, size);
            else if (nb == 3) sort_pass<3>(s, P, b, size);
            else if (nb == 2) sort_pass<2>(s, P, b, size);
            else sort_pass<1>(s, P, b, size);
            top = b;
        }
        sort_block<LG, false>(s, P, size);
    }
}

// s: sort_slots(P) keys of LDS owned by this wave, key i at s[SortSlot()(i)]; P a power of two >= 16.
__device__ inline void wave_sort_descending(key64_t* s, int P) {
    if (P <= 512) wave_sort_descending_by<3>(s, P);
    else wave_sort_descending_by<4>(s, P);
}

}  // namespace si
