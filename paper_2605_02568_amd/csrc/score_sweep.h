// The key sweep of the fused score kernel (Section 5, "fused score kernel"; Section 1 for the
// formula):
//   score[t, s] = sum_h w[t,h] * max(0, sum_d q[t,h,d] * K[s,d])
// for the queries of one workgroup (one per wave) against a run of consecutive keys.  bf16 operands, fp32
// MFMA accumulation, ReLU and the weighted head sum done on the MFMA result registers; the
// per-head values never leave the wave.
//
// Mapping (gfx950, wave64, v_mfma_f32_32x32x16_bf16):
//   - one wave owns one query for the whole key sweep.  The query's heads are the M side of
//     the MFMA (32 heads per block, HB blocks), kept in registers: HB * D/16 operands of
//     8 bf16.  Keys are the N side, 32 per MFMA, read from LDS.
//   - the 32x32 result puts one key per lane column (lane & 31) and 16 heads per lane, so the
//     head sum is 16 in-lane FMAs per head block plus one exchange between lane and lane^32.
//   - a workgroup is 8 (or 4, see SweepShape) waves = consecutive queries sharing each staged
//     block of 128 (64) keys.  Key blocks travel HBM/L2 -> LDS directly (buffer_load ... lds, no
//     register round trip) into a ring of three (four) buffers, two (three) blocks ahead of the
//     one being multiplied.
//   - the loop is a software pipeline over 32-key sub-blocks: MFMAs of sub-block g, epilogue
//     of sub-block g-1 and LDS reads for sub-block g+1 are interleaved instruction by
//     instruction, so the matrix pipe, the vector ALU and the LDS work at the same time.
// Every (query, key) score is produced by the same instruction sequence wherever the pair
// falls in a sweep, which is what makes results independent of the tiling.
//
// Two outputs, chosen at compile time:
//   dense  : the fp32 scores themselves (entry point si_score_tile);
//   filter : the per-tile mask (Section 5) and the first half of the per-tile select are
//            applied in registers: only legal entries that beat the row's threshold (the k-th
//            best score of an earlier prefix of the key axis) are appended, as 64-bit
//            (score, ~index) keys, to the row's buffer.  An entry that does not beat it can
//            never enter the final top-k: keys are visited in ascending index order, so on
//            equal score the entry already held has the smaller index and wins
//            (Section 4.1).  One wave owns one row, so the append needs no atomics.
#pragma once

#include "si_internal.h"

namespace si {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kWaves = 8;            // waves per workgroup of the wide shape, one query each
constexpr int kQB = kWaves;          // queries per workgroup
constexpr int kKeyChunk = 128;       // keys per LDS buffer
constexpr int kScoreThreads = 64 * kWaves;
constexpr int kLdsBuffers = 3;

// Two workgroup shapes share the sweep.
//   wide   (8 waves): 8 queries share every staged key chunk; chunks of 128 keys in a ring of three
//          buffers (96 KiB at D = 128), one workgroup per compute unit.  Least key traffic per
//          query: the shape for long key ranges and for the tiled schedule.
//   narrow (4 waves): 4 queries per workgroup, chunks of 64 keys in a ring of four buffers (64 KiB),
//          so that TWO workgroups fit a compute unit, each SIMD holding one wave of each.  While one
//          of them merges, sorts or writes out (no matrix work), the other one's sweep keeps the
//          matrix pipe busy: the shape for short key ranges, where those phases are a large share.
template <int WAVES> struct SweepShape;
template <> struct SweepShape<8> { static constexpr int kChunk = 128, kBuffers = 3; };
template <> struct SweepShape<4> { static constexpr int kChunk = 64, kBuffers = 4; };

// LDS bytes the sweep needs for head dimension D (1 KiB aligned).
template <int D, int WAVES = kWaves>
constexpr int sweep_lds_bytes() { return SweepShape<WAVES>::kBuffers * SweepShape<WAVES>::kChunk * D * 2; }

// max(x, 0) on the bit pattern: negative floats (and -0) are negative integers.
__device__ inline float relu(float x) { return __int_as_float(max(__float_as_int(x), 0)); }

// Query operand of this wave: head h = hb*32 + col, d = ks*16 + half*8 .. +8, plus the head
// weights in the layout of the MFMA result.  `qrow` is the query's row in q [B*S, H, D] and
// w [B*S, H]; `lane` is the caller's lane id.  A head slot past H reuses head H-1 with weight 0,
// which adds exactly +0.
template <int D, int HB>
__device__ __forceinline__ void load_query(const __bf16* __restrict__ q, const float* __restrict__ w,
                                           int64_t qrow, int H, int lane, bf16x8 (&a)[HB][D / 16],
                                           float (&wr)[HB][16]) {
    constexpr int KS = D / 16;
    const int col = lane & 31;
    const int half = lane >> 5;
#pragma unroll
    for (int hb = 0; hb < HB; ++hb) {
        const int h = min(hb * 32 + col, H - 1);
        const __bf16* src = q + (qrow * H + h) * D + half * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) a[hb][ks] = *reinterpret_cast<const bf16x8*>(src + ks * 16);
        // Result register j of this lane holds head hb*32 + 8*(j/4) + 4*half + j%4.
        float wv[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) {  // all loads first, so that they overlap
            const int hh = hb * 32 + 8 * (j >> 2) + 4 * half + (j & 3);
            wv[j] = w[qrow * H + min(hh, H - 1)];
        }
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int hh = hb * 32 + 8 * (j >> 2) + 4 * half + (j & 3);
            float v = hh < H ? wv[j] : 0.0f;
            asm volatile("" : "+v"(v));  // keep the masked weight in a register for the whole sweep
            wr[hb][j] = v;
        }
    }
}

// Byte offset, inside a 128-key chunk of head dimension D, of the 16-byte piece that lane `lane`
// moves with the wave-wide load number `blk` of the chunk (each load fills 1 KiB of LDS, lane l
// writing bytes [16 l, 16 l + 16) of it).  The XOR swizzle of the pieces of a key row is applied
// on this (global) side, so that LDS rows are unpadded yet bank-conflict free when read back.
template <int D>
__host__ __device__ constexpr int chunk_lane_offset(int blk, int lane) {
    constexpr int kRowBytes = D * 2;
    constexpr int kPieces = D / 8;                // 16-byte pieces per key row
    constexpr int kRowsPer256 = 256 / kRowBytes;  // key rows per 256 B of LDS (0 for D = 256: unsupported)
    constexpr int kRowsPerLoad = 64 / kPieces;    // key rows covered by one wave-wide load
    const int row = blk * kRowsPerLoad + lane / kPieces;
    const int piece = (lane % kPieces) ^ ((row / kRowsPer256) % kPieces);
    return row * kRowBytes + piece * 16;
}
// Checked at compile time for every head dimension the library accepts: the loads of one chunk
// read every 16-byte piece of the chunk exactly once and nothing outside it, so the largest
// address a load can form is (chunk base) + 128 * 2D - 16, which the descriptor of chunk_rsrc
// compares against the bytes that really exist.
template <int D>
constexpr bool chunk_offsets_cover_chunk_once() {
    constexpr int kChunkBytes = 128 * D * 2;
    bool seen[kChunkBytes / 16] = {};
    for (int blk = 0; blk < kChunkBytes / 1024; ++blk)
        for (int lane = 0; lane < 64; ++lane) {
            const int off = chunk_lane_offset<D>(blk, lane);
            if (off < 0 || off % 16 != 0 || off + 16 > kChunkBytes || seen[off / 16]) return false;
            seen[off / 16] = true;
        }
    for (int i = 0; i < kChunkBytes / 16; ++i)
        if (!seen[i]) return false;
    return true;
}
static_assert(chunk_offsets_cover_chunk_once<32>() && chunk_offsets_cover_chunk_once<64>() &&
              chunk_offsets_cover_chunk_once<128>(), "a chunk's loads must tile the chunk exactly");

// Buffer descriptor of the key rows [first_key, key_clamp) of Kb: raw buffer, stride 0, untyped
// 32-bit data, num_records = the bytes that exist from first_key on (0 when the chunk lies past the
// key range).  A chunk's loads address it with the lane's constant offset only (row inside the
// chunk, piece), which is the one part of a buffer address the hardware range-checks: a 16-byte
// piece at or past num_records is not read and lands as zero.  The chunk's position is folded into
// the base address and the record count with scalar arithmetic, never into the unchecked scalar
// offset operand, so no load can touch memory past the last key row.  key_clamp * 2D < 2^32.
template <int D>
__device__ __forceinline__ __amdgpu_buffer_rsrc_t chunk_rsrc(const __bf16* Kb, int key_clamp, int first_key) {
    constexpr unsigned kRowBytes = D * 2;
    const unsigned total = static_cast<unsigned>(key_clamp) * kRowBytes;
    const unsigned skip = static_cast<unsigned>(first_key) * kRowBytes;
    // (written with min / max so that it stays on the scalar unit)
    const unsigned start = min(skip, total);
    const unsigned remain = total - start;
    const char* base = reinterpret_cast<const char*>(Kb) + start;
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(base), 0, static_cast<int>(remain), 0x00020000);
}

// Starts the trip of the first chunks of a sweep over Kb (all but one buffer of the ring: two
// 128-key chunks in the wide shape, three 64-key chunks in the narrow one) into LDS buffers 0, 1, ...
// -- the same transfers the sweep's own prologue would issue.  A sweep called with
// PREFETCHED = true expects them in flight or landed and skips its own.  All waves call it.
template <int D, int WAVES = kWaves>
__device__ __forceinline__ void sweep_prefetch(unsigned char* lds, const __bf16* __restrict__ Kb,
                                               int key_clamp) {
#if defined(__HIP_DEVICE_COMPILE__)
    constexpr int kChunk = SweepShape<WAVES>::kChunk;
    constexpr int kBufBytes = kChunk * D * 2;
    constexpr int kLoads = kBufBytes / 1024 / WAVES;
    typedef __attribute__((address_space(3))) void lds_void;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int c = 0; c < SweepShape<WAVES>::kBuffers - 1; ++c) {
        const __amdgpu_buffer_rsrc_t krsrc = chunk_rsrc<D>(Kb, key_clamp, c * kChunk);
#pragma unroll
        for (int i = 0; i < kLoads; ++i) {
            const int blk = wave * kLoads + i;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(
                krsrc, (lds_void*)(lds + c * kBufBytes + blk * 1024), 16, chunk_lane_offset<D>(blk, lane), 0, 0, 0);
        }
    }
#else
    (void)lds; (void)Kb; (void)key_clamp;
#endif
}

// What the sweep does with the scores of this wave's query.
struct SweepOut {
    // filter mode
    int row_keys;      // this row's legal keys inside the sweep (keys >= row_keys are dropped)
    float theta;       // a key is appended only if its score beats this
    key64_t* cand;     // the row's buffer
    int cap;           // its capacity; the survivors of a block of 64 scores are appended only if
                       // all of them fit (always the case when the caller sizes the buffer as
                       // documented; kept as a bounds check on wave-uniform values)
    int n_cand;        // keys held (in/out)
    bool overflow;     // (in/out, sticky) some survivors did not fit: the row's result is invalid
                       // and the caller must report it (poison_row), never write a top-k from it
    uint32_t index0;   // key index of the sweep's first key
    // dense mode
    bool live;         // false: this wave's row does not exist, store nothing
    float* out_row;    // fp32 scores of the sweep's keys
};

// Sweeps keys [0, n_keys) of Kb (a multiple of 128 is covered: key rows from `key_clamp` on read
// as zero and are never emitted; key_clamp * 2D < 2^32).  All WAVES waves of the workgroup must call it together
// with the same Kb, key_clamp and n_keys > 0.
//
// STOPPABLE (filter mode): the sweep also ends, for the whole workgroup at the same key, once
// some wave holds at least `trigger` keys.  Such a wave sets flags[step parity] (LDS, 2 ints,
// zero on entry) after its step (one key chunk), and everybody reads the word of the previous step
// behind the step's barrier, so the decision is uniform without another barrier and nothing has to
// be cleared on the way.  A row can therefore grow to at most trigger + kSweepOvershoot (319) keys
// before the sweep returns (128-key chunks; 191 with 64-key chunks).
//
// Returns the number of keys swept (a multiple of the chunk, or >= n_keys at the natural end).  On
// return every global -> LDS transfer the workgroup issued has landed for the calling wave;
// a workgroup barrier must follow before the LDS is reused.
template <int D, int HB, bool FILTER, bool STOPPABLE, bool PREFETCHED = false, int WAVES = kWaves>
__device__ __forceinline__ int score_sweep(unsigned char* lds, const bf16x8 (&a)[HB][D / 16],
                                           const float (&wr)[HB][16], const __bf16* __restrict__ Kb,
                                           int key_clamp, int n_keys, SweepOut& o, int* flags,
                                           int trigger) {
#if defined(__HIP_DEVICE_COMPILE__)
    static_assert(!STOPPABLE || FILTER, "only the filtering sweep can be stopped");
    constexpr int KS = D / 16;             // MFMA steps along d
    constexpr int EPM = 16 / KS;           // epilogue elements handled next to one MFMA
    static_assert(16 % KS == 0, "epilogue elements must split evenly over the MFMA steps");
    // LDS key rows are unpadded (2*D bytes); the 16-byte pieces of a row are XOR-swizzled so
    // that the 16 lanes served together by one ds_read_b128 hit 16 different bank groups:
    // piece p of row r sits in slot p ^ swz(r), swz(r) = (r / rows per 256 B) mod pieces per row.
    constexpr int kRowBytes = D * 2;
    constexpr int kPieces = D / 8;         // 16-byte pieces per key row
    constexpr int kRowsPer256 = 256 / kRowBytes;
    constexpr int kChunk = SweepShape<WAVES>::kChunk;      // keys per LDS buffer
    constexpr int kBuffers = SweepShape<WAVES>::kBuffers;  // ring length; kBuffers - 1 chunks ahead
    constexpr int kBufBytes = kChunk * kRowBytes;
    constexpr int kLoads = kBufBytes / 1024 / WAVES;       // wave-wide 1 KiB loads per wave per chunk
    static_assert(kBufBytes % (1024 * WAVES) == 0 && kLoads >= 1, "chunk must split evenly over the waves");
    static_assert(kChunk == 128 || kChunk == 64, "the pipelined loop is written for 4 or 2 sub-blocks per chunk");
    static_assert(kLoads * (kBuffers - 2) <= 15, "the wait below counts loads in a 4-bit field");

    // wave-uniform values live in scalar registers
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int col = lane & 31;
    const int half = lane >> 5;
    // Row state is wave-uniform; readfirstlane tells the compiler so (the merge computes the count
    // and the threshold with cross-lane operations, which it would otherwise treat as per-lane
    // values: vector registers, exec-masked branches).
    const int row_keys = __builtin_amdgcn_readfirstlane(o.row_keys);
    const float theta = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(o.theta)));
    key64_t* const cand = o.cand;  // computed from the workgroup and wave numbers: uniform
    const int cap = __builtin_amdgcn_readfirstlane(o.cap);
    int n_cand = __builtin_amdgcn_readfirstlane(o.n_cand);
    bool overflow = o.overflow;
    const uint32_t index0 = __builtin_amdgcn_readfirstlane(o.index0);
    const bool live = o.live;
    float* const out_row = o.out_row;

    // Global -> LDS without a register round trip: each wave-wide load writes 1 KiB of LDS
    // (lane l to byte l*16 of the block); the lane picks the global piece that belongs there.
    // Buffer addressing: the lane's part of the address (key row inside the chunk, piece) is a
    // constant 32-bit offset, the chunk's part sits in the descriptor (chunk_rsrc: scalar work
    // only), and key rows past the end of the sweep's key range are not read and land as zero
    // (they are never emitted), so a load costs no vector ALU work.
    typedef __attribute__((address_space(3))) void lds_void;
    int kvoff[kLoads];
#pragma unroll
    for (int i = 0; i < kLoads; ++i)
        kvoff[i] = chunk_lane_offset<D>(wave * kLoads + i, lane);  // load wave*kLoads + i of the chunk

#define SI_FETCH(KC0, BUFOFF)                                                                      \
    {                                                                                               \
        const __amdgpu_buffer_rsrc_t krsrc_ = chunk_rsrc<D>(Kb, key_clamp, (KC0));                  \
        _Pragma("unroll") for (int i = 0; i < kLoads; ++i)                                          \
            __builtin_amdgcn_raw_ptr_buffer_load_lds(krsrc_,                                        \
                (lds_void*)(lds + (BUFOFF) + (wave * kLoads + i) * 1024), 16, kvoff[i], 0, 0, 0);   \
    }

    // This lane's byte offset, inside a 32-key sub-block, of the operand for MFMA step ks.
    const int swz = (col / kRowsPer256) % kPieces;
    // kaddr[ks] is kept absolute (buffer offset included) and moved from buffer to buffer once per
    // chunk, so that the sub-block and MFMA-step parts of a read's address are immediates.
    int kaddr[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) kaddr[ks] = col * kRowBytes + (((ks * 2 + half) ^ swz) * 16);
#define SI_KREAD(SUBBLOCK, KSTEP) \
    (*reinterpret_cast<const bf16x8*>(lds + kaddr[KSTEP] + (SUBBLOCK) * 32 * kRowBytes))

    // The first kBuffers - 1 chunks in flight; chunk 0 must have landed before its first read.
    // ring[0] is the buffer being read, ring[1] the next one, ..., ring[kBuffers - 1] the one filling.
    int ring[kBuffers];
#pragma unroll
    for (int i = 0; i < kBuffers; ++i) ring[i] = i * kBufBytes;
    if (!PREFETCHED) {
#pragma unroll
        for (int c = 0; c < kBuffers - 1; ++c) SI_FETCH(c * kChunk, ring[c])
    }
    // vmcnt: everything but the newest kBuffers - 2 chunks has landed
    __builtin_amdgcn_s_waitcnt(0x0F70 | (kLoads * (kBuffers - 2)));
    __syncthreads();

    bf16x8 bq[KS];  // key operand of the sub-block about to be multiplied
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) bq[ks] = SI_KREAD(0, ks);  // kaddr points into buffer 0 = off_cur

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
#define SI_STEP(CUR, PREV, OUT, NEXT_SUBBLOCK)                                                      \
    {                                                                                               \
        float s_ = 0.0f;                                                                            \
        _Pragma("unroll") for (int hb = 0; hb < HB; ++hb)                                           \
            _Pragma("unroll") for (int ks = 0; ks < KS; ++ks) {                                     \
                CUR[hb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[hb][ks], bq[ks],                \
                                                                  ks == 0 ? zero16 : CUR[hb], 0, 0, 0); \
                _Pragma("unroll") for (int e = (hb * KS + ks) * EPM; e < (hb * KS + ks + 1) * EPM; ++e)   \
                    s_ = fmaf(wr[e / 16][e % 16], relu(PREV[e / 16][e % 16]), s_);                  \
                if (hb == HB - 1) bq[ks] = SI_KREAD(NEXT_SUBBLOCK, ks);                             \
                __builtin_amdgcn_sched_barrier(0);                                                  \
            }                                                                                       \
        OUT = s_ + __shfl_xor(s_, 32);                                                              \
    }
    // 64 finished scores (lane l holds key KEY0 + l): append the kept ones / store them.
#define SI_EMIT(VAL, KEY0)                                                                         \
    {                                                                                               \
        if (FILTER) {                                                                               \
            /* KEY0 is wave-uniform and negative only in the first step of a sweep */               \
            if ((KEY0) >= 0) {                                                                      \
                const bool legal = lane < row_keys - (KEY0);                                        \
                const bool above = (VAL) > theta;                                                   \
                const unsigned long long mask =                                                     \
                    __builtin_amdgcn_ballot_w64(legal) & __builtin_amdgcn_ballot_w64(above);        \
                const int add = static_cast<int>(__popcll(mask));                                   \
                if (add != 0) {                                                                     \
                    if (n_cand + add <= cap) { /* always, when the buffer is sized as documented */ \
                        const unsigned below = __builtin_amdgcn_mbcnt_hi(static_cast<unsigned>(mask >> 32), \
                                               __builtin_amdgcn_mbcnt_lo(static_cast<unsigned>(mask), 0u)); \
                        const unsigned byte_off = (static_cast<unsigned>(n_cand) + below) * 8u;     \
                        if (legal && above)                                                         \
                            *reinterpret_cast<key64_t*>(reinterpret_cast<char*>(cand) + byte_off) = \
                                make_key((VAL), index0 + static_cast<uint32_t>((KEY0) + lane));     \
                        n_cand += add;                                                              \
                    } else {                                                                        \
                        overflow = true; /* wave-uniform; reported through the row's output */      \
                    }                                                                               \
                }                                                                                   \
            }                                                                                       \
        } else {                                                                                    \
            const int key = (KEY0) + lane;                                                          \
            if (live && key >= 0 && key < n_keys) out_row[key] = (VAL);                             \
        }                                                                                           \
    }

    float r_even = 0.0f;  // epilogue result of the last even sub-block, waiting for its odd partner
    int kc0 = 0;
    bool stop = false;
    // The next chunk must be in LDS, and visible to every wave, before its first read.
    // A bare barrier: __syncthreads() would add a release fence that waits for every vector
    // memory operation, i.e. also for the chunks that have just started their trip.  What the
    // barrier must order is waited for explicitly -- vmcnt: only the newest kBuffers - 2 chunks may
    // be in flight; lgkmcnt(0): this wave's LDS writes (the flags) are done -- and the empty
    // asm statements keep the compiler from moving memory accesses across it.
#define SI_NEXT_CHUNK_BARRIER()                                               \
    __builtin_amdgcn_s_waitcnt(0x0070 | (kLoads * (kBuffers - 2)));           \
    asm volatile("" ::: "memory");                                            \
    __builtin_amdgcn_s_barrier();                                             \
    asm volatile("" ::: "memory");
    for (; kc0 < n_keys && !stop; kc0 += kChunk) {
        // The chunk kBuffers - 1 ahead starts its trip to LDS.  Issued unconditionally (a chunk past
        // the key range reads nothing and its buffer is never used) so that the vmcnt arithmetic holds.
        SI_FETCH(kc0 + (kBuffers - 1) * kChunk, ring[kBuffers - 1])
        int posted = 0;
        if constexpr (kChunk == 128) {
            float sp, s0v, s1v, s2v;
            SI_STEP(accA, accB, sp, 1)
            SI_STEP(accB, accA, s0v, 2)
            SI_STEP(accA, accB, s1v, 3)
            SI_NEXT_CHUNK_BARRIER()
            if (STOPPABLE) posted = flags[((kc0 / kChunk) + 1) & 1];  // posted after the previous step
            {   // from here on the reads go to the next chunk's buffer
                const int delta = ring[1] - ring[0];
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) kaddr[ks] += delta;
            }
            SI_STEP(accB, accA, s2v, 0)
            // even sub-blocks stay in the low half-wave, odd ones in the high half
            const float res_prev = half ? sp : r_even;   // keys kc0 - 64 + lane (previous chunk)
            const float res_cur = half ? s1v : s0v;      // keys kc0 + lane
            r_even = s2v;
            if (!FILTER || __builtin_amdgcn_ballot_w64((res_prev > theta) | (res_cur > theta)) != 0ull) {
                SI_EMIT(res_prev, kc0 - 64)
                SI_EMIT(res_cur, kc0)
            }
        } else {
            // two sub-blocks per chunk: the scores of chunk c - 1 are complete after the first step
            // of chunk c (its odd sub-block's epilogue runs under the MFMAs of this chunk's even one)
            float e_odd, e_even;
            SI_STEP(accA, accB, e_odd, 1)
            SI_NEXT_CHUNK_BARRIER()
            if (STOPPABLE) posted = flags[((kc0 / kChunk) + 1) & 1];
            {
                const int delta = ring[1] - ring[0];
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) kaddr[ks] += delta;
            }
            SI_STEP(accB, accA, e_even, 0)
            const float res_prev = half ? e_odd : r_even;  // keys kc0 - 64 + lane (previous chunk)
            r_even = e_even;
            if (!FILTER || __builtin_amdgcn_ballot_w64(res_prev > theta) != 0ull) {
                SI_EMIT(res_prev, kc0 - 64)
            }
        }
        if (STOPPABLE) {
            if (n_cand >= trigger) {  // wave-uniform, rare
                if (lane == 0) flags[(kc0 / kChunk) & 1] = 1;
            }
            stop = __builtin_amdgcn_readfirstlane(posted) != 0;
        }
        {   // the ring moves on by one buffer
            const int t_ = ring[0];
#pragma unroll
            for (int i = 0; i + 1 < kBuffers; ++i) ring[i] = ring[i + 1];
            ring[kBuffers - 1] = t_;
        }
    }
#undef SI_NEXT_CHUNK_BARRIER
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
    o.n_cand = n_cand;
    o.overflow = overflow;
    // loads of chunks past the end may still be in flight: let them land before the LDS is reused
    __builtin_amdgcn_s_waitcnt(0x0F70);
    return kc0;
#else  // the host pass only needs the declaration (the buffer intrinsics are device-only)
    (void)lds; (void)a; (void)wr; (void)Kb; (void)key_clamp; (void)n_keys; (void)o; (void)flags; (void)trigger;
    return 0;
#endif
}

}  // namespace si
