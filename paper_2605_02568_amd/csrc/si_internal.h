// Internal declarations shared by the translation units of libstreamindex.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "streamindex.h"

namespace si {

// A (score, index) pair packed so that unsigned 64-bit comparison is the total order of
// Section 4.1: larger key = better entry.  High word: order-preserving image of the fp32
// score (-0 folded onto +0 so that they tie); low word: ~index, so that the smaller index
// wins among equal scores.  0 is below every real key and marks an empty slot.
typedef unsigned long long key64_t;

__host__ __device__ inline uint32_t score_to_ordered(uint32_t bits) {
    return bits ^ ((bits >> 31) ? 0xFFFFFFFFu : 0x80000000u);
}
__host__ __device__ inline uint32_t ordered_to_score(uint32_t ord) {
    return ord ^ ((ord >> 31) ? 0x80000000u : 0xFFFFFFFFu);
}
#ifdef __HIPCC__
__device__ inline key64_t make_key(float score, uint32_t idx) {
    const uint32_t ord = score_to_ordered(__float_as_uint(score + 0.0f));
    return (static_cast<key64_t>(ord) << 32) | static_cast<key64_t>(0xFFFFFFFFu - idx);
}
__device__ inline float key_score(key64_t key) {
    return __uint_as_float(ordered_to_score(static_cast<uint32_t>(key >> 32)));
}
__device__ inline int32_t key_index(key64_t key) {
    return static_cast<int32_t>(0xFFFFFFFFu - static_cast<uint32_t>(key));
}
// Section 4.2: number of legal keys of query position t.
__device__ inline int32_t legal_count(int32_t t, int32_t T, int32_t m, int32_t mask_mode) {
    if (mask_mode == SI_MASK_NONE) return T;
    const int64_t blocks = (static_cast<int64_t>(t) + 1) / m;
    return blocks < T ? static_cast<int32_t>(blocks) : T;
}
#endif

// A row whose candidate buffer overflowed has no valid top-k.  The sizes the library computes
// rule that out (a sweep appends at most its width / its overshoot to a row that is below its
// trigger), so this marks an internal invariant violation; it is written into the row's output
// (every slot: this index, NaN score) instead of a plausible-looking wrong answer.
constexpr int32_t kPoisonIndex = -2;
#ifdef __HIPCC__
__device__ inline void poison_row(int32_t* out_idx, float* out_score, int64_t out, int k) {
    for (int j = threadIdx.x & 63; j < k; j += 64) {
        out_idx[out + j] = kPoisonIndex;
        out_score[out + j] = __builtin_nanf("");
    }
}
#endif

constexpr int kMaxK = 4096;
constexpr int kMaxHeads = 64;
constexpr int kQueriesPerBlock = 8;  // score kernel: one query per wave, 8 waves (wide workgroup shape)

// Single-pass schedule (fused.hip): k up to kFusedMaxK (a row must fit a wave's registers); a row is merged once it holds
// kFusedTriggerMul * k keys; at most kFusedSlots workgroups are resident (one per compute unit
// of an MI355X), each with 8 row buffers.
constexpr int kFusedMaxK = 2048;
constexpr int kFusedTriggerMul = 2;
constexpr int kFusedSlots = 256;
// A stopped sweep notices the trigger one 128-key step late and then drains its pipeline: a row
// that held trigger - 1 keys before a step can grow by 128 in it, by 128 in the next one and by 64
// in the drain.  Row buffers of the single-pass schedule carry kFusedRowSlack keys beyond the trigger.
constexpr int kSweepOvershoot = 128 - 1 + 128 + 64;
constexpr int kFusedRowSlack = 384;
// Queries per launch when the caller does not say: the workgroups of a launch drift apart as they
// work through their items (and then miss each other's key rows in L2); a launch boundary brings
// them back in step.  131072 rows cost no time against a single launch and cut the key traffic
// to a third.
constexpr int kFusedDefaultRows = 131072;

// Per-row state of the current query tile, carved from the caller's workspace.
struct RowBuffers {
    key64_t* keys;   // [rows, cap] unsorted
    int32_t* count;  // [rows] keys held
    float* theta;    // [rows] score an entry must beat to be appended (-inf until k are known)
    int32_t cap;     // slots per row = 2k + c_T
    size_t bytes;
};
RowBuffers carve_workspace(void* base, int64_t rows, int64_t k, int64_t c_T);

// Words of the phase clock of the single-pass kernel, per workgroup (si_profile_phases).
enum PhaseWord {
    kPhaseSetup = 0,      // ticks: item start / merge end -> sweep call, and the barrier behind a sweep
    kPhaseSweep = 1,      // ticks: inside the key sweep (includes waiting for the query rows)
    kPhaseMerge = 2,      // ticks: in-kernel merges (radix cut of the rows that reached 2k keys)
    kPhaseFinal = 3,      // ticks: exact cut, sort, write-out of wave 0's row
    kPhaseFinalWait = 4,  // ticks: barrier behind the write-out (the slowest wave's write-out)
    kPhaseResident = 5,   // ticks: first instruction -> exit of the workgroup, summed over launches
    kPhaseItems = 6,      // count: work items
    kPhaseSweeps = 7,     // count: sweep calls
    kPhaseChunks = 8,     // count: 128-key steps swept
    kPhaseMerges = 9,     // count: merges
    kPhaseLaunches = 10,  // count: launches this workgroup took part in
    // ticks, parts of kPhaseMerge: barrier behind the stopped sweep + next key chunks requested,
    // row read into registers, radix descent, kept keys written back + barrier
    kPhaseMergeSync = 11, kPhaseMergeLoad = 12, kPhaseMergeRadix = 13, kPhaseMergeKeep = 14,
    // ticks, parts of kPhaseFinal: row read, exact radix cut, kept keys to LDS (+ pads), sort, write-out
    kPhaseFinalLoad = 15, kPhaseFinalRadix = 16, kPhaseFinalKeep = 17, kPhaseFinalSort = 18,
    kPhaseFinalWrite = 19,
    // set, not added: where the workgroup ran (hardware id register of its wave 0: compute unit,
    // shader array and engine; and the XCC id register), to see which workgroups shared a unit
    kPhaseHwId = 20, kPhaseXccId = 21,
    // ticks: first instruction of the workgroup, relative to the earliest tick the host finds
    kPhaseStartTick = 22,
    kPhaseWords = 32
};
// Phase-change log of two workgroups, behind the per-workgroup words (see fused.hip).
constexpr int kPhaseTraceEvents = 2048;

enum ProfileClass { kProfScore = 0, kProfFilterScores = 1, kProfCompact = 2, kProfFinalize = 3, kProfInit = 4, kProfFused = 5, kProfFusedNarrow = 6 };

// Kernel launchers (each enqueues exactly one kernel on `stream`).
// Dense fp32 tile [B, tile_rows, tile_cols] of queries [s0, s0+rows) x keys [t0, t0+width).
hipError_t launch_score_tile(const void* q, const void* K, const float* w, const si_dims& d,
                             int32_t m, int32_t mask_mode, int32_t s0, int32_t t0, int32_t rows,
                             int32_t width, int32_t tile_rows, int32_t tile_cols, float* tile,
                             hipStream_t stream);
// Score tile fused with the mask and the filter: appends, per row, the legal entries that beat
// the row's threshold to the row's buffer (row index = b*tile_rows + r).  A row holds fewer than
// 2k keys when the tile starts (the compaction cuts it at 2k) and gains at most `width`:
// rb.cap >= 2k + width is required and checked.
hipError_t launch_score_filter(const void* q, const void* K, const float* w, const si_dims& d,
                               int32_t m, int32_t mask_mode, int32_t k, int32_t s0, int32_t t0, int32_t rows,
                               int32_t width, int32_t tile_rows, const RowBuffers& rb,
                               hipStream_t stream);
hipError_t launch_init_rows(const RowBuffers& rb, int32_t n, hipStream_t stream);
hipError_t launch_filter_scores(const float* scores, int32_t R, int32_t n_cols, int32_t k, int32_t t0,
                                int32_t width, const int32_t* legal_rows, const RowBuffers& rb,
                                hipStream_t stream);
hipError_t launch_compact(const RowBuffers& rb, int32_t B, int32_t rows, int32_t tile_rows, int32_t k,
                          int32_t trigger, hipStream_t stream);
hipError_t launch_finalize(const RowBuffers& rb, int32_t B, int32_t rows, int32_t tile_rows, int32_t k,
                           int64_t out_batch_stride, int64_t out_row0, int32_t* out_idx,
                           float* out_score, hipStream_t stream);

// Single-pass schedule: queries [s_begin, s_begin + rows) of every batch in one launch.
// waves: 8 (wide workgroups, one per compute unit) or 4 (narrow, two per compute unit); at most
// n_workgroups are launched.  slots: n_workgroups * waves <= 2048 row buffers of slots.cap >=
// 2k + 384 keys; *counter must be zero.
// phase: nullptr, or n_slots * kPhaseWords words the instrumented kernel variant adds its phase
// times to: phase_slots >= n_workgroups blocks of kPhaseWords, then two logs of kPhaseTraceEvents
// words (D = 128, 33..64 heads, k <= 1024 only).
hipError_t launch_fused(const void* q, const void* K, const float* w, const si_dims& d, int32_t m,
                        int32_t mask_mode, int32_t k, int32_t s_begin, int32_t rows,
                        const RowBuffers& slots, int32_t waves, int32_t n_workgroups, int32_t* counter,
                        int32_t* out_idx, float* out_score, unsigned long long* phase, int32_t phase_slots,
                        hipStream_t stream);
hipError_t launch_zero_ints(int32_t* p, int32_t n, hipStream_t stream);

}  // namespace si
