// Single-pass schedule of Algorithm 2: one persistent workgroup takes 8 consecutive queries
// through their whole legal key range and does every step of the stream for them without
// leaving the kernel -- score sweep with the mask and threshold filter in registers, the
// merge (cutting a row back to its best k whenever it has collected 2k candidates) and the
// final exact cut, sort and write-out (Section 4.2 for the pad).  Compared with the tiled
// schedule the query operand is read once, there are no per-tile launches, a row's threshold
// is refreshed as soon as 2k candidates have accumulated, and the only scratch memory is one
// short row buffer per resident wave (tens of MB in total, L2 resident), independent of S.
// By the corollary of Section 4.3 the result is the same exact top-k under the total order of
// Section 4.1, so the output is bit-identical to the tiled schedule's.
//
// One wave owns one query row, as in the score sweep; the merge and the write-out are the
// wave-level routines of topk_wave.h, so no step needs an atomic or a cross-wave exchange.
// The only workgroup-wide decisions are "next work item" and "stop the sweep for a merge".
// Latencies at the seams are overlapped where that is free: the next work item is requested
// while the current one runs, the first two key chunks of every sweep are on their way before
// the query is (re)loaded and before a merge starts, and short items pull the next item's query
// rows into L2 while they sort.

#include "score_sweep.h"
#include "topk_wave.h"

namespace si {

// A sweep is stopped once a row holds `trigger` keys and can overshoot by kSweepOvershoot (see
// score_sweep): the row buffer must hold both.
__host__ __device__ constexpr int fused_trigger(int k) { return kFusedTriggerMul * k; }
__host__ __device__ constexpr int fused_row_cap(int k) { return fused_trigger(k) + kFusedRowSlack; }
static_assert(kFusedRowSlack >= kSweepOvershoot, "a stopped sweep must not run past the end of a row buffer");
// Items with at most this many keys warm L2 with the next item's query rows while they sort.
constexpr int kWarmupMaxKeys = 8192;

// The kernel is compiled for two ranges of k (KMAX = 1024 and kFusedMaxK = 2048): a whole row
// must fit the registers of a wave, and the sort area of the workgroup's waves must fit the LDS.
template <int KMAX>
constexpr int fused_reg_keys() { return (kFusedTriggerMul * KMAX + 384 + 63) / 64; }
template <int D, int KMAX, int WAVES>
constexpr int fused_lds_bytes() {
    constexpr int sort_bytes = WAVES * (KMAX + KMAX / 8) * 8;
    return sweep_lds_bytes<D, WAVES>() > sort_bytes ? sweep_lds_bytes<D, WAVES>() : sort_bytes;
}

// Queries [s_begin, s_begin + rows) of every batch; work item = (batch, group of WAVES
// consecutive queries), handed out through *counter (zero before the launch), longest key range
// first so that the workgroups running at any time have nearly equal work and walk the keys
// roughly together (which keeps the key rows they share in L2).  Workgroup j uses rows
// [WAVES j, WAVES j + WAVES) of `slots`.
//
// WAVES = 8 (wide shape, one workgroup per compute unit) or 4 (narrow shape, two per compute
// unit, see SweepShape).  In the narrow shape the point is that the two workgroups of a compute
// unit are NOT in step: while one merges or writes out, the other sweeps.  Workgroups that start
// together on equal work stay in step, so the second half of the grid (the workgroups that arrive
// second on each compute unit) starts with one of the shortest items instead of a longest one,
// which shifts it by about the length of a write-out phase.
//
// TIMED: workgroup j also adds, for its wave 0, the time spent in each phase (ticks of the constant
// wall clock) and event counts to phase[j * kPhaseWords ...] (layout: PhaseWord in si_internal.h).
// Every wave runs the same barriers, so wave 0's phases are the workgroup's.
template <int D, int HB, int KMAX, int WAVES, bool TIMED>
__global__ __launch_bounds__(64 * WAVES) __attribute__((amdgpu_waves_per_eu(2, 2)))
void indexer_fused_kernel(const __bf16* __restrict__ q, const __bf16* __restrict__ K,
                          const float* __restrict__ w, int B, int S, int H, int T, int m,
                          int mask_mode, int k, int pow2_k, int s_begin, int rows, RowBuffers slots,
                          int* __restrict__ counter, int32_t* __restrict__ out_idx,
                          float* __restrict__ out_score, unsigned long long* __restrict__ phase,
                          int phase_slots) {
    // One LDS object for everything (sweep buffers / sort area, histograms, flags, work item):
    // with several, the compiler orders every LDS read behind the global -> LDS transfers in
    // flight and the key prefetch of the sweep no longer overlaps anything.
    constexpr int kQB = WAVES;  // queries per work item
    constexpr int kHistOff = fused_lds_bytes<D, KMAX, WAVES>();
    constexpr int kFlagsOff = kHistOff + WAVES * 256 * 4;
    constexpr int kItemOff = kFlagsOff + 2 * 4;
    constexpr int kTouchOff = kItemOff + 8;  // 16-byte aligned; landing area of the query warm-up reads
    constexpr int kTouchLoads = 2;           // per wave: 2 x 64 lanes = 128 cache lines = one V4 query
    __shared__ __attribute__((aligned(1024))) unsigned char lds[kTouchOff + WAVES * kTouchLoads * 256];
    int (*s_hist)[256] = reinterpret_cast<int (*)[256]>(lds + kHistOff);
    int* s_flags = reinterpret_cast<int*>(lds + kFlagsOff);
    int& s_item = *reinterpret_cast<int*>(lds + kItemOff);
    int& s_next = *reinterpret_cast<int*>(lds + kItemOff + 4);

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int n_groups = (rows + kQB - 1) / kQB;
    const int n_items = n_groups * B;
    const int trigger = fused_trigger(k);
    const int limit = compact_limit(k);
    key64_t* const cand = slots.keys + (static_cast<int64_t>(blockIdx.x) * kQB + wave) * slots.cap;

    // phase clock (TIMED only): time since the last mark goes to the phase that just ended
    unsigned long long t_first = 0, t_mark = 0, acc[kPhaseWords] = {};
    if (TIMED) t_first = t_mark = __builtin_amdgcn_s_memrealtime();
    // Two workgroups that share a compute unit in the narrow shape (the first of each half of the
    // grid) also log their phase changes, (tick << 4) | phase that ended, behind the phase_slots
    // per-workgroup blocks of words: kPhaseTraceEvents words each.
    unsigned long long* trace = nullptr;
    int n_events = 0;
    if (TIMED && (blockIdx.x == 0 || blockIdx.x == gridDim.x / 2))
        trace = phase + static_cast<size_t>(phase_slots) * kPhaseWords + (blockIdx.x == 0 ? 0 : kPhaseTraceEvents);
#define SI_PHASE(P)                                                      \
    if (TIMED) {                                                         \
        const unsigned long long now_ = __builtin_amdgcn_s_memrealtime(); \
        acc[P] += now_ - t_mark;                                         \
        t_mark = now_;                                                   \
        if (trace != nullptr && n_events < kPhaseTraceEvents) {          \
            if (threadIdx.x == 0) trace[n_events] = (now_ << 4) | static_cast<unsigned long long>(P); \
            ++n_events;                                                  \
        }                                                                \
    }
#define SI_COUNT(P, N) \
    if (TIMED) acc[P] += static_cast<unsigned long long>(N);
    // sub-phases run on their own clock mark, so that they split a phase without disturbing it;
    // SI_SUB_WAIT first waits for the wave's outstanding memory operations (instrumented build only)
    unsigned long long t_sub = 0;
#define SI_SUB_START() \
    if (TIMED) t_sub = __builtin_amdgcn_s_memrealtime();
#define SI_SUB(P)                                                        \
    if (TIMED) {                                                         \
        const unsigned long long now_ = __builtin_amdgcn_s_memrealtime(); \
        acc[P] += now_ - t_sub;                                          \
        t_sub = now_;                                                    \
    }
#define SI_SUB_WAIT(P)                                  \
    if (TIMED) {                                        \
        __builtin_amdgcn_s_waitcnt(0x0070); /* vmcnt(0) lgkmcnt(0) */ \
        SI_SUB(P)                                       \
    }

    // Work items: the next one is requested from the counter while the current one is processed,
    // so its round trip costs nothing.  Narrow shape: the last n_tail items (the shortest) are not
    // handed out by the counter; each is the first item of one workgroup of the grid's second half.
    const int n_tail = (WAVES == 4 && n_items >= 4 * static_cast<int>(gridDim.x)) ? static_cast<int>(gridDim.x) / 2 : 0;
    const int n_head = n_items - n_tail;
    const int tail_slot = static_cast<int>(blockIdx.x) - (static_cast<int>(gridDim.x) - n_tail);
    int item;
    if (tail_slot >= 0) {
        item = n_head + tail_slot;
    } else {
        if (threadIdx.x == 0) s_item = atomicAdd(counter, 1);
        __syncthreads();
        item = s_item;
        if (item >= n_head) item = n_items;
    }
    for (;;) {
        if (item >= n_items) break;  // uniform: every wave of every workgroup ends here
        int next_item = 0;
        if (threadIdx.x == 0) next_item = atomicAdd(counter, 1);
        // (the sweep's first barrier orders this before any read of the flags)
        if (threadIdx.x < 2) s_flags[threadIdx.x] = 0;
        const int b = item % B;
        const int r_first = (n_groups - 1 - item / B) * kQB;
        const int r = r_first + wave;
        const bool live = r < rows;
        const int r_last = min(rows, r_first + kQB) - 1;
        const int group_keys = legal_count(s_begin + r_last, T, m, mask_mode);  // uniform
        const int row_keys = live ? legal_count(s_begin + r, T, m, mask_mode) : 0;
        const int64_t qrow = static_cast<int64_t>(b) * S + s_begin + (live ? r : rows - 1);

        SweepOut o;
        o.theta = -__builtin_huge_valf();
        o.cand = cand;
        o.cap = slots.cap;
        o.n_cand = 0;
        o.overflow = false;
        o.live = live;
        o.out_row = nullptr;
        // the first two key chunks of every sweep start their trip before the query is (re)loaded,
        // and, after a stop, before the merge
        if (group_keys > 0)
            sweep_prefetch<D, WAVES>(lds, K + static_cast<int64_t>(b) * T * D, T);
        SI_COUNT(kPhaseItems, 1)
        for (int kbeg = 0; kbeg < group_keys;) {
            SI_PHASE(kPhaseSetup)  // item start or merge -> the sweep call (the query load is only issued here)
            {
                bf16x8 a[HB][D / 16];
                float wr[HB][16];
                // (re)loaded for every sweep: the merge in between needs the registers.  Row and
                // lane are made opaque so that the address arithmetic is redone here instead of
                // being kept live (spilled) across the sweep.
                int64_t qrow_now = qrow;
                asm volatile("" : "+s"(qrow_now));
                int lane_now = lane;
                asm volatile("" : "+v"(lane_now));
                load_query<D, HB>(q, w, qrow_now, H, lane_now, a, wr);
                o.row_keys = row_keys - kbeg;
                o.index0 = static_cast<uint32_t>(kbeg);
                const __bf16* Kb = K + (static_cast<int64_t>(b) * T + kbeg) * D;
                // Narrow shape: the other workgroup's wave on this SIMD may be merging or sorting
                // (a dense vector-ALU stream); the sweep goes first at the shared issue port, so
                // that its epilogue never holds up the next matrix instruction.
                if (WAVES == 4) __builtin_amdgcn_s_setprio(3);
                const int swept = score_sweep<D, HB, true, true, true, WAVES>(lds, a, wr, Kb, T - kbeg,
                                                                              group_keys - kbeg, o, s_flags, trigger);
                kbeg += swept;
                if (WAVES == 4) __builtin_amdgcn_s_setprio(0);
                SI_COUNT(kPhaseChunks, (swept + 127) / 128)
                SI_COUNT(kPhaseSweeps, 1)
            }
            SI_PHASE(kPhaseSweep)
            SI_SUB_START()
            if (threadIdx.x == 0) s_next = next_item;  // (arrived long ago) for the warm-up below
            __syncthreads();  // the sweep's LDS and flags are free again
            if (kbeg >= group_keys) break;
            // Merge: the sweep stopped because some row reached the trigger.  Every row that
            // holds more than it would keep is cut back now, which also refreshes its threshold.
            if (threadIdx.x < 2) s_flags[threadIdx.x] = 0;
            SI_SUB(kPhaseMergeSync)
            // The row is requested before the next sweep's first key chunks: loads return in issue
            // order, so the radix cut starts as soon as the row is here and the chunks travel
            // while it runs.
            const __bf16* Knext = K + (static_cast<int64_t>(b) * T + kbeg) * D;
            if (o.n_cand > limit) {
                RegKeys<fused_reg_keys<KMAX>()> keys;
                keys.load(cand, o.n_cand);
                sweep_prefetch<D, WAVES>(lds, Knext, T - kbeg);
                SI_SUB_WAIT(kPhaseMergeLoad)
                int kept = 0;
                const key64_t thr = wave_radix_kth(keys, k, limit, s_hist[wave], &kept);
                SI_SUB(kPhaseMergeRadix)
                wave_keep(keys, thr, cand, slots.cap);
                o.n_cand = kept;
                o.theta = fmaxf(o.theta, key_score(thr));
            } else {
                sweep_prefetch<D, WAVES>(lds, Knext, T - kbeg);
            }
            // No wait and no barrier here: the kept keys are on their way to this wave's own row
            // (the sweep appends behind them, at other addresses, and the row is read again only
            // after the sweep's closing wait); the flags were cleared by wave 0 before its merge
            // and every wave meets it again at the next sweep's opening barrier.
            SI_SUB(kPhaseMergeKeep)
            SI_PHASE(kPhaseMerge)
            SI_COUNT(kPhaseMerges, 1)
        }
        SI_PHASE(kPhaseSetup)  // (items without a key, and the barrier after the last sweep)

        // Write-out: exact cut to k, sort best first in the wave's slice of the (now idle)
        // sweep LDS, decode, pad.
        if (live && o.overflow) {
            poison_row(out_idx, out_score, (static_cast<int64_t>(b) * S + s_begin + r) * k, k);
        } else if (live) {
            key64_t* s_sort = reinterpret_cast<key64_t*>(lds) + static_cast<size_t>(wave) * sort_slots(pow2_k);
            const SortSlot slot;
            const int n = o.n_cand;
            const int c = min(n, k);
            SI_SUB_START()
            {
                RegKeys<fused_reg_keys<KMAX>()> keys;
                keys.load(cand, n);
                SI_SUB_WAIT(kPhaseFinalLoad)
                key64_t thr = 0ull;
                int kept = 0;
                if (n > k) thr = wave_radix_kth(keys, k, k, s_hist[wave], &kept);  // limit k: exact
                SI_SUB(kPhaseFinalRadix)
                wave_keep(keys, thr, s_sort, pow2_k, slot);
            }
            // While this wave sorts, the next item's query rows start their trip from HBM to L2
            // (one 4-byte read per 128-byte line, landing in an LDS area nobody reads), so that
            // the query load at the start of the next item finds them there.  Only for short
            // items, where that latency is a visible share of the item (6 % at S = 32768); for
            // long ones the 128 KB per workgroup only compete with the key rows for L2.
            if (group_keys > 0 && group_keys <= kWarmupMaxKeys) {
                const int nx = s_next;
                if (nx < n_head) {
                    const int nr_first = (n_groups - 1 - nx / B) * kQB;
                    const int nrows = min(kQB, rows - nr_first);
                    const int64_t nqrow = static_cast<int64_t>(nx % B) * S + s_begin + nr_first;
                    const char* src = reinterpret_cast<const char*>(q + nqrow * H * D);
                    const int lines = (nrows * H * D * 2 + 127) / 128;
                    typedef __attribute__((address_space(3))) void lds_void;
                    typedef __attribute__((address_space(1))) const void gbl_void;
#pragma unroll
                    for (int j = 0; j < kTouchLoads; ++j) {
                        const int line = (j * WAVES + wave) * 64 + lane;
                        if (line < lines)
                            __builtin_amdgcn_global_load_lds(
                                (gbl_void*)(src + static_cast<int64_t>(line) * 128),
                                (lds_void*)(lds + kTouchOff + (wave * kTouchLoads + j) * 256), 4, 0, 0);
                    }
                }
            }
            int P = 16;
            while (P < c) P <<= 1;
            for (int i = c + lane; i < P; i += 64) s_sort[slot(i)] = 0ull;  // empty keys sort last
            __builtin_amdgcn_wave_barrier();
            SI_SUB_WAIT(kPhaseFinalKeep)
            wave_sort_descending(s_sort, P);
            SI_SUB_WAIT(kPhaseFinalSort)
            const int64_t out = (static_cast<int64_t>(b) * S + s_begin + r) * k;
            for (int j = lane; j < k; j += 64) {
                if (j < c) {
                    const key64_t key = s_sort[slot(j)];
                    out_idx[out + j] = key_index(key);
                    out_score[out + j] = key_score(key);
                } else {  // Section 4.2: pad
                    out_idx[out + j] = -1;
                    out_score[out + j] = -__builtin_huge_valf();
                }
            }
        }
        SI_SUB_WAIT(kPhaseFinalWrite)
        if (threadIdx.x == 0) s_item = next_item;
        SI_PHASE(kPhaseFinal)
        __syncthreads();  // the next item's sweep overwrites the LDS the sort used
        item = s_item;
        if (item >= n_head) item = n_items;  // the counter only hands out the head items
        SI_PHASE(kPhaseFinalWait)  // waiting for the slowest wave's write-out
    }
    if (TIMED && threadIdx.x == 0) {
        acc[kPhaseResident] = __builtin_amdgcn_s_memrealtime() - t_first;
        acc[kPhaseLaunches] = 1;
        for (int i = 0; i < kPhaseWords; ++i) phase[blockIdx.x * kPhaseWords + i] += acc[i];
        // (hardware registers HW_ID = 4 and XCC_ID = 20, all 32 bits)
        phase[blockIdx.x * kPhaseWords + kPhaseHwId] = __builtin_amdgcn_s_getreg((31 << 11) | 4);
        phase[blockIdx.x * kPhaseWords + kPhaseXccId] = __builtin_amdgcn_s_getreg((31 << 11) | 20);
        phase[blockIdx.x * kPhaseWords + kPhaseStartTick] = t_first;
    }
#undef SI_PHASE
#undef SI_COUNT
#undef SI_SUB_START
#undef SI_SUB
#undef SI_SUB_WAIT
}

__global__ void zero_ints_kernel(int* p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

hipError_t launch_zero_ints(int32_t* p, int32_t n, hipStream_t stream) {
    hipLaunchKernelGGL(zero_ints_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, p, n);
    return hipGetLastError();
}

hipError_t launch_fused(const void* q, const void* K, const float* w, const si_dims& d, int32_t m,
                        int32_t mask_mode, int32_t k, int32_t s_begin, int32_t rows,
                        const RowBuffers& slots, int32_t waves, int32_t n_workgroups, int32_t* counter,
                        int32_t* out_idx, float* out_score, unsigned long long* phase, int32_t phase_slots,
                        hipStream_t stream) {
    if (phase != nullptr && phase_slots < n_workgroups) return hipErrorInvalidValue;
    if (k < 1 || k > kFusedMaxK || slots.cap < fused_row_cap(k) || n_workgroups < 1) return hipErrorInvalidValue;
    if (waves != 4 && waves != 8) return hipErrorInvalidValue;
    // every workgroup owns `waves` row buffers of the workspace
    if (static_cast<int64_t>(n_workgroups) * waves > static_cast<int64_t>(kFusedSlots) * kQueriesPerBlock)
        return hipErrorInvalidValue;
    const int64_t items = static_cast<int64_t>((rows + waves - 1) / waves) * d.B;
    const dim3 grid(static_cast<unsigned>(std::min<int64_t>(items, n_workgroups)));
    const dim3 block(64 * waves);
    const __bf16* qp = static_cast<const __bf16*>(q);
    const __bf16* Kp = static_cast<const __bf16*>(K);
    const int HB = (d.H_I + 31) / 32;
    int pow2_k = 16;
    while (pow2_k < k) pow2_k <<= 1;
#define SI_LAUNCH_AS(DD, HH, KK, WW, TT)                                                            \
    hipLaunchKernelGGL((indexer_fused_kernel<DD, HH, KK, WW, TT>), grid, block, 0, stream, qp, Kp, \
                       w, d.B, d.S, d.H_I, d.T, m, mask_mode, k, pow2_k, s_begin, rows, slots,      \
                       counter, out_idx, out_score, phase, phase_slots)
#define SI_LAUNCH(DD, HH)                                                                          \
    if (waves == 8) {                                                                               \
        if (k <= 1024) SI_LAUNCH_AS(DD, HH, 1024, 8, false); else SI_LAUNCH_AS(DD, HH, kFusedMaxK, 8, false); \
    } else {                                                                                        \
        if (k <= 1024) SI_LAUNCH_AS(DD, HH, 1024, 4, false); else SI_LAUNCH_AS(DD, HH, kFusedMaxK, 4, false); \
    }
    // the phase clock exists for the evaluation head shape only (every variant is a full kernel)
    if (phase != nullptr && !(d.D == 128 && HB == 2 && k <= 1024)) return hipErrorInvalidValue;
    if (phase != nullptr && waves == 8) { SI_LAUNCH_AS(128, 2, 1024, 8, true); }
    else if (phase != nullptr) { SI_LAUNCH_AS(128, 2, 1024, 4, true); }
    else if (d.D == 128 && HB == 2) { SI_LAUNCH(128, 2) }
    else if (d.D == 128 && HB == 1) { SI_LAUNCH(128, 1) }
    else if (d.D == 64 && HB == 2) { SI_LAUNCH(64, 2) }
    else if (d.D == 64 && HB == 1) { SI_LAUNCH(64, 1) }
    else if (d.D == 32 && HB == 2) { SI_LAUNCH(32, 2) }
    else if (d.D == 32 && HB == 1) { SI_LAUNCH(32, 1) }
    else return hipErrorInvalidValue;
#undef SI_LAUNCH
#undef SI_LAUNCH_AS
    return hipGetLastError();
}

}  // namespace si
