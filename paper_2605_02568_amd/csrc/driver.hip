// Host driver: argument checks, tile planning, workspace carve-up and the nested tile loop
// of Algorithm 2 (outer loop over query tiles, inner loop over key tiles, per-query running
// state, write-out after the last key tile).  Per key tile: one score kernel that appends the
// surviving candidates to the row buffers, one compaction kernel; per query tile: one init and
// one finalize kernel.  Key tiles that hold no legal key for any query of the query tile are
// not visited (Algorithm 2 visits them; their masked entries can never be selected, so the
// result is the same).

#include <algorithm>
#include <atomic>
#include <mutex>
#include <vector>

#include "si_internal.h"

// Scratch of si_indexer_topk_static, the entry point that allocates nothing: the workspace of the
// single-pass schedule for k <= kStaticMaxK (launch counters, then 256 x 8 row buffers of
// 2k + 384 keys), as one static array in device memory.  Each GPU the library runs on holds its
// own copy from the moment the code object is loaded until the process ends.  In host code the
// name `scratch` is only a handle: the address kernels can use comes from hipGetSymbolAddress,
// once per device (static_scratch below), and only that pointer is ever passed on.
namespace {
constexpr int kStaticMaxK = 1024;
constexpr int kStaticMaxLaunches = 64;  // counters: one 256-byte block
constexpr size_t kStaticScratchBytes =
    256 + static_cast<size_t>(si::kFusedSlots) * si::kQueriesPerBlock *
              (si::kFusedTriggerMul * kStaticMaxK + si::kFusedRowSlack) * sizeof(si::key64_t);
}  // namespace
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace si {

namespace {

thread_local int32_t g_last_hip_error = 0;

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

si_status hip_fail(hipError_t e) {
    g_last_hip_error = static_cast<int32_t>(e);
    return SI_ERR_HIP;
}

// ---- per-kernel timing (benchmark aid) --------------------------------------------------
struct Profiler {
    std::mutex mu;  // every member below is read and written under it
    bool on = false;
    unsigned long long* phase = nullptr;  // device words of the single-pass kernel's phase clock
    int32_t phase_slots = 0;
    std::vector<hipEvent_t> pool;  // reused events
    size_t used = 0;
    struct Span { int cls; size_t begin, end; };
    std::vector<Span> spans;
    double ms[SI_PROFILE_CLASSES] = {0};
    int64_t launches[SI_PROFILE_CLASSES] = {0};

    hipError_t next_event(size_t* idx) {
        if (used == pool.size()) {
            hipEvent_t ev;
            hipError_t e = hipEventCreate(&ev);
            if (e != hipSuccess) return e;
            pool.push_back(ev);
        }
        *idx = used++;
        return hipSuccess;
    }
    // folds finished spans into the totals and frees the events for reuse
    hipError_t drain() {
        for (const Span& s : spans) {
            hipError_t e = hipEventSynchronize(pool[s.end]);
            if (e != hipSuccess) return e;
            float t = 0.f;
            e = hipEventElapsedTime(&t, pool[s.begin], pool[s.end]);
            if (e != hipSuccess) return e;
            ms[s.cls] += t;
            launches[s.cls] += 1;
        }
        spans.clear();
        used = 0;
        return hipSuccess;
    }
};
Profiler g_prof;

// Brackets one launch with events when profiling is on.
template <typename F>
hipError_t timed(int cls, hipStream_t stream, F&& launch) {
    std::lock_guard<std::mutex> hold(g_prof.mu);
    if (!g_prof.on) return launch();
    if (g_prof.spans.size() >= 8192) {  // bound the number of live events
        hipError_t e = g_prof.drain();
        if (e != hipSuccess) return e;
    }
    size_t b = 0, en = 0;
    hipError_t e = g_prof.next_event(&b);
    if (e != hipSuccess) return e;
    e = g_prof.next_event(&en);
    if (e != hipSuccess) return e;
    e = hipEventRecord(g_prof.pool[b], stream);
    if (e != hipSuccess) return e;
    e = launch();
    if (e != hipSuccess) return e;
    e = hipEventRecord(g_prof.pool[en], stream);
    if (e != hipSuccess) return e;
    g_prof.spans.push_back({cls, b, en});
    return hipSuccess;
}

si_status check_dims(const si_dims* d, int32_t m, int32_t k, int mask_mode) {
    if (!d) return SI_ERR_INVALID_ARG;
    if (d->B < 1 || d->S < 1 || d->H_I < 1 || d->D < 1 || d->T < 1) return SI_ERR_INVALID_ARG;
    if (m < 1 || k < 1) return SI_ERR_INVALID_ARG;
    if (mask_mode != SI_MASK_NONE && mask_mode != SI_MASK_CAUSAL_BLOCK) return SI_ERR_INVALID_ARG;
    if (d->D != 32 && d->D != 64 && d->D != 128) return SI_ERR_UNSUPPORTED_SHAPE;
    if (d->H_I > kMaxHeads || k > kMaxK) return SI_ERR_UNSUPPORTED_SHAPE;
    // the score sweep addresses one batch's keys through a 32-bit buffer range
    if (static_cast<int64_t>(d->T) * d->D * 2 >= (int64_t{1} << 32)) return SI_ERR_UNSUPPORTED_SHAPE;
    return SI_OK;
}

size_t workspace_bytes_for(int64_t B, int64_t c_S, int64_t c_T, int64_t k) {
    return carve_workspace(nullptr, B * c_S, k, std::max<int64_t>(c_T, 1)).bytes;
}

// Key tiles of one query tile: a narrow first tile, then widths that double up to c_T.  The
// first tile cannot be filtered (no k-th best exists yet), so it is kept small; each later
// tile is filtered against the top-k of everything before it.  The result does not depend on
// this schedule.
int64_t next_width(int64_t t0, int64_t c_T, int64_t k) {
    const int64_t first = std::max<int64_t>(2 * k, 1024);
    const int64_t w = t0 == 0 ? first : std::max<int64_t>(t0, first);
    return std::min<int64_t>(w, c_T);
}

// Workspace of the single-pass schedule: one launch counter per query tile, then the row
// buffers of the resident workgroups.
struct FusedLayout {
    int32_t* counters;
    int64_t n_launches;
    RowBuffers slots;
    size_t bytes;
};
int32_t fused_rows_per_launch(int32_t c_S, int32_t S) {
    if (c_S < 1) c_S = kFusedDefaultRows;
    return std::min(c_S, S);
}
FusedLayout carve_fused(void* base, int64_t S, int64_t k, int64_t c_S) {
    FusedLayout L;
    char* p = static_cast<char*>(base);
    L.n_launches = (S + c_S - 1) / c_S;
    size_t off = 0;
    L.counters = reinterpret_cast<int32_t*>(p + off);
    off = align_up(off + static_cast<size_t>(L.n_launches) * sizeof(int32_t), 256);
    L.slots.keys = reinterpret_cast<key64_t*>(p + off);
    L.slots.cap = static_cast<int32_t>(kFusedTriggerMul * k + kFusedRowSlack);
    off = align_up(off + static_cast<size_t>(kFusedSlots) * kQueriesPerBlock * L.slots.cap * sizeof(key64_t), 256);
    L.slots.count = nullptr;
    L.slots.theta = nullptr;
    L.slots.bytes = off;
    L.bytes = off;
    return L;
}

// Immutable facts about a device, looked up once per device and process.
struct DeviceInfo {
    std::atomic<int> compute_units{0};
    std::atomic<void*> static_scratch{nullptr};  // this device's copy of `scratch`
};
constexpr int kMaxDevices = 64;
DeviceInfo g_device[kMaxDevices];

// Workgroups the single-pass kernel is launched with: one wide (8-wave) or two narrow (4-wave)
// workgroups per compute unit of the current device -- either way 2 waves per SIMD, which is what
// their register budget allows -- and at most what the workspace has row buffers for.
hipError_t fused_workgroups(int32_t waves, int32_t* n) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    int cus = (dev >= 0 && dev < kMaxDevices) ? g_device[dev].compute_units.load(std::memory_order_acquire) : 0;
    if (cus == 0) {
        e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess) return e;
        if (cus < 1) return hipErrorInvalidDevice;
        if (dev >= 0 && dev < kMaxDevices) g_device[dev].compute_units.store(cus, std::memory_order_release);
    }
    const int32_t per_cu = kQueriesPerBlock / waves;
    *n = std::min<int32_t>(cus * per_cu, kFusedSlots * per_cu);
    return hipSuccess;
}

// Workgroup shape of the single-pass schedule when the caller does not choose (see SweepShape in
// score_sweep.h).  Per work item the merges, the final cut + sort and the write-out cost a time
// that depends on k but not on the item's key range, with the matrix pipe idle; two narrow
// workgroups per compute unit overlap one's such phases with the other's sweep, at the price of
// staging every key chunk for 4 queries instead of 8 and of a lone sweeping wave per SIMD that
// cannot hide its own stalls.  Measured on MI355X at the V4 head shape (S = 4 T, causal, k = 512
// and 1024): the narrow shape is 5-6 % faster at 8,192 keys per query, 1 % at 16,384, even at
// 32,768 and 3 % slower at 262,144.
constexpr int64_t kNarrowMaxKeys = 16384;
int32_t fused_shape_for(const si_dims& d, int32_t m, int32_t mask_mode) {
    int64_t longest = d.T;  // keys of the longest row
    if (mask_mode == SI_MASK_CAUSAL_BLOCK) longest = std::min<int64_t>(d.T, static_cast<int64_t>(d.S) / m);
    return longest <= kNarrowMaxKeys ? 4 : 8;
}

// Device address of the current device's copy of `scratch`: asked from the runtime on the first
// call on that device (with that device current), remembered afterwards.
hipError_t static_scratch(void** ptr) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const bool tracked = dev >= 0 && dev < kMaxDevices;
    void* p = tracked ? g_device[dev].static_scratch.load(std::memory_order_acquire) : nullptr;
    if (p == nullptr) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (p == nullptr) return hipErrorInvalidSymbol;
        if (tracked) g_device[dev].static_scratch.store(p, std::memory_order_release);
    }
    *ptr = p;
    return hipSuccess;
}

// The single-pass schedule on a carved workspace: one counter-clearing kernel, then one launch
// per c_S queries.  Arguments have been checked.
si_status run_fused(const void* q, const void* K, const float* w, const si_dims& d, int32_t m, int32_t k,
                    int32_t mask_mode, int32_t c_S, int32_t waves, const FusedLayout& L, int32_t* out_idx,
                    float* out_score, hipStream_t hs) {
    if (waves == 0) waves = fused_shape_for(d, m, mask_mode);
    int32_t n_wg = 0;
    hipError_t e = fused_workgroups(waves, &n_wg);
    if (e != hipSuccess) return hip_fail(e);
    e = timed(kProfInit, hs, [&] {
        return launch_zero_ints(L.counters, static_cast<int32_t>(L.n_launches), hs);
    });
    if (e != hipSuccess) return hip_fail(e);
    int64_t launch = 0;
    for (int64_t s0 = 0; s0 < d.S; s0 += c_S, ++launch) {
        const int32_t rows = static_cast<int32_t>(std::min<int64_t>(c_S, d.S - s0));
        e = timed(waves == 8 ? kProfFused : kProfFusedNarrow, hs, [&] {
            // (timed holds the profiler's lock: the phase clock's buffer is read under it)
            unsigned long long* phase = g_prof.phase_slots >= n_wg ? g_prof.phase : nullptr;
            if (phase != nullptr && !(d.D == 128 && d.H_I > 32 && k <= 1024)) phase = nullptr;
            return launch_fused(q, K, w, d, m, mask_mode, k, static_cast<int32_t>(s0), rows, L.slots,
                                waves, n_wg, L.counters + launch, out_idx, out_score, phase,
                                g_prof.phase_slots, hs);
        });
        if (e != hipSuccess) return hip_fail(e);
    }
    return SI_OK;
}
}  // namespace

// Per query row of a tile: a key buffer of 2k + c_T slots (a row is cut back to k as soon as
// it holds 2k, and one key tile adds at most c_T), a count and a threshold.
RowBuffers carve_workspace(void* base, int64_t rows_, int64_t k, int64_t c_T) {
    RowBuffers rb;
    const size_t rows = static_cast<size_t>(rows_);
    rb.cap = static_cast<int32_t>(2 * k + c_T);
    size_t off = 0;
    char* p = static_cast<char*>(base);
    rb.keys = reinterpret_cast<key64_t*>(p + off);
    off = align_up(off + rows * static_cast<size_t>(rb.cap) * sizeof(key64_t), 256);
    rb.count = reinterpret_cast<int32_t*>(p + off);
    off = align_up(off + rows * sizeof(int32_t), 256);
    rb.theta = reinterpret_cast<float*>(p + off);
    off = align_up(off + rows * sizeof(float), 256);
    rb.bytes = off;
    return rb;
}

}  // namespace si

using namespace si;

extern "C" {

size_t si_workspace_bytes(const si_dims* dims, int32_t k, int32_t c_S, int32_t c_T) {
    if (!dims || dims->B < 1 || dims->S < 1 || dims->T < 1 || k < 1 || c_S < 1 || c_T < 1) return 0;
    const int64_t cs = std::min<int64_t>(c_S, dims->S);
    const int64_t ct = std::min<int64_t>(c_T, dims->T);
    return workspace_bytes_for(dims->B, cs, ct, k);
}

si_status si_plan_tiles(const si_dims* dims, int32_t m, int32_t k, si_mask_mode mask_mode,
                        size_t hbm_budget_bytes, si_plan* out) {
    si_status st = check_dims(dims, m, k, mask_mode);
    if (st != SI_OK) return st;
    if (!out) return SI_ERR_INVALID_ARG;
    // Measured on MI355X (flash_1m, 8 GB budget): larger tiles win on both axes.  Fewer, longer
    // launches lose less to the drain at every kernel boundary, and every key tile costs one
    // pass of the compaction kernel over all rows.  The workgroups of a launch walk the key
    // tile in step, so the part of K in use at any moment is small whatever c_T is.  Rule:
    // the largest key tile (up to 32768) for which a query tile at least as long (up to 32768)
    // still fits the budget; failing that, the smallest query tile and a shrinking key tile.
    const int64_t B = dims->B;
    const int64_t s_cap = std::min<int64_t>(dims->S, std::max<int64_t>(kQueriesPerBlock, 32768 / B));
    auto fit_rows = [&](int64_t c_T) {  // longest query tile (multiple of 8, or all of S) within the budget
        int64_t lo = 0, hi = s_cap;     // workspace grows with c_S: bisect
        while (lo < hi) {
            const int64_t mid = (lo + hi + 1) / 2;
            if (workspace_bytes_for(B, mid, c_T, k) <= hbm_budget_bytes) lo = mid; else hi = mid - 1;
        }
        if (lo < dims->S) lo = lo / kQueriesPerBlock * kQueriesPerBlock;
        return lo;
    };
    static const int64_t key_tiles[] = {32768, 24576, 16384, 12288, 8192, 6144, 4096, 3072, 2048, 1024,
                                        512, 256, 128, 64, 32};
    int64_t best_S = 0, best_T = 0;
    for (int64_t cand : key_tiles) {
        const int64_t c_T = std::min<int64_t>(cand, dims->T);
        const int64_t c_S = fit_rows(c_T);
        if (c_S >= std::min<int64_t>(c_T, s_cap)) {  // balanced tile found
            best_S = c_S;
            best_T = c_T;
            break;
        }
        if (c_S >= kQueriesPerBlock || c_S == dims->S) {  // remember the widest key tile that fits at all
            if (best_S == 0 || c_S * c_T > best_S * best_T) {
                best_S = c_S;
                best_T = c_T;
            }
        }
    }
    if (best_S == 0) return SI_ERR_WORKSPACE_TOO_SMALL;
    out->c_S = static_cast<int32_t>(best_S);
    out->c_T = static_cast<int32_t>(best_T);
    out->workspace_bytes = workspace_bytes_for(B, best_S, best_T, k);
    return SI_OK;
}

si_status si_score_tile(const void* q, const void* K, const float* w, const si_dims* dims,
                        int32_t m, si_mask_mode mask_mode, int32_t s0, int32_t t0,
                        int32_t c_S, int32_t c_T, float* tile, void* stream) {
    si_status st = check_dims(dims, m, 1, mask_mode);
    if (st != SI_OK) return st;
    if (!q || !K || !w || !tile) return SI_ERR_INVALID_ARG;
    if (s0 < 0 || t0 < 0 || c_S < 1 || c_T < 1 || s0 >= dims->S || t0 >= dims->T) return SI_ERR_INVALID_ARG;
    const int32_t rows = std::min<int64_t>(c_S, static_cast<int64_t>(dims->S) - s0);
    const int32_t width = std::min<int64_t>(c_T, static_cast<int64_t>(dims->T) - t0);
    hipStream_t hs = static_cast<hipStream_t>(stream);
    hipError_t e = timed(kProfScore, hs, [&] {
        return launch_score_tile(q, K, w, *dims, m, mask_mode, s0, t0, rows, width, c_S, c_T, tile, hs);
    });
    return e == hipSuccess ? SI_OK : hip_fail(e);
}

si_status si_indexer_topk_tiled(const void* q, const void* K, const float* w,
                                const si_dims* dims, int32_t m, int32_t k,
                                si_mask_mode mask_mode, int32_t c_S, int32_t c_T,
                                int32_t* out_idx, float* out_score, void* workspace,
                                size_t workspace_bytes, void* stream) {
    si_status st = check_dims(dims, m, k, mask_mode);
    if (st != SI_OK) return st;
    if (!q || !K || !w || !out_idx || !out_score || !workspace) return SI_ERR_INVALID_ARG;
    if (c_S < 1 || c_T < 1) return SI_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(workspace) % 256 != 0) return SI_ERR_INVALID_ARG;
    const si_dims d = *dims;
    c_S = std::min(c_S, d.S);
    c_T = std::min(c_T, d.T);
    const RowBuffers rb = carve_workspace(workspace, static_cast<int64_t>(d.B) * c_S, k, c_T);
    if (rb.bytes > workspace_bytes) return SI_ERR_WORKSPACE_TOO_SMALL;
    hipStream_t hs = static_cast<hipStream_t>(stream);

    for (int64_t s0 = 0; s0 < d.S; s0 += c_S) {
        const int32_t rows = static_cast<int32_t>(std::min<int64_t>(c_S, d.S - s0));
        hipError_t e = timed(kProfInit, hs, [&] { return launch_init_rows(rb, d.B * c_S, hs); });
        if (e != hipSuccess) return hip_fail(e);
        // keys visible to the last query of this tile (Section 4.2); later key tiles are skipped
        int64_t t_hi = d.T;
        if (mask_mode == SI_MASK_CAUSAL_BLOCK) t_hi = std::min<int64_t>(d.T, (s0 + rows) / m);
        for (int64_t t0 = 0; t0 < t_hi;) {
            const int32_t width = static_cast<int32_t>(std::min<int64_t>(next_width(t0, c_T, k), d.T - t0));
            e = timed(kProfScore, hs, [&] {
                return launch_score_filter(q, K, w, d, m, mask_mode, k, static_cast<int32_t>(s0),
                                           static_cast<int32_t>(t0), rows, width, c_S, rb, hs);
            });
            if (e != hipSuccess) return hip_fail(e);
            e = timed(kProfCompact, hs, [&] { return launch_compact(rb, d.B, rows, c_S, k, 2 * k, hs); });
            if (e != hipSuccess) return hip_fail(e);
            t0 += width;
        }
        e = timed(kProfFinalize, hs, [&] {
            return launch_finalize(rb, d.B, rows, c_S, k, d.S, s0, out_idx, out_score, hs);
        });
        if (e != hipSuccess) return hip_fail(e);
    }
    return SI_OK;
}

si_status si_indexer_topk(const void* q, const void* K, const float* w, const si_dims* dims,
                          int32_t m, int32_t k, si_mask_mode mask_mode, int32_t* out_idx,
                          float* out_score, void* workspace, size_t workspace_bytes,
                          void* stream) {
    // The single-pass schedule whenever it applies (k <= 2048) and its small workspace fits;
    // otherwise the tiled schedule with the plan for this budget.
    const size_t fused_bytes = si_fused_workspace_bytes(dims, k, 0);
    if (fused_bytes != 0 && fused_bytes <= workspace_bytes)
        return si_indexer_topk_fused(q, K, w, dims, m, k, mask_mode, 0, out_idx, out_score, workspace,
                                     workspace_bytes, stream);
    si_plan plan;
    si_status st = si_plan_tiles(dims, m, k, mask_mode, workspace_bytes, &plan);
    if (st != SI_OK) return st;
    return si_indexer_topk_tiled(q, K, w, dims, m, k, mask_mode, plan.c_S, plan.c_T, out_idx,
                                 out_score, workspace, workspace_bytes, stream);
}

size_t si_fused_workspace_bytes(const si_dims* dims, int32_t k, int32_t c_S) {
    if (!dims || dims->S < 1 || k < 1 || k > kFusedMaxK) return 0;
    c_S = fused_rows_per_launch(c_S, dims->S);
    return carve_fused(nullptr, dims->S, k, c_S).bytes;
}

si_status si_indexer_topk_fused_shape(const void* q, const void* K, const float* w, const si_dims* dims,
                                      int32_t m, int32_t k, si_mask_mode mask_mode, int32_t c_S,
                                      int32_t queries_per_workgroup, int32_t* out_idx, float* out_score,
                                      void* workspace, size_t workspace_bytes, void* stream) {
    si_status st = check_dims(dims, m, k, mask_mode);
    if (st != SI_OK) return st;
    if (k > kFusedMaxK) return SI_ERR_UNSUPPORTED_SHAPE;
    if (!q || !K || !w || !out_idx || !out_score || !workspace) return SI_ERR_INVALID_ARG;
    if (queries_per_workgroup != 0 && queries_per_workgroup != 4 && queries_per_workgroup != 8)
        return SI_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(workspace) % 256 != 0) return SI_ERR_INVALID_ARG;
    c_S = fused_rows_per_launch(c_S, dims->S);
    const FusedLayout L = carve_fused(workspace, dims->S, k, c_S);
    if (L.bytes > workspace_bytes) return SI_ERR_WORKSPACE_TOO_SMALL;
    return run_fused(q, K, w, *dims, m, k, mask_mode, c_S, queries_per_workgroup, L, out_idx, out_score,
                     static_cast<hipStream_t>(stream));
}

si_status si_indexer_topk_fused(const void* q, const void* K, const float* w, const si_dims* dims,
                                int32_t m, int32_t k, si_mask_mode mask_mode, int32_t c_S,
                                int32_t* out_idx, float* out_score, void* workspace,
                                size_t workspace_bytes, void* stream) {
    return si_indexer_topk_fused_shape(q, K, w, dims, m, k, mask_mode, c_S, 0, out_idx, out_score,
                                       workspace, workspace_bytes, stream);
}

int32_t si_fused_shape_for(const si_dims* dims, int32_t m, int32_t k, si_mask_mode mask_mode) {
    if (check_dims(dims, m, k, mask_mode) != SI_OK || k > kFusedMaxK) return 0;
    return fused_shape_for(*dims, m, mask_mode);
}

si_status si_indexer_topk_static(const void* q, const void* K, const float* w, const si_dims* dims,
                                 int32_t m, int32_t k, si_mask_mode mask_mode, int32_t* out_idx,
                                 float* out_score, void* stream) {
    si_status st = check_dims(dims, m, k, mask_mode);
    if (st != SI_OK) return st;
    if (!q || !K || !w || !out_idx || !out_score) return SI_ERR_INVALID_ARG;
    // beyond what the static array was sized for: refuse, never spill over
    if (k > kStaticMaxK) return SI_ERR_UNSUPPORTED_SHAPE;
    const int32_t c_S = fused_rows_per_launch(0, dims->S);
    if ((static_cast<int64_t>(dims->S) + c_S - 1) / c_S > kStaticMaxLaunches) return SI_ERR_UNSUPPORTED_SHAPE;
    void* base = nullptr;
    hipError_t e = static_scratch(&base);
    if (e != hipSuccess) return hip_fail(e);
    const FusedLayout L = carve_fused(base, dims->S, k, c_S);
    if (L.bytes > kStaticScratchBytes) return SI_ERR_UNSUPPORTED_SHAPE;  // (cannot happen within the two limits)
    return run_fused(q, K, w, *dims, m, k, mask_mode, c_S, 0, L, out_idx, out_score,
                     static_cast<hipStream_t>(stream));
}

si_status si_topk_from_scores(const float* scores, int32_t R, int32_t n_cols,
                              const int32_t* legal, int32_t k, int32_t c_T, int32_t* out_idx,
                              float* out_score, void* workspace, size_t workspace_bytes,
                              void* stream) {
    if (!scores || !out_idx || !out_score || !workspace) return SI_ERR_INVALID_ARG;
    if (R < 1 || n_cols < 1 || k < 1 || c_T < 1) return SI_ERR_INVALID_ARG;
    if (k > kMaxK) return SI_ERR_UNSUPPORTED_SHAPE;
    if (reinterpret_cast<uintptr_t>(workspace) % 256 != 0) return SI_ERR_INVALID_ARG;
    c_T = std::min(c_T, n_cols);
    const RowBuffers rb = carve_workspace(workspace, R, k, c_T);
    if (rb.bytes > workspace_bytes) return SI_ERR_WORKSPACE_TOO_SMALL;
    hipStream_t hs = static_cast<hipStream_t>(stream);
    hipError_t e = timed(kProfInit, hs, [&] { return launch_init_rows(rb, R, hs); });
    if (e != hipSuccess) return hip_fail(e);
    for (int64_t t0 = 0; t0 < n_cols; t0 += c_T) {
        const int32_t width = static_cast<int32_t>(std::min<int64_t>(c_T, n_cols - t0));
        e = timed(kProfFilterScores, hs, [&] {
            return launch_filter_scores(scores, R, n_cols, k, static_cast<int32_t>(t0), width, legal, rb, hs);
        });
        if (e != hipSuccess) return hip_fail(e);
        e = timed(kProfCompact, hs, [&] { return launch_compact(rb, 1, R, R, k, 2 * k, hs); });
        if (e != hipSuccess) return hip_fail(e);
    }
    e = timed(kProfFinalize, hs, [&] { return launch_finalize(rb, 1, R, R, k, R, 0, out_idx, out_score, hs); });
    return e == hipSuccess ? SI_OK : hip_fail(e);
}

uint64_t si_materialize_bytes(const si_dims* dims) {
    if (!dims) return 0;
    return static_cast<uint64_t>(dims->B) * static_cast<uint64_t>(dims->S) *
           static_cast<uint64_t>(dims->H_I) * static_cast<uint64_t>(dims->T) * 4ull;
}

si_status si_profile_enable(int32_t on) {
    std::lock_guard<std::mutex> hold(g_prof.mu);
    g_prof.on = on != 0;
    return SI_OK;
}

si_status si_profile_phases(uint64_t* device_words, int32_t n_workgroups) {
    if (device_words != nullptr && n_workgroups < 1) return SI_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> hold(g_prof.mu);
    g_prof.phase = reinterpret_cast<unsigned long long*>(device_words);
    g_prof.phase_slots = device_words ? n_workgroups : 0;
    return SI_OK;
}

int32_t si_wall_clock_khz(void) {
    int dev = 0, khz = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) != hipSuccess) return 0;
    return khz;
}

si_status si_profile_reset(void) {
    std::lock_guard<std::mutex> hold(g_prof.mu);
    hipError_t e = g_prof.drain();
    if (e != hipSuccess) return hip_fail(e);
    for (int i = 0; i < SI_PROFILE_CLASSES; ++i) {
        g_prof.ms[i] = 0.0;
        g_prof.launches[i] = 0;
    }
    return SI_OK;
}

si_status si_profile_read(double* ms_per_class, int64_t* launches_per_class) {
    if (!ms_per_class || !launches_per_class) return SI_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> hold(g_prof.mu);
    hipError_t e = g_prof.drain();
    if (e != hipSuccess) return hip_fail(e);
    for (int i = 0; i < SI_PROFILE_CLASSES; ++i) {
        ms_per_class[i] = g_prof.ms[i];
        launches_per_class[i] = g_prof.launches[i];
    }
    return SI_OK;
}

const char* si_strerror(si_status status) {
    switch (status) {
        case SI_OK: return "ok";
        case SI_ERR_INVALID_ARG: return "invalid argument";
        case SI_ERR_UNSUPPORTED_SHAPE: return "unsupported shape (D in {32,64,128}, H_I <= 64, k <= 4096, T*D*2 < 2^32)";
        case SI_ERR_WORKSPACE_TOO_SMALL: return "workspace too small for this tiling";
        case SI_ERR_HIP: return "HIP runtime error (see si_last_hip_error)";
    }
    return "unknown status";
}

int32_t si_last_hip_error(void) { return g_last_hip_error; }

int32_t si_version(void) { return 100; }

}  // extern "C"
