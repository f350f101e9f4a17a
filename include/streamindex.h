/*
 * libstreamindex -- lightning-indexer score + exact per-query top-k on one MI355X (gfx950).
 *
 * The operation (StreamIndex, Sections 1, 3, 4 and 5):
 *
 *   I(t, s)  = sum_h w[t,h] * ReLU( sum_d q[t,h,d] * K[s,d] )            (Section 1, Section 3)
 *   legal(t) = T                          for SI_MASK_NONE
 *            = min(T, floor((t+1)/m))     for SI_MASK_CAUSAL_BLOCK        (Section 4.2, Section 5)
 *   out(t)   = the min(k, legal(t)) keys s < legal(t) that are largest under
 *              (a,i) > (b,j)  <=>  a > b or (a == b and i < j)            (Section 4.1)
 *              listed best first; the remaining slots hold idx = -1, score = -inf.
 *
 * It is computed as the chunked partition-merge stream of Algorithm 2: keys are visited in
 * chunks, a running top-k buffer per query absorbs each chunk's candidates.  The [B,S,H,T]
 * tensor is never formed.  Two schedules of the same stream are offered:
 *   tiled       one launch per (c_S x c_T) tile; the largest transient is one candidate list of
 *               at most c_T (score, index) pairs per query of the current query tile, inside
 *               `workspace` (O(B * c_S * c_T) bytes) -- the design-space axes of Section 6.5;
 *   single pass one persistent kernel; 8 (or 4) queries per workgroup walk their whole key range and
 *               the only transient is a short row buffer per resident wave (tens of MB).
 * The result does not depend on the schedule or on (c_S, c_T): it is bit-identical.
 *
 * Conventions for every entry point
 *   - q, K, w, out_idx, out_score, workspace and every other array argument marked "device"
 *     are caller-owned DEVICE pointers (HBM), contiguous row-major, 16-byte aligned.
 *     The library allocates no device memory and frees none.
 *   - q and K hold bfloat16; w, scores hold IEEE float32.  Inputs must be finite.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All work is
 *     enqueued on it; the call returns without synchronising.  Results are valid once the
 *     caller has synchronised the stream.  `workspace` contents are undefined afterwards.
 *     Only kernel launches are enqueued (no memset or copy nodes, no host synchronisation), so
 *     a call may be recorded into a HIP graph by stream capture and replayed, provided the
 *     profiler below is off and the pointers stay valid.
 *   - Argument errors are detected on the host before anything is launched and reported as
 *     a negative si_status; no exception crosses the boundary.
 *   - Calls that share a workspace must not overlap in time.
 *   - A row whose internal candidate buffer overflowed is reported in place: all k slots hold
 *     idx = -2 and score = NaN.  The buffer sizes the library computes rule this out; the
 *     marker exists so that a violated invariant can never look like a result.
 *   - State the library keeps between calls: the optional timing facility at the end of this
 *     file (off by default, guarded by a mutex), a per-thread last HIP error code, and per-device
 *     caches of two immutable facts (compute-unit count, the LDS limit already granted to the
 *     write-out kernel).  Nothing else; entry points may be called from several threads.
 */
#ifndef STREAMINDEX_H
#define STREAMINDEX_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SI_OK = 0,
    SI_ERR_INVALID_ARG = -1,        /* null pointer, non-positive size, bad enum               */
    SI_ERR_UNSUPPORTED_SHAPE = -2,  /* D not in {32,64,128}, H_I > 64, k > 4096, T*D*2 >= 2^32 */
    SI_ERR_WORKSPACE_TOO_SMALL = -3,
    SI_ERR_HIP = -4                 /* a HIP runtime call failed; see si_last_hip_error()      */
} si_status;

typedef enum {
    SI_MASK_NONE = 0,          /* every key is legal for every query                          */
    SI_MASK_CAUSAL_BLOCK = 1   /* key s legal for query t iff (s+1)*m <= t+1  (Section 4.2)    */
} si_mask_mode;

/* Problem size.  T is explicit (the causal mode does not require T == S/m). */
typedef struct {
    int32_t B;    /* batch                                  */
    int32_t S;    /* queries per batch                      */
    int32_t H_I;  /* indexer heads, 1..64                   */
    int32_t D;    /* head dimension: 32, 64 or 128          */
    int32_t T;    /* compressed keys per batch              */
} si_dims;

typedef struct {
    int32_t c_S;             /* query tile                                                    */
    int32_t c_T;             /* key tile                                                      */
    size_t workspace_bytes;  /* what si_workspace_bytes returns for (c_S, c_T)                */
} si_plan;

/* Chunk-size rule of Section 6.5 ("key tile as large as fits, then the query tile") as measured
 * on this chip: larger tiles win on both axes, so the plan is the largest key tile (up to 32768)
 * for which a query tile at least as long (up to 32768 rows over the batch) still fits
 * `hbm_budget_bytes`; for tiny budgets the query tile shrinks to 8 and the key tile follows.
 * Host only, no GPU call.  Fails with SI_ERR_WORKSPACE_TOO_SMALL when nothing fits. */
si_status si_plan_tiles(const si_dims* dims, int32_t m, int32_t k, si_mask_mode mask_mode,
                        size_t hbm_budget_bytes, si_plan* out);

/* Bytes of workspace needed for a tiling: per query row of a tile a buffer of 2k + c_T
 * 64-bit (score,index) keys (the running top-k plus the candidates of one key tile), an int32
 * count and an fp32 threshold; B*c_S rows (c_S, c_T clamped to S, T).  0 on invalid arguments. */
size_t si_workspace_bytes(const si_dims* dims, int32_t k, int32_t c_S, int32_t c_T);

/* The whole step (Algorithm 2).  Runs the single-pass schedule (si_indexer_topk_fused) when k <= 2048 and workspace_bytes >= si_fused_workspace_bytes(dims, k, 0); otherwise
 * the tiled schedule with the tiling si_plan_tiles chooses for budget = workspace_bytes.  Both
 * give the same bits.
 *   q         device [B,S,H_I,D] bf16        K  device [B,T,D] bf16      w  device [B,S,H_I] f32
 *   out_idx   device [B,S,k] int32           out_score  device [B,S,k] f32
 *   workspace device, workspace_bytes bytes, 256-byte aligned */
si_status si_indexer_topk(const void* q, const void* K, const float* w, const si_dims* dims,
                          int32_t m, int32_t k, si_mask_mode mask_mode, int32_t* out_idx,
                          float* out_score, void* workspace, size_t workspace_bytes,
                          void* stream);

/* Same with an explicit tiling (the design-space sweeps of Section 6.5).  Any c_S >= 1,
 * c_T >= 1 is accepted; values above S / T are clamped. */
si_status si_indexer_topk_tiled(const void* q, const void* K, const float* w,
                                const si_dims* dims, int32_t m, int32_t k,
                                si_mask_mode mask_mode, int32_t c_S, int32_t c_T,
                                int32_t* out_idx, float* out_score, void* workspace,
                                size_t workspace_bytes, void* stream);

/* The same result by the single-pass schedule: every group of 8 (or 4) consecutive queries is taken
 * through its whole legal key range by one resident workgroup, which filters, merges (a row is
 * cut back to its best k whenever it has collected 2k candidates) and writes out without
 * leaving the kernel.  No (c_S x c_T) candidate lists exist: the workspace holds one short row
 * buffer per resident wave plus one counter per launch, independent of S and T
 * (si_fused_workspace_bytes, about 40 MB at k = 1024).  Requires k <= 2048.
 * c_S = queries per kernel launch (<= 0: the library's default, 131072; values above S are
 * clamped).  The split only resynchronises the workgroups' walk over the keys; it does not
 * change the result. */
/* The kernel comes in two workgroup shapes that give the same bits: wide (8 queries per
 * workgroup, one workgroup per compute unit: every staged key chunk serves 8 queries) and narrow
 * (4 queries per workgroup, two workgroups per compute unit: while one of them merges, sorts or
 * writes out, the other one's sweep keeps the matrix pipe busy).  si_indexer_topk_fused picks the
 * narrow shape when the longest key range of a query is short (si_fused_shape_for tells which);
 * si_indexer_topk_fused_shape takes queries_per_workgroup = 8, 4 or 0 (= that choice). */
size_t si_fused_workspace_bytes(const si_dims* dims, int32_t k, int32_t c_S);
int32_t si_fused_shape_for(const si_dims* dims, int32_t m, int32_t k, si_mask_mode mask_mode);
si_status si_indexer_topk_fused_shape(const void* q, const void* K, const float* w, const si_dims* dims,
                                      int32_t m, int32_t k, si_mask_mode mask_mode, int32_t c_S,
                                      int32_t queries_per_workgroup, int32_t* out_idx, float* out_score,
                                      void* workspace, size_t workspace_bytes, void* stream);
si_status si_indexer_topk_fused(const void* q, const void* K, const float* w, const si_dims* dims,
                                int32_t m, int32_t k, si_mask_mode mask_mode, int32_t c_S,
                                int32_t* out_idx, float* out_score, void* workspace,
                                size_t workspace_bytes, void* stream);

/* For callers that cannot allocate device memory or hand over a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): the single-pass schedule of
 * si_indexer_topk_fused with its scratch memory in a static array inside the library instead of
 * a workspace argument.  Same arguments otherwise, same bits out.  Allocates nothing, frees
 * nothing, enqueues kernel launches only.
 *   Limits: k <= 1024 and S <= 64 * 131072 (SI_ERR_UNSUPPORTED_SHAPE beyond; nothing is launched).
 *   The array is 39,846,144 bytes and exists once per GPU the library runs on, for the life of
 *   the process.  Its device address is looked up on the first call on each device (make that
 *   call outside stream capture).  Every call on a GPU uses that GPU's one array: calls that
 *   overlap in time on the same GPU, from any stream or thread, race; the array keeps the last
 *   call's contents and each call clears what it needs cleared (its launch counters) itself. */
si_status si_indexer_topk_static(const void* q, const void* K, const float* w, const si_dims* dims,
                                 int32_t m, int32_t k, si_mask_mode mask_mode, int32_t* out_idx,
                                 float* out_score, void* stream);

/* Step "score tile" alone (the fused score kernel of Section 5): fp32 scores of queries
 * [s0, s0+c_S) against keys [t0, t0+c_T) of every batch, ReLU and the weighted head sum
 * done in registers.  tile: device [B, c_S, c_T] f32, row stride c_T.  Entries whose query
 * or key lies outside the problem are not written.  With SI_MASK_CAUSAL_BLOCK, entries of
 * keys that are illegal for their query may be left unwritten (they are never selected). */
si_status si_score_tile(const void* q, const void* K, const float* w, const si_dims* dims,
                        int32_t m, si_mask_mode mask_mode, int32_t s0, int32_t t0,
                        int32_t c_S, int32_t c_T, float* tile, void* stream);

/* Steps "per-tile select", "merge" and "write-out" alone, on scores the caller supplies
 * (Algorithm 2 without the score kernel; Section 4.3 corollary):
 *   scores  device [R, n_cols] f32;  legal  device [R] int32 or NULL (= n_cols for all rows)
 * Row r's result is the top-min(k, legal[r]) of scores[r, 0:legal[r]] under the total order,
 * reached by streaming column tiles of c_T through the running buffer.
 *   out_idx device [R,k] int32, out_score device [R,k] f32.
 * workspace needs si_workspace_bytes({B=1, S=R, T=n_cols, ..}, k, c_S=R, c_T) bytes. */
si_status si_topk_from_scores(const float* scores, int32_t R, int32_t n_cols,
                              const int32_t* legal, int32_t k, int32_t c_T, int32_t* out_idx,
                              float* out_score, void* workspace, size_t workspace_bytes,
                              void* stream);

/* B*S*H_I*T*4: bytes of the fp32 intermediate of the materialize path (Section 3), for
 * reporting only. */
uint64_t si_materialize_bytes(const si_dims* dims);

/* Per-kernel timing for benchmarks.  When enabled, every kernel launch made by the entry
 * points above is bracketed by HIP events on its stream.  si_profile_read synchronises
 * those events and returns, per kernel class, the summed duration in milliseconds and the
 * number of launches since the last reset.  Classes: 0 score tile (with its fused filter),
 * 1 filter of caller-supplied scores, 2 compaction (select + merge), 3 final sort + write-out,
 * 4 buffer / counter init, 5 single-pass kernel (wide shape), 6 single-pass kernel (narrow shape).  One set of totals per process: meant for a
 * single benchmarking thread (concurrent callers are serialised, their launches are summed). */
#define SI_PROFILE_CLASSES 7
si_status si_profile_enable(int32_t on);
si_status si_profile_reset(void);
si_status si_profile_read(double* ms_per_class, int64_t* launches_per_class);

/* Phase clock of the single-pass kernel, for the phase budget of a benchmark run.  While
 * device_words is non-NULL, launches of the single-pass schedule with D = 128, 33..64 heads and
 * k <= 1024 run an instrumented copy of the kernel in which workgroup j ADDS to
 * device_words[j*32 + i] (uint64, device memory, at least n_workgroups*32 + 4096 words,
 * n_workgroups >= twice the device's compute units, cleared by the caller):
 *   i = 0..5  time in ticks of the device's constant wall clock (hipDeviceAttributeWallClockRate):
 *             0 item set-up and barriers around sweeps, 1 key sweeps, 2 in-kernel merges,
 *             3 final cut + sort + write-out, 4 barrier behind the write-out, 5 residency
 *             (first instruction to exit, summed over launches);
 *   i = 6..10 counts: 6 work items, 7 sweep calls, 8 128-key steps, 9 merges, 10 launches;
 *   i = 11..14 parts of 2 (barrier + next chunks requested, row read, radix descent, write-back +
 *             barrier); i = 15..19 parts of 3 (row read, exact cut, keys to LDS, sort, write-out).
 *             The instrumented kernel waits for outstanding memory operations at these marks.
 *   i = 20, 21 set, not added: hardware id and XCC id registers of the workgroup's first wave
 *             (which compute unit it ran on); i = 22: tick of its first instruction.
 *   Behind the n_workgroups blocks of words: two logs of 2048 words, (tick << 4) | phase
 *   that ended (0..4), written by workgroup 0 and by the first workgroup of the grid's second half
 *   (in the narrow shape these two share a compute unit); unused entries stay as the caller left them.
 * Results are unchanged.  Pass NULL to switch back to the plain kernel.  The pointer is global to
 * the process: meant for one benchmarking thread. */
si_status si_profile_phases(uint64_t* device_words, int32_t n_workgroups);
/* Ticks per millisecond of the current device's constant wall clock (the unit of the phase
 * clock); 0 if the runtime cannot tell. */
int32_t si_wall_clock_khz(void);

const char* si_strerror(si_status status);
/* hipError_t of the last failed HIP call made by this library on this thread (0 = none). */
int32_t si_last_hip_error(void);
/* Library version, major*10000 + minor*100 + patch. */
int32_t si_version(void);

#ifdef __cplusplus
}
#endif
#endif /* STREAMINDEX_H */
