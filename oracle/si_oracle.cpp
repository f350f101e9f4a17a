// CPU oracle for the lightning-indexer top-k step.  TEST INFRASTRUCTURE ONLY:
// see si_oracle.h for what is computed and what pins it.  Plain loops, fp64,
// one query row at a time; nothing here is shared with the HIP library.

#include "si_oracle.h"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <limits>
#include <queue>
#include <set>
#include <thread>
#include <utility>
#include <vector>

namespace {

// bfloat16 is the top half of an IEEE float; widening is exact.
inline double bf16_to_double(uint16_t bits) {
    uint32_t u = static_cast<uint32_t>(bits) << 16;
    float f;
    std::memcpy(&f, &u, sizeof f);
    return static_cast<double>(f);
}

// Section 4.1: (a,i) is better than (b,j) iff a > b, or a == b and i < j.
struct Entry {
    double score;
    int64_t idx;
};
inline bool better(const Entry& x, const Entry& y) {
    if (x.score > y.score) return true;
    if (x.score < y.score) return false;
    return x.idx < y.idx;
}

// Section 1 / Section 3 score of one (query, key) pair from widened operands.
// qT: the query's heads stored [D][H] (head index fastest), kd: [D], w: [H],
// dot: scratch [H].  Each head's dot product is summed over d = 0, 1, ... in
// order; the d loop is outermost only so that the H independent sums advance
// together.
inline double pair_score(const double* qT, const double* kd, const float* w, int H, int D,
                         double* dot) {
    for (int h = 0; h < H; ++h) dot[h] = 0.0;
    for (int d = 0; d < D; ++d) {
        const double kv = kd[d];
        const double* qd = qT + static_cast<int64_t>(d) * H;
#pragma omp simd
        for (int h = 0; h < H; ++h) dot[h] += qd[h] * kv;
    }
    double acc = 0.0;
    for (int h = 0; h < H; ++h)
        if (dot[h] > 0.0) acc += static_cast<double>(w[h]) * dot[h];  // ReLU, then weight
    return acc;
}

// q_row [H][D] bf16 bits -> doubles stored [D][H]
void widen_query(const uint16_t* q_row, int H, int D, std::vector<double>& qT) {
    qT.resize(static_cast<size_t>(H) * static_cast<size_t>(D));
    for (int h = 0; h < H; ++h)
        for (int d = 0; d < D; ++d)
            qT[static_cast<size_t>(d) * H + h] = bf16_to_double(q_row[static_cast<int64_t>(h) * D + d]);
}

void write_sorted(std::vector<Entry>& e, int32_t k, int32_t* out_idx, double* out_score) {
    std::sort(e.begin(), e.end(), better);
    const int64_t keep = std::min<int64_t>(k, static_cast<int64_t>(e.size()));
    for (int64_t j = 0; j < keep; ++j) {
        out_idx[j] = static_cast<int32_t>(e[static_cast<size_t>(j)].idx);
        out_score[j] = e[static_cast<size_t>(j)].score;
    }
    for (int64_t j = keep; j < k; ++j) {
        out_idx[j] = -1;
        out_score[j] = -std::numeric_limits<double>::infinity();
    }
}

}  // namespace

extern "C" {

int64_t si_oracle_legal_count(int64_t t, int64_t T, int32_t m, int32_t mask_mode) {
    if (mask_mode == 0) return T;
    return std::min<int64_t>(T, (t + 1) / m);  // blocks fully in the past of t
}

int32_t si_oracle_score_row(const uint16_t* q_row, const uint16_t* K, const float* w_row,
                            int32_t H, int32_t D, int64_t n_keys, double* out) {
    if (!q_row || !K || !w_row || (!out && n_keys > 0) || H <= 0 || D <= 0 || n_keys < 0) return -1;
    std::vector<double> qT, kd(static_cast<size_t>(D)), dot(static_cast<size_t>(H));
    widen_query(q_row, H, D, qT);
    for (int64_t s = 0; s < n_keys; ++s) {
        for (int d = 0; d < D; ++d) kd[static_cast<size_t>(d)] = bf16_to_double(K[s * D + d]);
        out[s] = pair_score(qT.data(), kd.data(), w_row, H, D, dot.data());
    }
    return 0;
}

int32_t si_oracle_score_at(const uint16_t* q_row, const uint16_t* K, const float* w_row,
                           int32_t H, int32_t D, const int32_t* idx, int64_t n_idx,
                           double* out) {
    if (!q_row || !K || !w_row || !idx || !out || H <= 0 || D <= 0 || n_idx < 0) return -1;
    std::vector<double> qT, kd(static_cast<size_t>(D)), dot(static_cast<size_t>(H));
    widen_query(q_row, H, D, qT);
    for (int64_t i = 0; i < n_idx; ++i) {
        if (idx[i] < 0) {
            out[i] = std::numeric_limits<double>::quiet_NaN();
            continue;
        }
        const int64_t s = idx[i];
        for (int d = 0; d < D; ++d) kd[static_cast<size_t>(d)] = bf16_to_double(K[s * D + d]);
        out[i] = pair_score(qT.data(), kd.data(), w_row, H, D, dot.data());
    }
    return 0;
}

int32_t si_oracle_sort_topk(const double* scores, int64_t L, int32_t k, int32_t* out_idx,
                            double* out_score) {
    if ((!scores && L > 0) || !out_idx || !out_score || L < 0 || k < 1) return -1;
    std::vector<Entry> e(static_cast<size_t>(L));
    for (int64_t s = 0; s < L; ++s) e[static_cast<size_t>(s)] = Entry{scores[s], s};
    write_sorted(e, k, out_idx, out_score);
    return 0;
}

int32_t si_oracle_topk_rows(const uint16_t* q_rows, const float* w_rows, const uint16_t* K,
                            const int32_t* b_of_row, const int64_t* t_of_row, int64_t n_rows,
                            int32_t H, int32_t D, int64_t T, int32_t m, int32_t k,
                            int32_t mask_mode, int32_t* out_idx, double* out_score,
                            int32_t n_threads) {
    if (!q_rows || !w_rows || !K || !b_of_row || !t_of_row || !out_idx || !out_score) return -1;
    if (n_rows < 0 || H <= 0 || D <= 0 || T <= 0 || m < 1 || k < 1) return -1;
    if (mask_mode != 0 && mask_mode != 1) return -1;

    auto one_row = [&](int64_t r) {
        const int64_t L = si_oracle_legal_count(t_of_row[r], T, m, mask_mode);
        const uint16_t* Kb = K + static_cast<int64_t>(b_of_row[r]) * T * D;
        std::vector<double> sc(static_cast<size_t>(L));
        si_oracle_score_row(q_rows + r * H * D, Kb, w_rows + r * H, H, D, L, sc.data());
        si_oracle_sort_topk(sc.data(), L, k, out_idx + r * k, out_score + r * k);
    };

    if (n_threads <= 1) {
        for (int64_t r = 0; r < n_rows; ++r) one_row(r);
    } else {
        // Fan-out only: thread i takes rows i, i + n_threads, ...
        std::vector<std::thread> pool;
        for (int32_t i = 0; i < n_threads; ++i)
            pool.emplace_back([&, i] {
                for (int64_t r = i; r < n_rows; r += n_threads) one_row(r);
            });
        for (auto& th : pool) th.join();
    }
    return 0;
}

int32_t si_oracle_stream_topk(const double* scores, int64_t L, const int64_t* perm, int32_t k,
                              int32_t* out_idx, double* out_score) {
    if (!scores || !perm || !out_idx || !out_score || L < 0 || k < 1) return -1;
    // priority_queue keeps its "largest" on top; with `better` as less-than the
    // top is the worst kept entry, i.e. the heap's minimum under the order.
    auto worse_on_top = [](const Entry& x, const Entry& y) { return better(x, y); };
    std::priority_queue<Entry, std::vector<Entry>, decltype(worse_on_top)> heap(worse_on_top);
    for (int64_t j = 0; j < L; ++j) {
        const int64_t s = perm[j];
        if (s < 0 || s >= L) return -1;
        const Entry cand{scores[s], s};
        if (static_cast<int64_t>(heap.size()) < k) {
            heap.push(cand);
        } else if (better(cand, heap.top())) {
            heap.pop();
            heap.push(cand);
        }
    }
    std::vector<Entry> kept;
    while (!heap.empty()) {
        kept.push_back(heap.top());
        heap.pop();
    }
    write_sorted(kept, k, out_idx, out_score);
    return 0;
}

int32_t si_oracle_chunked_topk_row(const double* scores, int64_t T, int64_t legal, int32_t k,
                                   int64_t c_T, int32_t variant, int32_t* out_idx,
                                   double* out_score) {
    if (!scores || !out_idx || !out_score || T < 0 || legal < 0 || legal > T) return -1;
    if (k < 1 || c_T < 1 || variant < 0 || variant > 2) return -1;
    const double ninf = -std::numeric_limits<double>::infinity();
    // A pad is (-inf, no index).  Inside this routine "no index" is a value above
    // every key index, so that under the total order a pad loses to any entry
    // of equal score; it is written out as -1.
    const int64_t no_index = std::numeric_limits<int64_t>::max();
    std::vector<Entry> run(static_cast<size_t>(k), Entry{ninf, no_index});
    bool first_tile_done = false;
    for (int64_t t0 = 0; t0 < T; t0 += c_T) {
        const int64_t width = std::min<int64_t>(c_T, T - t0);
        // score tile row, then the per-tile causal mask from the offsets
        std::vector<Entry> tile(static_cast<size_t>(width));
        for (int64_t j = 0; j < width; ++j) {
            const int64_t s = t0 + j;
            tile[static_cast<size_t>(j)] = Entry{s < legal ? scores[s] : ninf, s};
        }
        if (variant == 2 && width < k) continue;  // ablation A2: saturated tile skipped
        // per-tile top-min(k, width); a saturated tile keeps all its entries
        std::sort(tile.begin(), tile.end(), better);
        tile.resize(static_cast<size_t>(std::min<int64_t>(k, width)));
        if (variant == 1 && first_tile_done) continue;  // ablation A1: no merge afterwards
        // merge: best k of (running buffer) U (tile top-k)
        std::vector<Entry> uni(run);
        uni.insert(uni.end(), tile.begin(), tile.end());
        std::sort(uni.begin(), uni.end(), better);
        uni.resize(static_cast<size_t>(k));
        run.swap(uni);
        first_tile_done = true;
    }
    // post-mask: a masked key that filled a slot is not a legal key
    for (int32_t j = 0; j < k; ++j) {
        const Entry& e = run[static_cast<size_t>(j)];
        const bool valid = e.idx < legal;
        out_idx[j] = valid ? static_cast<int32_t>(e.idx) : -1;
        out_score[j] = valid ? e.score : ninf;
    }
    return 0;
}

int32_t si_oracle_sparse_attention_rows(const uint16_t* qa_rows, const uint16_t* K,
                                        const int32_t* idx_rows, const int32_t* b_of_row,
                                        const int64_t* t_of_row, int64_t n_rows, int32_t H,
                                        int32_t D, int64_t T, int32_t m, int32_t k,
                                        int32_t mask_mode, int32_t n_win, double scale,
                                        double* out, int32_t n_threads) {
    if (!qa_rows || !K || !idx_rows || !b_of_row || !t_of_row || !out) return -1;
    if (n_rows < 0 || H <= 0 || D <= 0 || T <= 0 || m < 1 || k < 1 || n_win < 0) return -1;
    if (mask_mode != 0 && mask_mode != 1) return -1;
    for (int64_t i = 0; i < n_rows * k; ++i)
        if (idx_rows[i] < -1 || idx_rows[i] >= T) return -2;

    auto one_row = [&](int64_t r) {
        const int64_t L = si_oracle_legal_count(t_of_row[r], T, m, mask_mode);
        // U(t): the list's valid entries and the window, as a set, ascending
        std::set<int64_t> U;
        for (int32_t j = 0; j < k; ++j)
            if (idx_rows[r * k + j] >= 0) U.insert(idx_rows[r * k + j]);
        for (int64_t s = std::max<int64_t>(0, L - n_win); s < L; ++s) U.insert(s);
        const uint16_t* Kb = K + static_cast<int64_t>(b_of_row[r]) * T * D;
        double* o = out + r * H * D;
        for (int64_t i = 0; i < static_cast<int64_t>(H) * D; ++i) o[i] = 0.0;
        if (U.empty()) return;
        std::vector<double> logit(U.size()), p(U.size());
        for (int32_t h = 0; h < H; ++h) {
            const uint16_t* qh = qa_rows + (r * H + h) * D;
            size_t n = 0;
            double top = -std::numeric_limits<double>::infinity();
            for (int64_t s : U) {
                double dot = 0.0;
                for (int32_t d = 0; d < D; ++d) dot += bf16_to_double(qh[d]) * bf16_to_double(Kb[s * D + d]);
                logit[n] = scale * dot;
                top = std::max(top, logit[n]);
                ++n;
            }
            double denom = 0.0;
            for (size_t i = 0; i < n; ++i) {
                p[i] = std::exp(logit[i] - top);
                denom += p[i];
            }
            n = 0;
            for (int64_t s : U) {
                const double ps = p[n++] / denom;
                for (int32_t d = 0; d < D; ++d) o[h * D + d] += ps * bf16_to_double(Kb[s * D + d]);
            }
        }
    };
    if (n_threads <= 1) {
        for (int64_t r = 0; r < n_rows; ++r) one_row(r);
    } else {
        std::vector<std::thread> pool;
        for (int32_t i = 0; i < n_threads; ++i)
            pool.emplace_back([&, i] {
                for (int64_t r = i; r < n_rows; r += n_threads) one_row(r);
            });
        for (auto& th : pool) th.join();
    }
    return 0;
}

uint64_t si_oracle_materialize_bytes(int64_t B, int64_t S, int64_t H, int64_t T) {
    return static_cast<uint64_t>(B) * static_cast<uint64_t>(S) * static_cast<uint64_t>(H) *
           static_cast<uint64_t>(T) * 4u;
}

uint64_t si_oracle_mask_bytes(int64_t B, int64_t S, int64_t T) {
    return static_cast<uint64_t>(B) * static_cast<uint64_t>(S) * static_cast<uint64_t>(T);
}

}  // extern "C"
