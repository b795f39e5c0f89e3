// Host-side steps that turn measured action times into freeze ratios
// (TimelyFreeze Sec. 3.2: pipeline DAG, start times by longest path, the linear
// program; App. "Edge Construction Rules"; Sec. 3.3: progressive ratio).
// Nothing here touches the GPU: the inputs are the per-action times that the
// monitoring phase measured (e.g. with tf_profile_collect), the outputs are the
// ratios that tf_num_frozen / tf_select_row_blocks / tf_reconcile_mask turn
// into masks.
//
// Node numbering: action (a, m, s) with a = 0 forward / 1 backward, microbatch
// m in [0, M), stage s in [0, S) has id (a M + m) S + s; the source is 2 M S,
// the destination 2 M S + 1.
#include "../../include/tf.h"

#include <algorithm>
#include <cmath>
#include <set>
#include <utility>
#include <vector>

namespace {

inline int node_id(int a, int m, int s, int M, int S) { return (a * M + m) * S + s; }

struct Act { int a, m, s; };          // forward (0) / backward (1), microbatch, stage

// GPipe and 1F1B keep one stage per rank; interleaved 1F1B and ZBV place two (the training
// framework's choice for schedules with several stages per rank).
constexpr int kStagesPerRank = 2;

inline bool one_stage_per_rank(int schedule) { return schedule == TF_SCHEDULE_GPIPE || schedule == TF_SCHEDULE_1F1B; }

// TF_OK, or why (S, M) does not fit the schedule.
int check_schedule(int S, int M, int schedule) {
    if (schedule < TF_SCHEDULE_GPIPE || schedule > TF_SCHEDULE_ZBV) return TF_ERR_INVALID_ARG;
    if (one_stage_per_rank(schedule)) return TF_OK;
    if (S % kStagesPerRank != 0) return TF_ERR_SHAPE;
    if (schedule == TF_SCHEDULE_INTERLEAVED_1F1B) {
        const int R = S / kStagesPerRank, rounds = std::max(1, M / R);
        if (M % rounds != 0) return TF_ERR_SHAPE;                // a chunk takes M / rounds microbatches per visit
    }
    return TF_OK;
}

// GPipe: all forwards, then all backwards.  1F1B: rank s runs min(M, S - 1 - s) forwards ahead.
void one_stage_order(int s, int M, int S, int schedule, std::vector<Act>* o) {
    if (schedule == TF_SCHEDULE_GPIPE) {
        for (int m = 0; m < M; ++m) o->push_back({0, m, s});
        for (int m = 0; m < M; ++m) o->push_back({1, m, s});
        return;
    }
    const int warm = std::min(M, S - 1 - s);                 // forwards before the first backward
    for (int m = 0; m < warm; ++m) o->push_back({0, m, s});
    for (int i = 0; i < M - warm; ++i) { o->push_back({0, warm + i, s}); o->push_back({1, i, s}); }
    for (int m = M - warm; m < M; ++m) o->push_back({1, m, s});
}

// Interleaved 1F1B, rank r of R, V chunks per rank (chunk c is stage c R + r).  A rank visits its
// chunks in turn, g = M / max(1, M div R) microbatches per visit - forwards from the first chunk
// on, backwards from the last - so the k-th pass of either kind is visit k / g: chunk (k / g) mod V
// (mirrored for backwards), microbatch (k / g / V) g + k mod g.  (V - 1) g + 2 (R - 1 - r)
// forwards run ahead, then forward and backward passes alternate, then the backwards that are left.
void interleaved_order(int r, int M, int R, std::vector<Act>* o) {
    const int V = kStagesPerRank;
    const int g = M / std::max(1, M / R);
    const int total = V * M;
    const int warm = std::min((V - 1) * g + 2 * (R - 1 - r), total);
    auto pass = [&](int a, int k) {
        const int visit = k / g;
        const int chunk = a == 0 ? visit % V : V - 1 - visit % V;
        o->push_back({a, (visit / V) * g + k % g, chunk * R + r});
    };
    for (int k = 0; k < warm; ++k) pass(0, k);
    for (int k = 0; k + warm < total; ++k) { pass(0, warm + k); pass(1, k); }
    for (int k = total - warm; k < total; ++k) pass(1, k);
}

// Zero-bubble V schedule, rank r of R: chunk 0 is stage r, chunk 1 stage 2R - 1 - r (the V).  The
// schedule runs a backward as an input-gradient pass and a weight-gradient pass; a backward node
// of the DAG is both, placed where the input-gradient pass runs.  It is laid out for
// n = max(M, 2R - 1) microbatches, those past M left out:
//   2 (R - r) - 1 forwards of chunk 0;  r x (forward chunk 1, forward chunk 0);
//   (R - r) x (forward chunk 1, backward chunk 1);
//   n - R rounds of (forward chunk 0 - the first n - (2R - r - 1) rounds only -, backward chunk 0,
//   forward chunk 1, backward chunk 1), after which every forward has run;
//   r x (backward chunk 0, backward chunk 1);  (R - r) x backward chunk 0.
void zbv_order(int r, int M, int R, std::vector<Act>* o) {
    const int n = std::max(M, 2 * R - 1);
    const int stage[2] = {r, 2 * R - 1 - r};
    int next[2][2] = {{0, 0}, {0, 0}};                       // [a][chunk]: microbatch of the next such pass
    auto pass = [&](int a, int chunk) {
        const int m = next[a][chunk]++;
        if (m < M) o->push_back({a, m, stage[chunk]});
    };
    for (int i = 0; i < 2 * (R - r) - 1; ++i) pass(0, 0);
    for (int i = 0; i < r; ++i) { pass(0, 1); pass(0, 0); }
    for (int i = 0; i < R - r; ++i) { pass(0, 1); pass(1, 1); }
    const int rounds = n - R, with_forward0 = n - (2 * R - r - 1);
    for (int i = 0; i < rounds; ++i) {
        if (i < with_forward0) pass(0, 0);
        pass(1, 0); pass(0, 1); pass(1, 1);
    }
    for (int i = 0; i < r; ++i) { pass(1, 0); pass(1, 1); }
    for (int i = 0; i < R - r; ++i) pass(1, 0);
}

// The order in which every rank runs its actions.
std::vector<std::vector<Act>> rank_orders(int S, int M, int schedule) {
    const int R = one_stage_per_rank(schedule) ? S : S / kStagesPerRank;
    std::vector<std::vector<Act>> all(R);
    for (int r = 0; r < R; ++r) {
        if (schedule == TF_SCHEDULE_INTERLEAVED_1F1B) interleaved_order(r, M, R, &all[r]);
        else if (schedule == TF_SCHEDULE_ZBV) zbv_order(r, M, R, &all[r]);
        else one_stage_order(r, M, S, schedule, &all[r]);
    }
    return all;
}

std::vector<std::pair<int, int>> build_dag(int S, int M, int schedule) {
    std::set<std::pair<int, int>> E;
    auto nid = [&](int a, int m, int s) { return node_id(a, m, s, M, S); };
    const int src = 2 * M * S, dst = src + 1;
    E.insert({src, nid(0, 0, 0)});                                              // rule 1
    E.insert({nid(1, M - 1, 0), dst});
    for (int s = 0; s < S; ++s)                                                 // rule 2
        for (int m = 0; m < M; ++m) {
            E.insert({nid(0, m, s), nid(1, m, s)});
            if (m + 1 < M) { E.insert({nid(0, m, s), nid(0, m + 1, s)}); E.insert({nid(1, m, s), nid(1, m + 1, s)}); }
        }
    for (int m = 0; m < M; ++m)                                                 // rule 3
        for (int s = 0; s + 1 < S; ++s) { E.insert({nid(0, m, s), nid(0, m, s + 1)}); E.insert({nid(1, m, s + 1), nid(1, m, s)}); }
    for (const auto& o : rank_orders(S, M, schedule))                           // rule 4: each rank's own order
        for (size_t i = 0; i + 1 < o.size(); ++i) E.insert({nid(o[i].a, o[i].m, o[i].s), nid(o[i + 1].a, o[i + 1].m, o[i + 1].s)});
    return std::vector<std::pair<int, int>>(E.begin(), E.end());
}

// P_i = max over predecessors (P_j + w_j); false on a cycle.
bool longest_path(int n, const std::vector<std::pair<int, int>>& edges, const double* w, double* P) {
    std::vector<std::vector<int>> succ(n);
    std::vector<int> indeg(n, 0), ready;
    for (const auto& e : edges) { succ[e.first].push_back(e.second); ++indeg[e.second]; }
    for (int i = 0; i < n; ++i) { P[i] = 0.0; if (indeg[i] == 0) ready.push_back(i); }
    int seen = 0;
    while (!ready.empty()) {
        const int i = ready.back();
        ready.pop_back();
        ++seen;
        for (int j : succ[i]) {
            P[j] = std::max(P[j], P[i] + w[i]);
            if (--indeg[j] == 0) ready.push_back(j);
        }
    }
    return seen == n;
}

// Dense two-phase simplex with Bland's rule for  min c x,  A x = b (b >= 0),  x >= 0.
// Small problems only (a few hundred rows); returns false if infeasible or unbounded.
class Simplex {
  public:
    Simplex(int rows, int cols) : m_(rows), n_(cols), t_(size_t(rows) * (cols + 1), 0.0), basis_(rows, -1) {}
    double& a(int r, int c) { return t_[size_t(r) * (n_ + 1) + c]; }
    double& rhs(int r) { return t_[size_t(r) * (n_ + 1) + n_]; }
    void set_basic(int r, int col) { basis_[r] = col; }

    // cost: n_ entries; allowed[c] == false: column c may not enter (artificials in phase 2)
    bool run(const std::vector<double>& cost, const std::vector<char>& allowed, double* objective) {
        std::vector<double> red(n_ + 1, 0.0);                  // reduced costs, last = -objective
        for (int c = 0; c <= n_; ++c) {
            double v = c < n_ ? cost[c] : 0.0;
            for (int r = 0; r < m_; ++r) v -= cost[basis_[r]] * t_[size_t(r) * (n_ + 1) + c];
            red[c] = v;
        }
        const double eps = 1e-10;
        for (long it = 0; it < 200000; ++it) {
            int enter = -1;
            for (int c = 0; c < n_; ++c)
                if (allowed[c] && red[c] < -eps) { enter = c; break; }      // Bland: lowest index
            if (enter < 0) { *objective = -red[n_]; return true; }
            int leave = -1;
            double best = 0.0;
            for (int r = 0; r < m_; ++r) {
                const double p = a(r, enter);
                if (p > eps) {
                    const double q = rhs(r) / p;
                    if (leave < 0 || q < best - 1e-12 || (q < best + 1e-12 && basis_[r] < basis_[leave])) { leave = r; best = q; }
                }
            }
            if (leave < 0) return false;                                     // unbounded
            pivot(leave, enter, &red);
        }
        return false;
    }

    void pivot(int pr, int pc, std::vector<double>* red) {
        const double inv = 1.0 / a(pr, pc);
        double* prow = &t_[size_t(pr) * (n_ + 1)];
        for (int c = 0; c <= n_; ++c) prow[c] *= inv;
        prow[pc] = 1.0;
        for (int r = 0; r < m_; ++r) {
            if (r == pr) continue;
            double* row = &t_[size_t(r) * (n_ + 1)];
            const double f = row[pc];
            if (f == 0.0) continue;
            for (int c = 0; c <= n_; ++c) row[c] -= f * prow[c];
            row[pc] = 0.0;
        }
        if (red) {
            const double f = (*red)[pc];
            if (f != 0.0) {
                for (int c = 0; c <= n_; ++c) (*red)[c] -= f * prow[c];
                (*red)[pc] = 0.0;
            }
        }
        basis_[pr] = pc;
    }

    int rows() const { return m_; }
    int basic(int r) const { return basis_[r]; }
    double value(int col) const {
        for (int r = 0; r < m_; ++r)
            if (basis_[r] == col) return t_[size_t(r) * (n_ + 1) + n_];
        return 0.0;
    }

  private:
    int m_, n_;
    std::vector<double> t_;
    std::vector<int> basis_;
};

}  // namespace

extern "C" {

int tf_pipeline_dag(int32_t n_stages, int32_t n_microbatches, tf_schedule schedule,
                    int32_t capacity, int32_t* edges, int32_t* n_edges) {
    if (n_stages <= 0 || n_microbatches <= 0 || capacity < 0 || !n_edges) return TF_ERR_INVALID_ARG;
    if (int64_t(n_stages) * n_microbatches > (1 << 20)) return TF_ERR_SHAPE;
    const int fit = check_schedule(n_stages, n_microbatches, schedule);
    if (fit != TF_OK) return fit;
    const auto E = build_dag(n_stages, n_microbatches, schedule);
    *n_edges = int32_t(E.size());
    if (capacity > 0 && !edges) return TF_ERR_INVALID_ARG;
    for (int32_t i = 0; i < capacity && i < int32_t(E.size()); ++i) { edges[2 * i] = E[i].first; edges[2 * i + 1] = E[i].second; }
    return TF_OK;
}

int tf_dag_start_times(int32_t n_nodes, int32_t n_edges, const int32_t* edges, const double* w, double* P) {
    if (n_nodes <= 0 || n_edges < 0 || !w || !P || (n_edges > 0 && !edges)) return TF_ERR_INVALID_ARG;
    std::vector<std::pair<int, int>> E;
    for (int32_t i = 0; i < n_edges; ++i) {
        const int32_t a = edges[2 * i], b = edges[2 * i + 1];
        if (a < 0 || b < 0 || a >= n_nodes || b >= n_nodes) return TF_ERR_INVALID_ARG;
        E.push_back({a, b});
    }
    for (int32_t i = 0; i < n_nodes; ++i)
        if (!(w[i] >= 0.0) || !std::isfinite(w[i])) return TF_ERR_INVALID_ARG;
    return longest_path(n_nodes, E, w, P) ? TF_OK : TF_ERR_INVALID_ARG;        // a cycle is an invalid argument
}

int tf_freeze_ratio_lp(int32_t S, int32_t M, tf_schedule schedule,
                       const double* w_min, const double* w_max, double r_max, double lambda,
                       double* r, double* w, double* P, double* batch_time_max, double* batch_time) {
    if (S <= 0 || M <= 0 || !w_min || !w_max || !r) return TF_ERR_INVALID_ARG;
    if (!(r_max >= 0.0 && r_max <= 1.0) || !(lambda >= 0.0 && lambda < 1.0)) return TF_ERR_INVALID_ARG;
    if (int64_t(S) * M > 4096) return TF_ERR_SHAPE;                            // dense tableau: small schedules only
    const int fit = check_schedule(S, M, schedule);
    if (fit != TF_OK) return fit;
    const int n_act = 2 * M * S, N = n_act + 2, src = n_act, dst = n_act + 1;
    double scale = 0.0;
    for (int i = 0; i < n_act; ++i) {
        if (!std::isfinite(w_min[i]) || !std::isfinite(w_max[i]) || w_min[i] < 0.0 || w_max[i] < w_min[i]) return TF_ERR_INVALID_ARG;
        scale = std::max(scale, w_max[i]);
    }
    if (scale == 0.0) scale = 1.0;
    std::vector<double> lo(N, 0.0), range(N, 0.0), delta(N, 0.0);
    for (int i = 0; i < n_act; ++i) {
        lo[i] = w_min[i] / scale;
        range[i] = (w_max[i] - w_min[i]) / scale;
        delta[i] = range[i] > 0.0 ? 1.0 / range[i] : 0.0;
    }
    const auto E = build_dag(S, M, schedule);

    // columns: P of every node but the source, y_i = w_i - w_min_i of freezable nodes, one
    // slack per row, one artificial per row that needs one
    std::vector<int> pcol(N, -1), ycol(N, -1);
    int ncol = 0;
    for (int i = 0; i < N; ++i) if (i != src) pcol[i] = ncol++;
    std::vector<int> free_nodes;
    for (int i = 0; i < n_act; ++i) if (range[i] > 0.0) { ycol[i] = ncol++; free_nodes.push_back(i); }
    std::vector<std::vector<int>> stage_free(S);
    for (int i : free_nodes) stage_free[i % S].push_back(i);
    int n_budget = 0;
    for (int s = 0; s < S; ++s) if (!stage_free[s].empty()) ++n_budget;
    const int nE = int(E.size()), nF = int(free_nodes.size());
    const int rows = nE + nF + n_budget;
    const int slack0 = ncol;                 // one per row
    const int art0 = slack0 + rows;          // one per edge row and budget row
    const int cols = art0 + nE + n_budget;
    Simplex lp(rows, cols);
    int row = 0, art = art0;
    for (const auto& e : E) {                // P_j - P_i - y_i - s = w_min_i
        const int i = e.first, j = e.second;
        if (pcol[j] >= 0) lp.a(row, pcol[j]) += 1.0;
        if (pcol[i] >= 0) lp.a(row, pcol[i]) -= 1.0;
        if (ycol[i] >= 0) lp.a(row, ycol[i]) -= 1.0;
        lp.a(row, slack0 + row) = -1.0;
        lp.a(row, art) = 1.0;
        lp.rhs(row) = lo[i];
        lp.set_basic(row, art++);
        ++row;
    }
    for (int i : free_nodes) {               // y_i + u = range_i
        lp.a(row, ycol[i]) = 1.0;
        lp.a(row, slack0 + row) = 1.0;
        lp.rhs(row) = range[i];
        lp.set_basic(row, slack0 + row);
        ++row;
    }
    for (int s = 0; s < S; ++s) {            // sum delta_i y_i - t = n_s (1 - r_max)
        if (stage_free[s].empty()) continue;
        for (int i : stage_free[s]) lp.a(row, ycol[i]) = delta[i];
        lp.a(row, slack0 + row) = -1.0;
        lp.a(row, art) = 1.0;
        lp.rhs(row) = double(stage_free[s].size()) * (1.0 - r_max);
        lp.set_basic(row, art++);
        ++row;
    }
    // phase 1: drive the artificials to zero
    std::vector<double> cost(cols, 0.0);
    std::vector<char> allowed(cols, 1);
    for (int c = art0; c < cols; ++c) cost[c] = 1.0;
    double obj = 0.0;
    if (!lp.run(cost, allowed, &obj) || obj > 1e-7) return TF_ERR_INVALID_ARG;       // infeasible: cannot happen for valid input
    for (int rr = 0; rr < lp.rows(); ++rr) {                                           // artificials still basic (at zero): pivot them out
        if (lp.basic(rr) < art0) continue;
        for (int c = 0; c < art0; ++c)
            if (std::fabs(lp.a(rr, c)) > 1e-9) { lp.pivot(rr, c, nullptr); break; }
    }
    // phase 2: min P_d - lambda sum delta_i y_i
    std::fill(cost.begin(), cost.end(), 0.0);
    cost[pcol[dst]] = 1.0;
    for (int c = art0; c < cols; ++c) allowed[c] = 0;
    // lambda multiplies sum delta_i w_i of the unscaled problem while P_d is scaled by 1 / scale
    for (int i : free_nodes) cost[ycol[i]] = -(lambda / scale) * delta[i];
    if (!lp.run(cost, allowed, &obj)) return TF_ERR_INVALID_ARG;

    std::vector<double> wv(N, 0.0), Pv(N, 0.0);
    for (int i = 0; i < n_act; ++i) {
        double y = ycol[i] >= 0 ? lp.value(ycol[i]) : 0.0;
        y = std::min(std::max(y, 0.0), range[i]);
        wv[i] = (lo[i] + y) * scale;
        double ri = range[i] > 0.0 ? 1.0 - y * delta[i] : 0.0;
        r[i] = std::min(std::max(ri, 0.0), 1.0);
        if (w) w[i] = wv[i];
    }
    if (!longest_path(N, E, wv.data(), Pv.data())) return TF_ERR_INVALID_ARG;
    if (P) for (int i = 0; i < N; ++i) P[i] = Pv[i];
    if (batch_time) *batch_time = Pv[dst];
    if (batch_time_max) {
        std::vector<double> wm(N, 0.0), Pm(N, 0.0);
        for (int i = 0; i < n_act; ++i) wm[i] = w_max[i];
        longest_path(N, E, wm.data(), Pm.data());
        *batch_time_max = Pm[dst];
    }
    return TF_OK;
}

double tf_actual_freeze_ratio(double r, int64_t t, int64_t T_m, int64_t T_f) {
    if (t <= T_m || T_f <= T_m) return t > T_m ? r : 0.0;
    return std::min(r, r * double(t - T_m) / double(T_f - T_m));
}

}  // extern "C"
