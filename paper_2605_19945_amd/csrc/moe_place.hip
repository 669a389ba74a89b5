// Host-side steps of the paper's method that consume what the GPU path produces (all pointers here are
// HOST memory, everything runs on the CPU as in the paper):
//   * Sec. 3.3.2 "Step-2": which token counts the variability profiler samples and how the token-vs-latency
//     curve C_g(n) is rebuilt from the samples (moe_curve_*),
//   * Sec. 3.3.1 "Step-1" / Sec. 3.2: statistics of the expert-utilisation trace T[t][e] (moe_trace_*),
//   * Sec. 3.3.3 "Step-3", Eq. 1, appendix algorithms Initialmapping / Refine / Place: the expert-to-GPU
//     mapping search (moe_gem_*).
//
// Choices where the paper is silent: C_g(n) joins neighbouring curve samples by straight lines; every GPU
// hosts exactly E / G experts, so a placement only considers GPUs with a free slot; the "20 % noise" of
// restart i > 0 is u_e * (1 + 0.2 * noise[i][e]) with noise supplied by the caller; ties go to the lower
// index (expert order, GPU choice, first best swap in ascending pair order).
//
// Organisation of the search.  The score S(M) = sum_t max_g C_g(n_g(t)) is kept as a table of per-step,
// per-GPU latencies plus, for every step, the three largest latencies and the GPUs that hold them.  A
// candidate change touches one GPU (placing an expert) or two (a swap), so its score is the sum over steps
// of max(new latencies of the touched GPUs, largest cached latency of an untouched GPU): O(S) curve look-ups
// per candidate instead of O(S * G), and the per-step maxima are the same numbers a full re-scoring would
// give, added in the same order.  A swap can only lower the score if at least one of its two GPUs is a
// straggler (holds the maximum) in some step, so pairs between two GPUs that never are get skipped.  The
// K restarts are independent searches whose results are reduced to the lowest score (earliest on a tie).
#include <math.h>

#include <algorithm>
#include <numeric>
#include <vector>

#include "moe_internal.h"

namespace {

// One GPU's sampled curve: counts strictly ascending (latencies as float from the profiler, or double).
template <class V>
struct CurveViewT {
    const int32_t* counts;
    const V* ms;
    int n;
    // straight line between the neighbouring samples; the first sample's value below it, the last one's
    // above it, 0 for no tokens
    double at(long long tokens) const {
        if (tokens <= 0) return 0.0;
        // first sample with counts[i] >= tokens
        const int32_t* hit = std::lower_bound(counts, counts + n, tokens,
                                              [](int32_t c, long long v) { return (long long)c < v; });
        const int i = (int)(hit - counts);
        if (i == n) return (double)ms[n - 1];
        if (i == 0 || counts[i] == tokens) return (double)ms[i];
        const double pv = (double)ms[i - 1], v = (double)ms[i];
        return pv + (v - pv) * (double)(tokens - counts[i - 1]) / (double)(counts[i] - counts[i - 1]);
    }
};

using CurveView = CurveViewT<float>;

template <class V>
bool curve_ok(const int32_t* counts, const V* ms, int n) {
    if (counts == nullptr || ms == nullptr || n < 1) return false;
    for (int i = 1; i < n; ++i)
        if (counts[i] <= counts[i - 1]) return false;
    return true;
}

// ---- mapping search ------------------------------------------------------------------------------------
struct Problem {
    int S, E, G;
    const int32_t* T;  // [S][E]
    std::vector<CurveView> C;
    int tokens(int t, int e) const { return T[(size_t)t * E + e]; }
};

// The three largest per-GPU latencies of one step, descending, with their GPUs (-1: fewer than three GPUs).
struct Top3 {
    double v[3];
    int g[3];
    // largest latency among the GPUs other than x and y
    double max_excluding(int x, int y) const {
        for (int i = 0; i < 3; ++i)
            if (g[i] != x && g[i] != y) return g[i] < 0 ? 0.0 : v[i];
        return 0.0;  // G <= 2 and both excluded, or G == 3 never reaches here with all three excluded
    }
};

class Board {
  public:
    explicit Board(const Problem& p) : P(p), M(p.E, -1), load((size_t)p.S * p.G, 0), lat((size_t)p.S * p.G, 0.0), top(p.S) {
        for (int t = 0; t < P.S; ++t) rebuild_top(t);
    }
    const std::vector<int>& mapping() const { return M; }
    int gpu_of(int e) const { return M[e]; }

    double score() const {
        double total = 0.0;
        for (int t = 0; t < P.S; ++t) total += top[t].v[0];
        return total;
    }
    // score if the unplaced expert e went to GPU g
    double score_with(int e, int g) const {
        double total = 0.0;
        for (int t = 0; t < P.S; ++t) {
            const double mine = P.C[g].at(load[(size_t)t * P.G + g] + P.tokens(t, e));
            total += std::max(mine, top[t].max_excluding(g, g));
        }
        return total;
    }
    // score if the placed experts a and b (on different GPUs) changed places
    double score_swapped(int a, int b) const {
        const int ga = M[a], gb = M[b];
        double total = 0.0;
        for (int t = 0; t < P.S; ++t) {
            const long long ta = P.tokens(t, a), tb = P.tokens(t, b);
            const double la = P.C[ga].at(load[(size_t)t * P.G + ga] - ta + tb);
            const double lb = P.C[gb].at(load[(size_t)t * P.G + gb] - tb + ta);
            total += std::max(std::max(la, lb), top[t].max_excluding(ga, gb));
        }
        return total;
    }
    void place(int e, int g) {
        M[e] = g;
        shift(e, g, +1);
    }
    void swap(int a, int b) {
        const int ga = M[a], gb = M[b];
        shift(a, ga, -1);
        shift(b, gb, -1);
        M[a] = gb;
        M[b] = ga;
        shift(a, gb, +1);
        shift(b, ga, +1);
    }
    // GPUs that hold the largest latency of at least one step
    std::vector<char> stragglers() const {
        std::vector<char> is(P.G, 0);
        for (int t = 0; t < P.S; ++t)
            for (int g = 0; g < P.G; ++g)
                if (lat[(size_t)t * P.G + g] == top[t].v[0]) is[g] = 1;
        return is;
    }

  private:
    void shift(int e, int g, int sign) {
        for (int t = 0; t < P.S; ++t) {
            long long& n = load[(size_t)t * P.G + g];
            n += (long long)sign * P.tokens(t, e);
            lat[(size_t)t * P.G + g] = P.C[g].at(n);
            rebuild_top(t);
        }
    }
    void rebuild_top(int t) {
        Top3& k = top[t];
        for (int i = 0; i < 3; ++i) {
            k.v[i] = 0.0;
            k.g[i] = -1;
        }
        for (int g = 0; g < P.G; ++g) {
            const double v = lat[(size_t)t * P.G + g];
            int at = 0;  // position among the kept ones: behind every larger or equal (earlier) latency
            while (at < 3 && k.g[at] >= 0 && k.v[at] >= v) ++at;
            if (at == 3) continue;
            for (int i = 2; i > at; --i) {
                k.v[i] = k.v[i - 1];
                k.g[i] = k.g[i - 1];
            }
            k.v[at] = v;
            k.g[at] = g;
        }
    }
    const Problem& P;
    std::vector<int> M;
    std::vector<long long> load;  // [S][G] tokens
    std::vector<double> lat;      // [S][G] C_g(load)
    std::vector<Top3> top;        // [S]
};

struct SearchResult {
    std::vector<int> M;
    double score;
    int swaps;
};

// Greedy start: experts in descending order of (perturbed) mean utilisation, each to the GPU with a free
// slot under which the partial mapping scores lowest.
void greedy_start(Board& bd, const Problem& P, const std::vector<double>& weight) {
    std::vector<int> order(P.E);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int x, int y) { return weight[x] > weight[y]; });
    const int slots = P.E / P.G;
    std::vector<int> used(P.G, 0);
    for (int e : order) {
        int pick = -1;
        double pick_score = 0.0;
        for (int g = 0; g < P.G; ++g) {
            if (used[g] == slots) continue;
            const double s = bd.score_with(e, g);
            if (pick < 0 || s < pick_score) {
                pick = g;
                pick_score = s;
            }
        }
        bd.place(e, pick);
        ++used[pick];
    }
}

// Hill climbing over pair exchanges: every round commits the exchange with the largest score drop; the
// round after which that drop is under 0.1 % of the score is the last.  Returns the number of exchanges.
int improve_by_swaps(Board& bd, const Problem& P) {
    int committed = 0;
    for (bool again = true; again;) {
        const double before = bd.score();
        const std::vector<char> hot = bd.stragglers();
        double gain = 0.0;
        int pa = -1, pb = -1;
        for (int a = 0; a < P.E; ++a) {
            const int ga = bd.gpu_of(a);
            for (int b = a + 1; b < P.E; ++b) {
                const int gb = bd.gpu_of(b);
                if (ga == gb || !(hot[ga] || hot[gb])) continue;
                const double d = before - bd.score_swapped(a, b);
                if (d > gain) {
                    gain = d;
                    pa = a;
                    pb = b;
                }
            }
        }
        if (pa < 0) break;
        bd.swap(pa, pb);
        ++committed;
        again = gain / before >= 0.001;
    }
    return committed;
}

SearchResult search_once(const Problem& P, const std::vector<double>& weight) {
    Board bd(P);
    greedy_start(bd, P, weight);
    const int swaps = improve_by_swaps(bd, P);
    return SearchResult{bd.mapping(), bd.score(), swaps};
}

bool problem_from_args(Problem& P, const int32_t* trace, int S, int E, int G, const int32_t* cc, const float* cm,
                       const int32_t* co) {
    if (trace == nullptr || cc == nullptr || cm == nullptr || co == nullptr) return false;
    if (S < 1 || E < 1 || G < 1 || E % G != 0) return false;
    P.S = S;
    P.E = E;
    P.G = G;
    P.T = trace;
    for (int g = 0; g < G; ++g) {
        const int n = co[g + 1] - co[g];
        if (n < 1 || !curve_ok(cc + co[g], cm + co[g], n)) return false;
        P.C.push_back(CurveView{cc + co[g], cm + co[g], n});
    }
    for (size_t i = 0; i < (size_t)S * E; ++i)
        if (trace[i] < 0) return false;
    return true;
}

std::vector<double> mean_utilisation(const int32_t* trace, int S, int E) {
    std::vector<double> u(E);
    for (int e = 0; e < E; ++e) {
        long long sum = 0;
        for (int t = 0; t < S; ++t) sum += trace[(size_t)t * E + e];
        u[e] = (double)sum / (double)S;
    }
    return u;
}

}  // namespace

extern "C" {

// ---- Step-2: sampling plan and curve ---------------------------------------------------------------------
moe_status moe_curve_sample_counts(int32_t boundary, int32_t dense_max, int32_t n_max, int32_t sparse_step,
                                   int32_t after, int32_t* counts_out, int32_t cap, int32_t* n_out) {
    if (n_out == nullptr || boundary < 1 || sparse_step < 1 || n_max < 1 || after < 1 || after > boundary ||
        dense_max < 0 || cap < 0 || (cap > 0 && counts_out == nullptr))
        return MOE_ERR_INVALID_ARG;
    // ascending by construction: 1, then (m*b, m*b + after) for every sampled boundary, then the sparse counts
    const int dense_end = std::min(dense_max, n_max) / boundary * boundary;
    std::vector<int32_t> pts;
    pts.push_back(1);
    for (long long c = boundary; c <= dense_end; c += boundary) {
        pts.push_back((int32_t)c);
        if (c + after <= n_max) pts.push_back((int32_t)(c + after));
    }
    for (long long c = (long long)dense_end + sparse_step; c < n_max; c += sparse_step) pts.push_back((int32_t)c);
    pts.push_back(n_max);
    std::sort(pts.begin(), pts.end());
    pts.erase(std::unique(pts.begin(), pts.end()), pts.end());
    *n_out = (int32_t)pts.size();
    if ((int)pts.size() > cap) return cap == 0 ? MOE_OK : MOE_ERR_WORKSPACE_TOO_SMALL;
    std::copy(pts.begin(), pts.end(), counts_out);
    return MOE_OK;
}

moe_status moe_curve_eval(const int32_t* counts, const double* ms, int32_t n_samples, const int32_t* tokens,
                          int32_t n_tokens, double* ms_out) {
    if (!curve_ok(counts, ms, n_samples) || n_tokens < 0 || (n_tokens > 0 && (tokens == nullptr || ms_out == nullptr)))
        return MOE_ERR_INVALID_ARG;
    const CurveViewT<double> c{counts, ms, n_samples};
    for (int i = 0; i < n_tokens; ++i) ms_out[i] = c.at(tokens[i]);
    return MOE_OK;
}

moe_status moe_curve_sum(const int32_t* counts, const double* ms, int32_t n_samples, int32_t n_lo, int32_t n_hi,
                         double* sum_out) {
    if (!curve_ok(counts, ms, n_samples) || sum_out == nullptr) return MOE_ERR_INVALID_ARG;
    const CurveViewT<double> c{counts, ms, n_samples};
    double s = 0.0;
    for (long long n = n_lo; n <= n_hi; ++n) s += c.at(n);
    *sum_out = s;
    return MOE_OK;
}

// ---- Step-1: trace statistics ------------------------------------------------------------------------------
moe_status moe_trace_mean_utilisation(const int32_t* trace, int32_t S, int32_t E, double* u_out) {
    if (trace == nullptr || u_out == nullptr || S < 1 || E < 1) return MOE_ERR_INVALID_ARG;
    const std::vector<double> u = mean_utilisation(trace, S, E);
    std::copy(u.begin(), u.end(), u_out);
    return MOE_OK;
}

moe_status moe_trace_correlation(const int32_t* trace, int32_t S, int32_t E, double* r_out) {
    if (trace == nullptr || r_out == nullptr || S < 1 || E < 1) return MOE_ERR_INVALID_ARG;
    const std::vector<double> u = mean_utilisation(trace, S, E);
    // centred loads, column-major per expert
    std::vector<double> dev((size_t)E * S);
    std::vector<double> ss(E, 0.0);
    for (int e = 0; e < E; ++e)
        for (int t = 0; t < S; ++t) {
            const double v = (double)trace[(size_t)t * E + e] - u[e];
            dev[(size_t)e * S + t] = v;
            ss[e] += v * v;
        }
    for (int a = 0; a < E; ++a)
        for (int b = 0; b < E; ++b) {
            double dot = 0.0;
            for (int t = 0; t < S; ++t) dot += dev[(size_t)a * S + t] * dev[(size_t)b * S + t];
            const double den = sqrt(ss[a] * ss[b]);
            r_out[(size_t)a * E + b] = den > 0.0 ? dot / den : NAN;  // an expert with constant load has no r
        }
    return MOE_OK;
}

// ---- Step-3: score and search ------------------------------------------------------------------------------
moe_status moe_gem_score(const int32_t* trace, int32_t S, int32_t E, int32_t G, const int32_t* curve_counts,
                         const float* curve_ms, const int32_t* curve_offsets, const int32_t* mapping,
                         double* score_out) {
    Problem P;
    if (!problem_from_args(P, trace, S, E, G, curve_counts, curve_ms, curve_offsets) || mapping == nullptr ||
        score_out == nullptr)
        return MOE_ERR_INVALID_ARG;
    for (int e = 0; e < E; ++e)
        if (mapping[e] < 0 || mapping[e] >= G) return MOE_ERR_INVALID_ARG;
    Board bd(P);
    for (int e = 0; e < E; ++e) bd.place(e, mapping[e]);
    *score_out = bd.score();
    return MOE_OK;
}

moe_status moe_gem_place(const int32_t* trace, int32_t S, int32_t E, int32_t G, const int32_t* curve_counts,
                         const float* curve_ms, const int32_t* curve_offsets, const float* noise, int32_t K,
                         int32_t* mapping_out, double* score_out, int32_t* swaps_out) {
    Problem P;
    if (!problem_from_args(P, trace, S, E, G, curve_counts, curve_ms, curve_offsets) || mapping_out == nullptr ||
        score_out == nullptr || K < 1 || (K > 1 && noise == nullptr))
        return MOE_ERR_INVALID_ARG;
    const std::vector<double> u = mean_utilisation(trace, S, E);
    std::vector<SearchResult> runs;
    runs.reserve(K);
    for (int i = 0; i < K; ++i) {
        std::vector<double> weight(u);
        if (i > 0)
            for (int e = 0; e < E; ++e) weight[e] = u[e] * (1.0 + 0.2 * (double)noise[(size_t)i * E + e]);
        runs.push_back(search_once(P, weight));
    }
    const SearchResult& best = *std::min_element(runs.begin(), runs.end(), [](const SearchResult& x, const SearchResult& y) {
        return x.score < y.score;  // min_element returns the first of equal minima
    });
    std::copy(best.M.begin(), best.M.end(), mapping_out);
    *score_out = best.score;
    if (swaps_out != nullptr) *swaps_out = best.swaps;
    return MOE_OK;
}

}  // extern "C"
