// Host-side expert-to-GPU mapping search of the paper (Sec. 3.3.3 "Step-3": Eq. 1 and the search
// algorithm; appendix "Expert Mapping Algorithm": initial mapping, iterative refinement, K restarts).
// It consumes what the GPU path produces -- the per-GPU token-vs-latency curves C_g (moe_profile_ffn)
// and the expert-utilisation trace T[t][e] (counts_out rows) -- and runs on the CPU, as in the paper.
//
// Choices where the paper is silent: C_g(n) joins neighbouring curve samples by straight lines; every
// GPU hosts exactly E / G experts, so the greedy placement only considers GPUs with a free slot; the
// "20 % noise" of restart i > 0 is u_e * (1 + 0.2 * noise[i][e]) with noise supplied by the caller;
// ties go to the lower index (expert order, GPU choice, first best swap in ascending pair order).
#include <math.h>

#include <vector>

#include "moe_internal.h"

namespace {

struct Curves {
    const int32_t* counts;
    const float* ms;
    const int32_t* off;  // [G + 1]
    int G;
    double at(int g, long long n) const {
        if (n <= 0) return 0.0;
        const int lo = off[g], hi = off[g + 1];
        for (int i = lo; i < hi; ++i) {
            if (counts[i] == n) return (double)ms[i];
            if (counts[i] > n) {
                if (i == lo) return (double)ms[i];
                const double pv = (double)ms[i - 1], v = (double)ms[i];
                return pv + (v - pv) * (double)(n - counts[i - 1]) / (double)(counts[i] - counts[i - 1]);
            }
        }
        return (double)ms[hi - 1];
    }
};

// State of a (partial) mapping: per-step per-GPU token loads and their latencies.
struct State {
    int S, E, G;
    const int32_t* T;
    const Curves* C;
    std::vector<int> M;             // GPU of expert e, -1 = not placed
    std::vector<long long> load;    // [S][G]
    std::vector<double> lat;        // [S][G]
    double score() const {
        double total = 0.0;
        for (int t = 0; t < S; ++t) {
            double worst = 0.0;
            for (int g = 0; g < G; ++g) worst = lat[(size_t)t * G + g] > worst ? lat[(size_t)t * G + g] : worst;
            total += worst;
        }
        return total;
    }
    void add(int e, int g, int sign) {
        for (int t = 0; t < S; ++t) {
            long long& n = load[(size_t)t * G + g];
            n += (long long)sign * T[(size_t)t * E + e];
            lat[(size_t)t * G + g] = C->at(g, n);
        }
    }
    // score with experts a (on ga) and b (on gb) exchanged, without changing the state
    double score_swapped(int a, int b) const {
        const int ga = M[a], gb = M[b];
        double total = 0.0;
        for (int t = 0; t < S; ++t) {
            const long long ta = T[(size_t)t * E + a], tb = T[(size_t)t * E + b];
            const double la = C->at(ga, load[(size_t)t * G + ga] - ta + tb);
            const double lb = C->at(gb, load[(size_t)t * G + gb] - tb + ta);
            double worst = 0.0;
            for (int g = 0; g < G; ++g) {
                const double v = g == ga ? la : (g == gb ? lb : lat[(size_t)t * G + g]);
                worst = v > worst ? v : worst;
            }
            total += worst;
        }
        return total;
    }
};

bool place_args_ok(const int32_t* trace, int S, int E, int G, const int32_t* cc, const float* cm, const int32_t* co) {
    if (trace == nullptr || cc == nullptr || cm == nullptr || co == nullptr) return false;
    if (S < 1 || E < 1 || G < 1 || E % G != 0) return false;
    for (int g = 0; g < G; ++g) {
        if (co[g + 1] <= co[g]) return false;  // every GPU needs at least one curve sample
        for (int i = co[g] + 1; i < co[g + 1]; ++i)
            if (cc[i] <= cc[i - 1]) return false;  // ascending token counts
    }
    for (size_t i = 0; i < (size_t)S * E; ++i)
        if (trace[i] < 0) return false;
    return true;
}

State make_state(const int32_t* trace, int S, int E, int G, const Curves* C) {
    State st;
    st.S = S; st.E = E; st.G = G; st.T = trace; st.C = C;
    st.M.assign(E, -1);
    st.load.assign((size_t)S * G, 0);
    st.lat.assign((size_t)S * G, 0.0);
    return st;
}

}  // namespace

extern "C" {

moe_status moe_gem_score(const int32_t* trace, int32_t S, int32_t E, int32_t G, const int32_t* curve_counts,
                         const float* curve_ms, const int32_t* curve_offsets, const int32_t* mapping,
                         double* score_out) {
    if (!place_args_ok(trace, S, E, G, curve_counts, curve_ms, curve_offsets) || mapping == nullptr ||
        score_out == nullptr)
        return MOE_ERR_INVALID_ARG;
    for (int e = 0; e < E; ++e)
        if (mapping[e] < 0 || mapping[e] >= G) return MOE_ERR_INVALID_ARG;
    const Curves C{curve_counts, curve_ms, curve_offsets, G};
    State st = make_state(trace, S, E, G, &C);
    for (int e = 0; e < E; ++e) {
        st.M[e] = mapping[e];
        st.add(e, mapping[e], +1);
    }
    *score_out = st.score();
    return MOE_OK;
}

moe_status moe_gem_place(const int32_t* trace, int32_t S, int32_t E, int32_t G, const int32_t* curve_counts,
                         const float* curve_ms, const int32_t* curve_offsets, const float* noise, int32_t K,
                         int32_t* mapping_out, double* score_out, int32_t* swaps_out) {
    if (!place_args_ok(trace, S, E, G, curve_counts, curve_ms, curve_offsets) || mapping_out == nullptr ||
        score_out == nullptr || K < 1 || (K > 1 && noise == nullptr))
        return MOE_ERR_INVALID_ARG;
    const Curves C{curve_counts, curve_ms, curve_offsets, G};
    const int cap = E / G;
    // u: per-expert mean utilisation over the trace
    std::vector<double> u(E);
    for (int e = 0; e < E; ++e) {
        long long sum = 0;
        for (int t = 0; t < S; ++t) sum += trace[(size_t)t * E + e];
        u[e] = (double)sum / (double)S;
    }
    double best_score = INFINITY;
    int best_swaps = 0;
    std::vector<int> best_M(E, 0);
    for (int i = 0; i < K; ++i) {
        // ---- initial mapping: heaviest experts first, each on the GPU that adds least to S ----
        std::vector<double> key(E);
        for (int e = 0; e < E; ++e) key[e] = i > 0 ? u[e] * (1.0 + 0.2 * (double)noise[(size_t)i * E + e]) : u[e];
        std::vector<int> order(E);
        for (int e = 0; e < E; ++e) order[e] = e;
        for (int x = 1; x < E; ++x) {  // stable insertion sort, descending key (E <= a few hundred)
            const int e = order[x];
            int y = x - 1;
            while (y >= 0 && key[order[y]] < key[e]) {
                order[y + 1] = order[y];
                --y;
            }
            order[y + 1] = e;
        }
        State st = make_state(trace, S, E, G, &C);
        std::vector<int> used(G, 0);
        for (int x = 0; x < E; ++x) {
            const int e = order[x];
            int best_g = -1;
            double best_s = 0.0;
            for (int g = 0; g < G; ++g) {
                if (used[g] >= cap) continue;
                st.add(e, g, +1);
                const double s = st.score();
                st.add(e, g, -1);
                if (best_g < 0 || s < best_s) {
                    best_g = g;
                    best_s = s;
                }
            }
            st.M[e] = best_g;
            st.add(e, best_g, +1);
            ++used[best_g];
        }
        // ---- refinement: commit the cross-GPU swap with the largest drop until it is below 0.1 % ----
        int swaps = 0;
        for (;;) {
            const double s_prev = st.score();
            int ba = -1, bb = -1;
            double best_drop = 0.0;
            for (int a = 0; a < E; ++a)
                for (int b = a + 1; b < E; ++b) {
                    if (st.M[a] == st.M[b]) continue;
                    const double drop = s_prev - st.score_swapped(a, b);
                    if (drop > best_drop) {
                        best_drop = drop;
                        ba = a;
                        bb = b;
                    }
                }
            if (ba < 0) break;
            const int ga = st.M[ba], gb = st.M[bb];
            st.add(ba, ga, -1);
            st.add(bb, gb, -1);
            st.add(ba, gb, +1);
            st.add(bb, ga, +1);
            st.M[ba] = gb;
            st.M[bb] = ga;
            ++swaps;
            if (best_drop / s_prev < 0.001) break;
        }
        const double s = st.score();
        if (s < best_score) {
            best_score = s;
            best_M = st.M;
            best_swaps = swaps;
        }
    }
    for (int e = 0; e < E; ++e) mapping_out[e] = best_M[e];
    *score_out = best_score;
    if (swaps_out != nullptr) *swaps_out = best_swaps;
    return MOE_OK;
}

}  // extern "C"
