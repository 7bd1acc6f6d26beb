// CPU oracle for the forward pass of one Expert-Token Resonance MoE layer.
//
// TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, obviously-correct
// statement of what the layer computes, written from the paper's definitions.
// It shares no code with the GPU library and must never be called from the
// product path; only the tests, the smoke check and the benchmark's
// cpu-baseline leg use it.
//
// Everything is computed the slow way: double accumulators, full sorts,
// triple-loop matrix products, no blocking, no fusion.  All pointers are HOST
// pointers.  Floating-point inputs are fp32 or bf16 (dtype 0 / 1); bf16 values
// are widened exactly.
//
// What each function follows:
//   etr_ref_route       GrAP pooling (Sec. Cost-Efficient Sparse Expert-Token
//                       Affinity, Eqs. 2-3: each gate vector is 1/(group size)
//                       on its group, so x^T w_i is the group mean) and the
//                       cosine affinity (Eq. 4); gate = row softmax (Eq. 1 text)
//   etr_ref_select      token choice Top-l (Eq. 5); expert choice over the
//                       candidates (Eq. 6, "Bottom-C" read as top-C by
//                       affinity: the text around it says each expert keeps
//                       the tokens with the highest affinity); pure TCR keep
//                       rule "fewer than C earlier tokens went to the same
//                       expert" (Proof of Theorem, part 1); pure ECR keep rule
//                       "at most C-1 tokens score higher" (Proof, part 2)
//   etr_ref_dispatch    the capacity-bounded per-expert slot table I_{ki} of
//                       Eq. 6, materialised as rows
//   etr_ref_ffn_rows    the expert network: a SwiGLU feed-forward block
//   etr_ref_combine     the gate-weighted sum of Eq. 1
//   etr_ref_moe_forward the chain of the above
//   etr_ref_route_stats expert load distribution, mean gate and KL(D_c || D_l) of Sec. Locality Loss
//   etr_ref_capacity_lower_bound  C_min of the Remark in Sec. Dynamic Lower Bound Module
//   etr_ref_backward_tokens / _hidden_units   the chain rule through Eqs. 1-6 with the routing tables fixed
//
// Readings of points the paper leaves open (all listed in the design notes):
// ties go to the lowest index; slots inside an expert are in ascending token
// order; the gate is the softmax over all experts of the affinity row with no
// renormalisation over the selected set; a token kept by no expert gives a
// zero output row.
//
// Every function here is pinned by CPU tests against worked examples derived
// from the equations, closed forms, invariants and brute force (no "parity
// unpinned" function).

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <numeric>
#include <vector>
#ifdef _OPENMP
#include <omp.h>
#endif

namespace {

enum { DT_F32 = 0, DT_BF16 = 1 };
enum { MODE_TCR = 0, MODE_ECR = 1, MODE_BIDIR = 2, MODE_TCR_RANK = 3, MODE_BIDIR_STRICT = 4 };
enum { COS_FULL = 0, COS_POOLED = 1 };

inline float bf16_to_float(uint16_t b) {
    uint32_t u = static_cast<uint32_t>(b) << 16;
    float f;
    std::memcpy(&f, &u, 4);
    return f;
}

// Round a double to the nearest bf16 (ties to even), directly, without going
// through fp32 first (which could round twice).
inline uint16_t double_to_bf16(double v) {
    if (std::isnan(v)) return 0x7FC0;
    if (std::isinf(v)) return v > 0 ? 0x7F80 : 0xFF80;
    if (v == 0.0) return std::signbit(v) ? 0x8000 : 0x0000;
    int e = std::ilogb(v);                 // v = m * 2^e, 1 <= |m| < 2
    if (e < -126) e = -126;                // subnormal range: fixed quantum
    // bf16 keeps 8 significant bits: quantum is 2^(e-7)
    double q = std::nearbyint(std::ldexp(v, 7 - e));   // default mode: ties-to-even
    double r = std::ldexp(q, e - 7);
    float f = static_cast<float>(r);       // exact: r has <= 8 significant bits
    if (std::isinf(f)) return f > 0 ? 0x7F80 : 0xFF80;
    uint32_t u;
    std::memcpy(&u, &f, 4);
    return static_cast<uint16_t>(u >> 16);
}

inline double load_elem(const void* p, int dtype, size_t i) {
    if (dtype == DT_F32) return static_cast<double>(static_cast<const float*>(p)[i]);
    return static_cast<double>(bf16_to_float(static_cast<const uint16_t*>(p)[i]));
}

inline void store_elem(void* p, int dtype, size_t i, double v) {
    if (dtype == DT_F32) static_cast<float*>(p)[i] = static_cast<float>(v);
    else static_cast<uint16_t*>(p)[i] = double_to_bf16(v);
}

inline size_t elem_size(int dtype) { return dtype == DT_F32 ? 4 : 2; }

// "a ranks before b": higher score first, then lower index.  Compared on the
// fp32 values as stored (so -0.0 and +0.0 tie and the index decides).
struct ByScoreThenIndex {
    const float* s;   // score of candidate i is s[i * stride]
    size_t stride;
    bool operator()(int a, int b) const {
        float sa = s[a * stride], sb = s[b * stride];
        if (sa != sb) return sa > sb;
        return a < b;
    }
};

}  // namespace

extern "C" {

// ---------------------------------------------------------------------------
// Route: GrAP + cosine affinity + softmax gate.
//   x[T][d] (dtype), w_emb[E][P] fp32 with P = d/D  ->  score[T][E], gate[T][E] fp32
// cos_mode FULL: Eq. 4 literally, with the expert embedding lifted back to R^d
//   (every pooled coordinate spread evenly over its group of D inputs):
//   score = sqrt(D) * <g, w_e> / (|x| * |w_e|).
// cos_mode POOLED: cosine between the pooled token and the embedding:
//   score = <g, w_e> / (|g| * |w_e|).
// A zero-norm token (or embedding) scores 0.
// ---------------------------------------------------------------------------
int etr_ref_route(int T, int d, int E, int D, int dtype, int cos_mode,
                  const void* x, const float* w_emb, float* score, float* gate) {
    if (T < 0 || d <= 0 || E <= 0 || D <= 0 || d % D != 0) return 2;
    const int P = d / D;
    std::vector<double> wnorm(E);
    for (int e = 0; e < E; ++e) {
        double s = 0;
        for (int p = 0; p < P; ++p) s += double(w_emb[e * (size_t)P + p]) * double(w_emb[e * (size_t)P + p]);
        wnorm[e] = std::sqrt(s);
    }
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        std::vector<double> g(P);
        double xx = 0, gg = 0;
        for (int p = 0; p < P; ++p) {
            double s = 0;
            for (int j = 0; j < D; ++j) {
                double v = load_elem(x, dtype, (size_t)t * d + (size_t)p * D + j);
                s += v;
                xx += v * v;
            }
            g[p] = s / D;                       // group mean
            gg += g[p] * g[p];
        }
        std::vector<double> sc(E);
        double mx = -INFINITY;
        for (int e = 0; e < E; ++e) {
            double dot = 0;
            for (int p = 0; p < P; ++p) dot += g[p] * double(w_emb[e * (size_t)P + p]);
            double den = (cos_mode == COS_FULL) ? std::sqrt(xx) * wnorm[e] : std::sqrt(gg) * wnorm[e];
            double num = (cos_mode == COS_FULL) ? std::sqrt((double)D) * dot : dot;
            double v = (den > 0) ? num / den : 0.0;
            float vf = static_cast<float>(v);
            score[(size_t)t * E + e] = vf;
            sc[e] = v;
            mx = std::max(mx, v);
        }
        double z = 0;
        for (int e = 0; e < E; ++e) z += std::exp(sc[e] - mx);
        for (int e = 0; e < E; ++e) gate[(size_t)t * E + e] = static_cast<float>(std::exp(sc[e] - mx) / z);
    }
    return 0;
}

// ---------------------------------------------------------------------------
// Select: token choice, capacity-bounded keep, slots.
//   score[T][E] fp32 (any source)  ->
//   topk_expert[T][k] (descending score; may be NULL; not written in ECR mode),
//   slot_of[T][E] (slot of token t in expert e's buffer, -1 if not kept),
//   slot_token[E][capacity] (inverse; -1 = empty slot), counts[E].
// ---------------------------------------------------------------------------
// Fixed-point image of an affinity used for the adaptive token count: round(clamp(s,-1,1) * 2^30).
// Sums of these integers do not depend on the order of addition, so "the prefix sum reaches the
// threshold" is one well-defined integer decision on every implementation.
static long long affinity_fixed(float s) {
    double v = std::min(1.0, std::max(-1.0, (double)s));
    return std::llrint(v * 1073741824.0);
}

int etr_ref_select_adaptive(int T, int E, int k, int capacity, int mode, const float* score, float sum_threshold,
                            int32_t* topk_expert, int32_t* slot_of, int32_t* slot_token, int32_t* counts);

int etr_ref_select(int T, int E, int k, int capacity, int mode, const float* score,
                   int32_t* topk_expert, int32_t* slot_of, int32_t* slot_token, int32_t* counts) {
    return etr_ref_select_adaptive(T, E, k, capacity, mode, score, 0.0f, topk_expert, slot_of, slot_token, counts);
}

// Selection with the adaptive token count of Sec. Routing Strategy ("the expert chooses its Top-l
// tokens where l is determined by a threshold of the sum of affinity scores"; the paper gives no
// value for the threshold, so it is an argument).  Reading: expert e walks its candidates from the
// highest affinity down and stops at the first prefix whose affinity sum reaches sum_threshold;
// l_e is that prefix length, or all candidates if the sum of the positive affinities never gets
// there; the expert then keeps min(capacity, l_e) tokens.  sum_threshold <= 0 switches it off; it
// does not apply to pure token choice (TCR keeps by position, not by affinity).
int etr_ref_select_adaptive(int T, int E, int k, int capacity, int mode, const float* score, float sum_threshold,
                            int32_t* topk_expert, int32_t* slot_of, int32_t* slot_token, int32_t* counts) {
    if (T < 0 || E <= 0 || capacity < 1) return 2;
    if (mode != MODE_ECR && (k < 1 || k > E)) return 2;
    if (mode < 0 || mode > 4) return 3;
    if (sum_threshold > 0.0f && mode == MODE_BIDIR_STRICT) return 3;

    // Eq. 5: every token lists its k best experts.
    std::vector<std::vector<int>> candidates(E);     // per expert, ascending token index
    std::vector<std::vector<int>> cand_rank(E);      // position of the expert in that token's list
    if (mode == MODE_ECR) {
        for (int e = 0; e < E; ++e) {
            candidates[e].resize(T);
            std::iota(candidates[e].begin(), candidates[e].end(), 0);
        }
    } else {
        std::vector<int> order(E);
        for (int t = 0; t < T; ++t) {
            std::iota(order.begin(), order.end(), 0);
            std::stable_sort(order.begin(), order.end(), ByScoreThenIndex{score + (size_t)t * E, 1});
            for (int j = 0; j < k; ++j) {
                if (topk_expert) topk_expert[(size_t)t * k + j] = order[j];
                candidates[order[j]].push_back(t);
                cand_rank[order[j]].push_back(j);
            }
        }
    }

    for (size_t i = 0; i < (size_t)T * E; ++i) slot_of[i] = -1;
    for (size_t i = 0; i < (size_t)E * capacity; ++i) slot_token[i] = -1;

    for (int e = 0; e < E; ++e) {
        std::vector<int> cand = candidates[e];
        int n_keep = std::min<int>(capacity, (int)cand.size());
        std::vector<int> kept;
        if (mode == MODE_TCR) {
            // position priority: the first C tokens (in token order) that chose e
            kept.assign(cand.begin(), cand.begin() + n_keep);
        } else if (mode == MODE_TCR_RANK) {
            // Variant of the position priority for Top-l with l > 1 (the paper states the rule for one
            // choice per token only): every token's first choice is served before any second choice,
            // and so on; inside one rank, token order.  An expert keeps the first C of its choosers in
            // the order (rank, token index).
            std::vector<int> idx(cand.size());
            std::iota(idx.begin(), idx.end(), 0);
            const std::vector<int>& rk = cand_rank[e];
            std::stable_sort(idx.begin(), idx.end(), [&](int a, int b) { return rk[a] < rk[b]; });
            for (int m = 0; m < n_keep; ++m) kept.push_back(cand[idx[m]]);
            std::sort(kept.begin(), kept.end());
        } else if (mode == MODE_BIDIR_STRICT) {
            // Variant of the bidirectional rule: the pair (t, e) survives iff t lists e (Eq. 5) and t is
            // among e's top-min(C, T) tokens taken over ALL tokens (pure expert choice), i.e. the
            // intersection of the two pure phases.  A subset of what Eq. 6 keeps.
            std::vector<int> all(T);
            std::iota(all.begin(), all.end(), 0);
            std::stable_sort(all.begin(), all.end(), ByScoreThenIndex{score + e, (size_t)E});
            std::vector<char> top(T, 0);
            for (int m = 0; m < std::min(capacity, T); ++m) top[all[m]] = 1;
            for (int t : cand) if (top[t]) kept.push_back(t);     // cand is in ascending token order
            n_keep = (int)kept.size();
        } else {
            // Eq. 6 / pure ECR: the C candidates with the highest affinity to e
            std::stable_sort(cand.begin(), cand.end(), ByScoreThenIndex{score + e, (size_t)E});
            if (sum_threshold > 0.0f) {
                const long long need = std::max(1ll, std::llrint((double)sum_threshold * 1073741824.0));
                long long run = 0;
                int ell = (int)cand.size();
                for (int m = 0; m < (int)cand.size(); ++m) {
                    const float sc = score[(size_t)cand[m] * E + e];
                    if (!(sc > 0.0f)) break;                 // the sum cannot grow any further
                    run += affinity_fixed(sc);
                    if (run >= need) { ell = m + 1; break; }
                }
                n_keep = std::min(n_keep, ell);
            }
            kept.assign(cand.begin(), cand.begin() + n_keep);
            std::sort(kept.begin(), kept.end());      // slots in ascending token order
        }
        counts[e] = n_keep;
        for (int s = 0; s < n_keep; ++s) {
            slot_token[(size_t)e * capacity + s] = kept[s];
            slot_of[(size_t)kept[s] * E + e] = s;
        }
    }
    return 0;
}

// ---------------------------------------------------------------------------
// Dispatch: xp[e][s][:] = x[slot_token[e][s]][:] for s < counts[e].
// Rows past counts[e] are zero-filled here (the contract leaves them unspecified).
// ---------------------------------------------------------------------------
int etr_ref_dispatch(int T, int d, int E, int capacity, int dtype, const void* x,
                     const int32_t* slot_token, const int32_t* counts, void* xp) {
    const size_t es = elem_size(dtype);
    std::memset(xp, 0, (size_t)E * capacity * d * es);
    for (int e = 0; e < E; ++e)
        for (int s = 0; s < counts[e]; ++s) {
            int t = slot_token[(size_t)e * capacity + s];
            if (t < 0 || t >= T) return 2;
            std::memcpy(static_cast<char*>(xp) + ((size_t)e * capacity + s) * d * es,
                        static_cast<const char*>(x) + (size_t)t * d * es, (size_t)d * es);
        }
    return 0;
}

// ---------------------------------------------------------------------------
// Expert FFN on a list of rows:  y = W_down * ( SiLU(W_gate * x) .* (W_up * x) )
// with SiLU(a) = a / (1 + exp(-a)); no biases; no intermediate rounding.
//   rows[r][d] (dtype), expert_of_row[r], w_gate/w_up[E][H][d], w_down[E][d][H]
//   -> y[r][d] double
// ---------------------------------------------------------------------------
int etr_ref_ffn_rows(int n_rows, int d, int H, int dtype, const void* rows, const int32_t* expert_of_row,
                     const void* w_gate, const void* w_up, const void* w_down, double* y) {
#pragma omp parallel for schedule(dynamic, 1)
    for (int r = 0; r < n_rows; ++r) {
        const int e = expert_of_row[r];
        std::vector<double> xr(d), h(H);
        for (int j = 0; j < d; ++j) xr[j] = load_elem(rows, dtype, (size_t)r * d + j);
        for (int i = 0; i < H; ++i) {
            double a = 0, b = 0;
            const size_t base = ((size_t)e * H + i) * d;
            for (int j = 0; j < d; ++j) {
                a += load_elem(w_gate, dtype, base + j) * xr[j];
                b += load_elem(w_up, dtype, base + j) * xr[j];
            }
            h[i] = a / (1.0 + std::exp(-a)) * b;
        }
        for (int j = 0; j < d; ++j) {
            double s = 0;
            const size_t base = ((size_t)e * d + j) * H;
            for (int i = 0; i < H; ++i) s += load_elem(w_down, dtype, base + i) * h[i];
            y[(size_t)r * d + j] = s;
        }
    }
    return 0;
}

// Expert FFN over the capacity-bounded buffers: yp[e][s][:] for s < counts[e]; other rows 0.
int etr_ref_expert_ffn(int d, int E, int capacity, int H, int dtype, const void* xp, const int32_t* counts,
                       const void* w_gate, const void* w_up, const void* w_down, double* yp) {
    std::memset(yp, 0, sizeof(double) * (size_t)E * capacity * d);
    const size_t es = elem_size(dtype);
    for (int e = 0; e < E; ++e) {
        int n = counts[e];
        if (n < 0 || n > capacity) return 2;
        std::vector<int32_t> eid(n, e);
        int rc = etr_ref_ffn_rows(n, d, H, dtype, static_cast<const char*>(xp) + (size_t)e * capacity * d * es,
                                  eid.data(), w_gate, w_up, w_down, yp + (size_t)e * capacity * d);
        if (rc) return rc;
    }
    return 0;
}

// ---------------------------------------------------------------------------
// Combine (Eq. 1): out[t][:] = sum over experts e (ascending) that kept t of
// gate[t][e] * yp[e][slot_of[t][e]][:]; accumulated in double, rounded once.
// gate_norm = 1 is the variant in which the gate weights of a token are renormalised over the
// experts that kept it (they then sum to one, as in Top-l gating of the sparse baselines);
// gate_norm = 0 uses the softmax over all experts as it is.
// ---------------------------------------------------------------------------
}  // extern "C"
namespace {
template <typename G>
double kept_gate_sum(const G* gate_row, const int32_t* slot_row, int E, int gate_norm) {
    if (!gate_norm) return 1.0;
    double s = 0;
    for (int e = 0; e < E; ++e)
        if (slot_row[e] >= 0) s += double(gate_row[e]);
    return s > 0 ? s : 1.0;
}
}  // namespace
extern "C" {

int etr_ref_combine(int T, int d, int E, int capacity, int dtype, const double* yp, const float* gate,
                    const int32_t* slot_of, void* out, int gate_norm) {
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        std::vector<double> acc(d, 0.0);
        const double norm = kept_gate_sum(gate + (size_t)t * E, slot_of + (size_t)t * E, E, gate_norm);
        for (int e = 0; e < E; ++e) {
            int s = slot_of[(size_t)t * E + e];
            if (s < 0) continue;
            const double gt = gate[(size_t)t * E + e] / norm;
            const double* yr = yp + ((size_t)e * capacity + s) * d;
            for (int j = 0; j < d; ++j) acc[j] += gt * yr[j];
        }
        for (int j = 0; j < d; ++j) store_elem(out, dtype, (size_t)t * d + j, acc[j]);
    }
    return 0;
}

// ---------------------------------------------------------------------------
// Whole layer.  If score_in is non-NULL the routing starts from those fp32
// scores (gate is then their row softmax) instead of from x; this is how the
// tests compare the rest of the layer on identical routing inputs.
// If n_tokens >= 0, the FFN and the sum are evaluated only for the listed
// tokens and out holds n_tokens rows (out[i] = layer output of tokens[i]);
// routing is always done for all T tokens.  Routing tables are returned when
// the pointers are non-NULL.
// ---------------------------------------------------------------------------
int etr_ref_moe_forward(int T, int d, int E, int D, int k, int capacity, int H, int dtype, int mode, int cos_mode,
                        const void* x, const float* w_emb, const void* w_gate, const void* w_up,
                        const void* w_down, const float* score_in, const int32_t* tokens, int n_tokens,
                        void* out, float* score_out, float* gate_out, int32_t* topk_out, int32_t* slot_of_out,
                        int32_t* slot_token_out, int32_t* counts_out, int gate_norm) {
    std::vector<float> score((size_t)T * E), gate((size_t)T * E);
    int rc = 0;
    if (!score_in) {
        rc = etr_ref_route(T, d, E, D, dtype, cos_mode, x, w_emb, score.data(), gate.data());
        if (rc) return rc;
    } else {
        std::copy(score_in, score_in + (size_t)T * E, score.begin());
        for (int t = 0; t < T; ++t) {
            double mx = -INFINITY, z = 0;
            for (int e = 0; e < E; ++e) mx = std::max(mx, (double)score[(size_t)t * E + e]);
            for (int e = 0; e < E; ++e) z += std::exp((double)score[(size_t)t * E + e] - mx);
            for (int e = 0; e < E; ++e)
                gate[(size_t)t * E + e] = static_cast<float>(std::exp((double)score[(size_t)t * E + e] - mx) / z);
        }
    }
    std::vector<int32_t> topk((size_t)T * std::max(k, 1)), slot_of((size_t)T * E),
        slot_token((size_t)E * capacity), counts(E);
    rc = etr_ref_select(T, E, k, capacity, mode, score.data(), topk.data(), slot_of.data(), slot_token.data(),
                        counts.data());
    if (rc) return rc;

    std::vector<int32_t> all;
    if (n_tokens < 0) {
        all.resize(T);
        std::iota(all.begin(), all.end(), 0);
        tokens = all.data();
        n_tokens = T;
    }
    // one FFN row per kept (token, expert) pair of the requested tokens
    std::vector<int32_t> pair_expert, pair_token_pos;
    for (int i = 0; i < n_tokens; ++i) {
        int t = tokens[i];
        if (t < 0 || t >= T) return 2;
        for (int e = 0; e < E; ++e)
            if (slot_of[(size_t)t * E + e] >= 0) { pair_expert.push_back(e); pair_token_pos.push_back(i); }
    }
    const size_t es = elem_size(dtype);
    const int n_pairs = (int)pair_expert.size();
    std::vector<char> rows((size_t)n_pairs * d * es);
    for (int r = 0; r < n_pairs; ++r)
        std::memcpy(rows.data() + (size_t)r * d * es,
                    static_cast<const char*>(x) + (size_t)tokens[pair_token_pos[r]] * d * es, (size_t)d * es);
    std::vector<double> y((size_t)n_pairs * d);
    rc = etr_ref_ffn_rows(n_pairs, d, H, dtype, rows.data(), pair_expert.data(), w_gate, w_up, w_down, y.data());
    if (rc) return rc;
    std::vector<double> acc((size_t)n_tokens * d, 0.0);
    for (int r = 0; r < n_pairs; ++r) {          // pairs are listed token-major, experts ascending
        int i = pair_token_pos[r];
        double gt = gate[(size_t)tokens[i] * E + pair_expert[r]] /
                    kept_gate_sum(gate.data() + (size_t)tokens[i] * E, slot_of.data() + (size_t)tokens[i] * E, E, gate_norm);
        for (int j = 0; j < d; ++j) acc[(size_t)i * d + j] += gt * y[(size_t)r * d + j];
    }
    for (size_t i = 0; i < (size_t)n_tokens * d; ++i) store_elem(out, dtype, i, acc[i]);

    if (score_out) std::copy(score.begin(), score.end(), score_out);
    if (gate_out) std::copy(gate.begin(), gate.end(), gate_out);
    if (topk_out && mode != MODE_ECR) std::copy(topk.begin(), topk.begin() + (size_t)T * k, topk_out);
    if (slot_of_out) std::copy(slot_of.begin(), slot_of.end(), slot_of_out);
    if (slot_token_out) std::copy(slot_token.begin(), slot_token.end(), slot_token_out);
    if (counts_out) std::copy(counts.begin(), counts.end(), counts_out);
    return 0;
}

// ---------------------------------------------------------------------------
// Routing statistics that the losses of Sec. Locality Loss are built from:
//   load[e]      = counts[e] / sum(counts): the current distribution D_c of kept
//                  (token, expert) assignments over the experts (all 0 if nothing is kept)
//   mean_gate[e] = (1/T) sum_t gate[t][e]
//   kl           = KL(D_c || D_l) = sum_e D_c(e) ln(D_c(e) / D_l(e)) for a caller-given
//                  localized distribution D_l (`target`); terms with D_c(e) = 0 are 0,
//                  D_l(e) = 0 < D_c(e) gives +inf.  L_loc = mu * kl is left to the caller.
//   n_unrouted   = tokens kept by no expert
// ---------------------------------------------------------------------------
int etr_ref_route_stats(int T, int E, const float* gate, const int32_t* slot_of, const int32_t* counts,
                        const float* target, double* load, double* mean_gate, double* kl, int32_t* n_unrouted) {
    long long total = 0;
    for (int e = 0; e < E; ++e) total += counts[e];
    double k = 0;
    for (int e = 0; e < E; ++e) {
        load[e] = total > 0 ? double(counts[e]) / double(total) : 0.0;
        double s = 0;
        for (int t = 0; t < T; ++t) s += double(gate[(size_t)t * E + e]);
        mean_gate[e] = s / T;
        if (load[e] > 0) k += (target[e] > 0) ? load[e] * std::log(load[e] / double(target[e])) : INFINITY;
    }
    *kl = k;
    int32_t un = 0;
    for (int t = 0; t < T; ++t) {
        bool any = false;
        for (int e = 0; e < E; ++e) any = any || slot_of[(size_t)t * E + e] >= 0;
        un += any ? 0 : 1;
    }
    *n_unrouted = un;
    return 0;
}

// ---------------------------------------------------------------------------
// Lower bound of the expert capacity from the Remark of Sec. Dynamic Lower Bound Module:
//   C_min = (1/n) exp{ d * dmax^2 / (2 - dmax^2) },  dmax = largest affinity in the batch,
// returned as an integer capacity: ceil(C_min) clamped into [1, T].  The exponent is
// evaluated in double from the fp32 maximum; it is compared in the log domain so that
// huge exponents (real d) do not overflow.
// ---------------------------------------------------------------------------
int etr_ref_capacity_lower_bound(int T, int E, int d, const float* score, float* dmax_out, int32_t* capacity_out) {
    if (T < 1 || E < 1) return 2;
    float mx = score[0];
    for (size_t i = 0; i < (size_t)T * E; ++i) mx = std::max(mx, score[i]);
    const double dm = double(mx);
    const double log_c = double(d) * dm * dm / (2.0 - dm * dm) - std::log(double(E));
    int32_t c;
    if (log_c >= std::log(double(T))) c = T;
    else c = (int32_t)std::ceil(std::exp(log_c));
    if (c < 1) c = 1;
    if (c > T) c = T;
    *dmax_out = mx;
    *capacity_out = c;
    return 0;
}

// ---------------------------------------------------------------------------
// Backward of the layer: the chain rule applied to Eqs. 1-6 with the routing tables held fixed
// (which tokens an expert keeps is a piecewise-constant function of the input; the gate vectors
// of Eq. 3 are constants of the method, so there is no gradient for them).  With
//   out[t] = sum_{e kept t} gate[t][e] * y_te,   y_te = Wd_e h_te,   h_te = SiLU(a_te) .* b_te,
//   a_te = Wg_e x_t,  b_te = Wu_e x_t,  gate[t][.] = softmax(score[t][.]),  score = Eq. 4,
// and an upstream gradient dout[T][d]:
//   dgate[t][e]  = <dout[t], y_te>            (0 for pairs that are not kept)
//   dscore[t][e] = gate[t][e] * (dgate[t][e] - sum_e' dgate[t][e'] gate[t][e'])
//   dy_te = gate[t][e] dout[t];  dh = Wd^T dy;  da = dh .* b .* SiLU'(a);  db = dh .* SiLU(a)
//   dWd_e += dy h^T;  dWg_e += da x^T;  dWu_e += db x^T
//   dx[t] = sum_e (Wg_e^T da + Wu_e^T db) + sum_e dscore[t][e] * d score[t][e] / d x[t]
// Everything is evaluated in double from the stored inputs; nothing is rounded.
// The work is split so that any part can be evaluated on its own for sampled checks at sizes
// where the whole gradient is out of reach: per token (dx, dgate, dscore) and per hidden unit
// (row j of dWg_e and dWu_e, column j of dWd_e).
// ---------------------------------------------------------------------------
namespace {

struct TokenRoute {          // routing quantities of one token, all in double
    std::vector<double> g, score, gate;
    double xx = 0, gg = 0;
};

void route_token_double(int t, int d, int E, int D, int dtype, int cos_mode, const void* x, const float* w_emb,
                        const std::vector<double>& wnorm, TokenRoute& r) {
    const int P = d / D;
    r.g.assign(P, 0.0); r.score.assign(E, 0.0); r.gate.assign(E, 0.0);
    r.xx = 0; r.gg = 0;
    for (int p = 0; p < P; ++p) {
        double s = 0;
        for (int j = 0; j < D; ++j) {
            double v = load_elem(x, dtype, (size_t)t * d + (size_t)p * D + j);
            s += v; r.xx += v * v;
        }
        r.g[p] = s / D;
        r.gg += r.g[p] * r.g[p];
    }
    double mx = -INFINITY;
    for (int e = 0; e < E; ++e) {
        double dot = 0;
        for (int p = 0; p < P; ++p) dot += r.g[p] * double(w_emb[e * (size_t)P + p]);
        double den = (cos_mode == COS_FULL ? std::sqrt(r.xx) : std::sqrt(r.gg)) * wnorm[e];
        double num = (cos_mode == COS_FULL) ? std::sqrt((double)D) * dot : dot;
        r.score[e] = den > 0 ? num / den : 0.0;
        mx = std::max(mx, r.score[e]);
    }
    double z = 0;
    for (int e = 0; e < E; ++e) z += std::exp(r.score[e] - mx);
    for (int e = 0; e < E; ++e) r.gate[e] = std::exp(r.score[e] - mx) / z;
}

std::vector<double> embedding_norms(int E, int P, const float* w_emb) {
    std::vector<double> wnorm(E);
    for (int e = 0; e < E; ++e) {
        double s = 0;
        for (int p = 0; p < P; ++p) s += double(w_emb[e * (size_t)P + p]) * double(w_emb[e * (size_t)P + p]);
        wnorm[e] = std::sqrt(s);
    }
    return wnorm;
}

inline double sigmoid(double a) { return 1.0 / (1.0 + std::exp(-a)); }

}  // namespace

// Per-token part of the backward: for each listed token, dx (d values), dgate and dscore (E values each).
int etr_ref_backward_tokens(int T, int d, int E, int D, int H, int dtype, int cos_mode,
                            const void* x, const float* w_emb, const void* w_gate, const void* w_up,
                            const void* w_down, const int32_t* slot_of, const void* dout,
                            const int32_t* tokens, int n_tokens, double* dx, double* dgate, double* dscore,
                            int gate_norm) {
    if (d <= 0 || E <= 0 || D <= 0 || d % D != 0 || H <= 0) return 2;
    const int P = d / D;
    const std::vector<double> wnorm = embedding_norms(E, P, w_emb);
    int bad = 0;
#pragma omp parallel for schedule(dynamic)
    for (int i = 0; i < n_tokens; ++i) {
        const int t = tokens[i];
        if (t < 0 || t >= T) { bad = 1; continue; }
        TokenRoute r;
        route_token_double(t, d, E, D, dtype, cos_mode, x, w_emb, wnorm, r);
        std::vector<double> xt(d), go(d), acc(d, 0.0), a(H), b(H), h(H), dh(H), dg(E, 0.0);
        // effective weights: the softmax gate, or (variant) renormalised over the experts that kept the token
        const double norm = kept_gate_sum(r.gate.data(), slot_of + (size_t)t * E, E, gate_norm);
        for (int j = 0; j < d; ++j) {
            xt[j] = load_elem(x, dtype, (size_t)t * d + j);
            go[j] = load_elem(dout, dtype, (size_t)t * d + j);
        }
        for (int e = 0; e < E; ++e) {
            if (slot_of[(size_t)t * E + e] < 0) continue;
            for (int u = 0; u < H; ++u) {
                double sa = 0, sb = 0;
                const size_t base = ((size_t)e * H + u) * d;
                for (int j = 0; j < d; ++j) {
                    sa += load_elem(w_gate, dtype, base + j) * xt[j];
                    sb += load_elem(w_up, dtype, base + j) * xt[j];
                }
                a[u] = sa; b[u] = sb; h[u] = sa * sigmoid(sa) * sb; dh[u] = 0;
            }
            double dgte = 0;
            for (int j = 0; j < d; ++j) {
                const size_t base = ((size_t)e * d + j) * H;
                double y = 0;
                for (int u = 0; u < H; ++u) {
                    const double w = load_elem(w_down, dtype, base + u);
                    y += w * h[u];
                    dh[u] += w * (r.gate[e] / norm) * go[j];
                }
                dgte += go[j] * y;
            }
            dg[e] = dgte;
            for (int u = 0; u < H; ++u) {
                const double sg = sigmoid(a[u]);
                const double da = dh[u] * b[u] * (sg * (1.0 + a[u] * (1.0 - sg)));   // d/da [a sigma(a)]
                const double db = dh[u] * a[u] * sg;
                const size_t base = ((size_t)e * H + u) * d;
                for (int j = 0; j < d; ++j)
                    acc[j] += load_elem(w_gate, dtype, base + j) * da + load_elem(w_up, dtype, base + j) * db;
            }
        }
        // dg holds d out / d (effective weight); with renormalised weights g'_e = g_e / S, S = sum over the
        // kept experts: d / d g_e = (dg'_e - sum_kept dg'_i g'_i) / S for kept e, 0 otherwise
        if (gate_norm) {
            double m2 = 0;
            for (int e = 0; e < E; ++e) if (slot_of[(size_t)t * E + e] >= 0) m2 += dg[e] * r.gate[e] / norm;
            for (int e = 0; e < E; ++e) dg[e] = slot_of[(size_t)t * E + e] >= 0 ? (dg[e] - m2) / norm : 0.0;
        }
        // softmax backward, then the affinity's own derivative
        double mix = 0;
        for (int e = 0; e < E; ++e) mix += dg[e] * r.gate[e];
        std::vector<double> ds(E);
        for (int e = 0; e < E; ++e) ds[e] = r.gate[e] * (dg[e] - mix);
        const double nx = std::sqrt(r.xx), ng = std::sqrt(r.gg);
        for (int e = 0; e < E; ++e) {
            if (ds[e] == 0.0 || wnorm[e] == 0.0) continue;
            if (cos_mode == COS_FULL) {
                if (nx == 0.0) continue;
                // score = sqrt(D) <g,w> / (|x| |w|),  g_p = mean of group p
                for (int j = 0; j < d; ++j) {
                    const double w = double(w_emb[e * (size_t)P + j / D]);
                    acc[j] += ds[e] * (std::sqrt((double)D) * w / (D * nx * wnorm[e]) - r.score[e] * xt[j] / r.xx);
                }
            } else {
                if (ng == 0.0) continue;
                // score = <g,w> / (|g| |w|); d g_p / d x_j = 1/D inside the group
                for (int j = 0; j < d; ++j) {
                    const int p = j / D;
                    const double w = double(w_emb[e * (size_t)P + p]);
                    acc[j] += ds[e] * (w / (ng * wnorm[e]) - r.score[e] * r.g[p] / r.gg) / D;
                }
            }
        }
        for (int j = 0; j < d; ++j) dx[(size_t)i * d + j] = acc[j];
        if (dgate) for (int e = 0; e < E; ++e) dgate[(size_t)i * E + e] = dg[e];
        if (dscore) for (int e = 0; e < E; ++e) dscore[(size_t)i * E + e] = ds[e];
    }
    return bad ? 2 : 0;
}

// Per-hidden-unit part of the backward: for unit u = unit_index[i] of expert e = unit_expert[i],
// row u of dWg_e and of dWu_e (d values each) and column u of dWd_e (d values).
int etr_ref_backward_hidden_units(int T, int d, int E, int D, int H, int dtype, int cos_mode,
                                  const void* x, const float* w_emb, const void* w_gate, const void* w_up,
                                  const void* w_down, const int32_t* slot_of, const void* dout,
                                  const int32_t* unit_expert, const int32_t* unit_index, int n_units,
                                  double* dwg_rows, double* dwu_rows, double* dwd_cols, int gate_norm) {
    if (d <= 0 || E <= 0 || D <= 0 || d % D != 0 || H <= 0) return 2;
    const int P = d / D;
    const std::vector<double> wnorm = embedding_norms(E, P, w_emb);
    // gates of every token once (double)
    std::vector<double> gate((size_t)T * E);
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        TokenRoute r;
        route_token_double(t, d, E, D, dtype, cos_mode, x, w_emb, wnorm, r);
        const double norm = kept_gate_sum(r.gate.data(), slot_of + (size_t)t * E, E, gate_norm);
        for (int e = 0; e < E; ++e) gate[(size_t)t * E + e] = r.gate[e] / norm;      // effective weights
    }
    int bad = 0;
#pragma omp parallel for schedule(dynamic)
    for (int i = 0; i < n_units; ++i) {
        const int e = unit_expert[i], u = unit_index[i];
        if (e < 0 || e >= E || u < 0 || u >= H) { bad = 1; continue; }
        std::vector<double> gw(d, 0.0), uw(d, 0.0), dw(d, 0.0);
        const size_t wrow = ((size_t)e * H + u) * d;
        for (int t = 0; t < T; ++t) {
            if (slot_of[(size_t)t * E + e] < 0) continue;
            double a = 0, b = 0, dh = 0;
            for (int j = 0; j < d; ++j) {
                const double xv = load_elem(x, dtype, (size_t)t * d + j);
                a += load_elem(w_gate, dtype, wrow + j) * xv;
                b += load_elem(w_up, dtype, wrow + j) * xv;
            }
            const double gt = gate[(size_t)t * E + e];
            for (int j = 0; j < d; ++j)
                dh += load_elem(w_down, dtype, ((size_t)e * d + j) * H + u) * gt * load_elem(dout, dtype, (size_t)t * d + j);
            const double sg = sigmoid(a);
            const double h = a * sg * b;
            const double da = dh * b * (sg * (1.0 + a * (1.0 - sg)));
            const double db = dh * a * sg;
            for (int j = 0; j < d; ++j) {
                const double xv = load_elem(x, dtype, (size_t)t * d + j);
                gw[j] += da * xv;
                uw[j] += db * xv;
                dw[j] += gt * load_elem(dout, dtype, (size_t)t * d + j) * h;
            }
        }
        for (int j = 0; j < d; ++j) {
            dwg_rows[(size_t)i * d + j] = gw[j];
            dwu_rows[(size_t)i * d + j] = uw[j];
            dwd_cols[(size_t)i * d + j] = dw[j];
        }
    }
    return bad ? 2 : 0;
}

// helpers exposed for the tests
uint16_t etr_ref_double_to_bf16(double v) { return double_to_bf16(v); }
int etr_ref_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
// Number of OpenMP threads the loops above run on from now on (timing on one core; no arithmetic changes).
void etr_ref_set_num_threads(int n) {
#ifdef _OPENMP
    omp_set_num_threads(n < 1 ? 1 : n);
#else
    (void)n;
#endif
}

}  // extern "C"
