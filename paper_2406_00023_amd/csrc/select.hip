// Bidirectional selection under the capacity bound (Sec. Routing Strategy, Eqs. 5-6; keep
// rules of the pure phases from the Proof of the Theorem, parts 1 and 2) and the
// prefix-sum permutation tables.
//
// Three launches (four for long columns), no global atomics, integer counting only, so the result is
// bit-reproducible:
//   1. token_choice_kernel   one lane per (token, expert): k rounds of arg-max inside a lane group (DPP folds)
//                            give the token's Top-k list (Eq. 5); writes the candidate mask and, through an LDS
//                            tile, a column-major copy of the selection keys
//   2. expert_choice_kernel  one 1024-thread workgroup per expert, keys in registers as whole rows of the
//                            column: the key tau_e of the C-th best candidate (Eq. 6) by a radix search over the
//                            bits in which the candidates' order-preserving keys differ at all (11 bits per
//                            pass, one LDS histogram per pass, the digit picked by every wave for itself), then
//                            the (key > tau, key == tau) counts of each chunk are scanned into exclusive prefixes
//                            (long columns: the first digit is counted beforehand by key_histogram_kernel,
//                            up to 16 workgroups per expert)
//   3. slot_kernel           one lane per (expert, token): the position inside the chunk comes from a
//                            ballot, so slot_of / slot_token are written without any serial walk; the slots of
//                            64 tokens leave as whole rows of slot_of
// All three phases are one algorithm: in TCR every candidate has the same key, so
// "the C best, lowest token first among equals" is "the first C in token order".
#include <mutex>

#include "etr_internal.h"

// Scratch of the allocation-free entry point (etr_select_noalloc): device memory that belongs to the library, one
// copy per GPU the library runs on, held until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress; kernels and copies are given the address that call returns.
static __device__ __align__(256) unsigned char scratch[etr::kStaticSelectBytes];

namespace etr {
namespace {

// fp32 -> uint32 that preserves order; 0 is reserved for "not a candidate".
__device__ __forceinline__ uint32_t order_key(float s) {
    uint32_t u = __float_as_uint(s);
    if (u == 0x80000000u) u = 0u;                       // -0.0 ties with +0.0
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Key under which expert e ranks token t ("the C best keys, lowest token first among equals"):
//   TCR        1 for every chooser (position priority)
//   ECR/BIDIR  the affinity, for all tokens / for the choosers
//   TCR_RANK   k - (position of e in the token's list): first choices before second choices (variant)
//   STRICT     the affinity for ALL tokens; the chooser set is intersected afterwards (variant)
__device__ __forceinline__ uint32_t selection_key(float s, bool cand, int mode, int k = 0, int rank = 0) {
    if (mode == ETR_MODE_BIDIR_STRICT) return order_key(s);
    if (!cand) return 0u;
    if (mode == ETR_MODE_TCR) return 1u;
    if (mode == ETR_MODE_TCR_RANK) return static_cast<uint32_t>(k - rank);
    return order_key(s);
}

// ---------------------------------------------------------------------------------------
// 1. token choice
// ---------------------------------------------------------------------------------------
// Maximum (MAX) or minimum over aligned groups of G lanes, every lane of a group gets it: swaps inside quads, the
// mirror images of the half row and of the row (16 lanes) as data-parallel-primitive moves, then the row-pair and
// half-wave swaps.  Call with all lanes active.
template <bool MAX> __device__ __forceinline__ uint32_t pick(uint32_t a, uint32_t b) { return MAX ? max(a, b) : min(a, b); }
template <bool MAX, int CTRL>
__device__ __forceinline__ uint32_t dpp_fold(uint32_t v) {
    return pick<MAX>(v, static_cast<uint32_t>(__builtin_amdgcn_update_dpp(static_cast<int>(v), static_cast<int>(v), CTRL, 0xF, 0xF, false)));
}
template <int G, bool MAX>
__device__ __forceinline__ uint32_t lane_group_fold(uint32_t v) {
    if constexpr (G >= 2) v = dpp_fold<MAX, 0xB1>(v);        // quad_perm [1,0,3,2]
    if constexpr (G >= 4) v = dpp_fold<MAX, 0x4E>(v);        // quad_perm [2,3,0,1]
    if constexpr (G >= 8) v = dpp_fold<MAX, 0x141>(v);       // row_half_mirror
    if constexpr (G >= 16) v = dpp_fold<MAX, 0x140>(v);      // row_mirror
    if constexpr (G >= 32) {                                 // odd rows of one copy <-> even rows of the other
        const auto r = __builtin_amdgcn_permlane16_swap(v, v, false, false);
        v = pick<MAX>(r[0], r[1]);
    }
    if constexpr (G >= 64) {                                 // upper half of one copy <-> lower half of the other
        const auto r = __builtin_amdgcn_permlane32_swap(v, v, false, false);
        v = pick<MAX>(r[0], r[1]);
    }
    return v;
}

template <int G> constexpr int token_tile() { return G <= 4 ? 256 / G : 64; }       // tokens per workgroup
template <int G> constexpr int token_threads() { return G >= 16 ? 1024 : 256; }       // threads per workgroup

// G = lanes per token, a power of two >= E.  A workgroup takes token_tile<G>() tokens in one to four passes, all of
// whose affinities are requested before the first is used.  Each of the k rounds of Eq. 5 is a maximum over the
// token's lanes of the order-preserving affinities still in the contest, then a minimum over the experts that hold
// it (the lower expert wins among equals); the winner leaves the contest.  The keys of the tile go through LDS, so
// that each column of the column-major copy is written in whole stretches.
template <int G>
__global__ __launch_bounds__(token_threads<G>()) void token_choice_kernel(const float* __restrict__ score, int T, int E,
                                                                          int k, int mode, int32_t* __restrict__ topk,
                                                                          uint64_t* __restrict__ cmask,
                                                                          uint32_t* __restrict__ keyT, int Tpad) {
    constexpr int TT = token_tile<G>(), NT = token_threads<G>();
    constexpr int PASSES = TT * G / NT;
    static_assert(PASSES >= 1 && PASSES * NT == TT * G, "whole passes");
    __shared__ uint32_t tile[G][TT + 1];
    const int t_base = blockIdx.x * TT;
    const int e = threadIdx.x % G, tl0 = threadIdx.x / G;      // (NT is a multiple of G: the same expert in every pass)
    float vals[PASSES];
#pragma unroll
    for (int pass = 0; pass < PASSES; ++pass) {
        const int t = t_base + pass * (NT / G) + tl0;
        vals[pass] = (t < T && e < E) ? score[static_cast<size_t>(t) * E + e] : 0.f;
    }
#pragma unroll
    for (int pass = 0; pass < PASSES; ++pass) {
        const int tl = pass * (NT / G) + tl0;
        const int t = t_base + tl;
        const bool valid = t < T && e < E;
        const float val = vals[pass];
        uint64_t mask = 0;
        int my_rank = 0, choice = 0;
        if (mode != ETR_MODE_ECR) {
            // 0 = out of the contest (no such expert, or already chosen)
            uint32_t mine = valid ? max(order_key(val), 1u) : 0u;
            for (int r = 0; r < k; ++r) {
                const uint32_t best = lane_group_fold<G, true>(mine);
                const int bi = static_cast<int>(lane_group_fold<G, false>(mine == best && best != 0u ? static_cast<uint32_t>(e) : 255u));
                if (e == bi) { mine = 0u; my_rank = r; }
                if (e == r) choice = bi;
            }
            // the token's candidate set: the lanes of its group that have left the contest (one ballot after the
            // rounds, not a shifted bit per round)
            const uint64_t chosen = __ballot(valid && mine == 0u);
            mask = (chosen >> (threadIdx.x & (kWave - 1) & ~(G - 1))) & (G >= 64 ? ~0ull : ((1ull << G) - 1ull));
            if (topk && e < k && t < T) topk[static_cast<size_t>(t) * k + e] = choice;
        } else {
            mask = E >= 64 ? ~0ull : ((1ull << E) - 1ull);
        }
        tile[e][tl] = valid ? selection_key(val, (mask >> e) & 1ull, mode, k, my_rank) : 0u;
        if (e == 0 && t < T) cmask[t] = mask;
    }
    __syncthreads();
    for (int i = threadIdx.x; i < G * TT; i += NT) {
        const int ee = i / TT, tl = i % TT;
        const int t = t_base + tl;
        if (ee < E && t < T) keyT[static_cast<size_t>(ee) * Tpad + t] = tile[ee][tl];
    }
}

// ---------------------------------------------------------------------------------------
// 2a. first radix digit, spread over the chip (long columns only): workgroup (slice, expert) counts the top
// kRadixBits bits of the candidate keys of its slice of the column; expert_choice_kernel<IPT, true> adds the
// slices up instead of walking all of its keys once more (its per-key work is what bounds it: one CU per expert).
// Integer counts, so the result does not depend on the split.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void key_histogram_kernel(const uint32_t* __restrict__ keyT, int Tpad, int T,
                                                            int slice, uint32_t* __restrict__ hist1) {
    constexpr int NBINS = 1 << 11;
    __shared__ uint32_t h[NBINS];
    const int b = blockIdx.x, e = blockIdx.y, nb = gridDim.x, tid = threadIdx.x;
    for (int i = tid; i < NBINS; i += 256) h[i] = 0u;
    __syncthreads();
    const uint32_t* col = keyT + static_cast<size_t>(e) * Tpad;
    const int t_end = min(T, (b + 1) * slice);
    for (int t = b * slice + tid * 4; t < t_end; t += 1024) {       // slice and Tpad are multiples of 4
        const uint4 v = *reinterpret_cast<const uint4*>(col + t);
        const uint32_t k4[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (t + j < T && k4[j] != 0u) atomicAdd(&h[k4[j] >> (32 - 11)], 1u);
    }
    __syncthreads();
    uint32_t* out = hist1 + (static_cast<size_t>(e) * nb + b) * NBINS;
    for (int i = tid; i < NBINS; i += 256) out[i] = h[i];
}

// ---------------------------------------------------------------------------------------
// 2. expert choice: threshold search + chunk prefixes
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ int wave_sum_i(int v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, kWave);
    return v;
}

// Inclusive prefix sum over the 64 lanes of a wave, lane 0 first, by data-parallel-primitive moves: shifts by
// 1, 2, 4, 8 inside each row of 16 lanes (a lane whose source lies outside its row adds nothing), then lane 15 of
// row 0 / 2 is added to all of row 1 / 3 and lane 31 to all of rows 2 and 3.  Call with all lanes active.
__device__ __forceinline__ int wave_scan_incl(int v) {
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xF, 0xF, false);   // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xF, 0xF, false);   // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xF, 0xF, false);   // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xF, 0xF, false);   // row_shr:8
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xA, 0xF, false);   // row_bcast:15 -> rows 1, 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xC, 0xF, false);   // row_bcast:31 -> rows 2, 3
    return v;
}

// Sum over aligned groups of Q lanes (Q = 1, 2, 4, 8, 16), every lane of a group gets the group's total:
// swaps inside quads, then the mirror images of the half row and of the row.  Call with all lanes active.
template <int Q>
__device__ __forceinline__ int lane_group_sum(int v) {
    if constexpr (Q >= 2) v += __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xF, 0xF, false);    // quad_perm [1,0,3,2]
    if constexpr (Q >= 4) v += __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xF, 0xF, false);    // quad_perm [2,3,0,1]
    if constexpr (Q >= 8) v += __builtin_amdgcn_update_dpp(0, v, 0x141, 0xF, 0xF, false);   // row_half_mirror
    if constexpr (Q >= 16) v += __builtin_amdgcn_update_dpp(0, v, 0x140, 0xF, 0xF, false);  // row_mirror
    return v;
}

// Block-wide sums of three counters (all threads get the totals).
__device__ __forceinline__ void block_sum3(int& a, int& b, int& c, int (*red)[3]) {
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    a = wave_sum_i(a); b = wave_sum_i(b); c = wave_sum_i(c);
    __syncthreads();                                   // previous readers of red are done
    if (lane == 0) { red[wave][0] = a; red[wave][1] = b; red[wave][2] = c; }
    __syncthreads();
    a = b = c = 0;
#pragma unroll
    for (int w = 0; w < kSelThreads / kWave; ++w) { a += red[w][0]; b += red[w][1]; c += red[w][2]; }
}

constexpr int kRadixBits = 11;           // digit width of the threshold search
constexpr int kBins = 1 << kRadixBits;   // 2048 bins: 32 per lane of a wave
constexpr int kMaxDigits = 3;            // 32 key bits in digits of at most 11
constexpr int kMaxSlices = 16;           // workgroups per expert that count the first digit of a long column

// A wave's view of one histogram of kBins counters in LDS (narrower digits leave the upper bins zero), walked
// from the largest digit down: lane g owns the 32 bins [kBins - 32 (g + 1), kBins - 32 g).  Every wave of the
// workgroup takes the same view by itself, so no barrier is needed between the histogram and its use.
struct DigitView {
    int own;       // candidates in this lane's 32 bins
    int upto;      // candidates in the bins of lanes 0..g (inclusive scan)
    int total;     // candidates in all bins
};

__device__ __forceinline__ DigitView digit_view(const uint32_t* hist) {
    const int lane = threadIdx.x & (kWave - 1);
    const uint4* q4 = reinterpret_cast<const uint4*>(hist) + 8 * (kWave - 1 - lane);
    int s = 0;
#pragma unroll
    for (int q = 0; q < 8; ++q) {                       // the lane's eight quads, rotated by the lane: no bank conflicts
        const uint4 v = q4[(q + lane) & 7];
        s += static_cast<int>(v.x + v.y + v.z + v.w);
    }
    DigitView d;
    d.own = s;
    d.upto = wave_scan_incl(s);
    d.total = __builtin_amdgcn_readlane(d.upto, kWave - 1);
    return d;
}

// The digit that holds the need-th largest candidate (1 <= need <= total) and the number of candidates with a
// larger digit.
__device__ __forceinline__ void digit_pick(const uint32_t* hist, const DigitView& d, int need, int& digit, int& above) {
    const int lane = threadIdx.x & (kWave - 1);
    const uint64_t m1 = __ballot(d.upto >= need);
    const int g = m1 ? __builtin_ctzll(m1) : kWave - 1;                       // the lane whose bins hold it
    const int before = __builtin_amdgcn_readlane(d.upto - d.own, g);
    const int h = lane < 32 ? static_cast<int>(hist[kBins - 1 - 32 * g - lane]) : 0;   // its bins, largest first
    const int upto = wave_scan_incl(h);
    const uint64_t m2 = __ballot(before + upto >= need);
    const int j = m2 ? __builtin_ctzll(m2) : 31;
    digit = kBins - 1 - 32 * g - j;
    above = before + __builtin_amdgcn_readlane(upto - h, j);
}

// One 1024-thread workgroup per expert.
// IPT > 0 (4, 8, 16, 32, 64; equal to ipt): the column's keys live in registers.  Wave w holds the 64 chunks
//   [64 w, 64 w + 64) of IPT tokens each, as IPT/4 rows of 64 pieces of four keys: row r, lane l is piece
//   64 r + l of the wave's stretch of the column, so every load instruction reads 1 KiB in one piece.  The search
//   does not care which lane holds which key; only the last step, the per-chunk counts, puts the pieces of a
//   chunk (IPT/4 neighbouring lanes of one row) together.
// IPT == 0: keys streamed from memory, thread t owns chunk t (columns longer than 64 keys per thread).
// PRE: the histogram of the first digit (the top kRadixBits bits) comes from key_histogram_kernel (hist1, n_slices).
// ADAPT: with the adaptive token count (an instantiation of its own: its double-precision sums over the keys in
//   registers would otherwise cost the plain search of the long columns a hundred spilled registers).
template <int IPT, bool PRE = false, bool ADAPT = false>
__global__ __launch_bounds__(kSelThreads) void expert_choice_kernel(const uint32_t* __restrict__ keyT, int Tpad, int T,
                                                                    int ipt, int capacity_host, int mode,
                                                                    const int32_t* __restrict__ capacity_dev,
                                                                    long long sum_need,
                                                                    uint32_t* __restrict__ tau_out,
                                                                    int32_t* __restrict__ need_eq_out,
                                                                    int32_t* __restrict__ pre_gt,
                                                                    int32_t* __restrict__ pre_eq,
                                                                    int32_t* __restrict__ counts,
                                                                    const uint32_t* __restrict__ hist1, int n_slices) {
    constexpr int Q = IPT > 0 ? IPT / 4 : 1;            // rows of a wave = pieces of a chunk
    static_assert(IPT == 0 || (IPT >= 4 && IPT <= 64 && (IPT & (IPT - 1)) == 0), "chunk lengths held in registers");
    __shared__ int red[kSelThreads / kWave][3];
    __shared__ int wave_tot[kSelThreads / kWave][2];
    __shared__ uint32_t range[kSelThreads / kWave][2];
    __shared__ __attribute__((aligned(16))) uint32_t hist[kMaxDigits][kBins];
    __shared__ int chunk_cnt[kSelThreads / kWave][kWave];
    const int e = blockIdx.x, tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wave = tid / kWave;
    // a capacity computed on the device (e.g. the lower bound of the Remark) may tighten the host one
    const int capacity = capacity_dev ? min(capacity_host, max(1, *capacity_dev)) : capacity_host;
    const uint32_t* col = keyT + static_cast<size_t>(e) * Tpad;

    uint32_t keys[IPT > 0 ? IPT : 1];
    if constexpr (IPT > 0) {
        const int seg = wave * kWave * IPT;             // first token of the wave's stretch
#pragma unroll
        for (int r = 0; r < Q; ++r) {
            const int idx = seg + (r * kWave + lane) * 4;
            uint4 v = make_uint4(0u, 0u, 0u, 0u);
            if (idx < Tpad) v = *reinterpret_cast<const uint4*>(col + idx);     // Tpad is a multiple of 4
            keys[4 * r + 0] = idx + 0 < T ? v.x : 0u;
            keys[4 * r + 1] = idx + 1 < T ? v.y : 0u;
            keys[4 * r + 2] = idx + 2 < T ? v.z : 0u;
            keys[4 * r + 3] = idx + 3 < T ? v.w : 0u;
        }
    }
    // The histograms of all digits start at zero; the first barrier below lies between this and their first use.
    if constexpr (PRE) {
        // first digit: the slices' counts of this thread's two bins, added up (integer sums, any order)
        static_assert(kSelThreads * 2 == kBins, "two bins of the first digit per thread");
        const uint32_t* hp = hist1 + static_cast<size_t>(e) * n_slices * kBins + 2 * tid;
        uint32_t s0 = 0u, s1 = 0u;
#pragma unroll
        for (int b = 0; b < kMaxSlices; ++b) {          // all loads in flight at once; slices past the last count as zero
            const uint2 v = *reinterpret_cast<const uint2*>(hp + static_cast<size_t>(b < n_slices ? b : 0) * kBins);
            const uint32_t on = b < n_slices ? 0xFFFFFFFFu : 0u;
            s0 += v.x & on; s1 += v.y & on;
        }
        hist[0][2 * tid] = s0; hist[0][2 * tid + 1] = s1;
    } else {
        hist[0][2 * tid] = 0u; hist[0][2 * tid + 1] = 0u;
    }
#pragma unroll
    for (int p = 1; p < kMaxDigits; ++p) { hist[p][2 * tid] = 0u; hist[p][2 * tid + 1] = 0u; }

    int ncand;
    DigitView first{0, 0, 0};                           // PRE: the view of the first digit
    if constexpr (PRE) {
        __syncthreads();
        first = digit_view(hist[0]);
        ncand = first.total;
    } else {
        int d1 = 0, d2 = 0;
        ncand = 0;
        if constexpr (IPT > 0) {
#pragma unroll
            for (int j = 0; j < IPT; ++j) ncand += keys[j] != 0u;
        } else {
            for (int idx = tid; idx < T; idx += kSelThreads) ncand += col[idx] != 0u;
        }
        block_sum3(ncand, d1, d2, red);
    }
    int n_keep = ncand < capacity ? ncand : capacity;

    // Adaptive token count (Sec. Routing Strategy: "l is determined by a threshold of the sum of
    // affinity scores"): walking the candidates from the highest affinity down, stop at the first
    // prefix whose affinity sum reaches the threshold.  Affinities are summed as fixed-point
    // integers round(clamp(s,-1,1) * 2^30), so the sum of "all candidates with key >= theta" is
    // exact and order-free, and the prefix length follows from a bisection over theta.
    if constexpr (ADAPT) if (sum_need > 0 && (mode == ETR_MODE_ECR || mode == ETR_MODE_BIDIR) && n_keep > 0) {
        __shared__ long long red_sum[kSelThreads / kWave];
        __shared__ int red_cnt[kSelThreads / kWave];
        // sum and count over the candidates with key >= thr (thr >= key(+0): positive affinities only)
        auto sum_ge = [&](uint32_t thr, long long& sum, int& cnt) {
            sum = 0; cnt = 0;
            auto add = [&](uint32_t key) {
                if (key >= thr) {
                    const float sc = __uint_as_float(key & 0x7FFFFFFFu);
                    sum += llrint(static_cast<double>(fminf(sc, 1.0f)) * 1073741824.0);
                    ++cnt;
                }
            };
            if constexpr (IPT > 0) {
#pragma unroll
                for (int j = 0; j < IPT; ++j) add(keys[j]);
            } else {
                for (int idx = tid; idx < T; idx += kSelThreads) add(col[idx]);
            }
#pragma unroll
            for (int m = 32; m >= 1; m >>= 1) { sum += __shfl_xor(sum, m, kWave); cnt += __shfl_xor(cnt, m, kWave); }
            __syncthreads();
            if (lane == 0) { red_sum[wave] = sum; red_cnt[wave] = cnt; }
            __syncthreads();
            sum = 0; cnt = 0;
#pragma unroll
            for (int w = 0; w < kSelThreads / kWave; ++w) { sum += red_sum[w]; cnt += red_cnt[w]; }
        };
        long long s_all; int c_all;
        sum_ge(0x80000000u, s_all, c_all);
        if (s_all >= sum_need) {                        // otherwise the positive affinities never get there: take all
            uint32_t th = 0x80000000u;                  // largest theta with sum_ge(theta) >= need
            for (int bit = 30; bit >= 0; --bit) {
                long long sv; int cv;
                sum_ge(th | (1u << bit), sv, cv);
                if (sv >= sum_need) th |= 1u << bit;
            }
            long long s_gt = 0; int n_gt = 0;
            if (th != 0xFFFFFFFFu) sum_ge(th + 1u, s_gt, n_gt);
            const long long q_th = llrint(static_cast<double>(fminf(__uint_as_float(th & 0x7FFFFFFFu), 1.0f)) * 1073741824.0);
            const long long j = q_th > 0 ? (sum_need - s_gt + q_th - 1) / q_th : 1;
            const long long ell = n_gt + j;
            if (ell < n_keep) n_keep = static_cast<int>(ell);
        }
    }

    uint32_t tau;
    if (n_keep == 0) {
        tau = 0xFFFFFFFFu;
    } else if (mode == ETR_MODE_TCR) {
        tau = 1u;                                       // every candidate carries key 1
    } else {
        // The n_keep-th largest key, by radix search from the top.  Only the bits in which the candidates differ
        // have to be resolved (affinities of one expert share sign, exponent and often leading mantissa bits), so
        // the search starts below the common prefix of the largest and the smallest candidate key.
        int shift = 32;                                              // low bits still to resolve
        uint32_t prefix = 0u;
        if constexpr (!PRE) {
            uint32_t kmax = 0u, kmin = 0xFFFFFFFFu;
            auto fold = [&](uint32_t key) { if (key != 0u) { kmax = max(kmax, key); kmin = min(kmin, key); } };
            if constexpr (IPT > 0) {
#pragma unroll
                for (int j = 0; j < IPT; ++j) fold(keys[j]);
            } else {
                for (int idx = tid; idx < T; idx += kSelThreads) fold(col[idx]);
            }
#pragma unroll
            for (int m = 32; m >= 1; m >>= 1) {
                kmax = max(kmax, static_cast<uint32_t>(__shfl_xor(static_cast<int>(kmax), m, kWave)));
                kmin = min(kmin, static_cast<uint32_t>(__shfl_xor(static_cast<int>(kmin), m, kWave)));
            }
            if (lane == 0) { range[wave][0] = kmax; range[wave][1] = kmin; }
            __syncthreads();
#pragma unroll
            for (int w = 0; w < kSelThreads / kWave; ++w) { kmax = max(kmax, range[w][0]); kmin = min(kmin, range[w][1]); }
            const uint32_t diff = kmax ^ kmin;
            shift = diff ? 32 - __builtin_clz(diff) : 0;             // low bits that vary among the candidates
            prefix = shift >= 32 ? 0u : (kmax >> shift) << shift;
        }
        int need = n_keep;
        for (int p = 0; p < kMaxDigits && shift > 0; ++p) {
            const int w = shift < kRadixBits ? shift : kRadixBits;
            const int top = shift;                                   // bits [31:top] are settled
            shift -= w;
            int digit, above;
            if (PRE && p == 0) {
                digit_pick(hist[0], first, need, digit, above);      // the first digit was counted by the slices
            } else {
                // candidates whose settled bits equal the prefix: lo <= key <= lo + span
                const uint32_t lo = prefix > 1u ? prefix : 1u;
                const uint32_t span = (top >= 32 ? 0xFFFFFFFFu : prefix + ((1u << top) - 1u)) - lo;
                const uint32_t dmask = (1u << w) - 1u;
                uint32_t* h = hist[p];
                auto bin = [&](uint32_t key) {
                    if (key - lo <= span) atomicAdd(&h[(key >> shift) & dmask], 1u);   // LDS; integer adds, so order-free
                };
                if constexpr (IPT > 0) {
#pragma unroll
                    for (int j = 0; j < IPT; ++j) bin(keys[j]);
                } else {
                    for (int idx = tid; idx < T; idx += kSelThreads) bin(col[idx]);
                }
                __syncthreads();
                const DigitView d = digit_view(h);
                digit_pick(h, d, need, digit, above);
            }
            prefix |= static_cast<uint32_t>(digit) << shift;
            need -= above;
        }
        tau = prefix;
    }

    // per-chunk counts of (key > tau, key == tau) in token order, then an exclusive block scan
    int gt = 0, eq = 0;
    if constexpr (IPT > 0) {
        const bool some = tau != 0u;                    // (a key of 0 is no candidate)
        int cnt[Q];
#pragma unroll
        for (int r = 0; r < Q; ++r) {
            int g = 0, q = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) { g += keys[4 * r + j] > tau; q += (keys[4 * r + j] == tau) && some; }
            cnt[r] = lane_group_sum<Q>(g | (q << 16));  // at most 64 each: the halves do not meet
        }
        if constexpr (Q > 1) {
            // row r, lanes [Q c', Q c' + Q) hold chunk r (64 / Q) + c' of the wave; lane c takes chunk c
            if ((lane & (Q - 1)) == 0) {
#pragma unroll
                for (int r = 0; r < Q; ++r) chunk_cnt[wave][r * (kWave / Q) + lane / Q] = cnt[r];
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            const int mine = chunk_cnt[wave][lane];
            gt = mine & 0xFFFF; eq = mine >> 16;
        } else {
            gt = cnt[0] & 0xFFFF; eq = cnt[0] >> 16;
        }
    } else {
        const int base = tid * ipt;
        for (int j = 0; j < ipt; ++j) {
            const int idx = base + j;
            uint32_t key = idx < T ? col[idx] : 0u;
            gt += key > tau; eq += (key == tau) && key != 0u;
        }
    }
    const int igt = wave_scan_incl(gt), ieq = wave_scan_incl(eq);
    if (lane == kWave - 1) { wave_tot[wave][0] = igt; wave_tot[wave][1] = ieq; }
    __syncthreads();
    int off_gt = 0, off_eq = 0, tot_gt = 0;
#pragma unroll
    for (int w = 0; w < kSelThreads / kWave; ++w) {
        if (w < wave) { off_gt += wave_tot[w][0]; off_eq += wave_tot[w][1]; }
        tot_gt += wave_tot[w][0];
    }
    pre_gt[e * kSelThreads + tid] = off_gt + igt - gt;
    pre_eq[e * kSelThreads + tid] = off_eq + ieq - eq;
    if (tid == 0) {
        tau_out[e] = tau;
        need_eq_out[e] = n_keep - tot_gt;
        counts[e] = n_keep;
    }
}

// ---------------------------------------------------------------------------------------
// 2b. strict intersection (variant): expert_choice_kernel has ranked ALL tokens; a pair survives
// only if the token also lists the expert.  One workgroup per expert, thread = chunk: count the
// survivors of the chunk, scan, and replace counts[e] by the number of survivors.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(kSelThreads) void strict_filter_kernel(const uint32_t* __restrict__ keyT, int Tpad, int T,
                                                                    int ipt, const uint64_t* __restrict__ cmask,
                                                                    const uint32_t* __restrict__ tau_in,
                                                                    const int32_t* __restrict__ need_eq_in,
                                                                    const int32_t* __restrict__ pre_eq,
                                                                    int32_t* __restrict__ pre_kept,
                                                                    int32_t* __restrict__ counts) {
    __shared__ int wave_tot[kSelThreads / kWave];
    const int e = blockIdx.x, tid = threadIdx.x;
    const uint32_t tau = tau_in[e];
    const int need = need_eq_in[e];
    int eq = pre_eq[e * kSelThreads + tid], n = 0;
    const int t_end = min(T, (tid + 1) * ipt);
    for (int t = tid * ipt; t < t_end; ++t) {
        const uint32_t key = keyT[static_cast<size_t>(e) * Tpad + t];
        bool member = key > tau;
        if (key == tau && key != 0u) { member = eq < need; ++eq; }
        n += member && ((cmask[t] >> e) & 1ull);
    }
    const int lane = tid & (kWave - 1), wave = tid / kWave;
    int inc = n;
#pragma unroll
    for (int m = 1; m < kWave; m <<= 1) {
        int a = __shfl_up(inc, m, kWave);
        if (lane >= m) inc += a;
    }
    if (lane == kWave - 1) wave_tot[wave] = inc;
    __syncthreads();
    int off = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < kSelThreads / kWave; ++w) {
        if (w < wave) off += wave_tot[w];
        tot += wave_tot[w];
    }
    pre_kept[e * kSelThreads + tid] = off + inc - n;
    if (tid == 0) counts[e] = tot;
}

// ---------------------------------------------------------------------------------------
// 3. slots
// ---------------------------------------------------------------------------------------
// A workgroup takes a tile of max(64, ipt) tokens (whole chunks) and all experts, 64 tokens at a time: wave w of W
// does experts w, w + W, ...  Lane = token, so the keys are read in whole stretches of the column-major copy and the
// number of kept tokens in front of a token inside its chunk is a popcount of a ballot (chunks longer than 64
// tokens carry their running counts from one stretch of 64 to the next).  The slots of the 64 x E tile are
// gathered in LDS and leave as whole rows of slot_of.
__global__ __launch_bounds__(kSelThreads) void slot_kernel(const uint64_t* __restrict__ cmask, int T, int E, int capacity,
                                                   int mode, int ipt,
                                                   const uint32_t* __restrict__ tau_in,
                                                   const int32_t* __restrict__ need_eq_in,
                                                   const int32_t* __restrict__ pre_gt,
                                                   const int32_t* __restrict__ pre_eq,
                                                   const int32_t* __restrict__ counts, int32_t* __restrict__ slot_of,
                                                   int32_t* __restrict__ slot_token,
                                                   const uint32_t* __restrict__ keyT, int Tpad,
                                                   const int32_t* __restrict__ pre_kept) {          // STRICT: see strict_filter_kernel
    __shared__ int32_t tile[kWave * (kWave + 1)];       // [token][E + 1]
    __shared__ int carry[kWave][3];                     // per expert: kept-before counts of a long chunk so far
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave, nthreads = blockDim.x;
    const bool long_chunk = ipt > kWave;
    const int TT = long_chunk ? ipt : kWave;
    const int t_tile = blockIdx.x * TT;
    const int G = long_chunk ? kWave : ipt;             // lanes per chunk inside a stretch (a power of two)
    const uint64_t group_mask = (G >= 64 ? ~0ull : ((1ull << G) - 1ull)) << (lane & ~(G - 1));
    const uint64_t below = (1ull << lane) - 1ull;
    const int ld = E + 1;
    if (tid < kWave) { carry[tid][0] = 0; carry[tid][1] = 0; carry[tid][2] = 0; }
    __syncthreads();
    for (int j0 = 0; j0 < TT; j0 += kWave) {
        const int t = t_tile + j0 + lane;
        const bool on = t < T && j0 + lane < TT;
        const int c = long_chunk ? static_cast<int>(blockIdx.x) : t / ipt;
        for (int e = wave; e < E; e += nthreads / kWave) {
            const uint32_t tau = tau_in[e];
            const int need = need_eq_in[e];
            const int gt = (on ? pre_gt[e * kSelThreads + c] : 0) + carry[e][0];
            const int eq = (on ? pre_eq[e * kSelThreads + c] : 0) + carry[e][1];
            const uint32_t key = on ? keyT[static_cast<size_t>(e) * Tpad + t] : 0u;
            const bool is_gt = key > tau, is_eq = key == tau && key != 0u;
            const uint64_t w_gt = __ballot(is_gt), w_eq = __ballot(is_eq);
            const int gt_before = gt + __popcll(w_gt & group_mask & below), eq_before = eq + __popcll(w_eq & group_mask & below);
            int slot = -1;
            if (is_gt) slot = gt_before + min(eq_before, need);
            else if (is_eq && eq_before < need) slot = gt_before + eq_before;
            uint64_t w_k = 0ull;
            if (mode == ETR_MODE_BIDIR_STRICT) {        // renumber inside the chooser set
                const int kept = (on ? pre_kept[e * kSelThreads + c] : 0) + carry[e][2];
                const bool keep = slot >= 0 && on && ((cmask[t] >> e) & 1ull);
                w_k = __ballot(keep);
                slot = keep ? kept + __popcll(w_k & group_mask & below) : -1;
            }
            tile[lane * ld + e] = slot;
            if (on && slot >= 0) slot_token[static_cast<size_t>(e) * capacity + slot] = t;
            if (long_chunk && lane == 0) {              // (the whole wave is one chunk here)
                carry[e][0] += __popcll(w_gt); carry[e][1] += __popcll(w_eq); carry[e][2] += __popcll(w_k);
            }
        }
        __syncthreads();
        int rows = T - (t_tile + j0);
        rows = rows < TT - j0 ? rows : TT - j0;
        rows = rows < kWave ? rows : kWave;
        int32_t* out = slot_of + static_cast<size_t>(t_tile + j0) * E;
        for (int i = tid; i < rows * E; i += nthreads) out[i] = tile[(i / E) * ld + i % E];
        __syncthreads();
    }
    // empty slots
    const long long gid = static_cast<long long>(blockIdx.x) * nthreads + tid;
    const long long total = static_cast<long long>(gridDim.x) * nthreads;
    for (long long i = gid; i < static_cast<long long>(E) * capacity; i += total) {
        const int ee = static_cast<int>(i / capacity), sl = static_cast<int>(i - static_cast<long long>(ee) * capacity);
        if (sl >= counts[ee]) slot_token[i] = -1;
    }
}

}  // namespace

// Tokens per chunk (= per thread of the per-expert kernel): a power of two from 4 to 64 while the column fits
// that kernel's registers, else a multiple of 4.
static int chunk_tokens(int T) {
    const int ipt = (T + kSelThreads - 1) / kSelThreads;
    for (int p = 4; p <= 64; p <<= 1)
        if (ipt <= p) return p;
    return (ipt + 3) / 4 * 4;
}

// Long columns (more than 32 keys per thread of the per-expert kernel) get their first radix digit counted by
// up to 16 workgroups per expert.
static int select_slices(int T) {
    if (chunk_tokens(T) <= 32) return 0;
    const int n = (T + 4095) / 4096;
    return n > kMaxSlices ? kMaxSlices : n;
}

size_t select_ws_bytes(int T, int E) {
    const size_t Tpad = align_up(static_cast<size_t>(T), 64);
    return align_up(sizeof(uint64_t) * T) + align_up(sizeof(uint32_t) * E * Tpad) + 2 * align_up(sizeof(int32_t) * E) +
           3 * align_up(sizeof(int32_t) * E * kSelThreads) +
           align_up(sizeof(uint32_t) * E * select_slices(T) * 2048);
}

SelectWs select_ws_carve(void* ws, int T, int E) {
    SelectWs w;
    char* p = static_cast<char*>(ws);
    w.Tpad = static_cast<int>(align_up(static_cast<size_t>(T), 64));
    w.cmask = reinterpret_cast<uint64_t*>(p);  p += align_up(sizeof(uint64_t) * T);
    w.keyT = reinterpret_cast<uint32_t*>(p);   p += align_up(sizeof(uint32_t) * E * w.Tpad);
    w.tau = reinterpret_cast<uint32_t*>(p);    p += align_up(sizeof(int32_t) * E);
    w.need_eq = reinterpret_cast<int32_t*>(p); p += align_up(sizeof(int32_t) * E);
    w.pre_gt = reinterpret_cast<int32_t*>(p);  p += align_up(sizeof(int32_t) * E * kSelThreads);
    w.pre_eq = reinterpret_cast<int32_t*>(p);  p += align_up(sizeof(int32_t) * E * kSelThreads);
    w.pre_kept = reinterpret_cast<int32_t*>(p); p += align_up(sizeof(int32_t) * E * kSelThreads);
    w.hist1 = reinterpret_cast<uint32_t*>(p);
    w.ipt = chunk_tokens(T);
    w.n_slices = select_slices(T);
    w.slice = w.n_slices ? ((T + w.n_slices - 1) / w.n_slices + 3) / 4 * 4 : 0;
    return w;
}

hipError_t static_select_scratch(void** out) {
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static void* ptrs[kMaxDevices] = {};
    int dev = 0;
    hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess) return err;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (!ptrs[dev]) {
        void* p = nullptr;
        err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (err != hipSuccess) return err;
        if (!p) return hipErrorInvalidSymbol;
        ptrs[dev] = p;
    }
    *out = ptrs[dev];
    return hipSuccess;
}

hipError_t launch_select(const etr_config& c, const float* score, int32_t* topk_expert, int32_t* slot_of,
                         int32_t* slot_token, int32_t* counts, const SelectWs& w, hipStream_t st,
                         const int32_t* capacity_dev, long long sum_need) {
    int G = 1;
    while (G < c.E) G <<= 1;
#define ETR_TC(GG)                                                                                              \
    hipLaunchKernelGGL(token_choice_kernel<GG>, dim3((c.T + token_tile<GG>() - 1) / token_tile<GG>()),         \
                       dim3(token_threads<GG>()), 0, st,                                                        \
                       score, c.T, c.E, c.k, c.mode, topk_expert, w.cmask, w.keyT, w.Tpad)
    switch (G) {
        case 1: ETR_TC(1); break;
        case 2: ETR_TC(2); break;
        case 4: ETR_TC(4); break;
        case 8: ETR_TC(8); break;
        case 16: ETR_TC(16); break;
        case 32: ETR_TC(32); break;
        default: ETR_TC(64); break;
    }
#undef ETR_TC
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;

    // TCR keeps by position and searches nothing, so it skips the pre-pass
    const bool pre = w.n_slices > 0 && c.mode != ETR_MODE_TCR;
    if (pre) {
        hipLaunchKernelGGL(key_histogram_kernel, dim3(w.n_slices, c.E), dim3(256), 0, st, w.keyT, w.Tpad, c.T, w.slice,
                           w.hist1);
        err = hipGetLastError();
        if (err != hipSuccess) return err;
    }
    const bool adapt = sum_need > 0;
#define ETR_EC1(II, PP, AA)                                                                                           \
    hipLaunchKernelGGL((expert_choice_kernel<II, PP, AA>), dim3(c.E), dim3(kSelThreads), 0, st, w.keyT, w.Tpad, c.T, w.ipt, \
                       c.capacity, c.mode, capacity_dev, sum_need, w.tau, w.need_eq, w.pre_gt, w.pre_eq, counts, w.hist1, \
                       w.n_slices)
#define ETR_EC(II, PP) do { if (adapt) ETR_EC1(II, PP, true); else ETR_EC1(II, PP, false); } while (0)
    if (w.ipt == 4) ETR_EC(4, false);                       // (the register variants take exactly their chunk length)
    else if (w.ipt == 8) ETR_EC(8, false);
    else if (w.ipt == 16) ETR_EC(16, false);
    else if (w.ipt == 32) ETR_EC(32, false);                // (no pre-pass up to here, see select_slices)
    else if (w.ipt == 64) { if (pre) ETR_EC(64, true); else ETR_EC(64, false); }
    else { if (pre) ETR_EC(0, true); else ETR_EC(0, false); }
#undef ETR_EC
#undef ETR_EC1
    err = hipGetLastError();
    if (err != hipSuccess) return err;

    if (c.mode == ETR_MODE_BIDIR_STRICT) {
        hipLaunchKernelGGL(strict_filter_kernel, dim3(c.E), dim3(kSelThreads), 0, st, w.keyT, w.Tpad, c.T, w.ipt, w.cmask,
                           w.tau, w.need_eq, w.pre_eq, w.pre_kept, counts);
        err = hipGetLastError();
        if (err != hipSuccess) return err;
    }
    const int tile3 = w.ipt > kWave ? w.ipt : kWave;     // tokens per workgroup of slot_kernel
    const int blocks3 = (c.T + tile3 - 1) / tile3;
    const int waves3 = c.E < 4 ? 4 : (c.E > 16 ? 16 : c.E);   // one expert per wave up to 16 waves
    hipLaunchKernelGGL(slot_kernel, dim3(blocks3), dim3(waves3 * kWave), 0, st, w.cmask, c.T, c.E, c.capacity, c.mode, w.ipt,
                       w.tau, w.need_eq, w.pre_gt, w.pre_eq, counts, slot_of, slot_token, w.keyT, w.Tpad, w.pre_kept);
    return hipGetLastError();
}

}  // namespace etr
