// Reductions over the routing outputs that the training side of the method consumes:
//  * the statistics behind the losses of Sec. Locality Loss: expert load distribution D_c,
//    mean gate per expert, KL(D_c || D_l) against a caller-given localized distribution;
//  * the capacity lower bound C_min of the Remark in Sec. Dynamic Lower Bound Module,
//    C_min = (1/n) exp{ d * dmax^2 / (2 - dmax^2) }, from the largest affinity of the batch.
// Both are two-level reductions with a fixed summation order (no float atomics), so results
// are bit-reproducible; they read T*E*4..8 bytes and are latency-bound.
#include "etr_internal.h"

namespace etr {
namespace {

constexpr int kStatThreads = 256;

// partial[b][e] = sum of gate[t][e] over the block's tokens, partial[b][E] = its unrouted tokens (as int bits)
template <int G>   // lanes per token, power of two >= E
__global__ __launch_bounds__(kStatThreads) void stats_partial_kernel(const float* __restrict__ gate,
                                                                     const int32_t* __restrict__ slot_of, int T, int E,
                                                                     int tokens_per_block, float* __restrict__ partial) {
    constexpr int TPP = kStatThreads / G;              // tokens per pass
    __shared__ float red[TPP][G];
    __shared__ int unrouted[TPP];
    const int tid = threadIdx.x, e = tid % G, j = tid / G;
    const int t_begin = blockIdx.x * tokens_per_block;
    const int t_end = min(T, t_begin + tokens_per_block);
    float acc = 0.f;
    int un = 0;
    for (int t = t_begin + j; t < t_end + j; t += TPP) {     // uniform trip count per block (shuffles inside)
        const bool ok = t < t_end && e < E;
        if (ok) acc += gate[static_cast<size_t>(t) * E + e];
        int kept = ok && slot_of[static_cast<size_t>(t) * E + e] >= 0;
#pragma unroll
        for (int m = 1; m < G; m <<= 1) kept |= __shfl_xor(kept, m, kWave);
        if (e == 0 && t < t_end) un += kept ? 0 : 1;
    }
    red[j][e] = acc;
    if (e == 0) unrouted[j] = un;
    __syncthreads();
    if (tid < E) {
        float s = 0.f;
        for (int q = 0; q < TPP; ++q) s += red[q][tid];        // fixed order
        partial[static_cast<size_t>(blockIdx.x) * (E + 1) + tid] = s;
    }
    if (tid == 0) {
        int u = 0;
        for (int q = 0; q < TPP; ++q) u += unrouted[q];
        partial[static_cast<size_t>(blockIdx.x) * (E + 1) + E] = __int_as_float(u);
    }
}

__global__ __launch_bounds__(64) void stats_final_kernel(const float* __restrict__ partial, int nblk, int T, int E,
                                                         const int32_t* __restrict__ counts,
                                                         const float* __restrict__ target, float* __restrict__ load,
                                                         float* __restrict__ mean_gate, float* __restrict__ kl,
                                                         int32_t* __restrict__ n_unrouted) {
    const int e = threadIdx.x;
    long long total = 0;
    for (int q = 0; q < E; ++q) total += counts[q];
    double term = 0.0;
    if (e < E) {
        double s = 0.0;
        for (int b = 0; b < nblk; ++b) s += static_cast<double>(partial[static_cast<size_t>(b) * (E + 1) + e]);
        mean_gate[e] = static_cast<float>(s / T);
        const double l = total > 0 ? static_cast<double>(counts[e]) / static_cast<double>(total) : 0.0;
        load[e] = static_cast<float>(l);
        if (l > 0.0) term = target[e] > 0.f ? l * log(l / static_cast<double>(target[e])) : INFINITY;
    }
    // sum of the E terms in ascending expert order (one wave, E <= 64)
    __shared__ double terms[64];
    terms[e] = term;
    __syncthreads();
    if (e == 0) {
        double k = 0.0;
        for (int q = 0; q < E; ++q) k += terms[q];
        *kl = static_cast<float>(k);
        int u = 0;
        for (int b = 0; b < nblk; ++b) u += __float_as_int(partial[static_cast<size_t>(b) * (E + 1) + E]);
        *n_unrouted = u;
    }
}

__global__ __launch_bounds__(kStatThreads) void max_partial_kernel(const float* __restrict__ score, long long n,
                                                                   float* __restrict__ partial) {
    __shared__ float red[kStatThreads / kWave];
    float m = -INFINITY;
    for (long long i = static_cast<long long>(blockIdx.x) * kStatThreads + threadIdx.x; i < n;
         i += static_cast<long long>(gridDim.x) * kStatThreads)
        m = fmaxf(m, score[i]);
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) m = fmaxf(m, __shfl_xor(m, s, kWave));
    if ((threadIdx.x & (kWave - 1)) == 0) red[threadIdx.x / kWave] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < kStatThreads / kWave; ++w) m = fmaxf(m, red[w]);
        partial[blockIdx.x] = m;
    }
}

__global__ __launch_bounds__(64) void capacity_final_kernel(const float* __restrict__ partial, int nblk, int T, int E,
                                                            int d, float* __restrict__ dmax,
                                                            int32_t* __restrict__ capacity) {
    float m = -INFINITY;
    for (int b = threadIdx.x; b < nblk; b += 64) m = fmaxf(m, partial[b]);
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) m = fmaxf(m, __shfl_xor(m, s, kWave));
    if (threadIdx.x == 0) {
        const double dm = static_cast<double>(m);
        // ln C_min = d dmax^2 / (2 - dmax^2) - ln n, compared in the log domain against ln T
        const double log_c = static_cast<double>(d) * dm * dm / (2.0 - dm * dm) - log(static_cast<double>(E));
        int c;
        if (log_c >= log(static_cast<double>(T))) c = T;
        else c = static_cast<int>(ceil(exp(log_c)));
        c = c < 1 ? 1 : (c > T ? T : c);
        *dmax = m;
        *capacity = c;
    }
}

int stats_blocks(int T) {
    int nb = (T + kStatThreads - 1) / kStatThreads;
    return nb < 1 ? 1 : (nb > 1024 ? 1024 : nb);
}

}  // namespace

size_t stats_ws_bytes(int T, int E) { return align_up(sizeof(float) * static_cast<size_t>(stats_blocks(T)) * (E + 1)); }

hipError_t launch_route_stats(const etr_config& c, const float* gate, const int32_t* slot_of, const int32_t* counts,
                              const float* target, float* load, float* mean_gate, float* kl, int32_t* n_unrouted,
                              void* ws, hipStream_t st) {
    const int nblk = stats_blocks(c.T);
    const int tpb = (c.T + nblk - 1) / nblk;
    float* partial = static_cast<float*>(ws);
    int G = 1;
    while (G < c.E) G <<= 1;
#define ETR_SP(GG)                                                                                             \
    hipLaunchKernelGGL(stats_partial_kernel<GG>, dim3(nblk), dim3(kStatThreads), 0, st, gate, slot_of, c.T, c.E, \
                       tpb, partial)
    switch (G) {
        case 1: ETR_SP(1); break;
        case 2: ETR_SP(2); break;
        case 4: ETR_SP(4); break;
        case 8: ETR_SP(8); break;
        case 16: ETR_SP(16); break;
        case 32: ETR_SP(32); break;
        default: ETR_SP(64); break;
    }
#undef ETR_SP
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    hipLaunchKernelGGL(stats_final_kernel, dim3(1), dim3(64), 0, st, partial, nblk, c.T, c.E, counts, target, load,
                       mean_gate, kl, n_unrouted);
    return hipGetLastError();
}

hipError_t launch_capacity_lower_bound(const etr_config& c, const float* score, float* dmax, int32_t* capacity,
                                       void* ws, hipStream_t st) {
    const int nblk = stats_blocks(c.T);
    float* partial = static_cast<float*>(ws);
    hipLaunchKernelGGL(max_partial_kernel, dim3(nblk), dim3(kStatThreads), 0, st, score,
                       static_cast<long long>(c.T) * c.E, partial);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    hipLaunchKernelGGL(capacity_final_kernel, dim3(1), dim3(64), 0, st, partial, nblk, c.T, c.E, c.d, dmax, capacity);
    return hipGetLastError();
}

}  // namespace etr
