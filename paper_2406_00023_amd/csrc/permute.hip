// Token rearrangement into the capacity-bounded per-expert buffers (the slot table
// I_{ki} of Eq. 6) and the gate-weighted sum of Eq. 1 that undoes it.
//
// Both are HBM-bound row movers: one wavefront per row, 16 bytes per lane per
// access, every load of a row issued before its first use.
#include "etr_internal.h"

namespace etr {
namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
constexpr int kRowThreads = 256;
constexpr int kRowWaves = kRowThreads / kWave;

// xp[e][s][:] = x[slot_token[e][s]][:]  for s < counts[e]
// A wave walks rows r, r + stride, ...  The source index of the next row is fetched while the
// current row is copied (otherwise every row pays two dependent memory latencies before its first
// load), and all loads of a row are in flight before its first store.
__global__ __launch_bounds__(kRowThreads) void dispatch_kernel(const uint4* __restrict__ x,
                                                               const int32_t* __restrict__ slot_token,
                                                               const int32_t* __restrict__ counts,
                                                               uint4* __restrict__ xp, int T, int capacity,
                                                               long long rows, int row_vecs) {
    const int lane = threadIdx.x & (kWave - 1);
    const long long stride = static_cast<long long>(gridDim.x) * kRowWaves;
    constexpr int U = 8;
    // source row of buffer row r, or -1 when the slot is empty / the table does not belong to this x
    auto source_of = [&](long long r) -> int {
        if (r >= rows) return -1;
        const int e = static_cast<int>(r / capacity), s = static_cast<int>(r - static_cast<long long>(e) * capacity);
        if (s >= counts[e]) return -1;
        const int t = slot_token[r];
        return (t < 0 || t >= T) ? -1 : t;
    };
    long long r = static_cast<long long>(blockIdx.x) * kRowWaves + threadIdx.x / kWave;
    int t = source_of(r);
    for (; r < rows; r += stride) {
        const int t_next = source_of(r + stride);
        if (t >= 0) {
            const uint4* src = x + static_cast<size_t>(t) * row_vecs;
            uint4* dst = xp + static_cast<size_t>(r) * row_vecs;
            for (int c0 = 0; c0 < row_vecs; c0 += kWave * U) {
                uint4 v[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    int c = c0 + u * kWave + lane;
                    if (c < row_vecs) v[u] = src[c];
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    int c = c0 + u * kWave + lane;
                    // streaming store: the permuted rows are not read again by this kernel
                    if (c < row_vecs)
                        __builtin_nontemporal_store(__builtin_bit_cast(u32x4, v[u]), reinterpret_cast<u32x4*>(dst) + c);
                }
            }
        }
        t = t_next;
    }
}

template <bool BF16>
struct Row;
template <>
struct Row<false> {
    static constexpr int kVec = 4;
    __device__ static void unpack(const uint4& v, float* f) {
        f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y); f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
    }
    __device__ static uint4 pack(const float* f) {
        return make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3]));
    }
};
__device__ __forceinline__ uint32_t bf16_rne(float f) {       // fp32 -> bf16 bits, round to nearest even
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return 0x7FC0u;        // NaN stays NaN
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}
template <>
struct Row<true> {
    static constexpr int kVec = 8;
    __device__ static void unpack(const uint4& v, float* f) {
        f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xFFFF0000u);
        f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xFFFF0000u);
        f[4] = __uint_as_float(v.z << 16); f[5] = __uint_as_float(v.z & 0xFFFF0000u);
        f[6] = __uint_as_float(v.w << 16); f[7] = __uint_as_float(v.w & 0xFFFF0000u);
    }
    __device__ static uint4 pack(const float* f) {
        return make_uint4(bf16_rne(f[0]) | (bf16_rne(f[1]) << 16), bf16_rne(f[2]) | (bf16_rne(f[3]) << 16),
                          bf16_rne(f[4]) | (bf16_rne(f[5]) << 16), bf16_rne(f[6]) | (bf16_rne(f[7]) << 16));
    }
};

// out[t][:] = sum_{e ascending, slot_of[t][e] >= 0} gate[t][e] * yp[e][slot_of[t][e]][:]
template <bool BF16>
__global__ __launch_bounds__(kRowThreads) void combine_kernel(const uint4* __restrict__ yp,
                                                              const float* __restrict__ gate,
                                                              const int32_t* __restrict__ slot_of,
                                                              uint4* __restrict__ out, int T, int E, int capacity,
                                                              int row_vecs, int gate_norm) {
    using R = Row<BF16>;
    constexpr int V = R::kVec;
    const int lane = threadIdx.x & (kWave - 1);
    const int t = blockIdx.x * kRowWaves + threadIdx.x / kWave;
    if (t >= T) return;
    int my_slot = -1;
    float my_gate = 0.f;
    if (lane < E) {
        my_slot = slot_of[static_cast<size_t>(t) * E + lane];
        my_gate = gate[static_cast<size_t>(t) * E + lane];
    }
    const uint64_t kept = __ballot(my_slot >= 0 && my_slot < capacity);
    if (gate_norm) {                                             // variant: weights renormalised over the kept experts
        float sum = (my_slot >= 0 && my_slot < capacity) ? my_gate : 0.f;
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) sum += __shfl_xor(sum, m, kWave);
        if (sum > 0.f) my_gate /= sum;
    }
    constexpr int U = 4;
    for (int c0 = 0; c0 < row_vecs; c0 += kWave * U) {
        float acc[U][V];
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int j = 0; j < V; ++j) acc[u][j] = 0.f;
        uint64_t m = kept;
        while (m) {                                              // ascending expert index
            const int e = __ffsll(static_cast<unsigned long long>(m)) - 1;
            m &= m - 1;
            const int s = __shfl(my_slot, e, kWave);
            const float g = __shfl(my_gate, e, kWave);
            const uint4* src = yp + (static_cast<size_t>(e) * capacity + s) * row_vecs;
            uint4 v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                int c = c0 + u * kWave + lane;
                v[u] = c < row_vecs ? src[c] : make_uint4(0u, 0u, 0u, 0u);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float f[V];
                R::unpack(v[u], f);
#pragma unroll
                for (int j = 0; j < V; ++j) acc[u][j] = fmaf(g, f[j], acc[u][j]);
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            int c = c0 + u * kWave + lane;
            // streaming store: the layer output is not read again here
            if (c < row_vecs)
                __builtin_nontemporal_store(__builtin_bit_cast(u32x4, R::pack(acc[u])),
                                            reinterpret_cast<u32x4*>(out) + static_cast<size_t>(t) * row_vecs + c);
        }
    }
}

}  // namespace

hipError_t launch_dispatch(const etr_config& c, const void* x, const int32_t* slot_token, const int32_t* counts,
                           void* xp, hipStream_t st) {
    const long long rows = static_cast<long long>(c.E) * c.capacity;
    const int row_vecs = static_cast<int>(static_cast<size_t>(c.d) * elt_bytes(c.dtype) / 16);
    long long blocks = (rows + kRowWaves - 1) / kRowWaves;
    if (blocks > 256 * 16) blocks = 256 * 16;          // 16 workgroups per CU, each wave walks several rows
    hipLaunchKernelGGL(dispatch_kernel, dim3(static_cast<unsigned>(blocks)), dim3(kRowThreads), 0, st,
                       static_cast<const uint4*>(x), slot_token, counts, static_cast<uint4*>(xp), c.T, c.capacity,
                       rows, row_vecs);
    return hipGetLastError();
}

hipError_t launch_combine(const etr_config& c, const void* yp, const float* gate, const int32_t* slot_of,
                          void* out, hipStream_t st) {
    const int row_vecs = static_cast<int>(static_cast<size_t>(c.d) * elt_bytes(c.dtype) / 16);
    const int blocks = (c.T + kRowWaves - 1) / kRowWaves;
    if (c.dtype == ETR_BF16)
        hipLaunchKernelGGL(combine_kernel<true>, dim3(blocks), dim3(kRowThreads), 0, st, static_cast<const uint4*>(yp),
                           gate, slot_of, static_cast<uint4*>(out), c.T, c.E, c.capacity, row_vecs, c.gate_norm);
    else
        hipLaunchKernelGGL(combine_kernel<false>, dim3(blocks), dim3(kRowThreads), 0, st, static_cast<const uint4*>(yp),
                           gate, slot_of, static_cast<uint4*>(out), c.T, c.E, c.capacity, row_vecs, c.gate_norm);
    return hipGetLastError();
}

}  // namespace etr
