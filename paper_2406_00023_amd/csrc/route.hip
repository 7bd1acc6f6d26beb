// GrAP pooling, cosine affinity and gate (Sec. Cost-Efficient Sparse Expert-Token
// Affinity, Eqs. 2-4; gate = row softmax of Eq. 1's text).
//
// HBM-bound: every token row is read exactly once with 16-byte loads; one
// wavefront owns one token.  The pooled vector g (P floats) is reduced inside
// the wave with lane shuffles and staged in LDS; the expert embeddings sit in
// LDS with a padded row stride so that the E x L lane grid of the dot-product
// stage reads conflict-free.  Scores and gates leave as fp32.
#include "etr_internal.h"

namespace etr {
namespace {

constexpr int kRouteThreads = 256;
constexpr int kRouteWaves = kRouteThreads / kWave;
constexpr int kUnroll = 8;
// Workgroups resident per CU.  Measured on the 32-expert workload (57 us at 4): 5 and 6 per CU need 96 / 80 registers,
// spill, and take 66 / 99 us; keeping a lane's share of its embedding row in registers (172 registers, two waves
// per SIMD) takes 83 us.  The kernel lives on loads in flight, but not at the price of spills.
constexpr int kRouteBlocksPerCU = 4;

// g lives in a per-wave LDS region: a wave's LDS instructions execute in issue order, so ordering
// them in the instruction stream is all that is needed (no workgroup barrier, no waiting)
__device__ __forceinline__ void wave_lds_fence() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, kWave);
    return v;
}

template <bool BF16>
struct Chunk;   // one 16-byte piece of a token row

__device__ __forceinline__ uint4 load_chunk(const void* row, int c, bool ok) {
    return ok ? reinterpret_cast<const uint4*>(row)[c] : make_uint4(0u, 0u, 0u, 0u);
}

template <>
struct Chunk<false> {
    static constexpr int kVec = 4;
    __device__ static void unpack(const uint4& v, float* f) {
        f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y); f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
    }
    __device__ static float scalar(const void* row, int i) { return reinterpret_cast<const float*>(row)[i]; }
    // s += sum of the chunk, xx += sum of squares
    __device__ static void accumulate(const uint4& v, float& s, float& xx) {
        float f[4];
        unpack(v, f);
#pragma unroll
        for (int j = 0; j < 4; ++j) { s += f[j]; xx = fmaf(f[j], f[j], xx); }
    }
};

template <>
struct Chunk<true> {
    static constexpr int kVec = 8;
    __device__ static void unpack(const uint4& v, float* f) {
        f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xFFFF0000u);
        f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xFFFF0000u);
        f[4] = __uint_as_float(v.z << 16); f[5] = __uint_as_float(v.z & 0xFFFF0000u);
        f[6] = __uint_as_float(v.w << 16); f[7] = __uint_as_float(v.w & 0xFFFF0000u);
    }
    __device__ static float scalar(const void* row, int i) {
        return __uint_as_float(static_cast<uint32_t>(reinterpret_cast<const uint16_t*>(row)[i]) << 16);
    }
    // s += sum of the chunk, xx += sum of squares: two-element bf16 dot products with fp32 accumulation
    // (v_dot2c_f32_bf16), one instruction per pair instead of unpack + add + fma
    __device__ static void accumulate(const uint4& v, float& s, float& xx) {
        typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
        const bf16x2 one = __builtin_bit_cast(bf16x2, 0x3F803F80u);
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const bf16x2 p2 = __builtin_bit_cast(bf16x2, w[j]);
            s = __builtin_amdgcn_fdot2_f32_bf16(p2, one, s, false);
            xx = __builtin_amdgcn_fdot2_f32_bf16(p2, p2, xx, false);
        }
    }
};

struct RouteParams {
    int T, d, E, D, P;
    int cos_mode;
    int L;          // lanes cooperating on one expert in the dot-product stage (power of two, E*L <= 64)
    int w_stride;   // padded LDS row stride of the embeddings (floats)
    int R;          // 16-byte chunks per pooling group when that is a power of two <= 64, else 0
};

// FAST: the whole row fits one pass of kUnroll loads per lane and pools with lane shuffles;
// otherwise the general walk (several passes, or one lane per pooled feature).
template <bool BF16, bool FAST>
__global__ __launch_bounds__(kRouteThreads, kRouteBlocksPerCU) void route_kernel(RouteParams p, const void* __restrict__ x,
                                                              const float* __restrict__ w_emb,
                                                              float* __restrict__ score, float* __restrict__ gate) {
    using C = Chunk<BF16>;
    constexpr int V = C::kVec;
    extern __shared__ float smem[];
    float* Ws = smem;                                  // [E][w_stride]
    float* wn = Ws + p.E * p.w_stride;                 // [64] embedding norms
    float* gs = wn + 64;                               // [waves][P]

    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int nchunks = p.d / V;
    const size_t row_bytes = static_cast<size_t>(p.d) * (BF16 ? 2 : 4);
    // one pass of kUnroll 16-byte loads per lane covers d <= 64 * kUnroll * V elements (4096 bf16):
    // then the row of the NEXT token is fetched while the current one is reduced
    constexpr bool one_pass = FAST;
    uint4 raw[FAST ? kUnroll : 1];                                 // the row stays packed until it is reduced
    auto fetch = [&](int t) {
        if constexpr (FAST) {
            const bool live = t < p.T;
            const char* row = reinterpret_cast<const char*>(x) + static_cast<size_t>(live ? t : 0) * row_bytes;
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                int c = u * kWave + lane;
                raw[u] = load_chunk(row, c, live && c < nchunks);
            }
        }
    };
    // the first row is requested before the embeddings are staged, so both latencies overlap
    if (one_pass) fetch(blockIdx.x * kRouteWaves + wave);

    for (int i = tid; i < p.E * p.P; i += kRouteThreads) {
        int e = i / p.P, q = i - e * p.P;
        Ws[e * p.w_stride + q] = w_emb[i];
    }
    __syncthreads();
    for (int e = wave; e < p.E; e += kRouteWaves) {
        float s = 0.f;
        for (int q = lane; q < p.P; q += kWave) { float w = Ws[e * p.w_stride + q]; s += w * w; }
        s = wave_sum(s);
        if (lane == 0) wn[e] = sqrtf(s);
    }
    __syncthreads();

    float* g = gs + wave * p.P;
    const float invD = 1.0f / static_cast<float>(p.D);
    const float sqrtD = sqrtf(static_cast<float>(p.D));
    const int e_lane = lane / p.L, sub = lane & (p.L - 1);

    for (int t0 = blockIdx.x * kRouteWaves; t0 < p.T; t0 += gridDim.x * kRouteWaves) {
        const int t = t0 + wave;
        const bool live = t < p.T;
        const char* row = reinterpret_cast<const char*>(x) + static_cast<size_t>(live ? t : 0) * row_bytes;
        float xx = 0.f;
        if constexpr (one_pass) {
            float s[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                s[u] = 0.f;
                C::accumulate(raw[u], s[u], xx);
            }
            fetch(t + gridDim.x * kRouteWaves);          // next token of this wave (masked past T)
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int c = u * kWave + lane;
                float v = s[u];
                for (int m = 1; m < p.R; m <<= 1) v += __shfl_xor(v, m, kWave);
                if ((lane & (p.R - 1)) == 0 && c < nchunks) g[c / p.R] = v * invD;
            }
        } else if (p.R > 0) {
            for (int c0 = 0; c0 < nchunks; c0 += kWave * kUnroll) {
                uint4 rr[kUnroll];
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) {
                    int c = c0 + u * kWave + lane;
                    rr[u] = load_chunk(row, c, live && c < nchunks);
                }
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) {
                    int c = c0 + u * kWave + lane;
                    float ff[V];
                    C::unpack(rr[u], ff);
                    float s = 0.f;
#pragma unroll
                    for (int j = 0; j < V; ++j) { s += ff[j]; xx += ff[j] * ff[j]; }
                    for (int m = 1; m < p.R; m <<= 1) s += __shfl_xor(s, m, kWave);
                    if ((lane & (p.R - 1)) == 0 && c < nchunks) g[c / p.R] = s * invD;
                }
            }
        } else {
            // group size not a multiple of the 16-byte vector: scalar walk, one lane per pooled feature
            for (int q = lane; q < p.P; q += kWave) {
                float s = 0.f;
                for (int j = 0; j < p.D; ++j) {
                    float v = live ? C::scalar(row, q * p.D + j) : 0.f;
                    s += v; xx += v * v;
                }
                g[q] = s * invD;
            }
        }
        xx = wave_sum(xx);
        wave_lds_fence();                               // g was written by other lanes of this wave

        float acc = 0.f, gg = 0.f;
        if (e_lane < p.E) {
            const float* wr = Ws + e_lane * p.w_stride;
            if ((p.P & 3) == 0) {
                // four pooled features per LDS access and four independent accumulators: the loop is bound by
                // LDS latency, not bandwidth (the row stride makes the 16-byte reads conflict-free, see launch_route)
                const float4* g4 = reinterpret_cast<const float4*>(g);
                const float4* w4 = reinterpret_cast<const float4*>(wr);
                float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
#pragma unroll 4
                for (int q = sub; q < (p.P >> 2); q += p.L) {
                    const float4 gv = g4[q], wv = w4[q];
                    a0 = fmaf(gv.x, wv.x, a0); a1 = fmaf(gv.y, wv.y, a1);
                    a2 = fmaf(gv.z, wv.z, a2); a3 = fmaf(gv.w, wv.w, a3);
                }
                acc = (a0 + a1) + (a2 + a3);
            } else {
                for (int q = sub; q < p.P; q += p.L) acc += g[q] * wr[q];
            }
        }
        for (int m = 1; m < p.L; m <<= 1) acc += __shfl_xor(acc, m, kWave);
        float den;
        if (p.cos_mode == ETR_COS_POOLED) {
            for (int q = lane; q < p.P; q += kWave) gg += g[q] * g[q];
            gg = wave_sum(gg);
            den = sqrtf(gg);
        } else {
            den = sqrtf(xx);
            acc *= sqrtD;
        }
        const bool is_e = e_lane < p.E;
        den *= is_e ? wn[e_lane] : 0.f;
        const float sc = (is_e && den > 0.f) ? acc / den : 0.f;
        float mx = is_e ? sc : -INFINITY;
        for (int m = p.L; m < kWave; m <<= 1) mx = fmaxf(mx, __shfl_xor(mx, m, kWave));
        const float ex = is_e ? expf(sc - mx) : 0.f;
        float z = ex;
        for (int m = p.L; m < kWave; m <<= 1) z += __shfl_xor(z, m, kWave);
        if (live && is_e && sub == 0) {
            score[static_cast<size_t>(t) * p.E + e_lane] = sc;
            gate[static_cast<size_t>(t) * p.E + e_lane] = ex / z;
        }
        wave_lds_fence();                               // g is rewritten by the next iteration
    }
}

}  // namespace

hipError_t launch_route(const etr_config& c, const void* x, const float* w_emb, float* score, float* gate,
                        hipStream_t st) {
    RouteParams p;
    p.T = c.T; p.d = c.d; p.E = c.E; p.D = c.D; p.P = c.d / c.D; p.cos_mode = c.cos;
    int e2 = 1;
    while (e2 < c.E) e2 <<= 1;
    p.L = kWave / e2;
    // LDS row stride of the embeddings.  Scalar walk (P % 4 != 0): stride = L (mod 64 banks), so the E x L lane grid
    // reads distinct banks.  Vector walk: a 16-byte read is served 16 lanes at a time = 16/L experts x L lanes x 4
    // banks, conflict-free when consecutive rows start 4L banks apart.
    const int step = (p.P % 4 == 0) ? 4 * p.L : p.L;
    p.w_stride = p.P + ((step - p.P % 64) % 64 + 64) % 64;
    const int V = c.dtype == ETR_BF16 ? 8 : 4;
    p.R = 0;
    if (c.D % V == 0) {
        int r = c.D / V;
        if (r <= 64 && (r & (r - 1)) == 0) p.R = r;
    }
    const size_t lds = sizeof(float) * (static_cast<size_t>(p.E) * p.w_stride + 64 + kRouteWaves * p.P);
    if (lds > 160 * 1024) return hipErrorInvalidValue;
    int blocks = (c.T + kRouteWaves - 1) / kRouteWaves;
    const int resident = cu_count() * kRouteBlocksPerCU;    // what is resident at once: the embeddings are staged once per workgroup
    if (blocks > resident) blocks = resident;
    if (blocks < 1) blocks = 1;
    const bool fast = p.R > 0 && p.d / V <= kWave * kUnroll;
    auto kern = c.dtype == ETR_BF16 ? (fast ? route_kernel<true, true> : route_kernel<true, false>)
                                    : (fast ? route_kernel<false, true> : route_kernel<false, false>);
    hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(kRouteThreads), lds, st, p, x, w_emb, score, gate);
    return hipGetLastError();
}

}  // namespace etr
