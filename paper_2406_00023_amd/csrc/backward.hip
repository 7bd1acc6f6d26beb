// Backward of the layer: the chain rule through Eqs. 1-6 with the routing tables held fixed
// (the kept sets are piecewise constant in the input; the gate vectors of Eq. 3 are constants).
//
//   out[t] = sum_{e kept t} gate[t][e] * Wd_e (SiLU(Wg_e x_t) .* (Wu_e x_t)),  gate = softmax(score), score = Eq. 4
//
// Stages (all on one stream, nothing leaves the device):
//   1. a = Xp Wg^T, b = Xp Wu^T recomputed (rows gathered through slot_token), u = dOut_p Wd
//   2. element-wise: h = SiLU(a) b, da = gate u b SiLU'(a), db = gate u SiLU(a), <u, h> per row (= d out / d gate)
//   3. dXp = da Wg + db Wu;  dWd = (gate dOut_p)^T h;  dWg = da^T Xp;  dWu = db^T Xp
//   4. dx[t] = sum_e dXp[e][slot] + sum_e dscore[t][e] * d score[t][e] / d x[t]  (softmax and Eq. 4 differentiated)
// Every matrix product runs on the grouped "NT" kernel of ffn.hip (both operands contiguous along
// the contraction), so operands whose contraction index is the slow one are transposed first:
// the weights once per call, the per-row quantities straight out of the element-wise kernel.
#include "etr_internal.h"

namespace etr {
namespace {

constexpr int kTile = 64;
constexpr int kTileThreads = 256;

template <typename T> struct Elt;
template <> struct Elt<float> {
    __device__ static float load(const float* p, size_t i) { return p[i]; }
    __device__ static void store(float* p, size_t i, float v) { p[i] = v; }
};
template <> struct Elt<uint16_t> {          // bf16 bit patterns
    __device__ static float load(const uint16_t* p, size_t i) { return __uint_as_float(static_cast<uint32_t>(p[i]) << 16); }
    __device__ static void store(uint16_t* p, size_t i, float v) {
        uint32_t u = __float_as_uint(v);
        p[i] = static_cast<uint16_t>((u & 0x7FFFFFFFu) > 0x7F800000u ? 0x7FC0u : (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
    }
};

__device__ __forceinline__ int round_up64(int v) { return (v + 63) & ~63; }

// dst[b][c][col0 + r] = src[b][r][c]   for r < R, c < Cc   (dst rows have ld_dst elements)
template <typename T>
__global__ __launch_bounds__(kTileThreads) void transpose_kernel(const T* __restrict__ src, T* __restrict__ dst, int R,
                                                                 int Cc, int ld_dst, int col0) {
    __shared__ T tile[kTile][kTile + 2];
    const int b = blockIdx.z, r0 = blockIdx.y * kTile, c0 = blockIdx.x * kTile;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const T* s = src + static_cast<size_t>(b) * R * Cc;
    T* d = dst + static_cast<size_t>(b) * Cc * ld_dst;
#pragma unroll 4
    for (int i = ty; i < kTile; i += 4)
        if (r0 + i < R && c0 + tx < Cc) tile[i][tx] = s[static_cast<size_t>(r0 + i) * Cc + c0 + tx];
    __syncthreads();
#pragma unroll 4
    for (int i = ty; i < kTile; i += 4)
        if (c0 + i < Cc && r0 + tx < R) d[static_cast<size_t>(c0 + i) * ld_dst + col0 + r0 + tx] = tile[tx][i];
}

// dst[e][j][s] = src[slot_token[e][s]][j] (* gate[slot_token[e][s]][e])  for s < counts[e];
// zeros for counts[e] <= s < round_up64(counts[e]); nothing beyond.
template <typename T, bool SCALE>
__global__ __launch_bounds__(kTileThreads) void gather_transpose_kernel(const T* __restrict__ src,
                                                                        const int32_t* __restrict__ slot_token,
                                                                        const int32_t* __restrict__ counts,
                                                                        const float* __restrict__ gate, T* __restrict__ dst,
                                                                        int T_, int d, int E, int C, int Cp) {
    __shared__ float tile[kTile][kTile + 1];
    const int e = blockIdx.z, s0 = blockIdx.y * kTile, j0 = blockIdx.x * kTile;
    const int count = min(counts[e], C);
    if (s0 >= round_up64(count)) return;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
#pragma unroll 4
    for (int i = ty; i < kTile; i += 4) {
        const int s = s0 + i;
        float v = 0.f;
        if (s < count && j0 + tx < d) {
            const int t = slot_token[static_cast<size_t>(e) * C + s];
            if (t >= 0 && t < T_) {
                v = Elt<T>::load(src, static_cast<size_t>(t) * d + j0 + tx);
                if (SCALE) v *= gate[static_cast<size_t>(t) * E + e];
            }
        }
        tile[i][tx] = v;
    }
    __syncthreads();
    T* de = dst + static_cast<size_t>(e) * d * Cp;
#pragma unroll 4
    for (int i = ty; i < kTile; i += 4)
        if (j0 + i < d && s0 + tx < Cp) Elt<T>::store(de, static_cast<size_t>(j0 + i) * Cp + s0 + tx, tile[tx][i]);
}

// Element-wise middle of the FFN backward for one block of 64 buffer rows of one expert.
//   in : u, a, b [E][C][H];  gate through slot_token
//   out: dab [E][C][2H] = (da | db);  daT, dbT, hT [E][H][Cp];  dgate_slot [E][C] = <u, h>
template <typename T>
__global__ __launch_bounds__(kTileThreads) void swiglu_backward_kernel(
    const T* __restrict__ u, const T* __restrict__ a, const T* __restrict__ b, const float* __restrict__ gate,
    const int32_t* __restrict__ slot_token, const int32_t* __restrict__ counts, T* __restrict__ dab, T* __restrict__ daT,
    T* __restrict__ dbT, T* __restrict__ hT, float* __restrict__ dgate_slot, int T_, int E, int C, int Cp, int H) {
    __shared__ float th[kTile][kTile + 1], ta[kTile][kTile + 1], tb[kTile][kTile + 1];
    const int e = blockIdx.y, s0 = blockIdx.x * kTile;
    const int count = min(counts[e], C);
    if (s0 >= round_up64(count)) return;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    constexpr int R = kTile / 4;                     // rows per thread: ty, ty + 4, ...
    float g_row[R], dot[R];
#pragma unroll
    for (int i = 0; i < R; ++i) {
        const int s = s0 + ty + 4 * i;
        g_row[i] = 0.f; dot[i] = 0.f;
        if (s < count) {
            const int t = slot_token[static_cast<size_t>(e) * C + s];
            if (t >= 0 && t < T_) g_row[i] = gate[static_cast<size_t>(t) * E + e];
        }
    }
    const size_t ebase = static_cast<size_t>(e) * C;
    for (int n0 = 0; n0 < H; n0 += kTile) {
        const int n = n0 + tx;
#pragma unroll
        for (int i = 0; i < R; ++i) {
            const int r = ty + 4 * i, s = s0 + r;
            float hv = 0.f, dav = 0.f, dbv = 0.f;
            if (s < count && n < H) {
                const size_t idx = (ebase + s) * H + n;
                const float uv = Elt<T>::load(u, idx), av = Elt<T>::load(a, idx), bv = Elt<T>::load(b, idx);
                const float sg = 1.0f / (1.0f + __expf(-av));
                const float sl = av * sg;
                hv = sl * bv;
                const float dh = g_row[i] * uv;
                dav = dh * bv * (sg * (1.0f + av * (1.0f - sg)));
                dbv = dh * sl;
                dot[i] += uv * hv;
                Elt<T>::store(dab, (ebase + s) * 2 * H + n, dav);
                Elt<T>::store(dab, (ebase + s) * 2 * H + H + n, dbv);
            }
            th[r][tx] = hv; ta[r][tx] = dav; tb[r][tx] = dbv;
        }
        __syncthreads();
        if (s0 + tx < Cp) {
#pragma unroll
            for (int i = 0; i < R; ++i) {
                const int c = ty + 4 * i;
                if (n0 + c < H) {
                    const size_t o = (static_cast<size_t>(e) * H + n0 + c) * Cp + s0 + tx;
                    Elt<T>::store(hT, o, th[tx][c]);
                    Elt<T>::store(daT, o, ta[tx][c]);
                    Elt<T>::store(dbT, o, tb[tx][c]);
                }
            }
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < R; ++i) {
        float v = dot[i];
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
        const int s = s0 + ty + 4 * i;
        if (tx == 0 && s < count) dgate_slot[ebase + s] = v;
    }
}

// dx[t] = sum_e dXp[e][slot_of[t][e]] + router term; one wavefront per token.
// Router term: dscore[e] = gate[e] (dgate[e] - sum_e' dgate[e'] gate[e']); with Eq. 4 in the form
//   FULL:   score = sqrt(D) <g, w> / (|x| |w|)  ->  d score / d x_j = sqrt(D) w[p(j)] / (D |x| |w|) - score x_j / |x|^2
//   POOLED: score = <g, w> / (|g| |w|)          ->  d score / d x_j = (w[p(j)] / (|g| |w|) - score g[p(j)] / |g|^2) / D
template <typename T>
__global__ __launch_bounds__(256) void dx_kernel(const T* __restrict__ x, const float* __restrict__ w_emb,
                                                 const float* __restrict__ score, const float* __restrict__ gate,
                                                 const int32_t* __restrict__ slot_of, const float* __restrict__ dgate_slot,
                                                 const T* __restrict__ dxp, T* __restrict__ dx, float* __restrict__ dgate_out,
                                                 float* __restrict__ dscore_out, int T_, int d, int E, int D, int C,
                                                 int cos_mode) {
    extern __shared__ float sm[];
    const int P = d / D;
    float* w = sm;                       // [E][P]
    float* wn = w + E * P;               // [E] 1 / |w_e| (0 for a zero embedding)
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    float* g = wn + E + wave * (2 * P + 2 * E);   // per wave: g[P], v[P], ds[E], slot (as int)[E]
    float* v = g + P;
    float* ds = v + P;
    int* sl = reinterpret_cast<int*>(ds + E);
    for (int i = threadIdx.x; i < E * P; i += blockDim.x) w[i] = w_emb[i];
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += blockDim.x) {
        float s = 0.f;
        for (int p = 0; p < P; ++p) s += w[e * P + p] * w[e * P + p];
        wn[e] = s > 0.f ? rsqrtf(s) : 0.f;
    }
    __syncthreads();
    const int t = blockIdx.x * 4 + wave;
    if (t >= T_) return;                 // no block-wide barrier below
    const T* xr = x + static_cast<size_t>(t) * d;
    // pooled features and norms
    float xx = 0.f, gg = 0.f;
    for (int p = lane; p < P; p += 64) {
        float s = 0.f;
        for (int j = 0; j < D; ++j) {
            const float xv = Elt<T>::load(xr, static_cast<size_t>(p) * D + j);
            s += xv; xx += xv * xv;
        }
        s /= D;
        g[p] = s; gg += s * s;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) { xx += __shfl_xor(xx, o, 64); gg += __shfl_xor(gg, o, 64); }
    // softmax backward (E <= 64: lane e)
    float dg = 0.f, gt = 0.f, sc = 0.f;
    int slot = -1;
    if (lane < E) {
        slot = slot_of[static_cast<size_t>(t) * E + lane];
        gt = gate[static_cast<size_t>(t) * E + lane];
        sc = score[static_cast<size_t>(t) * E + lane];
        if (slot >= 0 && slot < C) dg = dgate_slot[static_cast<size_t>(lane) * C + slot]; else slot = -1;
    }
    float mix = dg * gt;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mix += __shfl_xor(mix, o, 64);
    const float dsv = gt * (dg - mix);
    float beta = dsv * sc;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) beta += __shfl_xor(beta, o, 64);
    if (lane < E) {
        ds[lane] = dsv; sl[lane] = slot;
        if (dgate_out) dgate_out[static_cast<size_t>(t) * E + lane] = dg;
        if (dscore_out) dscore_out[static_cast<size_t>(t) * E + lane] = dsv;
    }
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_s_waitcnt(0xC07F);          // lgkmcnt(0): this wave's LDS writes are visible to its lanes
    const bool full = cos_mode == ETR_COS_FULL;
    const float nrm2 = full ? xx : gg;
    const float inv_n = nrm2 > 0.f ? rsqrtf(nrm2) : 0.f;
    // v[p] = sum_e ds[e] * w_e[p] / |w_e| * (FULL: sqrt(D) / (D |x|); POOLED: 1 / (D |g|))
    const float cv = inv_n * (full ? sqrtf(static_cast<float>(D)) : 1.0f) / D;
    for (int p = lane; p < P; p += 64) {
        float s = 0.f;
        for (int e = 0; e < E; ++e) s += ds[e] * wn[e] * w[e * P + p];
        v[p] = s * cv;
    }
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_s_waitcnt(0xC07F);
    // FULL: - beta x_j / |x|^2 ; POOLED: - beta g_p / (D |g|^2)
    const float cb = nrm2 > 0.f ? beta / nrm2 * (full ? 1.0f : 1.0f / D) : 0.f;
    T* out = dx + static_cast<size_t>(t) * d;
    for (int j = lane; j < d; j += 64) {
        const int p = j / D;
        float acc = v[p] - cb * (full ? Elt<T>::load(xr, j) : g[p]);
        for (int e = 0; e < E; ++e) {
            const int s = sl[e];
            if (s >= 0) acc += Elt<T>::load(dxp, (static_cast<size_t>(e) * C + s) * d + j);
        }
        Elt<T>::store(out, j, acc);
    }
}

struct BackwardWs {
    size_t wdT, wguT, a, b, u, dab, daT, dbT, hT, xpT, dypT, dxp, dgate_slot, total;
};

BackwardWs backward_layout(const etr_config& c) {
    BackwardWs w{};
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes); return o; };
    const size_t es = elt_bytes(c.dtype), E = c.E, C = c.capacity, H = c.H, d = c.d;
    const size_t Cp = (C + 63) / 64 * 64;
    w.wdT = take(E * H * d * es);
    w.wguT = take(E * d * 2 * H * es);
    w.a = take(E * C * H * es);
    w.b = take(E * C * H * es);
    w.u = take(E * C * H * es);
    w.dab = take(E * C * 2 * H * es);
    w.daT = take(E * H * Cp * es);
    w.dbT = take(E * H * Cp * es);
    w.hT = take(E * H * Cp * es);
    w.xpT = take(E * d * Cp * es);
    w.dypT = take(E * d * Cp * es);
    w.dxp = take(E * C * d * es);
    w.dgate_slot = take(E * C * 4);
    w.total = off;
    return w;
}

template <typename T>
hipError_t backward_impl(const etr_config& c, const void* x, const float* w_emb, const void* w_gate, const void* w_up,
                         const void* w_down, const float* score, const float* gate, const int32_t* slot_of,
                         const int32_t* slot_token, const int32_t* counts, const void* dout, void* dx, void* dw_gate,
                         void* dw_up, void* dw_down, float* dgate, float* dscore, void* ws, hipStream_t st) {
    const BackwardWs L = backward_layout(c);
    char* base = static_cast<char*>(ws);
    auto at = [&](size_t off) { return reinterpret_cast<T*>(base + off); };
    const int E = c.E, C = c.capacity, H = c.H, d = c.d, Tn = c.T;
    const int Cp = (C + 63) / 64 * 64;
    const unsigned cd = (d + kTile - 1) / kTile, cH = (H + kTile - 1) / kTile, cC = Cp / kTile;
    hipError_t err;
#define ETR_BW(call) do { if ((err = (call)) != hipSuccess) return err; } while (0)
    // weights with the contraction index made contiguous: WdT[e][H][d], WguT[e][d][2H] = (Wg^T | Wu^T)
    hipLaunchKernelGGL(transpose_kernel<T>, dim3(cH, cd, E), dim3(kTileThreads), 0, st, static_cast<const T*>(w_down),
                       at(L.wdT), d, H, d, 0);
    hipLaunchKernelGGL(transpose_kernel<T>, dim3(cd, cH, E), dim3(kTileThreads), 0, st, static_cast<const T*>(w_gate),
                       at(L.wguT), H, d, 2 * H, 0);
    hipLaunchKernelGGL(transpose_kernel<T>, dim3(cd, cH, E), dim3(kTileThreads), 0, st, static_cast<const T*>(w_up),
                       at(L.wguT), H, d, 2 * H, H);
    ETR_BW(hipGetLastError());
    // a, b recomputed from the gathered token rows; u = gathered upstream gradient times Wd
    GroupedGemm g1{x, w_gate, w_up, at(L.a), at(L.b), counts, nullptr, slot_token, E, C, H, d, 0, 0, Tn, GEMM_DUAL, c.dtype};
    ETR_BW(launch_grouped_gemm(g1, st));
    GroupedGemm g2{dout, at(L.wdT), nullptr, at(L.u), nullptr, counts, nullptr, slot_token, E, C, H, d, 0, 0, Tn, GEMM_PLAIN, c.dtype};
    ETR_BW(launch_grouped_gemm(g2, st));
    hipLaunchKernelGGL(swiglu_backward_kernel<T>, dim3(cC, E), dim3(kTileThreads), 0, st, at(L.u), at(L.a), at(L.b), gate,
                       slot_token, counts, at(L.dab), at(L.daT), at(L.dbT), at(L.hT),
                       reinterpret_cast<float*>(base + L.dgate_slot), Tn, E, C, Cp, H);
    hipLaunchKernelGGL((gather_transpose_kernel<T, false>), dim3(cd, cC, E), dim3(kTileThreads), 0, st,
                       static_cast<const T*>(x), slot_token, counts, gate, at(L.xpT), Tn, d, E, C, Cp);
    hipLaunchKernelGGL((gather_transpose_kernel<T, true>), dim3(cd, cC, E), dim3(kTileThreads), 0, st,
                       static_cast<const T*>(dout), slot_token, counts, gate, at(L.dypT), Tn, d, E, C, Cp);
    ETR_BW(hipGetLastError());
    // dXp = (da | db) (Wg^T | Wu^T)^T
    GroupedGemm g3{at(L.dab), at(L.wguT), nullptr, at(L.dxp), nullptr, counts, nullptr, nullptr, E, C, d, 2 * H, 0, 0, C, GEMM_PLAIN, c.dtype};
    ETR_BW(launch_grouped_gemm(g3, st));
    // weight gradients: contraction over the kept rows of each expert
    GroupedGemm g4{at(L.dypT), at(L.hT), nullptr, dw_down, nullptr, nullptr, counts, nullptr, E, d, H, Cp, Cp, Cp, d, GEMM_PLAIN, c.dtype};
    ETR_BW(launch_grouped_gemm(g4, st));
    GroupedGemm g5{at(L.daT), at(L.xpT), nullptr, dw_gate, nullptr, nullptr, counts, nullptr, E, H, d, Cp, Cp, Cp, H, GEMM_PLAIN, c.dtype};
    ETR_BW(launch_grouped_gemm(g5, st));
    GroupedGemm g6{at(L.dbT), at(L.xpT), nullptr, dw_up, nullptr, nullptr, counts, nullptr, E, H, d, Cp, Cp, Cp, H, GEMM_PLAIN, c.dtype};
    ETR_BW(launch_grouped_gemm(g6, st));
    const int P = d / c.D;
    const size_t lds = (static_cast<size_t>(E) * P + E + 4 * (2 * P + 2 * E)) * 4;
    auto kern = dx_kernel<T>;
    if (lds > 64 * 1024)
        ETR_BW(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                   static_cast<int>(lds)));
    hipLaunchKernelGGL(kern, dim3((Tn + 3) / 4), dim3(256), lds, st, static_cast<const T*>(x), w_emb, score, gate, slot_of,
                       reinterpret_cast<const float*>(base + L.dgate_slot), at(L.dxp), static_cast<T*>(dx), dgate, dscore,
                       Tn, d, E, c.D, C, static_cast<int>(c.cos));
#undef ETR_BW
    return hipGetLastError();
}

}  // namespace

size_t backward_ws_bytes(const etr_config& c) { return backward_layout(c).total; }

hipError_t launch_moe_backward(const etr_config& c, const void* x, const float* w_emb, const void* w_gate,
                               const void* w_up, const void* w_down, const float* score, const float* gate,
                               const int32_t* slot_of, const int32_t* slot_token, const int32_t* counts,
                               const void* dout, void* dx, void* dw_gate, void* dw_up, void* dw_down, float* dgate,
                               float* dscore, void* ws, hipStream_t st) {
    if (static_cast<size_t>(c.E) * (c.d / c.D) * 4 > 120 * 1024) return hipErrorInvalidValue;   // embeddings must fit in LDS
    if (c.dtype == ETR_BF16)
        return backward_impl<uint16_t>(c, x, w_emb, w_gate, w_up, w_down, score, gate, slot_of, slot_token, counts, dout,
                                       dx, dw_gate, dw_up, dw_down, dgate, dscore, ws, st);
    return backward_impl<float>(c, x, w_emb, w_gate, w_up, w_down, score, gate, slot_of, slot_token, counts, dout, dx,
                                dw_gate, dw_up, dw_down, dgate, dscore, ws, st);
}

}  // namespace etr
