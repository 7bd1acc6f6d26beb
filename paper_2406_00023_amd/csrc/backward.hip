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
// Every matrix product runs on the grouped kernels of ffn.hip.  Operands whose contraction index is the
// slow one in memory (Wd for u, Wg / Wu for dXp, the row-major activations for the weight gradients) are
// read as they lie: the persistent kernel stages such k-tiles k-major in LDS and takes its MFMA fragments
// through transposing LDS reads, so nothing is transposed in memory.  Only shapes that kernel does not take
// (fp32, H % 64 != 0, fewer than 128 padded rows) go through the fall-back that transposes the weights once per
// call and has the element-wise kernel write transposed copies of the per-row quantities.
#include "etr_internal.h"

namespace etr {
namespace {

constexpr int kTile = 64;
constexpr int kTileThreads = 256;

template <typename T> struct Elt;
template <> struct Elt<float> {
    static constexpr int kVec = 4;           // elements per 16 bytes
    static constexpr int kPad = 1;           // LDS tile padding (elements): odd dword stride
    __device__ static float load(const float* p, size_t i) { return p[i]; }
    __device__ static void store(float* p, size_t i, float v) { p[i] = v; }
    __device__ static void load_vec(const float* p, float* f) {
        const float4 v = *reinterpret_cast<const float4*>(p);
        f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
    }
    __device__ static void store_vec(float* p, const float* f) { *reinterpret_cast<float4*>(p) = make_float4(f[0], f[1], f[2], f[3]); }
    __device__ static float widen(float v) { return v; }
    __device__ static float narrow(float v) { return v; }
};
__device__ __forceinline__ uint16_t bf16_bits(float v) {     // round to nearest even
    const uint32_t u = __float_as_uint(v);
    return static_cast<uint16_t>((u & 0x7FFFFFFFu) > 0x7F800000u ? 0x7FC0u : (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}
template <> struct Elt<uint16_t> {          // bf16 bit patterns
    static constexpr int kVec = 8;
    static constexpr int kPad = 2;
    __device__ static float load(const uint16_t* p, size_t i) { return __uint_as_float(static_cast<uint32_t>(p[i]) << 16); }
    __device__ static void store(uint16_t* p, size_t i, float v) { p[i] = bf16_bits(v); }
    __device__ static void load_vec(const uint16_t* p, float* f) {
        const uint4 v = *reinterpret_cast<const uint4*>(p);
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) { f[2 * i] = __uint_as_float(w[i] << 16); f[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u); }
    }
    __device__ static void store_vec(uint16_t* p, const float* f) {
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) w[i] = bf16_bits(f[2 * i]) | (static_cast<uint32_t>(bf16_bits(f[2 * i + 1])) << 16);
        *reinterpret_cast<uint4*>(p) = make_uint4(w[0], w[1], w[2], w[3]);
    }
    __device__ static float widen(uint16_t v) { return __uint_as_float(static_cast<uint32_t>(v) << 16); }
    __device__ static uint16_t narrow(float v) { return bf16_bits(v); }
};

// Columns of the transposed per-expert buffers that the weight-gradient products read: the kept rows rounded up
// to a multiple of 64, at least 256 (the grouped product's rule for per-group contraction lengths is 128, or 256
// where it fetches its rows through an index), at most Cp.
__device__ __forceinline__ int padded_rows(int count, int Cp) { return min(max((count + 63) & ~63, 256), Cp); }

// A 64 x 64 tile in LDS, stored [row][col] in the tensor's own element type.
template <typename T> struct Tile { T v[kTile][kTile + Elt<T>::kPad]; };

// Writes the transpose of the tile: dst[(c0 + c) * ld + r0 + r] = tile[r][c], 16 bytes per store,
// eight consecutive lanes on one output row.  Bounds: c0 + c < c_end, r0 + r < r_end (both multiples
// of the vector width away from the tile origin, so a vector is all in or all out).
template <typename T>
__device__ __forceinline__ void store_transposed(const Tile<T>& t, T* dst, size_t ld, int c0, int c_end, int r0, int r_end) {
    constexpr int V = Elt<T>::kVec, CH = kTile / V;            // chunks per output row
    for (int q = threadIdx.x; q < kTile * CH; q += kTileThreads) {
        const int c = q / CH, rc = (q % CH) * V;
        if (c0 + c >= c_end || r0 + rc >= r_end) continue;
        alignas(16) T out[V];
#pragma unroll
        for (int i = 0; i < V; ++i) out[i] = t.v[rc + i][c];
        *reinterpret_cast<uint4*>(dst + static_cast<size_t>(c0 + c) * ld + r0 + rc) = *reinterpret_cast<const uint4*>(out);
    }
}

// dst[b][c][col0 + r] = src[b][r][c]   for r < R, c < Cc   (dst rows have ld_dst elements; R, Cc, col0,
// ld_dst multiples of the 16-byte vector width)
template <typename T>
__global__ __launch_bounds__(kTileThreads) void transpose_kernel(const T* __restrict__ src, T* __restrict__ dst, int R,
                                                                 int Cc, int ld_dst, int col0) {
    __shared__ __attribute__((aligned(16))) Tile<T> tile;
    constexpr int V = Elt<T>::kVec, CH = kTile / V;
    const int b = blockIdx.z, r0 = blockIdx.y * kTile, c0 = blockIdx.x * kTile;
    const T* s = src + static_cast<size_t>(b) * R * Cc;
    T* d = dst + static_cast<size_t>(b) * Cc * ld_dst + col0;
    for (int q = threadIdx.x; q < kTile * CH; q += kTileThreads) {
        const int r = q / CH, cc = (q % CH) * V;
        if (r0 + r < R && c0 + cc < Cc) {
            const uint4 v = *reinterpret_cast<const uint4*>(s + static_cast<size_t>(r0 + r) * Cc + c0 + cc);
            const T* e = reinterpret_cast<const T*>(&v);
#pragma unroll
            for (int i = 0; i < V; ++i) tile.v[r][cc + i] = e[i];
        }
    }
    __syncthreads();
    store_transposed<T>(tile, d, ld_dst, c0, Cc, r0, R);
}

// dst[e][j][s] = src[slot_token[e][s]][j] (* gate[slot_token[e][s]][e])  for s < counts[e];
// zeros for counts[e] <= s < padded_rows(counts[e]); nothing beyond.
template <typename T, bool SCALE>
__global__ __launch_bounds__(kTileThreads) void gather_transpose_kernel(const T* __restrict__ src,
                                                                        const int32_t* __restrict__ slot_token,
                                                                        const int32_t* __restrict__ counts,
                                                                        const float* __restrict__ gate, T* __restrict__ dst,
                                                                        int T_, int d, int E, int C, int Cp) {
    __shared__ __attribute__((aligned(16))) Tile<T> tile;
    constexpr int V = Elt<T>::kVec, CH = kTile / V;
    const int e = blockIdx.z, s0 = blockIdx.y * kTile, j0 = blockIdx.x * kTile;
    const int count = min(counts[e], C);
    if (s0 >= padded_rows(count, Cp)) return;
    for (int q = threadIdx.x; q < kTile * CH; q += kTileThreads) {
        const int r = q / CH, cc = (q % CH) * V, s = s0 + r;
        float f[V];
#pragma unroll
        for (int i = 0; i < V; ++i) f[i] = 0.f;
        if (s < count && j0 + cc < d) {
            const int t = slot_token[static_cast<size_t>(e) * C + s];
            if (t >= 0 && t < T_) {
                Elt<T>::load_vec(src + static_cast<size_t>(t) * d + j0 + cc, f);
                if (SCALE) {
                    const float gt = gate[static_cast<size_t>(t) * E + e];
#pragma unroll
                    for (int i = 0; i < V; ++i) f[i] *= gt;
                }
            }
        }
#pragma unroll
        for (int i = 0; i < V; ++i) tile.v[r][cc + i] = Elt<T>::narrow(f[i]);
    }
    __syncthreads();
    store_transposed<T>(tile, dst + static_cast<size_t>(e) * d * Cp, Cp, j0, d, s0, Cp);
}

// Element-wise middle of the FFN backward for one 64 x 64 tile (buffer rows x hidden units) of one expert.
//   in : u, a, b [E][C][H];  gate through slot_token
//   out: dab [E][C][2H] = (da | db);  daT, dbT, hT [E][H][Cp];
//        dgate_part [H/64][E][C]: this tile's share of <u, h> per row (summed by dx_kernel in tile order)
// ROWS: no transposed copies; dab and h are [E][Cp][.] row-major with zero rows from counts[e] to padded_rows (the
// products that contract over the rows read them through transposing LDS reads); hT then is that row-major h.
// SCALE_H (with ROWS): hT holds gate * h, so that dW_down = dOut_p^T (gate h) needs no scaled copy of dOut's rows.
template <typename T, bool ROWS, bool SCALE_H = false>
__global__ __launch_bounds__(kTileThreads) void swiglu_backward_kernel(
    const T* __restrict__ u, const T* __restrict__ a, const T* __restrict__ b, const float* __restrict__ gate,
    const int32_t* __restrict__ slot_token, const int32_t* __restrict__ counts, T* __restrict__ dab, T* __restrict__ daT,
    T* __restrict__ dbT, T* __restrict__ hT, float* __restrict__ dgate_part, int T_, int E, int C, int Cp, int H) {
    __shared__ __attribute__((aligned(16))) Tile<T> th, ta, tb;
    constexpr int V = Elt<T>::kVec, CH = kTile / V;
    const size_t obase = static_cast<size_t>(blockIdx.z) * (ROWS ? Cp : C);     // first row of this expert in dab
    const int e = blockIdx.z, s0 = blockIdx.y * kTile, n0 = blockIdx.x * kTile;
    const int count = min(counts[e], C);
    if (s0 >= padded_rows(count, Cp)) return;
    const size_t ebase = static_cast<size_t>(e) * C;
    for (int q = threadIdx.x; q < kTile * CH; q += kTileThreads) {
        const int r = q / CH, cc = (q % CH) * V, s = s0 + r, n = n0 + cc;
        float hv[V], dav[V], dbv[V], dot = 0.f, g_row = 0.f;
#pragma unroll
        for (int i = 0; i < V; ++i) { hv[i] = 0.f; dav[i] = 0.f; dbv[i] = 0.f; }
        if (s < count && n < H) {
            const int t = slot_token[ebase + s];
            g_row = (t >= 0 && t < T_) ? gate[static_cast<size_t>(t) * E + e] : 0.f;
            const size_t idx = (ebase + s) * H + n;
            float uv[V], av[V], bv[V];
            Elt<T>::load_vec(u + idx, uv); Elt<T>::load_vec(a + idx, av); Elt<T>::load_vec(b + idx, bv);
#pragma unroll
            for (int i = 0; i < V; ++i) {
                const float sg = 1.0f / (1.0f + __expf(-av[i]));
                const float sl = av[i] * sg;
                hv[i] = sl * bv[i];
                const float dh = g_row * uv[i];
                dav[i] = dh * bv[i] * (sg * (1.0f + av[i] * (1.0f - sg)));
                dbv[i] = dh * sl;
                dot += uv[i] * hv[i];
            }
            if constexpr (!ROWS) {
                Elt<T>::store_vec(dab + (obase + s) * 2 * H + n, dav);
                Elt<T>::store_vec(dab + (obase + s) * 2 * H + H + n, dbv);
            }
        }
        if constexpr (ROWS) {
            if (s < Cp && n < H) {                                   // (s < padded_rows: the block starts below it)
                Elt<T>::store_vec(dab + (obase + s) * 2 * H + n, dav);
                Elt<T>::store_vec(dab + (obase + s) * 2 * H + H + n, dbv);
                if constexpr (SCALE_H) {
#pragma unroll
                    for (int i = 0; i < V; ++i) hv[i] *= g_row;
                }
                Elt<T>::store_vec(hT + (obase + s) * H + n, hv);
            }
        } else {
#pragma unroll
            for (int i = 0; i < V; ++i) {
                th.v[r][cc + i] = Elt<T>::narrow(hv[i]); ta.v[r][cc + i] = Elt<T>::narrow(dav[i]); tb.v[r][cc + i] = Elt<T>::narrow(dbv[i]);
            }
        }
        // the CH consecutive lanes of one row add up their shares (fixed order)
#pragma unroll
        for (int o = CH / 2; o > 0; o >>= 1) dot += __shfl_xor(dot, o, 64);
        if ((q % CH) == 0 && s < count)
            dgate_part[(static_cast<size_t>(blockIdx.x) * E + e) * C + s] = dot;
    }
    if constexpr (!ROWS) {
        __syncthreads();
        const size_t tb_off = static_cast<size_t>(e) * H * Cp;
        store_transposed<T>(th, hT + tb_off, Cp, n0, H, s0, Cp);
        store_transposed<T>(ta, daT + tb_off, Cp, n0, H, s0, Cp);
        store_transposed<T>(tb, dbT + tb_off, Cp, n0, H, s0, Cp);
    }
}

// dst[e][s][:] = src[slot_token[e][s]][:] (* gate[slot_token[e][s]][e]) for s < counts[e], zero rows from counts[e] to
// padded_rows; dst is [E][Cp][d].  One wavefront per row, 16 bytes per lane and access.
template <typename T, bool SCALE>
__global__ __launch_bounds__(256) void gather_rows_kernel(const T* __restrict__ src, const int32_t* __restrict__ slot_token,
                                                          const int32_t* __restrict__ counts, const float* __restrict__ gate,
                                                          T* __restrict__ dst, int T_, int d, int E, int C, int Cp) {
    constexpr int V = Elt<T>::kVec;
    const int lane = threadIdx.x & 63;
    const long long row = static_cast<long long>(blockIdx.x) * 4 + (threadIdx.x >> 6);
    if (row >= static_cast<long long>(E) * Cp) return;
    const int e = static_cast<int>(row / Cp), s = static_cast<int>(row - static_cast<long long>(e) * Cp);
    const int count = min(counts[e], C);
    if (s >= padded_rows(count, Cp)) return;
    int t = -1;
    float gt = 1.0f;
    if (s < count) {
        t = slot_token[static_cast<size_t>(e) * C + s];
        if (t < 0 || t >= T_) t = -1;
        else if (SCALE) gt = gate[static_cast<size_t>(t) * E + e];
    }
    T* out = dst + static_cast<size_t>(row) * d;
    for (int j = lane * V; j < d; j += 64 * V) {
        float f[V];
#pragma unroll
        for (int i = 0; i < V; ++i) f[i] = 0.f;
        if (t >= 0) {
            Elt<T>::load_vec(src + static_cast<size_t>(t) * d + j, f);
            if (SCALE) {
#pragma unroll
                for (int i = 0; i < V; ++i) f[i] *= gt;
            }
        }
        Elt<T>::store_vec(out + j, f);
    }
}

// Variant with renormalised weights: gate_eff[t][e] = gate[t][e] / (sum of gate[t][.] over the experts that kept t)
// for kept pairs, 0 otherwise.  One thread per token.
__global__ __launch_bounds__(256) void gate_eff_kernel(const float* __restrict__ gate, const int32_t* __restrict__ slot_of,
                                                       float* __restrict__ gate_eff, int T_, int E) {
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t >= T_) return;
    float sum = 0.f;
    for (int e = 0; e < E; ++e)
        if (slot_of[static_cast<size_t>(t) * E + e] >= 0) sum += gate[static_cast<size_t>(t) * E + e];
    const float inv = sum > 0.f ? 1.0f / sum : 0.f;
    for (int e = 0; e < E; ++e)
        gate_eff[static_cast<size_t>(t) * E + e] =
            slot_of[static_cast<size_t>(t) * E + e] >= 0 ? gate[static_cast<size_t>(t) * E + e] * inv : 0.f;
}

// dx[t] = sum_e dXp[e][slot_of[t][e]] + router term; one wavefront per token.
// Router term: dscore[e] = gate[e] (dgate[e] - sum_e' dgate[e'] gate[e']); with Eq. 4 in the form
//   FULL:   score = sqrt(D) <g, w> / (|x| |w|)  ->  d score / d x_j = sqrt(D) w[p(j)] / (D |x| |w|) - score x_j / |x|^2
//   POOLED: score = <g, w> / (|g| |w|)          ->  d score / d x_j = (w[p(j)] / (|g| |w|) - score g[p(j)] / |g|^2) / D
template <typename T>
__global__ __launch_bounds__(256) void dx_kernel(const T* __restrict__ x, const float* __restrict__ w_emb,
                                                 const float* __restrict__ score, const float* __restrict__ gate,
                                                 const int32_t* __restrict__ slot_of, const float* __restrict__ dgate_part, int n_part,
                                                 const T* __restrict__ dxp, T* __restrict__ dx, float* __restrict__ dgate_out,
                                                 float* __restrict__ dscore_out, int T_, int d, int E, int D, int C,
                                                 int cos_mode, int gate_norm, int Cx) {     // Cx: rows per expert of dxp
    extern __shared__ float sm[];
    const int P = d / D;
    float* w = sm;                       // [E][P]
    float* wn = w + E * P;               // [E] 1 / |w_e| (0 for a zero embedding)
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    float* g = wn + E + wave * (2 * P + 2 * E);   // per wave: g[P], v[P], ds[E], rows of the kept pairs (as int)[E]
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
    // softmax backward (E <= 64: lane e); its scattered reads are requested first and land while the row is walked
    float dg = 0.f, gt = 0.f, sc = 0.f;
    int slot = -1;
    if (lane < E) {
        slot = slot_of[static_cast<size_t>(t) * E + lane];
        gt = gate[static_cast<size_t>(t) * E + lane];
        sc = score[static_cast<size_t>(t) * E + lane];
        if (slot >= 0 && slot < C) {
            for (int i = 0; i < n_part; ++i) dg += dgate_part[(static_cast<size_t>(i) * E + lane) * C + slot];
        } else {
            slot = -1;
        }
    }
    // pooled features and norms
    float xx = 0.f, gg = 0.f;
    constexpr int VX = Elt<T>::kVec;
    const int LPG = D / VX;                                  // lanes that share a pooled group in the coalesced walk
    const bool row_walk = D % VX == 0 && LPG <= 64 && (LPG & (LPG - 1)) == 0 && d % (64 * VX) == 0;
    if (row_walk) {
        // the row in whole 16-byte pieces, lane after lane; the LPG neighbouring lanes of a group add up by swaps
        for (int c = lane; c < d / VX; c += 64) {
            float f[VX], s = 0.f;
            Elt<T>::load_vec(xr + static_cast<size_t>(c) * VX, f);
#pragma unroll
            for (int i = 0; i < VX; ++i) { s += f[i]; xx += f[i] * f[i]; }
            for (int o = 1; o < LPG; o <<= 1) s += __shfl_xor(s, o, 64);
            if ((lane & (LPG - 1)) == 0) {
                s /= D;
                g[c / LPG] = s; gg += s * s;
            }
        }
    }
    for (int p = lane; p < P && !row_walk; p += 64) {
        float s = 0.f;
        if (D % Elt<T>::kVec == 0) {
            for (int j = 0; j < D; j += Elt<T>::kVec) {
                float f[Elt<T>::kVec];
                Elt<T>::load_vec(xr + static_cast<size_t>(p) * D + j, f);
#pragma unroll
                for (int i = 0; i < Elt<T>::kVec; ++i) { s += f[i]; xx += f[i] * f[i]; }
            }
        } else {
            for (int j = 0; j < D; ++j) {
                const float xv = Elt<T>::load(xr, static_cast<size_t>(p) * D + j);
                s += xv; xx += xv * xv;
            }
        }
        s /= D;
        g[p] = s; gg += s * s;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) { xx += __shfl_xor(xx, o, 64); gg += __shfl_xor(gg, o, 64); }
    if (gate_norm) {
        // dg is the gradient of the renormalised weight g' = g / S (S = sum of g over the kept experts);
        // d / d g_e = (dg'_e - sum_kept dg'_i g'_i) / S for kept e, 0 otherwise
        float S = slot >= 0 ? gt : 0.f;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) S += __shfl_xor(S, o, 64);
        const float inv = S > 0.f ? 1.0f / S : 0.f;
        float m2 = slot >= 0 ? dg * gt * inv : 0.f;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) m2 += __shfl_xor(m2, o, 64);
        dg = slot >= 0 ? (dg - m2) * inv : 0.f;
    }
    float mix = dg * gt;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mix += __shfl_xor(mix, o, 64);
    const float dsv = gt * (dg - mix);
    float beta = dsv * sc;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) beta += __shfl_xor(beta, o, 64);
    // the token's kept pairs in ascending expert order, as rows of dxp (sl[i], i < n_kept)
    const uint64_t kept_mask = __ballot(slot >= 0);
    const int n_kept = __popcll(kept_mask);
    if (lane < E) {
        ds[lane] = dsv;
        if (slot >= 0) sl[__popcll(kept_mask & ((1ull << lane) - 1ull))] = lane * Cx + slot;
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
    constexpr int V = Elt<T>::kVec;
    for (int j = lane * V; j < d; j += 64 * V) {
        float acc[V], f[V];
        if (full) Elt<T>::load_vec(xr + j, f);
#pragma unroll
        for (int i = 0; i < V; ++i) {
            const int p = (j + i) / D;
            acc[i] = v[p] - cb * (full ? f[i] : g[p]);
        }
        // ascending expert order, as in the forward sum; four rows requested at a time (past the last kept pair the
        // last one is requested again and not added)
        for (int i0 = 0; i0 < n_kept; i0 += 4) {
            float r[4][V];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int row = sl[min(i0 + q, n_kept - 1)];
                Elt<T>::load_vec(dxp + static_cast<size_t>(row) * d + j, r[q]);
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                if (i0 + q < n_kept) {
#pragma unroll
                    for (int i = 0; i < V; ++i) acc[i] += r[q][i];
                }
            }
        }
        Elt<T>::store_vec(out + j, acc);
    }
}

struct BackwardWs {
    size_t wdT, wguT, a, b, u, dab, daT, dbT, hT, xpT, dypT, dxp, dgate_part, gate_eff, total;
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
    w.dab = take(E * Cp * 2 * H * es);
    w.daT = take(E * H * Cp * es);
    w.dbT = take(E * H * Cp * es);
    w.hT = take(E * H * Cp * es);
    w.xpT = take(E * d * Cp * es);
    w.dypT = take(E * d * Cp * es);
    w.dxp = take(E * Cp * d * es);
    w.dgate_part = take((H + kTile - 1) / kTile * E * C * 4);
    w.gate_eff = take(static_cast<size_t>(c.T) * E * 4);
    w.total = off;
    return w;
}

template <typename T>
hipError_t backward_impl(const etr_config& c, const void* x, const float* w_emb, const void* w_gate, const void* w_up,
                         const void* w_down, const float* score, const float* gate, const int32_t* slot_of,
                         const int32_t* slot_token, const int32_t* counts, const void* dout, void* dx, void* dw_gate,
                         void* dw_up, void* dw_down, float* dgate, float* dscore, void* ws, hipStream_t st,
                         const void* a_saved, const void* b_saved) {
    const BackwardWs L = backward_layout(c);
    char* base = static_cast<char*>(ws);
    auto at = [&](size_t off) { return reinterpret_cast<T*>(base + off); };
    const int E = c.E, C = c.capacity, H = c.H, d = c.d, Tn = c.T;
    const int Cp = (C + 63) / 64 * 64;
    const unsigned cd = (d + kTile - 1) / kTile, cH = (H + kTile - 1) / kTile, cC = Cp / kTile;
    hipError_t err;
#define ETR_BW(call) do { if ((err = (call)) != hipSuccess) return err; } while (0)
    // weights of Eq. 1 as the forward applied them
    const float* gate_w = gate;
    if (c.gate_norm) {
        float* ge = reinterpret_cast<float*>(base + L.gate_eff);
        hipLaunchKernelGGL(gate_eff_kernel, dim3((Tn + 255) / 256), dim3(256), 0, st, gate, slot_of, ge, Tn, E);
        gate_w = ge;
    }
    float* dgate_part = reinterpret_cast<float*>(base + L.dgate_part);
    const T* pre_a = static_cast<const T*>(a_saved);
    const T* pre_b = static_cast<const T*>(b_saved);
    if (!pre_a || !pre_b) {                              // nothing kept from the forward call: recompute
        GroupedGemm g1{x, w_gate, w_up, at(L.a), at(L.b), counts, nullptr, slot_token, E, C, H, d, 0, 0, Tn, GEMM_DUAL, c.dtype};
        ETR_BW(launch_grouped_gemm(g1, st));
        pre_a = at(L.a); pre_b = at(L.b);
    }

    // Direct path: the grouped product reads operands whose contraction index is the slow one through transposing
    // LDS reads, so neither the weights nor the per-row quantities are transposed in memory.
    //   u = dOut_p Wd (Wd as [d][H]);  dXp = (da|db) (Wg ; Wu) (two [H][d] halves of the contraction);
    //   dWd = dYp^T h;  dWg = da^T Xp;  dWu = db^T Xp  (contraction over the rows, all operands row-major)
    GroupedGemm t2{dout, w_down, nullptr, at(L.u), nullptr, counts, nullptr, slot_token, E, C, H, d, 0, H, Tn, GEMM_PLAIN, c.dtype};
    t2.tb = true;
    GroupedGemm t3{at(L.dab), w_gate, w_up, at(L.dxp), nullptr, counts, nullptr, nullptr, E, Cp, d, 2 * H, 0, d, Cp, GEMM_PLAIN, c.dtype};
    t3.tb = true;
    GroupedGemm t4{at(L.dypT), at(L.hT), nullptr, dw_down, nullptr, nullptr, counts, nullptr, E, d, H, Cp, d, H, d, GEMM_PLAIN, c.dtype};
    t4.ta = t4.tb = true;
    GroupedGemm t5{at(L.dab), at(L.xpT), nullptr, dw_gate, nullptr, nullptr, counts, nullptr, E, H, d, Cp, 2 * H, d, H, GEMM_PLAIN, c.dtype};
    t5.ta = t5.tb = true;
    GroupedGemm t6 = t5;
    t6.A = at(L.dab) + H; t6.C = dw_up;
    const bool direct = grouped_gemm_transposed_ok(t2) && grouped_gemm_transposed_ok(t3) && grouped_gemm_transposed_ok(t4) &&
                        grouped_gemm_transposed_ok(t5) && grouped_gemm_transposed_ok(t6);
    // The same three weight-gradient products with the rows of dOut and x fetched through slot_token by the
    // products themselves: dWd = dOut_p^T (gate h), dWg = da^T x_p, dWu = db^T x_p.  (da, db, h hold zeros from
    // counts[e] on, so whatever row an empty slot fetches is multiplied by zero.)
    GroupedGemm k4 = t4, k5 = t5, k6 = t6;
    k4.A = dout; k4.k_gather = 1; k5.B0 = x; k5.k_gather = 2; k6.B0 = x; k6.k_gather = 2;
    for (GroupedGemm* g : {&k4, &k5, &k6}) { g->k_index = slot_token; g->k_index_stride = C; g->k_rows = Tn; }
    // It pays where the copies are large: 8 experts x 32 000 rows, 23.0 -> 21.9 ms per call (the fetching products are
    // 3-8 % slower than the plain ones, the two copies cost 1.6 ms); 16-64 experts with 500-2000 rows each, equal or
    // 1.5 % slower.  As above, the capacity stands in for the row count.
    // dWg and dWu share x_p: one product with the 2H rows of (da | db)^T, its output rows split between the two
    // gradients (H = 1408: 11 whole row tiles instead of twice 5.5)
    GroupedGemm k56 = k5;
    k56.M = 2 * H; k56.a_rows = 2 * H; k56.C = dw_gate; k56.C2 = dw_up; k56.split_m = H;
    const bool both_gates = H % 32 == 0 && grouped_gemm_transposed_ok(k56);
    const bool fetch_rows = C >= 8192 && direct && grouped_gemm_transposed_ok(k4) && grouped_gemm_transposed_ok(k5) &&
                            grouped_gemm_transposed_ok(k6);
    int dxp_rows = C;
    if (direct) {
        // The two products whose only awkward operand is a weight matrix run faster on the row-major kernel with
        // that weight transposed once per call: the 64-wide row-major kernel sustains a tenth to a fifth more than
        // the transposing one.  The copy moves E*d*H elements, the product works on every kept row, so it pays
        // from a few thousand rows per expert on (8-expert workload, 32 000 rows per expert: the input-gradient
        // product 5.1 -> 4.7 ms for 0.08 ms of copies; 16 experts with 760 rows each: 0.43 ms of copies for less
        // than 0.1 ms).  The row count lives on the device; the capacity stands in for it.  The kernel wants at least
        // one whole 256-column tile of the output.
        const bool many_rows = C >= 8192;
        const bool nt_dxp = many_rows && d >= 256 && d % 8 == 0, nt_u = many_rows && H >= 256 && H % 8 == 0;
        if (nt_u) {
            hipLaunchKernelGGL(transpose_kernel<T>, dim3(cH, cd, E), dim3(kTileThreads), 0, st, static_cast<const T*>(w_down),
                               at(L.wdT), d, H, d, 0);
            ETR_BW(hipGetLastError());
            GroupedGemm g2{dout, at(L.wdT), nullptr, at(L.u), nullptr, counts, nullptr, slot_token, E, C, H, d, 0, 0, Tn, GEMM_PLAIN, c.dtype};
            ETR_BW(launch_grouped_gemm(g2, st));
        } else {
            ETR_BW(launch_grouped_gemm(t2, st));
        }
        if (fetch_rows) {
            hipLaunchKernelGGL((swiglu_backward_kernel<T, true, true>), dim3(cH, cC, E), dim3(kTileThreads), 0, st, at(L.u), pre_a,
                               pre_b, gate_w, slot_token, counts, at(L.dab), static_cast<T*>(nullptr), static_cast<T*>(nullptr),
                               at(L.hT), dgate_part, Tn, E, C, Cp, H);
        } else {
            hipLaunchKernelGGL((swiglu_backward_kernel<T, true>), dim3(cH, cC, E), dim3(kTileThreads), 0, st, at(L.u), pre_a, pre_b,
                               gate_w, slot_token, counts, at(L.dab), static_cast<T*>(nullptr), static_cast<T*>(nullptr), at(L.hT),
                               dgate_part, Tn, E, C, Cp, H);
            const unsigned row_blocks = static_cast<unsigned>((static_cast<long long>(E) * Cp + 3) / 4);
            hipLaunchKernelGGL((gather_rows_kernel<T, false>), dim3(row_blocks), dim3(256), 0, st, static_cast<const T*>(x),
                               slot_token, counts, gate, at(L.xpT), Tn, d, E, C, Cp);
            hipLaunchKernelGGL((gather_rows_kernel<T, true>), dim3(row_blocks), dim3(256), 0, st, static_cast<const T*>(dout),
                               slot_token, counts, gate_w, at(L.dypT), Tn, d, E, C, Cp);
        }
        ETR_BW(hipGetLastError());
        if (nt_dxp) {
            hipLaunchKernelGGL(transpose_kernel<T>, dim3(cd, cH, E), dim3(kTileThreads), 0, st, static_cast<const T*>(w_gate),
                               at(L.wguT), H, d, 2 * H, 0);
            hipLaunchKernelGGL(transpose_kernel<T>, dim3(cd, cH, E), dim3(kTileThreads), 0, st, static_cast<const T*>(w_up),
                               at(L.wguT), H, d, 2 * H, H);
            ETR_BW(hipGetLastError());
            GroupedGemm g3{at(L.dab), at(L.wguT), nullptr, at(L.dxp), nullptr, counts, nullptr, nullptr, E, Cp, d, 2 * H, 0, 0, Cp, GEMM_PLAIN, c.dtype};
            ETR_BW(launch_grouped_gemm(g3, st));
        } else {
            ETR_BW(launch_grouped_gemm(t3, st));
        }
        ETR_BW(launch_grouped_gemm(fetch_rows ? k4 : t4, st));
        if (fetch_rows && both_gates) {
            ETR_BW(launch_grouped_gemm(k56, st));
        } else {
            ETR_BW(launch_grouped_gemm(fetch_rows ? k5 : t5, st));
            ETR_BW(launch_grouped_gemm(fetch_rows ? k6 : t6, st));
        }
        dxp_rows = Cp;
    } else {
        // Fallback (fp32, or shapes the transposing kernel does not take): every product on the "NT" kernel, with
        // the weights transposed once per call and transposed copies of the per-row quantities.
        // WdT[e][H][d], WguT[e][d][2H] = (Wg^T | Wu^T)
        hipLaunchKernelGGL(transpose_kernel<T>, dim3(cH, cd, E), dim3(kTileThreads), 0, st, static_cast<const T*>(w_down),
                           at(L.wdT), d, H, d, 0);
        hipLaunchKernelGGL(transpose_kernel<T>, dim3(cd, cH, E), dim3(kTileThreads), 0, st, static_cast<const T*>(w_gate),
                           at(L.wguT), H, d, 2 * H, 0);
        hipLaunchKernelGGL(transpose_kernel<T>, dim3(cd, cH, E), dim3(kTileThreads), 0, st, static_cast<const T*>(w_up),
                           at(L.wguT), H, d, 2 * H, H);
        ETR_BW(hipGetLastError());
        GroupedGemm g2{dout, at(L.wdT), nullptr, at(L.u), nullptr, counts, nullptr, slot_token, E, C, H, d, 0, 0, Tn, GEMM_PLAIN, c.dtype};
        ETR_BW(launch_grouped_gemm(g2, st));
        hipLaunchKernelGGL((swiglu_backward_kernel<T, false>), dim3(cH, cC, E), dim3(kTileThreads), 0, st, at(L.u), pre_a, pre_b,
                           gate_w, slot_token, counts, at(L.dab), at(L.daT), at(L.dbT), at(L.hT), dgate_part, Tn, E, C, Cp, H);
        hipLaunchKernelGGL((gather_transpose_kernel<T, false>), dim3(cd, cC, E), dim3(kTileThreads), 0, st,
                           static_cast<const T*>(x), slot_token, counts, gate, at(L.xpT), Tn, d, E, C, Cp);
        hipLaunchKernelGGL((gather_transpose_kernel<T, true>), dim3(cd, cC, E), dim3(kTileThreads), 0, st,
                           static_cast<const T*>(dout), slot_token, counts, gate_w, at(L.dypT), Tn, d, E, C, Cp);
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
    }
    const int P = d / c.D;
    const size_t lds = (static_cast<size_t>(E) * P + E + 4 * (2 * P + 2 * E)) * 4;
    auto kern = dx_kernel<T>;
    ETR_BW(ensure_dynamic_lds(reinterpret_cast<const void*>(kern), lds));
    hipLaunchKernelGGL(kern, dim3((Tn + 3) / 4), dim3(256), lds, st, static_cast<const T*>(x), w_emb, score, gate, slot_of,
                       dgate_part, static_cast<int>(cH), at(L.dxp), static_cast<T*>(dx), dgate, dscore,
                       Tn, d, E, c.D, C, static_cast<int>(c.cos), static_cast<int>(c.gate_norm), dxp_rows);
#undef ETR_BW
    return hipGetLastError();
}

}  // namespace

size_t backward_ws_bytes(const etr_config& c) { return backward_layout(c).total; }

hipError_t launch_moe_backward(const etr_config& c, const void* x, const float* w_emb, const void* w_gate,
                               const void* w_up, const void* w_down, const float* score, const float* gate,
                               const int32_t* slot_of, const int32_t* slot_token, const int32_t* counts,
                               const void* dout, void* dx, void* dw_gate, void* dw_up, void* dw_down, float* dgate,
                               float* dscore, void* ws, hipStream_t st, const void* a_saved, const void* b_saved) {
    if (static_cast<size_t>(c.E) * (c.d / c.D) * 4 > 120 * 1024) return hipErrorInvalidValue;   // embeddings must fit in LDS
    if (c.dtype == ETR_BF16)
        return backward_impl<uint16_t>(c, x, w_emb, w_gate, w_up, w_down, score, gate, slot_of, slot_token, counts, dout,
                                       dx, dw_gate, dw_up, dw_down, dgate, dscore, ws, st, a_saved, b_saved);
    return backward_impl<float>(c, x, w_emb, w_gate, w_up, w_down, score, gate, slot_of, slot_token, counts, dout, dx,
                                dw_gate, dw_up, dw_down, dgate, dscore, ws, st, a_saved, b_saved);
}

}  // namespace etr
