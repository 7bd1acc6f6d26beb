// Expert networks on the kept rows: yp = W_down (SiLU(W_gate x) .* (W_up x)), one SwiGLU
// feed-forward block per expert (Sec. Locality Loss: experts are FFN layers; Sec.
// Experimental Setup: Mixtral experts).  This is the one dense contraction of the layer
// and the operator the paper reports as dominant ("FFN MatMul").
//
// bf16: two grouped "NT" GEMMs on the MFMA units (v_mfma_f32_32x32x16_bf16), fp32
// accumulation.  Both operands are K-contiguous, staged through LDS in 16-byte chunks
// with an XOR swizzle, double-buffered.  GEMM-1 computes the gate and the up projection
// of the same output tile so that SiLU(g)*u is its epilogue and the hidden activation
// crosses HBM once, in bf16.  The grid is sized for `capacity`; a workgroup whose row
// tile starts past counts[e] exits at once, so counts never leave the device.
// fp32: plain LDS-tiled FMA kernels (parity path for small layers).
#include "etr_internal.h"

namespace etr {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

struct GemmParams {
    const void* A;        // [E][capacity][K]
    const void* B0;       // [E][N][K]
    const void* B1;       // [E][N][K] (GLU only)
    void* C;              // [E][capacity][N]
    const int32_t* counts;
    int E, capacity, N, K;
    int MT, NT;           // row tiles per expert, column tiles
};

__device__ __forceinline__ uint32_t f2bf(float f) {            // fp32 -> bf16 bits, round to nearest even
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return 0x7FC0u;
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

__device__ __forceinline__ float silu(float a) { return a / (1.0f + __expf(-a)); }

// Workgroup -> (expert, column tile, row tile).  Hardware deals consecutive workgroups
// round-robin to the 8 XCDs, each with its own L2: a "band" = all row tiles of one
// (expert, column tile) shares one weight tile, so a whole band goes to one XCD, row tile
// fastest, and the weight tile is fetched from HBM once.
__device__ __forceinline__ bool decode_tile(const GemmParams& p, int& e, int& mt, int& nt) {
    const int pid = blockIdx.x;
    const int xcd = pid & 7, j = pid >> 3;
    const int band = (j / p.MT) * 8 + xcd;
    mt = j % p.MT;
    if (band >= p.E * p.NT) return false;
    e = band / p.NT;
    nt = band - e * p.NT;
    return true;
}

// ---------------------------------------------------------------------------------------
// bf16 MFMA grouped GEMM:  C[e][m][n] = sum_k A[e][m][k] * B[e][n][k]   (+ SwiGLU epilogue)
// ---------------------------------------------------------------------------------------
template <int BM, int BN, int BK, int WGM, int WGN, bool GLU, int SWZ>
__global__ __launch_bounds__(WGM* WGN * 64) void gemm_bf16_kernel(GemmParams p) {
    constexpr int NTH = WGM * WGN * 64;
    constexpr int BROWS = GLU ? 2 * BN : BN;       // weight rows staged per tile
    constexpr int CPR = BK / 8;                    // 16-byte chunks per tile row
    constexpr int WTM = BM / WGM, WTN = BN / WGN;  // per-wave output tile
    constexpr int TM = WTM / 32, TN = WTN / 32;    // 32x32 MFMA blocks per wave
    constexpr int NB = GLU ? 2 : 1;
    constexpr int A_CH = BM * CPR / NTH, B_CH = BROWS * CPR / NTH;
    static_assert(BM * CPR % NTH == 0 && BROWS * CPR % NTH == 0, "tile must divide over the threads");
    static_assert(WTM % 32 == 0 && WTN % 32 == 0 && BK % 16 == 0, "MFMA shape");

    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    uint4* As = reinterpret_cast<uint4*>(lds_raw);                  // [2][BM][CPR]
    uint4* Bs = As + 2 * BM * CPR;                                  // [2][BROWS][CPR]

    int e, mt, nt;
    if (!decode_tile(p, e, mt, nt)) return;
    const int count = min(p.counts[e], p.capacity);
    const int m0 = mt * BM, n0 = nt * BN;
    if (m0 >= count) return;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave / WGN) * WTM, wn0 = (wave % WGN) * WTN;
    const int K = p.K;
    const uint4* Ag = reinterpret_cast<const uint4*>(p.A) + static_cast<size_t>(e) * p.capacity * (K / 8);
    const uint4* B0g = reinterpret_cast<const uint4*>(p.B0) + static_cast<size_t>(e) * p.N * (K / 8);
    const uint4* B1g = GLU ? reinterpret_cast<const uint4*>(p.B1) + static_cast<size_t>(e) * p.N * (K / 8) : nullptr;

    // per-thread staging slots: chunk q -> (row, ck)
    const uint4* a_src[A_CH];
    const uint4* b_src[B_CH];
    int a_dst[A_CH], b_dst[B_CH], a_ck[A_CH], b_ck[B_CH];
#pragma unroll
    for (int i = 0; i < A_CH; ++i) {
        const int q = tid + i * NTH, row = q / CPR, ck = q % CPR;
        int m = m0 + row;
        m = m < p.capacity ? m : p.capacity - 1;                   // stay inside the buffer; such rows are never stored
        a_src[i] = Ag + static_cast<size_t>(m) * (K / 8) + ck;
        a_dst[i] = row * CPR + (ck ^ ((row >> SWZ) & (CPR - 1)));
        a_ck[i] = ck;
    }
#pragma unroll
    for (int i = 0; i < B_CH; ++i) {
        const int q = tid + i * NTH, row = q / CPR, ck = q % CPR;
        const bool up = GLU && row >= BN;
        int n = n0 + (up ? row - BN : row);
        n = n < p.N ? n : p.N - 1;
        b_src[i] = (up ? B1g : B0g) + static_cast<size_t>(n) * (K / 8) + ck;
        b_dst[i] = row * CPR + (ck ^ ((row >> SWZ) & (CPR - 1)));
        b_ck[i] = ck;
    }

    f32x16 acc[NB][TM][TN];
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[b][i][j][v] = 0.f;

    uint4 ra[A_CH], rb[B_CH];
    const int KC = K / 8;                          // chunks per full row
    auto load_global = [&](int kt) {
        const int kc0 = kt * CPR;
#pragma unroll
        for (int i = 0; i < A_CH; ++i)
            ra[i] = (kc0 + a_ck[i] < KC) ? a_src[i][kc0] : make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
        for (int i = 0; i < B_CH; ++i)
            rb[i] = (kc0 + b_ck[i] < KC) ? b_src[i][kc0] : make_uint4(0u, 0u, 0u, 0u);
    };
    auto store_lds = [&](int buf) {
#pragma unroll
        for (int i = 0; i < A_CH; ++i) As[buf * BM * CPR + a_dst[i]] = ra[i];
#pragma unroll
        for (int i = 0; i < B_CH; ++i) Bs[buf * BROWS * CPR + b_dst[i]] = rb[i];
    };

    const int KT = (K + BK - 1) / BK;
    load_global(0);
    store_lds(0);
    __syncthreads();

    const int r32 = lane & 31, half = lane >> 5;
    for (int kt = 0; kt < KT; ++kt) {
        const int cur = kt & 1;
        if (kt + 1 < KT) load_global(kt + 1);
        const uint4* Ab = As + cur * BM * CPR;
        const uint4* Bb = Bs + cur * BROWS * CPR;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            const int ck = ks * 2 + half;
            bf16x8 af[TM], bfr[NB][TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const int row = wm0 + i * 32 + r32;
                af[i] = __builtin_bit_cast(bf16x8, Ab[row * CPR + (ck ^ ((row >> SWZ) & (CPR - 1)))]);
            }
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const int row = b * BN + wn0 + j * 32 + r32;
                    bfr[b][j] = __builtin_bit_cast(bf16x8, Bb[row * CPR + (ck ^ ((row >> SWZ) & (CPR - 1)))]);
                }
            // D[n][m] += W[n][k] * X[m][k]: the weight fragment is the row operand, so a lane
            // ends up with 4 consecutive output columns n of one row m (8-byte stores).
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[b][i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[b][j], af[i], acc[b][i][j], 0, 0, 0);
        }
        if (kt + 1 < KT) store_lds(cur ^ 1);
        __syncthreads();
    }

    // epilogue: lane holds, per 32x32 block, row m = lane%32 and columns (v/4)*8 + (lane/32)*4 + v%4
    uint16_t* Cg = reinterpret_cast<uint16_t*>(p.C) + static_cast<size_t>(e) * p.capacity * p.N;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int m = m0 + wm0 + i * 32 + r32;
        if (m >= count) continue;
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int n = n0 + wn0 + j * 32 + q * 8 + half * 4;
                if (n >= p.N) continue;
                float o[4];
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    if constexpr (GLU) o[v] = silu(acc[0][i][j][q * 4 + v]) * acc[1][i][j][q * 4 + v];
                    else o[v] = acc[0][i][j][q * 4 + v];
                }
                uint2 pk = make_uint2(f2bf(o[0]) | (f2bf(o[1]) << 16), f2bf(o[2]) | (f2bf(o[3]) << 16));
                *reinterpret_cast<uint2*>(Cg + static_cast<size_t>(m) * p.N + n) = pk;
            }
    }
}

// ---------------------------------------------------------------------------------------
// fp32 grouped GEMM, 64x64 tile, 4x4 outputs per thread, plain FMA
// ---------------------------------------------------------------------------------------
template <bool GLU>
__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmParams p) {
    constexpr int BM = 64, BN = 64, BK = 16, LD = BM + 4;
    __shared__ float As[BK][LD];
    __shared__ float Bs[GLU ? 2 : 1][BK][LD];
    int e, mt, nt;
    if (!decode_tile(p, e, mt, nt)) return;
    const int count = min(p.counts[e], p.capacity);
    const int m0 = mt * BM, n0 = nt * BN;
    if (m0 >= count) return;
    const int tid = threadIdx.x, K = p.K;
    const float* Ag = static_cast<const float*>(p.A) + static_cast<size_t>(e) * p.capacity * K;
    const float* B0g = static_cast<const float*>(p.B0) + static_cast<size_t>(e) * p.N * K;
    const float* B1g = GLU ? static_cast<const float*>(p.B1) + static_cast<size_t>(e) * p.N * K : nullptr;
    const int lr = tid >> 2, lk = (tid & 3) * 4;                  // staging: row, k offset
    const int am = min(m0 + lr, p.capacity - 1), bn = min(n0 + lr, p.N - 1);
    const int ty = tid >> 4, tx = tid & 15;
    float acc[GLU ? 2 : 1][4][4] = {};
    for (int k0 = 0; k0 < K; k0 += BK) {
        const bool kin = k0 + lk < K;                             // K % 4 == 0: a float4 is all in or all out
        const float4 z = make_float4(0.f, 0.f, 0.f, 0.f);
        float4 va = kin ? *reinterpret_cast<const float4*>(Ag + static_cast<size_t>(am) * K + k0 + lk) : z;
        float4 vb = kin ? *reinterpret_cast<const float4*>(B0g + static_cast<size_t>(bn) * K + k0 + lk) : z;
        As[lk + 0][lr] = va.x; As[lk + 1][lr] = va.y; As[lk + 2][lr] = va.z; As[lk + 3][lr] = va.w;
        Bs[0][lk + 0][lr] = vb.x; Bs[0][lk + 1][lr] = vb.y; Bs[0][lk + 2][lr] = vb.z; Bs[0][lk + 3][lr] = vb.w;
        if constexpr (GLU) {
            float4 vc = kin ? *reinterpret_cast<const float4*>(B1g + static_cast<size_t>(bn) * K + k0 + lk) : z;
            Bs[1][lk + 0][lr] = vc.x; Bs[1][lk + 1][lr] = vc.y; Bs[1][lk + 2][lr] = vc.z; Bs[1][lk + 3][lr] = vc.w;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < BK; ++k) {
            const float4 a = *reinterpret_cast<const float4*>(&As[k][ty * 4]);
            const float av[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
            for (int b = 0; b < (GLU ? 2 : 1); ++b) {
                const float4 w = *reinterpret_cast<const float4*>(&Bs[b][k][tx * 4]);
                const float wv[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[b][i][j] = fmaf(av[i], wv[j], acc[b][i][j]);
            }
        }
        __syncthreads();
    }
    float* Cg = static_cast<float*>(p.C) + static_cast<size_t>(e) * p.capacity * p.N;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = m0 + ty * 4 + i;
        if (m >= count) continue;
        const int n = n0 + tx * 4;
        if (n >= p.N) continue;                                   // N % 4 == 0
        float o[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if constexpr (GLU) {
                const float g = acc[0][i][j];
                o[j] = g / (1.0f + expf(-g)) * acc[1][i][j];
            } else {
                o[j] = acc[0][i][j];
            }
        }
        *reinterpret_cast<float4*>(Cg + static_cast<size_t>(m) * p.N + n) = make_float4(o[0], o[1], o[2], o[3]);
    }
}

template <int BM, int BN, int BK, int WGM, int WGN, bool GLU, int SWZ>
hipError_t launch_bf16(GemmParams p, hipStream_t st) {
    constexpr int BROWS = GLU ? 2 * BN : BN;
    constexpr size_t lds = 2ull * (BM + BROWS) * BK * 2;
    p.MT = (p.capacity + BM - 1) / BM;
    p.NT = (p.N + BN - 1) / BN;
    const long long bands = static_cast<long long>(p.E) * p.NT;
    const long long blocks = (bands + 7) / 8 * 8 * p.MT;
    auto kern = gemm_bf16_kernel<BM, BN, BK, WGM, WGN, GLU, SWZ>;
    if (lds > 64 * 1024) {
        hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
        if (err != hipSuccess) return err;
    }
    hipLaunchKernelGGL(kern, dim3(static_cast<unsigned>(blocks)), dim3(WGM * WGN * 64), lds, st, p);
    return hipGetLastError();
}

template <bool GLU>
hipError_t launch_f32(GemmParams p, hipStream_t st) {
    p.MT = (p.capacity + 63) / 64;
    p.NT = (p.N + 63) / 64;
    const long long bands = static_cast<long long>(p.E) * p.NT;
    const long long blocks = (bands + 7) / 8 * 8 * p.MT;
    hipLaunchKernelGGL(gemm_f32_kernel<GLU>, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, st, p);
    return hipGetLastError();
}

}  // namespace

size_t ffn_ws_bytes(const etr_config& c) {
    return align_up(static_cast<size_t>(c.E) * c.capacity * c.H * elt_bytes(c.dtype));
}

hipError_t launch_expert_ffn(const etr_config& c, const void* xp, const int32_t* counts, const void* w_gate,
                             const void* w_up, const void* w_down, void* yp, void* hidden, hipStream_t st,
                             hipEvent_t between) {
    GemmParams g1{xp, w_gate, w_up, hidden, counts, c.E, c.capacity, c.H, c.d, 0, 0};
    GemmParams g2{hidden, w_down, nullptr, yp, counts, c.E, c.capacity, c.d, c.H, 0, 0};
    hipError_t err;
    if (c.dtype == ETR_BF16) {
        err = launch_bf16<128, 64, 64, 2, 2, true, 0>(g1, st);
        if (err != hipSuccess) return err;
        if (between && (err = hipEventRecord(between, st)) != hipSuccess) return err;
        return launch_bf16<128, 128, 64, 2, 2, false, 0>(g2, st);
    }
    err = launch_f32<true>(g1, st);
    if (err != hipSuccess) return err;
    if (between && (err = hipEventRecord(between, st)) != hipSuccess) return err;
    return launch_f32<false>(g2, st);
}

}  // namespace etr
