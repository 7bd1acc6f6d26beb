// Expert networks on the kept rows: yp = W_down (SiLU(W_gate x) .* (W_up x)), one SwiGLU
// feed-forward block per expert (Sec. Locality Loss: experts are FFN layers; Sec.
// Experimental Setup: Mixtral experts).  This is the one dense contraction of the layer
// and the operator the paper reports as dominant ("FFN MatMul").
//
// bf16: two grouped "NT" GEMMs on the MFMA units (v_mfma_f32_16x16x32_bf16 in the persistent
// kernel the layer launches, v_mfma_f32_32x32x16_bf16 in the other forms), fp32
// accumulation.  Both operands are K-contiguous, staged through LDS in 16-byte chunks
// with an XOR swizzle, double-buffered.  GEMM-1 computes the gate and the up projection
// of the same output tile so that SiLU(g)*u is its epilogue and the hidden activation
// crosses HBM once, in bf16.  The kernel the layer launches is the persistent one
// (gemm_bf16_persistent_kernel: one workgroup per CU walks the live tiles, the copies run on
// across tile boundaries); the per-tile kernels size the grid for `capacity` and a workgroup
// whose row tile starts past counts[e] exits at once.  Either way counts never leave the device.
// fp32: plain LDS-tiled FMA kernels (parity path for small layers).

#include "etr_internal.h"

namespace etr {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

struct GemmParams {
    const void* A;        // [E][capacity][K]
    const void* B0;       // [E][N][K]
    const void* B1;       // [E][N][K] (GLU only)
    void* C;              // [E][capacity][N]
    const int32_t* counts;
    int E, capacity, N, K;
    int MT, NT;           // row tiles per expert, column tiles
    int SM, SN;           // super-tile shape (see decode_tile)
    const int32_t* row_index;   // optional [E][capacity]: A row m of expert e is row row_index[e][m] of A
    int a_rows;                 // rows of A that row_index may name (indices are clamped into [0, a_rows))
    int lda = 0, ldb = 0;       // row strides of A and B in elements (0: K)
    const int32_t* k_counts = nullptr;   // optional per-group contraction length; it is rounded up to a multiple
                                         // of 64, at least 128 (at most K), and the operands must hold zeros in
                                         // that padding
    void* C2 = nullptr;         // DUAL epilogue: the B1 product goes here, the B0 product to C, no activation
    void* C3 = nullptr;         // SwiGLU epilogue that also keeps the two products: B0 product to C2, B1 product to C3
    // Contraction rows fetched through an index (transposing kernel only; k_gather 1: A, 2: B0): row k of group g of
    // that operand is row k_index[g * k_index_stride + min(k, k_index_stride - 1)] of a [k_rows][ld] matrix, clamped
    // into [0, k_rows).  The per-group contraction length is then at least 256.
    const int32_t* k_index = nullptr;
    int k_index_stride = 0, k_rows = 0, k_gather = 0;
    // Plain epilogue of the transposing kernel with the output rows split between two arrays: rows below split_m go
    // to C, the others (as rows m - split_m) to C2, both [E][split_m][N] (a multiple of 32, capacity = 2 split_m).
    int split_m = 0;
};

// rows of group e (counts may be absent: every group has `capacity` rows) and its contraction length
__device__ __forceinline__ int group_rows(const GemmParams& p, int e) {
    return p.counts ? min(p.counts[e], p.capacity) : p.capacity;
}
__device__ __forceinline__ int group_k(const GemmParams& p, int e) {
    return p.k_counts ? min(max((max(p.k_counts[e], 0) + 63) & ~63, p.k_gather ? 256 : 128), p.K) : p.K;
}

// Two fp32 values -> packed bf16 pair, round to nearest even (v_cvt_pk_bf16_f32).
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    typedef __attribute__((ext_vector_type(2))) float f32x2;
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
__device__ __forceinline__ uint2 pack_bf16x4(float a, float b, float c, float d) {
    return make_uint2(pack_bf16(a, b), pack_bf16(c, d));
}

// SiLU(a) = a / (1 + exp(-a)) with the hardware exponential and reciprocal (about 1 ulp each; the result
// is rounded to bf16 right after)
__device__ __forceinline__ float silu(float a) {
    return a * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.44269504088896341f * a));
}

// Epilogue shared by the MFMA kernels.  acc[i][j] is the 32 x 32 block at rows m_base + 32 i, staged weight rows
// 32 j of this wave (GLU: the first TB/2 blocks are gate rows, the others the up rows of the same output columns).
// A lane holds, per block, row m = lane % 32 and the columns (v / 4) * 8 + (lane / 32) * 4 + v % 4, so every store is
// four consecutive bf16 of one row.
// KEEP (SwiGLU epilogue only): the two products are stored as well (C2, C3), for the training-mode forward.
template <bool GLU, bool DUAL, int TI, int TB, bool KEEP = false>
__device__ __forceinline__ void store_blocks(const GemmParams& p, const f32x16 (&acc)[TI][TB], int e, int m_base,
                                             int n_base, int count, int r32, int half) {
    constexpr int TO = GLU ? TB / 2 : TB;
    uint16_t* Cg = reinterpret_cast<uint16_t*>(p.C) + static_cast<size_t>(e) * p.capacity * p.N;
    uint16_t* C2g = (GLU && (DUAL || KEEP)) ? reinterpret_cast<uint16_t*>(p.C2) + static_cast<size_t>(e) * p.capacity * p.N : nullptr;
    uint16_t* C3g = (GLU && !DUAL && KEEP) ? reinterpret_cast<uint16_t*>(p.C3) + static_cast<size_t>(e) * p.capacity * p.N : nullptr;
#pragma unroll
    for (int i = 0; i < TI; ++i) {
        const int m = m_base + i * 32 + r32;
        if (m >= count) continue;
#pragma unroll
        for (int j = 0; j < TO; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int n = n_base + j * 32 + q * 8 + half * 4;
                if (n >= p.N) continue;
                const size_t o = static_cast<size_t>(m) * p.N + n;
                const f32x16& g0 = acc[i][j];
                if constexpr (GLU) {
                    const f32x16& g1 = acc[i][TO + j];
                    if constexpr (DUAL) {                           // both products, no activation
                        *reinterpret_cast<uint2*>(Cg + o) = pack_bf16x4(g0[q * 4], g0[q * 4 + 1], g0[q * 4 + 2], g0[q * 4 + 3]);
                        *reinterpret_cast<uint2*>(C2g + o) = pack_bf16x4(g1[q * 4], g1[q * 4 + 1], g1[q * 4 + 2], g1[q * 4 + 3]);
                    } else {
                        *reinterpret_cast<uint2*>(Cg + o) =
                            pack_bf16x4(silu(g0[q * 4]) * g1[q * 4], silu(g0[q * 4 + 1]) * g1[q * 4 + 1],
                                        silu(g0[q * 4 + 2]) * g1[q * 4 + 2], silu(g0[q * 4 + 3]) * g1[q * 4 + 3]);
                        if constexpr (KEEP) {                       // keep the pre-activations (training-mode forward)
                            *reinterpret_cast<uint2*>(C2g + o) = pack_bf16x4(g0[q * 4], g0[q * 4 + 1], g0[q * 4 + 2], g0[q * 4 + 3]);
                            *reinterpret_cast<uint2*>(C3g + o) = pack_bf16x4(g1[q * 4], g1[q * 4 + 1], g1[q * 4 + 2], g1[q * 4 + 3]);
                        }
                    }
                } else {
                    uint16_t* dst = Cg + o;
                    if (p.split_m) {
                        const bool second = m >= p.split_m;
                        dst = reinterpret_cast<uint16_t*>(second ? p.C2 : p.C) +
                              (static_cast<size_t>(e) * p.split_m + (second ? m - p.split_m : m)) * p.N + n;
                    }
                    *reinterpret_cast<uint2*>(dst) = pack_bf16x4(g0[q * 4], g0[q * 4 + 1], g0[q * 4 + 2], g0[q * 4 + 3]);
                }
            }
        __builtin_amdgcn_sched_barrier(0);               // one row of blocks at a time: keeps the live set small
    }
}

// Workgroup -> (expert, row tile, column tile).  Hardware deals consecutive workgroups round-robin
// to the 8 XCDs, each with its own 4 MiB L2 and 32 CUs.  Tiles are grouped into "super-tiles" of
// SM row tiles x SN column tiles (SM*SN = 32 = the workgroups that run together on one XCD); a whole
// super-tile goes to one XCD, so while its 32 workgroups stream along K together every token-row
// slice is shared by SN of them and every weight slice by SM of them through that XCD's L2.
__device__ __forceinline__ bool decode_tile(const GemmParams& p, int& e, int& mt, int& nt) {
    const int pid = blockIdx.x;
    const int xcd = pid & 7, j = pid >> 3;
    const int per = p.SM * p.SN;
    const int sidx = (j / per) * 8 + xcd, l = j % per;
    const int MG = (p.MT + p.SM - 1) / p.SM, NG = (p.NT + p.SN - 1) / p.SN;
    if (sidx >= p.E * MG * NG) return false;
    e = sidx / (MG * NG);
    const int r = sidx - e * (MG * NG);
    mt = (r % MG) * p.SM + l % p.SM;
    nt = (r / MG) * p.SN + l / p.SM;
    return mt < p.MT && nt < p.NT;
}

// Fills MT, NT and the super-tile shape; returns the number of workgroups to launch.
// `wide`: the persistent kernel with 64-wide k-tiles, where a group has many row tiles (the 8-expert workload: 141):
// 8 row tiles x 4 column tiles, except where a row of column tiles is short and not a multiple of 4 (the 11 column
// tiles of that workload's gate/up product): then all of them in one super-tile, 2 x 11, so that no column group
// is left ragged.  Same box, whole layer: 7.42 -> 7.36 ms.  With 4-8 row tiles per group 4 x 8 stays (8 x 4 was
// 1 % slower there); 1 x 32 and 16 x 2 lose 3-8 % everywhere.
inline long long plan_tiles(GemmParams& p, int BM, int BN, bool wide = false) {
    p.MT = (p.capacity + BM - 1) / BM;
    p.NT = (p.N + BN - 1) / BN;
    if (wide && p.MT >= 16) {
        if (p.NT % 4 != 0 && p.NT <= 16) { p.SN = p.NT; p.SM = 32 / p.NT > 0 ? 32 / p.NT : 1; }
        else { p.SM = 8; p.SN = 4; }
        if (p.SM > p.MT) p.SM = p.MT;
    } else {
        p.SM = p.MT < 4 ? p.MT : 4;
        p.SN = 32 / p.SM;
    }
    if (p.SN > p.NT) p.SN = p.NT;
    const long long MG = (p.MT + p.SM - 1) / p.SM, NG = (p.NT + p.SN - 1) / p.SN;
    const long long supers = static_cast<long long>(p.E) * MG * NG;
    return (supers + 7) / 8 * 8 * (p.SM * p.SN);
}

// ---------------------------------------------------------------------------------------
// bf16 MFMA grouped GEMM:  C[e][m][n] = sum_k A[e][m][k] * B[e][n][k]   (+ SwiGLU epilogue)
// ---------------------------------------------------------------------------------------
template <int BM, int BN, int BK, int WGM, int WGN, bool GLU, int SWZ, bool DUAL = false>
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
    const int count = group_rows(p, e);
    const int m0 = mt * BM, n0 = nt * BN;
    if (m0 >= count) return;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave / WGN) * WTM, wn0 = (wave % WGN) * WTN;
    const int K = group_k(p, e);
    const int LA = (p.lda ? p.lda : p.K) / 8, LB = (p.ldb ? p.ldb : p.K) / 8;     // 16-byte chunks per operand row
    const uint4* Ag = reinterpret_cast<const uint4*>(p.A) + (p.row_index ? 0 : static_cast<size_t>(e) * p.capacity * LA);
    const uint4* B0g = reinterpret_cast<const uint4*>(p.B0) + static_cast<size_t>(e) * p.N * LB;
    const uint4* B1g = GLU ? reinterpret_cast<const uint4*>(p.B1) + static_cast<size_t>(e) * p.N * LB : nullptr;

    // per-thread staging slots: chunk q -> (row, ck)
    const uint4* a_src[A_CH];
    const uint4* b_src[B_CH];
    int a_dst[A_CH], b_dst[B_CH], a_ck[A_CH], b_ck[B_CH];
#pragma unroll
    for (int i = 0; i < A_CH; ++i) {
        const int q = tid + i * NTH, row = q / CPR, ck = q % CPR;
        int m = m0 + row;
        m = m < p.capacity ? m : p.capacity - 1;                   // stay inside the buffer; such rows are never stored
        if (p.row_index) m = min(max(p.row_index[static_cast<size_t>(e) * p.capacity + m], 0), p.a_rows - 1);
        a_src[i] = Ag + static_cast<size_t>(m) * LA + ck;
        a_dst[i] = row * CPR + (ck ^ ((row >> SWZ) & (CPR - 1)));
        a_ck[i] = ck;
    }
#pragma unroll
    for (int i = 0; i < B_CH; ++i) {
        const int q = tid + i * NTH, row = q / CPR, ck = q % CPR;
        const bool up = GLU && row >= BN;
        int n = n0 + (up ? row - BN : row);
        n = n < p.N ? n : p.N - 1;
        b_src[i] = (up ? B1g : B0g) + static_cast<size_t>(n) * LB + ck;
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
    load_global(0);                                 // (all zeros when K == 0)
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
    uint16_t* C2g = DUAL ? reinterpret_cast<uint16_t*>(p.C2) + static_cast<size_t>(e) * p.capacity * p.N : nullptr;
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
                const f32x16& g0 = acc[0][i][j];
                const f32x16& g1 = acc[NB - 1][i][j];
                float o[4];
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    if constexpr (GLU && !DUAL) o[v] = silu(g0[q * 4 + v]) * g1[q * 4 + v];
                    else o[v] = g0[q * 4 + v];
                }
                *reinterpret_cast<uint2*>(Cg + static_cast<size_t>(m) * p.N + n) = pack_bf16x4(o[0], o[1], o[2], o[3]);
                if constexpr (GLU && DUAL)
                    *reinterpret_cast<uint2*>(C2g + static_cast<size_t>(m) * p.N + n) =
                        pack_bf16x4(g1[q * 4], g1[q * 4 + 1], g1[q * 4 + 2], g1[q * 4 + 3]);
                if constexpr (GLU && !DUAL) {
                    if (p.C3) {                                     // keep the pre-activations (training-mode forward)
                        const size_t o3 = (static_cast<size_t>(e) * p.capacity + m) * p.N + n;
                        *reinterpret_cast<uint2*>(static_cast<uint16_t*>(p.C2) + o3) =
                            pack_bf16x4(g0[q * 4], g0[q * 4 + 1], g0[q * 4 + 2], g0[q * 4 + 3]);
                        *reinterpret_cast<uint2*>(static_cast<uint16_t*>(p.C3) + o3) =
                            pack_bf16x4(g1[q * 4], g1[q * 4 + 1], g1[q * 4 + 2], g1[q * 4 + 3]);
                    }
                }
            }
    }
}

// The epilogue of the persistent 64-wide kernel: the output passes through a small per-wave LDS patch, so that
// memory sees whole or half lines of a row instead of 8-byte pieces.  In the accumulator layout a lane owns four
// consecutive columns of one row, so a direct store instruction writes 16 rows x 32 bytes (32 x 16 with the
// 32x32x16 accumulators this was first built for): for a 256 x 256 tile that is thousands of write requests next to
// the 512 read requests of each k-step, a third of all requests of a product with a short contraction.  Here a
// 32 x 32 block is written to LDS as it lies in the registers (row stride 80 bytes), read back with four lanes per
// row (16 bytes each) and stored as 16 rows x 64 bytes per instruction (measured when it went in: the down
// projection of the 8-expert workload, whose contraction is 22 k-steps, 1009 -> 1119 TFLOP/s; 1-4 % elsewhere).
// The patch belongs to the wave (LDS instructions of one wave execute in order), so there is no barrier.  Requires
// whole column tiles (no column mask).
constexpr int kStageStride = 80;                         // bytes per staged row: 64 of data + 16 so that rows spread over the banks
constexpr int kStageBytes = 32 * kStageStride;           // per wave

// The patch is written and read back in assembly.  Through ordinary LDS accesses the compiler puts a vmcnt(0) in
// front of every one of them while asynchronous copies into LDS are in flight (it cannot tell that the next tile's
// k-tiles land elsewhere), and that wait also covers the stores this epilogue has just issued: every block then
// waited for the previous block's stores to reach memory, 4-7 thousand cycles per tile.  LDS instructions of one
// wave execute in order, so a write followed by a read needs no wait in between; each statement ends with its
// own lgkmcnt(0), so its outputs are ordinary, fully written registers.
typedef int epi_v2i __attribute__((ext_vector_type(2)));
typedef int epi_v4i __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint32_t lds_address(const void* p) {
    return static_cast<uint32_t>(reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) const char*)p));
}
__device__ __forceinline__ epi_v2i as_v2i(const uint2& v) { return epi_v2i{static_cast<int>(v.x), static_cast<int>(v.y)}; }
__device__ __forceinline__ uint4 as_uint4(const epi_v4i& v) {
    return make_uint4(static_cast<uint32_t>(v.x), static_cast<uint32_t>(v.y), static_cast<uint32_t>(v.z), static_cast<uint32_t>(v.w));
}

// One 32 x 32 output block = four 16 x 16 accumulators (bi, bj) of v_mfma_f32_16x16x32_bf16; in each, lane l holds
// row 16 bi + l % 16 and the four columns 16 bj + 4 (l / 16) .. + 3: pk[2 bi + bj] is that group packed.
// dst = the block's first element.
__device__ __forceinline__ void store_block_staged16(const uint2 (&pk)[4], uint16_t* dst, int ldc, int rows_live,
                                                     unsigned char* stage, int lane) {
    const int l16 = lane & 15, kq = lane >> 4;
    const uint32_t wa = lds_address(stage) + l16 * kStageStride + kq * 8;          // + 32 bj + 16 rows * bi
    const uint32_t ra = lds_address(stage) + (lane >> 2) * kStageStride + (lane & 3) * 16;
    epi_v4i v0, v1;
    static_assert(16 * kStageStride == 1280, "offsets in the statement below");
    asm volatile(
        "ds_write_b64 %2, %4\n\t"
        "ds_write_b64 %2, %5 offset:32\n\t"
        "ds_write_b64 %2, %6 offset:1280\n\t"
        "ds_write_b64 %2, %7 offset:1312\n\t"
        "ds_read_b128 %0, %3\n\t"
        "ds_read_b128 %1, %3 offset:1280\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&v"(v0), "=&v"(v1)
        : "v"(wa), "v"(ra), "v"(as_v2i(pk[0])), "v"(as_v2i(pk[1])), "v"(as_v2i(pk[2])), "v"(as_v2i(pk[3]))
        : "memory");
    const int row = lane >> 2, ch = lane & 3;
    if (row < rows_live) *reinterpret_cast<uint4*>(dst + static_cast<size_t>(row) * ldc + ch * 8) = as_uint4(v0);
    if (row + 16 < rows_live) *reinterpret_cast<uint4*>(dst + static_cast<size_t>(row + 16) * ldc + ch * 8) = as_uint4(v1);
}

// Two horizontally adjacent 32 x 32 blocks (64 columns = one 128-byte line per row), 16 rows at a time (row stride
// 144 bytes): eight lanes read one row back and a store instruction writes 8 rows x 128 bytes, whole lines (down
// projection of the 8-expert workload another 1.5 % over the 64-byte pieces).
constexpr int kPairStride = 144;
static_assert(16 * kPairStride <= kStageBytes, "the pair patch must fit the per-wave patch");
__device__ __forceinline__ void store_block_pair_staged16(const uint2 (&pk0)[4], const uint2 (&pk1)[4], uint16_t* dst, int ldc,
                                                          int rows_live, unsigned char* stage, int lane) {
    const int l16 = lane & 15, kq = lane >> 4;
    const uint32_t wa = lds_address(stage) + l16 * kPairStride + kq * 8;
    const uint32_t ra = lds_address(stage) + (lane >> 3) * kPairStride + (lane & 7) * 16;
    static_assert(8 * kPairStride == 1152, "offset in the statement below");
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {                // rows 16 pass .. + 15: every lane owns a piece of them
        epi_v4i v0, v1;
        asm volatile(
            "ds_write_b64 %2, %4\n\t"
            "ds_write_b64 %2, %5 offset:32\n\t"
            "ds_write_b64 %2, %6 offset:64\n\t"
            "ds_write_b64 %2, %7 offset:96\n\t"
            "ds_read_b128 %0, %3\n\t"
            "ds_read_b128 %1, %3 offset:1152\n\t"
            "s_waitcnt lgkmcnt(0)"
            : "=&v"(v0), "=&v"(v1)
            : "v"(wa), "v"(ra), "v"(as_v2i(pk0[pass * 2])), "v"(as_v2i(pk0[pass * 2 + 1])), "v"(as_v2i(pk1[pass * 2])),
              "v"(as_v2i(pk1[pass * 2 + 1]))
            : "memory");
        const int r = pass * 16 + (lane >> 3), ch = lane & 7;
        if (r < rows_live) *reinterpret_cast<uint4*>(dst + static_cast<size_t>(r) * ldc + ch * 8) = as_uint4(v0);
        if (r + 8 < rows_live) *reinterpret_cast<uint4*>(dst + static_cast<size_t>(r + 8) * ldc + ch * 8) = as_uint4(v1);
    }
}
// acc[i][j]: token block i (16 rows) x weight block j (16 rows of the staged weights; SwiGLU: 0, 1 gate and 2, 3 up
// rows of the same 32 columns; plain: 64 columns)
template <bool GLU, bool DUAL, bool KEEP = false>
__device__ __forceinline__ void store_blocks_staged16(const GemmParams& p, const f32x4 (&acc)[8][4], int e, int m_base,
                                                      int n_base, int count, int lane, unsigned char* stage) {
    const size_t eoff = static_cast<size_t>(e) * p.capacity * p.N;
    uint16_t* Cg = reinterpret_cast<uint16_t*>(p.C) + eoff;
    uint16_t* C2g = (GLU && (DUAL || KEEP)) ? reinterpret_cast<uint16_t*>(p.C2) + eoff : nullptr;
    uint16_t* C3g = (GLU && !DUAL && KEEP) ? reinterpret_cast<uint16_t*>(p.C3) + eoff : nullptr;
    auto pack4 = [](const f32x4& v) { return pack_bf16x4(v[0], v[1], v[2], v[3]); };
#pragma unroll
    for (int ib = 0; ib < 4; ++ib) {
        const int mb = m_base + ib * 32;
        const int live = count - mb;
        if (live <= 0) continue;                         // wave-uniform
        const size_t o = static_cast<size_t>(mb) * p.N + n_base;
        uint2 pk[4], pk1[4];
        if constexpr (!GLU) {
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                pk[b] = pack4(acc[2 * ib + (b >> 1)][b & 1]);
                pk1[b] = pack4(acc[2 * ib + (b >> 1)][2 + (b & 1)]);
            }
            store_block_pair_staged16(pk, pk1, Cg + o, p.N, live, stage, lane);
        } else {
            if constexpr (!DUAL) {
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const f32x4& g0 = acc[2 * ib + (b >> 1)][b & 1];
                    const f32x4& g1 = acc[2 * ib + (b >> 1)][2 + (b & 1)];
                    pk[b] = pack_bf16x4(silu(g0[0]) * g1[0], silu(g0[1]) * g1[1], silu(g0[2]) * g1[2], silu(g0[3]) * g1[3]);
                }
            } else {
#pragma unroll
                for (int b = 0; b < 4; ++b) pk[b] = pack4(acc[2 * ib + (b >> 1)][b & 1]);
            }
            store_block_staged16(pk, Cg + o, p.N, live, stage, lane);
            if constexpr (DUAL || KEEP) {                    // the two products themselves
                if constexpr (KEEP) {
#pragma unroll
                    for (int b = 0; b < 4; ++b) pk[b] = pack4(acc[2 * ib + (b >> 1)][b & 1]);
                    store_block_staged16(pk, C2g + o, p.N, live, stage, lane);
                }
#pragma unroll
                for (int b = 0; b < 4; ++b) pk[b] = pack4(acc[2 * ib + (b >> 1)][2 + (b & 1)]);
                store_block_staged16(pk, (KEEP ? C3g : C2g) + o, p.N, live, stage, lane);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

typedef const __attribute__((address_space(1))) void* global_cptr;
typedef __attribute__((address_space(3))) void* lds_ptr;

// ---------------------------------------------------------------------------------------
// Pipelined bf16 MFMA grouped GEMM (launched for K % 64 == 0; one workgroup per tile; the fall-back of the
// persistent kernels below): 256 x 256 staged rows, BK = 32, a ring of four 32 KiB LDS buffers.
//   * global -> LDS copies bypass the registers (global_load_lds_dwordx4); the XOR swizzle is
//     applied on the source side (lane l fetches the chunk that belongs in LDS slot l);
//   * the copies of tile kt+3 are spread one by one between the MFMAs of iteration kt (a copy
//     issued in a burst blocks the wave's MFMA issue for about 25 cycles each), and they have two
//     full iterations to land: before barrier(kt) a wave waits only until at most 12 copies are
//     outstanding (s_waitcnt vmcnt(12)), i.e. until its share of tile kt+1 is in LDS;
//   * MFMA operands are double-buffered in registers: the ds_reads of k-substep s+1 are issued
//     before the MFMAs of substep s; one barrier per iteration.
// With GLU the 256 staged weight rows are 128 gate rows + 128 up rows of the same output columns
// and the epilogue is SiLU(gate)*up.  With row_index the A rows are gathered straight from the
// token matrix (dispatch folded into the load).
// ---------------------------------------------------------------------------------------
// s_waitcnt immediate: vmcnt(n) (6 bits, split 3:0 and 15:14), expcnt untouched, lgkmcnt(0) or untouched
constexpr int waitcnt_imm(int vm, bool lgkm0) { return (vm & 15) | ((vm >> 4) << 14) | 0x70 | (lgkm0 ? 0 : 0x0F00); }

template <bool GLU, int WN = 2, bool DUAL = false, int NBUF = 4>
__global__ __launch_bounds__(128 * WN) void gemm_bf16_ring_kernel(GemmParams p) {
    constexpr int BM = 256, BR = 256, CPR = 4;
    constexpr int BN = GLU ? 128 : 256;
    constexpr int STAGE = (BM + BR) * CPR;              // uint4 per LDS buffer (32 KiB)
    constexpr int NW = 2 * WN;                          // waves: 2 row groups x WN column groups
    constexpr int TB = 4 / (WN / 2);                    // weight fragments per wave and k-substep (4 or 2)
    constexpr int NCP = 16 / NW;                        // row groups (of 16 rows) each wave copies per operand
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    uint4* lds = reinterpret_cast<uint4*>(lds_raw);

    int e, mt, nt;
    if (!decode_tile(p, e, mt, nt)) return;
    const int count = group_rows(p, e);
    const int m0 = mt * BM, n0 = nt * BN;
    if (m0 >= count) return;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int r32 = lane & 31, half = lane >> 5;
    const int KCA = (p.lda ? p.lda : p.K) / 8, KCB = (p.ldb ? p.ldb : p.K) / 8;   // 16-byte chunks per operand row
    const int KT = group_k(p, e) / 32;

    // ---- copy sources: wave w fills row groups w*NCP .. (16 rows x 4 chunks = 1 KiB each)
    // Addresses are a wave-uniform 64-bit base (scalar registers, advanced by 64 bytes per tile)
    // plus a per-lane 32-bit byte offset that never changes (the host checks that it fits).
    const char* Abase = reinterpret_cast<const char*>(p.A) +
                        (p.row_index ? 0 : static_cast<size_t>(e) * p.capacity * KCA * 16);
    const char* Bbase = reinterpret_cast<const char*>((GLU && wave >= NW / 2) ? p.B1 : p.B0) +
                        static_cast<size_t>(e) * p.N * KCB * 16;
    uint32_t off[2 * NCP];                              // first NCP: A groups, then B groups
#pragma unroll
    for (int i = 0; i < NCP; ++i) {
        const int r = (wave * NCP + i) * 16 + (lane >> 2);
        const int c = (lane & 3) ^ ((r >> 2) & 3);
        int m = m0 + r;
        m = m < count ? m : count - 1;                   // rows past the count replay a valid row; never stored
        const int row = p.row_index ? min(max(p.row_index[static_cast<size_t>(e) * p.capacity + m], 0), p.a_rows - 1) : m;
        off[i] = (static_cast<uint32_t>(row) * KCA + c) * 16u;
        int n = n0 + (GLU ? (r & 127) : r);
        n = n < p.N ? n : p.N - 1;
        off[NCP + i] = (static_cast<uint32_t>(n) * KCB + c) * 16u;
    }
    auto issue_copy = [&](int kt, int j) {
        uint4* dst = lds + (kt % NBUF) * STAGE + (j / NCP) * (BM * CPR) + (wave * NCP + (j % NCP)) * 64;
        // re-materialise the tile base as a scalar every time, so that the address stays
        // "scalar base + 32-bit lane offset" instead of a per-lane 64-bit pointer
        const uint64_t b64 = reinterpret_cast<uint64_t>(j < NCP ? Abase : Bbase) + static_cast<uint64_t>(kt) * (CPR * 16);
        const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(b64));
        const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(b64 >> 32));
        const char* base = reinterpret_cast<const char*>((static_cast<uint64_t>(hi) << 32) | lo);
        __builtin_amdgcn_global_load_lds((global_cptr)(base + off[j]), (lds_ptr)dst, 16, 0, 0);
    };

    const int sw = (r32 >> 2) & 3;
    int a_row[4], b_row[TB];
#pragma unroll
    for (int i = 0; i < 4; ++i) a_row[i] = (wm * 128 + i * 32 + r32) * CPR;
#pragma unroll
    for (int j = 0; j < TB; ++j) {
        const int br = GLU ? ((j / (TB / 2)) * 128 + wn * (16 * TB) + (j % (TB / 2)) * 32) : (wn * (32 * TB) + j * 32);
        b_row[j] = BM * CPR + (br + r32) * CPR;
    }
    const int ck0 = half ^ sw, ck1 = (2 + half) ^ sw;

    f32x16 acc[4][TB];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < TB; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    bf16x8 fa[2][4], fb[2][TB];
    auto load_frags = [&](int set, int kt, int ck) {
        const uint4* base = lds + (kt % NBUF) * STAGE + ck;
#pragma unroll
        for (int i = 0; i < 4; ++i) fa[set][i] = __builtin_bit_cast(bf16x8, base[a_row[i]]);
#pragma unroll
        for (int j = 0; j < TB; ++j) fb[set][j] = __builtin_bit_cast(bf16x8, base[b_row[j]]);
    };
    // the MFMAs of one k-substep; with `copy`, NCP copies of tile kt_copy go in between, one per 4 MFMAs
    auto mfma_step = [&](int set, bool copy, int kt_copy, int j0) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
#pragma unroll
            for (int j = 0; j < TB; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[set][j], fa[set][i], acc[i][j], 0, 0, 0);
            if (copy && (i + 1) % (4 / NCP) == 0) issue_copy(kt_copy, j0 + i / (4 / NCP));
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // ---- prologue: NBUF - 1 tiles in flight, wait for the first
    constexpr int AHEAD = NBUF - 1;
    const int pre = KT < AHEAD ? KT : AHEAD;
    for (int t = 0; t < pre; ++t)
#pragma unroll
        for (int j = 0; j < 2 * NCP; ++j) issue_copy(t, j);
    if (pre == AHEAD) __builtin_amdgcn_s_waitcnt(waitcnt_imm((AHEAD - 1) * 2 * NCP, false));
    else if (pre == 3) __builtin_amdgcn_s_waitcnt(waitcnt_imm(4 * NCP, false));
    else if (pre == 2) __builtin_amdgcn_s_waitcnt(waitcnt_imm(2 * NCP, false));
    else __builtin_amdgcn_s_waitcnt(waitcnt_imm(0, false));
    __builtin_amdgcn_s_barrier();
    load_frags(0, 0, ck0);

    int kt = 0;
    for (; kt + AHEAD < KT; ++kt) {                          // steady state: tile kt+AHEAD is being fetched
        __builtin_amdgcn_sched_barrier(0);
        load_frags(1, kt, ck1);
        mfma_step(0, true, kt + AHEAD, 0);
        // tile kt+1 is in LDS once at most tiles kt+2 .. kt+AHEAD-1 and half of kt+AHEAD are outstanding
        __builtin_amdgcn_s_waitcnt(waitcnt_imm((2 * (AHEAD - 2) + 1) * NCP, true));
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        load_frags(0, kt + 1, ck0);
        mfma_step(1, true, kt + AHEAD, NCP);
    }
    for (; kt < KT; ++kt) {                                  // drain: nothing left to fetch
        __builtin_amdgcn_sched_barrier(0);
        load_frags(1, kt, ck1);
        mfma_step(0, false, 0, 0);
        __builtin_amdgcn_s_waitcnt(0x0070);                  // vmcnt(0) lgkmcnt(0)
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        if (kt + 1 < KT) load_frags(0, kt + 1, ck0);
        mfma_step(1, false, 0, 0);
    }

    constexpr int TO = GLU ? TB / 2 : TB;
    if (GLU && !DUAL && p.C3) store_blocks<GLU, DUAL, 4, TB, GLU && !DUAL>(p, acc, e, m0 + wm * 128, n0 + wn * (32 * TO), count, r32, half);
    else store_blocks<GLU, DUAL, 4, TB>(p, acc, e, m0 + wm * 128, n0 + wn * (32 * TO), count, r32, half);
}

// ---------------------------------------------------------------------------------------
// Persistent form of the ring kernel: one workgroup per CU walks a list of tiles, and the ring
// of copies runs on across tile boundaries: while the last k-tiles of one tile are multiplied
// the first k-tiles of the next are already being fetched, and the stores of the epilogue
// overlap with them.  (A workgroup per tile pays launch, address set-up, the first-tile latency
// and the epilogue with the matrix pipe idle: about 5 us per tile, 5-10 % at K = 2048.)
//
// Tile list: only tiles that hold rows (m0 < counts[e]) are enumerated, super-tile by super-tile
// (see decode_tile), from an exclusive prefix over the super-tiles that every workgroup builds in
// LDS at start.  Consecutive groups of gridDim.x / 8 tiles go round-robin to the 8 XCDs, so the
// tiles that run together on one XCD are still (pieces of) one super-tile and share operand
// slices through its L2, and every workgroup gets the same number of tiles +- 1.
// No atomics, no flags: the schedule is a pure function of counts[].
//
// Waits: copies and stores complete in issue order, so "at most 3*NCP operations outstanding"
// always implies that everything older than the newest 3*NCP has landed; operations that are not
// copies of the ring (the epilogue's stores) only make that wait conservative, never unsafe.
// ---------------------------------------------------------------------------------------
constexpr int kMaxSuper = 4096;          // super-tiles the LDS prefix can hold (16 KiB)
constexpr int kMaxSuperWide = 2048;      // the same for the 64-wide kernel, whose two 64 KiB buffers leave less room

//
// Operands whose contraction index is the slow one (TRA: A is [K][M], TRB: B is [K][N], row strides lda / ldb,
// group stride K * ld; with TRB and B1 the contraction is split in the middle: first half from B0, second half
// from B1, each [K/2][N]).  Such a tile is staged in LDS as [block of 32 rows][32 k][32 rows] (64 bytes per k) and
// the MFMA fragments come out through the transposing read ds_read_b64_tr_b16: inside a group of 16 lanes, lane i
// supplies the address of 4 consecutive elements and receives element i % 4 of lanes i/4, i/4 + 4, i/4 + 8,
// i/4 + 12.  With lane (q = i % 4, j = i / 4) pointing at (k0 + j, r0 + 4 q) lane i receives rows r0 + i at
// k0 .. k0 + 3: two reads give the 8 consecutive k of one row that the MFMA operand layout wants.  The four k of a
// group are 64 bytes apart, so 32 lanes cover all 64 banks once: conflict-free without a swizzle.
//
// KG (1: A, 2: B): the contraction rows of that operand are fetched through p.k_index (a gather along the slow
// index).  The indices of a k-tile (32 of them) travel like the tiles themselves: wave 0 copies them into a ring
// of 16 LDS slots seven k-tiles before the tile is multiplied, i.e. four iterations before its copies are issued,
// so that its wait and the barrier of an earlier iteration have made them visible to every wave by the time a lane
// reads its row number; the per-lane source address of a copy is then
// base + row * row bytes + the lane's fixed column offset.  Every row number is clamped into [0, k_rows), so a
// stale or foreign ring word can at worst fetch a wrong but existing row.
template <bool GLU, bool DUAL = false, bool TRA = false, bool TRB = false, int KG = 0>
__global__ __launch_bounds__(512) void gemm_bf16_persist_kernel(GemmParams p) {
    static_assert(!(GLU && TRB), "the transposed B operand is for plain products");
    static_assert(KG == 0 || (KG == 1 && TRA) || (KG == 2 && TRB), "the gathered operand is a transposed one");
    constexpr int IDX_AHEAD = 7, IDX_SLOTS = 16;        // index prefetch distance in k-tiles, ring slots of 32 indices
    constexpr int BM = 256, BR = 256, CPR = 4, NBUF = 4, AHEAD = NBUF - 1;
    constexpr int BN = GLU ? 128 : 256;
    constexpr int STAGE = (BM + BR) * CPR;
    constexpr int WN = 4, NW = 8, TB = 2, NCP = 2;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    uint4* lds = reinterpret_cast<uint4*>(lds_raw);
    __shared__ int pre[kMaxSuper + 1];
    __shared__ int wave_tot[NW];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int r32 = lane & 31, half = lane >> 5;
    const int KCA = (p.lda ? p.lda : p.K) / 8, KCB = (p.ldb ? p.ldb : p.K) / 8;
    // bytes from one k-tile of an operand to the next
    const size_t stepA = TRA ? static_cast<size_t>(32) * KCA * 16 : CPR * 16;
    const size_t stepB = TRB ? static_cast<size_t>(32) * KCB * 16 : CPR * 16;
    const bool splitB = TRB && p.B1 != nullptr;
    const uint32_t kg_row_bytes = static_cast<uint32_t>(KG == 1 ? KCA : KCB) * 16u;
    int32_t* idx_ring = reinterpret_cast<int32_t*>(lds_raw + static_cast<size_t>(NBUF) * STAGE * 16);

    // ---- exclusive prefix of the number of live tiles per super-tile
    const int MG = (p.MT + p.SM - 1) / p.SM, NG = (p.NT + p.SN - 1) / p.SN;
    const int S = p.E * MG * NG;
    auto live_rows = [&](int e, int mg) {                // live row tiles of super-tile row mg of expert e
        const int mtv = (group_rows(p, e) + BM - 1) / BM;
        return min(max(mtv - mg * p.SM, 0), p.SM);
    };
    auto live_cols = [&](int ng) { return min(p.NT - ng * p.SN, p.SN); };
    {
        const int CH = (S + 511) / 512;
        int sum = 0;
        for (int i = 0; i < CH; ++i) {
            const int s = tid * CH + i;
            if (s < S) {
                const int e = s / (MG * NG), r = s - e * (MG * NG);
                sum += live_rows(e, r % MG) * live_cols(r / MG);
            }
        }
        int inc = sum;
#pragma unroll
        for (int m = 1; m < 64; m <<= 1) {
            const int o = __shfl_up(inc, m, 64);
            if (lane >= m) inc += o;
        }
        if (lane == 63) wave_tot[wave] = inc;
        __syncthreads();
        int run = inc - sum;
        for (int w = 0; w < wave; ++w) run += wave_tot[w];
        for (int i = 0; i < CH; ++i) {
            const int s = tid * CH + i;
            if (s < S) {
                pre[s] = run;
                const int e = s / (MG * NG), r = s - e * (MG * NG);
                run += live_rows(e, r % MG) * live_cols(r / MG);
            }
        }
        if (tid == 511) pre[S] = run;                    // thread 511 owns the last chunk (or nothing): run = total
        __syncthreads();
    }
    const int total = pre[S];
    const int GS = gridDim.x >> 3;                       // tiles per group = workgroups per XCD
    const int xcd = blockIdx.x & 7, slot_l = blockIdx.x >> 3;

    struct Tile {
        int e, m0, n0, count, KT;
        const char* Abase;
        const char* Bbase;
        const char* Bbase1;                              // second half of a split transposed B
        uint32_t off[2 * NCP];
    };
    // per-lane byte offset inside a k-tile of a [K][rows] operand.  Copy unit u = (block of 32 rows, half of the 32 k):
    // 16 k x 64 bytes, four lanes per k, the access shape of the row-major copies (64-byte pieces of 16 memory rows)
    auto kmajor_off = [&](int u, int r0, int limit, int kc, bool gathered) -> uint32_t {
        const int krow = gathered ? 0 : (u & 1) * 16 + (lane >> 2);      // (a gathered row comes from the index ring)
        int r = r0 + (u >> 1) * 32 + (lane & 3) * 8;
        r = r + 8 <= limit ? r : limit - 8;              // stay inside the row; such columns are never stored
        return (static_cast<uint32_t>(krow) * kc * 8 + r) * 2u;
    };
    // the tile with list index q (q < total)
    auto setup = [&](int q, Tile& t) {
        int lo = 0, hi = S;                              // largest s with pre[s] <= q
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (pre[mid] <= q) lo = mid; else hi = mid;
        }
        const int s = __builtin_amdgcn_readfirstlane(lo);
        const int u = __builtin_amdgcn_readfirstlane(q - pre[s]);
        const int e = s / (MG * NG), r = s - e * (MG * NG);
        const int mg = r % MG, ng = r / MG;
        const int vm = live_rows(e, mg);
        const int mt = mg * p.SM + u % vm, nt = ng * p.SN + u / vm;
        t.e = e; t.m0 = mt * BM; t.n0 = nt * BN;
        t.count = group_rows(p, e);
        t.KT = group_k(p, e) / 32;
        if constexpr (KG == 1) t.Abase = reinterpret_cast<const char*>(p.A);
        else if constexpr (TRA) t.Abase = reinterpret_cast<const char*>(p.A) + static_cast<size_t>(e) * p.K * KCA * 16;
        else t.Abase = reinterpret_cast<const char*>(p.A) + (p.row_index ? 0 : static_cast<size_t>(e) * p.capacity * KCA * 16);
        if constexpr (TRB) {
            const size_t per_group = KG == 2 ? 0 : static_cast<size_t>(splitB ? p.K / 2 : p.K) * KCB * 16;
            t.Bbase = reinterpret_cast<const char*>(p.B0) + e * per_group;
            t.Bbase1 = splitB ? reinterpret_cast<const char*>(p.B1) + e * per_group : t.Bbase;
        } else {
            t.Bbase = reinterpret_cast<const char*>((GLU && wave >= NW / 2) ? p.B1 : p.B0) + static_cast<size_t>(e) * p.N * KCB * 16;
            t.Bbase1 = t.Bbase;
        }
#pragma unroll
        for (int i = 0; i < NCP; ++i) {
            const int rr = (wave * NCP + i) * 16 + (lane >> 2);
            const int c = (lane & 3) ^ ((rr >> 2) & 3);
            if constexpr (TRA) {
                t.off[i] = kmajor_off(wave * NCP + i, t.m0, p.capacity, KCA, KG == 1);
            } else {
                int m = t.m0 + rr;
                m = m < t.count ? m : t.count - 1;
                const int row = p.row_index ? min(max(p.row_index[static_cast<size_t>(e) * p.capacity + m], 0), p.a_rows - 1) : m;
                t.off[i] = (static_cast<uint32_t>(row) * KCA + c) * 16u;
            }
            if constexpr (TRB) {
                t.off[NCP + i] = kmajor_off(wave * NCP + i, t.n0, p.N, KCB, KG == 2);
            } else {
                int n = t.n0 + (GLU ? (rr & 127) : rr);
                n = n < p.N ? n : p.N - 1;
                t.off[NCP + i] = (static_cast<uint32_t>(n) * KCB + c) * 16u;
            }
        }
    };
    // address of k-tile k of the B operand (wave-uniform); all arguments by value, so that the tile records stay in
    // registers
    auto b_ktile = [&](const char* b0, const char* b1, int kt_count, int k) -> uint64_t {
        const bool second = splitB && k >= (kt_count >> 1);
        const int kk = second ? k - (kt_count >> 1) : k;
        return reinterpret_cast<uint64_t>(second ? b1 : b0) + kk * stepB;
    };
    // copy j (0..NCP-1: A row groups, NCP..2NCP-1: B row groups) of k-tile k of tile t into the ring slot of step g
    auto issue_copy = [&](const Tile& t, int k, int g, int j, uint32_t row_off) {
        uint4* dst = lds + (g & (NBUF - 1)) * STAGE + (j / NCP) * (BM * CPR) + (wave * NCP + (j % NCP)) * 64;
        const bool gathered = (KG == 1 && j < NCP) || (KG == 2 && j >= NCP);
        const uint64_t b64 = gathered ? reinterpret_cast<uint64_t>(j < NCP ? t.Abase : t.Bbase)
                           : j < NCP ? reinterpret_cast<uint64_t>(t.Abase) + k * stepA : b_ktile(t.Bbase, t.Bbase1, t.KT, k);
        const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(b64));
        const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(b64 >> 32));
        const char* base = reinterpret_cast<const char*>((static_cast<uint64_t>(hi) << 32) | lo);
        __builtin_amdgcn_global_load_lds((global_cptr)(base + t.off[j] + row_off), (lds_ptr)dst, 16, 0, 0);
    };
    // KG: the 32 row numbers of k-tile kl of group e go to the ring slot of global step gstep (lanes 0..31 of the
    // calling wave); positions past the index row are clamped onto its last entry
    auto issue_idx = [&](int e, int kl, int gstep) {
        int pos = kl * 32 + (lane & 31);
        pos = pos < p.k_index_stride ? pos : p.k_index_stride - 1;
        const int32_t* src = p.k_index + static_cast<size_t>(e) * p.k_index_stride + pos;
        int32_t* dst = idx_ring + (gstep & (IDX_SLOTS - 1)) * 32;
        if (lane < 32) __builtin_amdgcn_global_load_lds((global_cptr)src, (lds_ptr)dst, 4, 0, 0);
    };

    const int sw = (r32 >> 2) & 3;
    int a_row[4], b_row[TB];
#pragma unroll
    for (int i = 0; i < 4; ++i) a_row[i] = (wm * 128 + i * 32 + r32) * CPR;
#pragma unroll
    for (int j = 0; j < TB; ++j) {
        const int br = GLU ? ((j / (TB / 2)) * 128 + wn * (16 * TB) + (j % (TB / 2)) * 32) : (wn * (32 * TB) + j * 32);
        b_row[j] = BM * CPR + (br + r32) * CPR;
    }
    const int ck0 = half ^ sw, ck1 = (2 + half) ^ sw;
    // transposing reads: byte offset, inside the operand's part of a ring slot, of this lane's 4 elements for the
    // 32-row fragment that starts at row rf (first k-substep, first half of its 8 k)
    auto tr_off = [&](int rf) -> uint32_t {
        const int r = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);           // inside the block of 32 rows
        const int kb = 8 * (lane >> 5) + ((lane & 15) >> 2);
        return static_cast<uint32_t>((rf >> 5) * 2048 + kb * 64 + r * 2);
    };
    uint32_t a_tr[4], b_tr[TB];
#pragma unroll
    for (int i = 0; i < 4; ++i) a_tr[i] = tr_off(wm * 128 + i * 32);
#pragma unroll
    for (int j = 0; j < TB; ++j) b_tr[j] = BM * CPR * 16 + tr_off(wn * (32 * TB) + j * 32);
    // The reads are written as assembly: through the compiler's builtin every such read waits for ALL outstanding
    // copies (vmcnt(0)), because it is taken to alias the asynchronous LDS writes.  The compiler does not track the
    // LDS counter for assembly, so every statement below carries its own wait (lgkmcnt(0)) behind its reads: when
    // the statement ends its outputs are ordinary, fully written registers, and nothing depends on how the register
    // allocator treats them afterwards.  All reads of one statement are in flight together; the statement is placed
    // one k-substep before the fragments are used, so the wait overlaps with the MFMAs of the other wave of the SIMD.
    typedef int v2i __attribute__((ext_vector_type(2)));
    typedef int v4i __attribute__((ext_vector_type(4)));
    const uint32_t lds_base = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) char*)lds_raw));
    // KG: byte offsets of the source rows of this wave's two copies (k rows lane / 4 and 16 + lane / 4) of the k-tile
    // of global step gstep, from the index ring (its words are visible: see the kernel's header)
    auto idx_addr = [&](int gstep) -> uint32_t {
        return lds_base + static_cast<uint32_t>(NBUF) * STAGE * 16 + (gstep & (IDX_SLOTS - 1)) * 128 + (lane >> 2) * 4;
    };
    auto idx_rows = [&](int gstep, uint32_t& r0, uint32_t& r1) {
        const uint32_t a = idx_addr(gstep);
        int i0, i1;
        asm volatile("ds_read_b32 %0, %2\n\t"
                     "ds_read_b32 %1, %2 offset:64\n\t"
                     "s_waitcnt lgkmcnt(0)"
                     : "=&v"(i0), "=&v"(i1) : "v"(a));
        r0 = static_cast<uint32_t>(min(max(i0, 0), p.k_rows - 1)) * kg_row_bytes;
        r1 = static_cast<uint32_t>(min(max(i1, 0), p.k_rows - 1)) * kg_row_bytes;
    };
    auto tr_pack = [](v2i lo, v2i hi) -> bf16x8 {          // k .. k+3 and k+4 .. k+7 of one row
        const v4i r = {lo.x, lo.y, hi.x, hi.y};
        return __builtin_bit_cast(bf16x8, r);
    };
    auto tr_frags4 = [&](bf16x8* f, uint32_t slot, const uint32_t* off) {
        const uint32_t a0 = lds_base + slot + off[0], a1 = lds_base + slot + off[1];
        const uint32_t a2 = lds_base + slot + off[2], a3 = lds_base + slot + off[3];
        v2i x0, x1, x2, x3, x4, x5, x6, x7;
        asm volatile(
            "ds_read_b64_tr_b16 %0, %8\n\t"
            "ds_read_b64_tr_b16 %1, %8 offset:256\n\t"
            "ds_read_b64_tr_b16 %2, %9\n\t"
            "ds_read_b64_tr_b16 %3, %9 offset:256\n\t"
            "ds_read_b64_tr_b16 %4, %10\n\t"
            "ds_read_b64_tr_b16 %5, %10 offset:256\n\t"
            "ds_read_b64_tr_b16 %6, %11\n\t"
            "ds_read_b64_tr_b16 %7, %11 offset:256\n\t"
            "s_waitcnt lgkmcnt(0)"
            : "=&v"(x0), "=&v"(x1), "=&v"(x2), "=&v"(x3), "=&v"(x4), "=&v"(x5), "=&v"(x6), "=&v"(x7)
            : "v"(a0), "v"(a1), "v"(a2), "v"(a3));
        f[0] = tr_pack(x0, x1); f[1] = tr_pack(x2, x3); f[2] = tr_pack(x4, x5); f[3] = tr_pack(x6, x7);
    };
    auto tr_frags2 = [&](bf16x8* f, uint32_t slot, const uint32_t* off) {
        const uint32_t a0 = lds_base + slot + off[0], a1 = lds_base + slot + off[1];
        v2i x0, x1, x2, x3;
        asm volatile(
            "ds_read_b64_tr_b16 %0, %4\n\t"
            "ds_read_b64_tr_b16 %1, %4 offset:256\n\t"
            "ds_read_b64_tr_b16 %2, %5\n\t"
            "ds_read_b64_tr_b16 %3, %5 offset:256\n\t"
            "s_waitcnt lgkmcnt(0)"
            : "=&v"(x0), "=&v"(x1), "=&v"(x2), "=&v"(x3)
            : "v"(a0), "v"(a1));
        f[0] = tr_pack(x0, x1); f[1] = tr_pack(x2, x3);
    };
    auto tr_frags6 = [&](bf16x8* f, bf16x8* h, uint32_t slot, const uint32_t* off, const uint32_t* off2) {
        const uint32_t a0 = lds_base + slot + off[0], a1 = lds_base + slot + off[1];
        const uint32_t a2 = lds_base + slot + off[2], a3 = lds_base + slot + off[3];
        const uint32_t a4 = lds_base + slot + off2[0], a5 = lds_base + slot + off2[1];
        v2i x0, x1, x2, x3, x4, x5, x6, x7, x8, x9, x10, x11;
        asm volatile(
            "ds_read_b64_tr_b16 %0, %12\n\t"
            "ds_read_b64_tr_b16 %1, %12 offset:256\n\t"
            "ds_read_b64_tr_b16 %2, %13\n\t"
            "ds_read_b64_tr_b16 %3, %13 offset:256\n\t"
            "ds_read_b64_tr_b16 %4, %14\n\t"
            "ds_read_b64_tr_b16 %5, %14 offset:256\n\t"
            "ds_read_b64_tr_b16 %6, %15\n\t"
            "ds_read_b64_tr_b16 %7, %15 offset:256\n\t"
            "ds_read_b64_tr_b16 %8, %16\n\t"
            "ds_read_b64_tr_b16 %9, %16 offset:256\n\t"
            "ds_read_b64_tr_b16 %10, %17\n\t"
            "ds_read_b64_tr_b16 %11, %17 offset:256\n\t"
            "s_waitcnt lgkmcnt(0)"
            : "=&v"(x0), "=&v"(x1), "=&v"(x2), "=&v"(x3), "=&v"(x4), "=&v"(x5), "=&v"(x6), "=&v"(x7), "=&v"(x8),
              "=&v"(x9), "=&v"(x10), "=&v"(x11)
            : "v"(a0), "v"(a1), "v"(a2), "v"(a3), "v"(a4), "v"(a5));
        f[0] = tr_pack(x0, x1); f[1] = tr_pack(x2, x3); f[2] = tr_pack(x4, x5); f[3] = tr_pack(x6, x7);
        h[0] = tr_pack(x8, x9); h[1] = tr_pack(x10, x11);
    };
    // the same with the two row numbers of a gathered operand's next copies riding on the statement's wait
    auto tr_frags6_idx = [&](bf16x8* f, bf16x8* h, uint32_t slot, const uint32_t* off, const uint32_t* off2, uint32_t ia,
                             int& i0, int& i1) {
        const uint32_t a0 = lds_base + slot + off[0], a1 = lds_base + slot + off[1];
        const uint32_t a2 = lds_base + slot + off[2], a3 = lds_base + slot + off[3];
        const uint32_t a4 = lds_base + slot + off2[0], a5 = lds_base + slot + off2[1];
        v2i x0, x1, x2, x3, x4, x5, x6, x7, x8, x9, x10, x11;
        asm volatile(
            "ds_read_b64_tr_b16 %0, %14\n\t"
            "ds_read_b64_tr_b16 %1, %14 offset:256\n\t"
            "ds_read_b64_tr_b16 %2, %15\n\t"
            "ds_read_b64_tr_b16 %3, %15 offset:256\n\t"
            "ds_read_b64_tr_b16 %4, %16\n\t"
            "ds_read_b64_tr_b16 %5, %16 offset:256\n\t"
            "ds_read_b64_tr_b16 %6, %17\n\t"
            "ds_read_b64_tr_b16 %7, %17 offset:256\n\t"
            "ds_read_b64_tr_b16 %8, %18\n\t"
            "ds_read_b64_tr_b16 %9, %18 offset:256\n\t"
            "ds_read_b64_tr_b16 %10, %19\n\t"
            "ds_read_b64_tr_b16 %11, %19 offset:256\n\t"
            "ds_read_b32 %12, %20\n\t"
            "ds_read_b32 %13, %20 offset:64\n\t"
            "s_waitcnt lgkmcnt(0)"
            : "=&v"(x0), "=&v"(x1), "=&v"(x2), "=&v"(x3), "=&v"(x4), "=&v"(x5), "=&v"(x6), "=&v"(x7), "=&v"(x8),
              "=&v"(x9), "=&v"(x10), "=&v"(x11), "=&v"(i0), "=&v"(i1)
            : "v"(a0), "v"(a1), "v"(a2), "v"(a3), "v"(a4), "v"(a5), "v"(ia));
        f[0] = tr_pack(x0, x1); f[1] = tr_pack(x2, x3); f[2] = tr_pack(x4, x5); f[3] = tr_pack(x6, x7);
        h[0] = tr_pack(x8, x9); h[1] = tr_pack(x10, x11);
    };
    static_assert(TB == 2, "tr_frags2 / tr_frags6 read the two weight fragments of a wave");

    f32x16 acc[4][TB];
    bf16x8 fa[2][4], fb[2][TB];
    // set = k-substep (0: k 0..15 of the tile, 1: k 16..31); ck is the swizzled chunk of the row-major layout
    auto load_frags = [&](int set, int g, int ck) {
        const uint4* base = lds + (g & (NBUF - 1)) * STAGE + ck;
        const uint32_t slot = static_cast<uint32_t>(g & (NBUF - 1)) * (STAGE * 16) + set * 1024;
        // row-major operands first: their reads are in flight while the transposing statement waits
        if constexpr (!TRA) {
#pragma unroll
            for (int i = 0; i < 4; ++i) fa[set][i] = __builtin_bit_cast(bf16x8, base[a_row[i]]);
        }
        if constexpr (!TRB) {
#pragma unroll
            for (int j = 0; j < TB; ++j) fb[set][j] = __builtin_bit_cast(bf16x8, base[b_row[j]]);
        }
        if constexpr (TRA && TRB) tr_frags6(fa[set], fb[set], slot, a_tr, b_tr);
        else if constexpr (TRA) tr_frags4(fa[set], slot, a_tr);
        else if constexpr (TRB) tr_frags2(fb[set], slot, b_tr);
    };

    int q = xcd * GS + slot_l;                           // first pass over the list
    if (q >= total) return;                              // uniform: nothing for this workgroup
    Tile cur, nxt;
    setup(q, cur);
    int g = 0;                                           // global step (ring position) of the next k-tile to multiply
    if constexpr (KG != 0) {                             // row numbers of k-tiles 0 .. AHEAD + 1, before anything else
        for (int t = 0; t < AHEAD + 2; ++t) issue_idx(cur.e, t, t);
        __builtin_amdgcn_s_waitcnt(waitcnt_imm(0, false));
        __builtin_amdgcn_s_barrier();
    }
    for (int t = 0; t < AHEAD; ++t) {                    // KT >= AHEAD is a launch condition (KG: KT >= 8)
        uint32_t kr[NCP] = {};
        if constexpr (KG != 0) idx_rows(t, kr[0], kr[1]);
#pragma unroll
        for (int j = 0; j < 2 * NCP; ++j)
            issue_copy(cur, t, t, j, (KG == 1 && j < NCP) ? kr[j] : (KG == 2 && j >= NCP) ? kr[j - NCP] : 0u);
        // the order of the steady state: ... tile, tile, indices, tile, indices, so that its wait counts hold from
        // the first iteration on
        if constexpr (KG != 0) if (t >= 1 && wave == 0) issue_idx(cur.e, t + AHEAD + 1, t + AHEAD + 1);
    }
    __builtin_amdgcn_s_waitcnt(waitcnt_imm((AHEAD - 1) * 2 * NCP, false));
    __builtin_amdgcn_s_barrier();
    load_frags(0, 0, ck0);

    for (;;) {
        const int qn = q + 8 * GS;                       // same XCD, next round
        const bool has_next = qn < total;
        if (has_next) setup(qn, nxt);
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < TB; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
        const int KT = cur.KT;
        // Fetching part: k-tile kt + AHEAD, which past KT is a k-tile of the next tile.  The source is
        // chosen with selects outside the unrolled MFMA sequences, which carry no branches.
        const int kt_fetch = has_next ? KT : KT - AHEAD;
        int kt = 0;
        for (; kt < kt_fetch; ++kt, ++g) {
            const bool in_cur = kt + AHEAD < KT;
            const int kf = in_cur ? kt + AHEAD : kt + AHEAD - KT;
            const char* srcA = in_cur ? cur.Abase : nxt.Abase;
            const char* srcB0 = in_cur ? cur.Bbase : nxt.Bbase;
            const char* srcB1 = in_cur ? cur.Bbase1 : nxt.Bbase1;
            const uint64_t baseA = reinterpret_cast<uint64_t>(srcA) + kf * stepA;
            const uint64_t baseB = b_ktile(srcB0, srcB1, in_cur ? KT : nxt.KT, kf);
            uint32_t offs[2 * NCP];
#pragma unroll
            for (int j = 0; j < 2 * NCP; ++j) offs[j] = in_cur ? cur.off[j] : nxt.off[j];

            auto copy = [&](int j) {
                uint4* dst = lds + ((g + AHEAD) & (NBUF - 1)) * STAGE + (j / NCP) * (BM * CPR) + (wave * NCP + (j % NCP)) * 64;
                const bool gathered = (KG == 1 && j < NCP) || (KG == 2 && j >= NCP);
                const uint64_t b64 = gathered ? reinterpret_cast<uint64_t>(j < NCP ? srcA : srcB0) : j < NCP ? baseA : baseB;
                const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(b64));
                const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(b64 >> 32));
                const char* base = reinterpret_cast<const char*>((static_cast<uint64_t>(hi) << 32) | lo);
                __builtin_amdgcn_global_load_lds((global_cptr)(base + offs[j]), (lds_ptr)dst, 16, 0, 0);
            };
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (KG != 0) {
                // the fragments of the second k-substep and, on the same wait, the rows of the gathered operand for
                // k-tile step g + AHEAD
                int i0, i1;
                tr_frags6_idx(fa[1], fb[1], static_cast<uint32_t>(g & (NBUF - 1)) * (STAGE * 16) + 1024, a_tr, b_tr,
                              idx_addr(g + AHEAD), i0, i1);
                offs[(KG - 1) * NCP] += static_cast<uint32_t>(min(max(i0, 0), p.k_rows - 1)) * kg_row_bytes;
                offs[(KG - 1) * NCP + 1] += static_cast<uint32_t>(min(max(i1, 0), p.k_rows - 1)) * kg_row_bytes;
            } else {
                load_frags(1, g, ck1);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
#pragma unroll
                for (int j = 0; j < TB; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[0][j], fa[0][i], acc[i][j], 0, 0, 0);
                if (i & 1) copy(i >> 1);
                __builtin_amdgcn_sched_barrier(0);
            }
            // step g+1 is in LDS (KG, wave 0: two index copies lie between its tile copies and now)
            if (KG != 0 && wave == 0) __builtin_amdgcn_s_waitcnt(waitcnt_imm(3 * NCP + 2, true));
            else __builtin_amdgcn_s_waitcnt(waitcnt_imm(3 * NCP, true));
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);
            load_frags(0, g + 1, ck0);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
#pragma unroll
                for (int j = 0; j < TB; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[1][j], fa[1][i], acc[i][j], 0, 0, 0);
                if (i & 1) copy(NCP + (i >> 1));
                if constexpr (KG != 0) {
                    if (i == 3 && wave == 0) {           // row numbers of the k-tile IDX_AHEAD steps on (one copy per
                        const bool in7 = kt + IDX_AHEAD < KT;        // iteration, whether anything needs it or not)
                        const int e7 = in7 ? cur.e : (has_next ? nxt.e : cur.e);
                        const int k7 = in7 ? kt + IDX_AHEAD : (has_next ? kt + IDX_AHEAD - KT : 0);
                        issue_idx(e7, k7, g + IDX_AHEAD);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        for (; kt < KT; ++kt, ++g) {                                 // tail of this workgroup's last tile: nothing to fetch
            __builtin_amdgcn_sched_barrier(0);
            load_frags(1, g, ck1);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
#pragma unroll
                for (int j = 0; j < TB; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[0][j], fa[0][i], acc[i][j], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
            __builtin_amdgcn_s_waitcnt(waitcnt_imm(0, true));
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);
            if (kt + 1 < KT) load_frags(0, g + 1, ck0);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
#pragma unroll
                for (int j = 0; j < TB; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[1][j], fa[1][i], acc[i][j], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        // ---- epilogue of cur (the copies of the next tile are in flight)
        constexpr int TO = GLU ? TB / 2 : TB;
        if (GLU && !DUAL && p.C3)
            store_blocks<GLU, DUAL, 4, TB, GLU && !DUAL>(p, acc, cur.e, cur.m0 + wm * 128, cur.n0 + wn * (32 * TO), cur.count, r32, half);
        else
            store_blocks<GLU, DUAL, 4, TB>(p, acc, cur.e, cur.m0 + wm * 128, cur.n0 + wn * (32 * TO), cur.count, r32, half);
        if (!has_next) break;
        cur = nxt;
        q = qn;
    }
}

__device__ __forceinline__ int live_row_tiles(const GemmParams& p, int e, int mg, int BM) {
    const int mtv = (group_rows(p, e) + BM - 1) / BM;
    return min(max(mtv - mg * p.SM, 0), p.SM);
}
__device__ __forceinline__ int live_col_tiles(const GemmParams& p, int ng) { return min(p.NT - ng * p.SN, p.SN); }

// pre[s] = number of live tiles in the super-tiles before s (s <= S = E * MG * NG), by NTH threads
template <int NTH = 512>
__device__ __forceinline__ void live_tile_prefix(const GemmParams& p, int BM, int MG, int NG, int* pre, int* wave_tot) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int S = p.E * MG * NG;
    const int CH = (S + NTH - 1) / NTH;
    auto tiles_of = [&](int s) {
        const int e = s / (MG * NG), r = s - e * (MG * NG);
        return live_row_tiles(p, e, r % MG, BM) * live_col_tiles(p, r / MG);
    };
    int sum = 0;
    for (int i = 0; i < CH; ++i) {
        const int s = tid * CH + i;
        if (s < S) sum += tiles_of(s);
    }
    int inc = sum;
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) {
        const int o = __shfl_up(inc, m, 64);
        if (lane >= m) inc += o;
    }
    if (lane == 63) wave_tot[wave] = inc;
    __syncthreads();
    int run = inc - sum;
    for (int w = 0; w < wave; ++w) run += wave_tot[w];
    for (int i = 0; i < CH; ++i) {
        const int s = tid * CH + i;
        if (s < S) {
            pre[s] = run;
            run += tiles_of(s);
        }
    }
    if (tid == NTH - 1) pre[S] = run;                    // the last thread owns the last chunk (or nothing): run = total
    __syncthreads();
}

// ---------------------------------------------------------------------------------------
// Persistent kernel with 64-wide k-tiles for row-major operands (the one the forward pass and every row-major
// product of the backward pass run): the tile list and the run-on across tile boundaries of the ring form above,
// but every copy instruction fetches whole 128-byte lines (8 rows x 128 bytes instead of 16 rows x 64 bytes).
// Measured on a copy-only loop over L2-resident data the line-sized pieces move 1.6 times the bytes per cycle of
// the half-line ones, and in the ring kernel the copies, not the matrix pipe, set the cycle count.
//
// Matrix instruction: v_mfma_f32_16x16x32_bf16.  The part is power-limited under this kernel, and a register-
// resident loop on random operands sustains 2.0 PFLOP/s with this shape against 1.77 with 32x32x16 (a fifth fewer
// register operands per flop).  Eight waves, two per SIMD; a wave's 128 x 64 slice of the 256 x 256 tile is 8 x 4
// accumulators of 16 x 16 (128 registers).  In an accumulator lane l holds token row l % 16 and the four output
// columns 4 (l / 16) .. + 3 (the weight fragment is the row operand).
//
// Two LDS buffers of 64 KiB (256 token rows + 256 weight rows x 128 bytes).  Step g multiplies buffer g & 1: two
// k-steps of 32 (ks), each split into the token blocks 0..3 and 4..7 (h), four substeps u = 2 ks + h of 16 MFMAs.
// Fragments: lane l reads row l % 16 of a 16-row block and the 16-byte chunk 4 ks + l / 16 of the k-tile (the
// chunk index is XORed with bits of the row on the copy's source side, which keeps each group of 16 lanes on 64
// distinct banks).  Token fragments are double-buffered by h, weight fragments by ks; every fragment read sits
// behind one MFMA of the substep before the one that needs it.  When the fourth substep's fragments have been asked
// for nobody reads that buffer any more: behind one wait (all copies landed, all own LDS reads done) and one
// barrier it is released.
//
// Copies (global_load_lds, no registers).  A wave's copies of k-tile g + 2 go out behind every other MFMA of the
// first half of two substeps: its groups of token rows in the fourth substep of step g (right behind the barrier),
// its groups of weight rows in the first substep of step g + 1.  All eight in one substep is twice what a CU's
// address unit takes in that time, and a wave that waits for a slot there issues no MFMA either (7 % slower); half
// a substep later in each costs 1-4 %.  All of them land before the barrier of step g + 1.  The weight rows of a
// tile are whole column tiles (a launch condition), so their addresses are a wave-uniform base plus one of two
// per-lane offsets that never change; only the token rows carry per-tile lane offsets.  There is always something
// to copy: past the end of a workgroup's list the last k-tile is fetched again into a buffer nobody reads any
// more, which keeps the unrolled MFMA sequences free of branches.
//
// Gathered token rows (row_index).  The 256 row indices of a tile travel through LDS as well: 4-byte
// asynchronous copies by waves 0..3, requested two tiles ahead, so no wave ever waits for a global load while it
// sets up a tile.  Three slots rotate; a slot is read one tile after it was requested (at least two barriers with
// vmcnt(0) lie in between) and rewritten two tiles after it was read.
//
// Measured and not kept in this kernel (per-wave cycle stamps around the barrier, 16-expert 11008-wide workload):
// a step of the 32x32x16 form took 2900 cycles for 2048 cycles of MFMA work at 1.67 GHz, 320 of them waiting for
// copies.  Staging the operands through registers (plain loads issued a whole step ahead and evenly spread, LDS
// writes behind the barrier) removed that wait and brought the step to 2540 cycles, and the clock fell to
// 1.49 GHz: the same time.  One wave per SIMD with 128 x 128 slices (a third fewer LDS bytes per flop) needs
// 2700-2900 cycles of issue alone.  One memory instruction behind each MFMA instead of groups: the same time.
// ---------------------------------------------------------------------------------------
template <bool GLU, bool DUAL = false, bool KEEP = false>
__global__ __launch_bounds__(512) void gemm_bf16_persistent_kernel(GemmParams p) {
    static_assert(!KEEP || (GLU && !DUAL), "the pre-activations are kept by the SwiGLU epilogue only");
    constexpr int NW = 8;                                // waves: 2 (token halves) x 4 (weight quarters)
    constexpr int BM = 256, BR = 256, CPR = 8, SWZ = 1;
    constexpr int BN = GLU ? 128 : 256;
    constexpr int STAGE = (BM + BR) * CPR;               // uint4 per LDS buffer (64 KiB)
    constexpr int NCP = 32 / NW;                         // groups of 8 rows each wave copies per operand
    constexpr int WROWS = 8 * NCP;                       // staged rows of each operand a wave copies
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    uint4* lds = reinterpret_cast<uint4*>(lds_raw);
    __shared__ int pre[kMaxSuperWide + 1];
    __shared__ int wave_tot[NW];
    __shared__ int row_ids[3][BM];                       // gathered rows of a tile: this, the next, the one after
    __shared__ __attribute__((aligned(16))) unsigned char stage_all[NW * kStageBytes];   // epilogue patches, one per wave

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 2, wn = wave & 3;
    const int KCA = (p.lda ? p.lda : p.K) / 8, KCB = (p.ldb ? p.ldb : p.K) / 8;
    const bool gather = p.row_index != nullptr;

    const int MG = (p.MT + p.SM - 1) / p.SM, NG = (p.NT + p.SN - 1) / p.SN;
    const int S = p.E * MG * NG;
    live_tile_prefix<NW * 64>(p, BM, MG, NG, pre, wave_tot);
    const int total = pre[S];
    const int GS = gridDim.x >> 3;                       // tiles per group = workgroups per XCD
    const int xcd = blockIdx.x & 7, slot_l = blockIdx.x >> 3;

    struct Tile {
        int e, m0, n0, count, KT;
        uint64_t Abase, Bbase;                           // wave-uniform; Bbase includes the wave's first weight row
        uint32_t offA[NCP];                              // per-lane byte offsets of the wave's token-row groups
    };
    // row group i of this wave: rows rr0 + 8 i, chunk c0 ^ 4 (i & 1) of the swizzle (8 rows further on flips bit 2)
    const int rr0 = wave * WROWS + (lane >> 3);
    const int c0 = (lane & 7) ^ ((rr0 >> SWZ) & 7);
    const uint32_t laneB[2] = {(static_cast<uint32_t>(lane >> 3) * KCB + ((lane & 7) ^ ((lane >> 4) & 7))) * 16u,
                               (static_cast<uint32_t>(lane >> 3) * KCB + ((lane & 7) ^ ((lane >> 4) & 7) ^ 4)) * 16u};
    const uint64_t strideB8 = static_cast<uint64_t>(8) * KCB * 16;      // 8 weight rows further on

    auto decode = [&](int q, Tile& t) {                  // scalar part of the tile with list index q
        int lo = 0, hi = S;                              // largest s with pre[s] <= q
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (pre[mid] <= q) lo = mid; else hi = mid;
        }
        const int s = __builtin_amdgcn_readfirstlane(lo);
        const int u = __builtin_amdgcn_readfirstlane(q - pre[s]);
        const int e = s / (MG * NG), r = s - e * (MG * NG);
        const int mg = r % MG, ng = r / MG;
        const int vm = live_row_tiles(p, e, mg, BM);
        const int mt = mg * p.SM + u % vm, nt = ng * p.SN + u / vm;
        // (a ragged last column tile is moved back to end on the last column: it computes some columns of its left
        // neighbour once more and stores the same values, and no weight-row address or store needs a bound)
        t.e = e; t.m0 = mt * BM; t.n0 = min(nt * BN, p.N - BN);
        t.count = group_rows(p, e);
        t.KT = group_k(p, e) / 64;
        t.Abase = reinterpret_cast<uint64_t>(p.A) + (gather ? 0 : static_cast<uint64_t>(e) * p.capacity * KCA * 16);
        // this wave's staged weight rows: GLU stages 128 gate rows, then the 128 up rows of the same columns
        const int nrow = t.n0 + (GLU ? (wave % (NW / 2)) * WROWS : wave * WROWS);
        t.Bbase = reinterpret_cast<uint64_t>((GLU && wave >= NW / 2) ? p.B1 : p.B0) +
                  (static_cast<uint64_t>(e) * p.N + nrow) * KCB * 16;
    };
    // asynchronous copy of the tile's row indices into slot `slot` (waves 0..3, 64 rows each)
    auto request_rows = [&](const Tile& t, int slot) {
        if (wave < 4) {
            int m = t.m0 + wave * 64 + lane;
            m = m < t.count ? m : t.count - 1;           // rows past the count replay a valid row; never stored
            const int32_t* src = p.row_index + static_cast<size_t>(t.e) * p.capacity + m;
            __builtin_amdgcn_global_load_lds((global_cptr)src, (lds_ptr)(&row_ids[slot][wave * 64]), 4, 0, 0);
        }
    };
    // per-lane offsets of the token rows; with `gather` the indices have landed in slot `slot`
    auto finish = [&](Tile& t, int slot) {
        int row[NCP];
        if (gather) {                                    // one uniform branch around straight-line code
#pragma unroll
            for (int i = 0; i < NCP; ++i) row[i] = min(max(row_ids[slot][rr0 + 8 * i], 0), p.a_rows - 1);
        } else {
#pragma unroll
            for (int i = 0; i < NCP; ++i) row[i] = min(t.m0 + rr0 + 8 * i, t.count - 1);
        }
#pragma unroll
        for (int i = 0; i < NCP; ++i) t.offA[i] = (static_cast<uint32_t>(row[i]) * KCA + (c0 ^ (4 * (i & 1)))) * 16u;
    };
    auto copy_to = [&](uint64_t b64, uint32_t off, uint4* dst) {
        const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(b64));
        const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(b64 >> 32));
        const char* base = reinterpret_cast<const char*>((static_cast<uint64_t>(hi) << 32) | lo);
        __builtin_amdgcn_global_load_lds((global_cptr)(base + off), (lds_ptr)dst, 16, 0, 0);
    };
    // token-row group i / weight-row group i of the k-tile at abase / bbase into buffer buf
    auto copy_a = [&](uint64_t abase, uint32_t off, int buf, int i) {
        copy_to(abase, off, lds + buf * STAGE + (wave * NCP + i) * 64);
    };
    auto copy_b = [&](uint64_t bbase, int buf, int i) {
        copy_to(bbase + i * strideB8, laneB[i & 1], lds + buf * STAGE + BM * CPR + (wave * NCP + i) * 64);
    };

    // fragments: fah[h][i] = token block 4 h + i, fbk[ks][j] = weight block j of k-step ks
    f32x4 acc[8][4];
    bf16x8 fah[2][4], fbk[2][4];
    const int l16 = lane & 15, kq = lane >> 4;
    const int a_row = (wm * 128 + l16) * CPR;
    int b_row[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        // SwiGLU: blocks 0, 1 are gate rows and 2, 3 the up rows of the same 32 output columns; plain: 64 columns
        const int br = GLU ? ((j >> 1) * 128 + wn * 32 + (j & 1) * 16) : (wn * 64 + j * 16);
        b_row[j] = BM * CPR + (br + l16) * CPR;
    }
    const int ck[2] = {kq ^ ((l16 >> SWZ) & 7), (4 + kq) ^ ((l16 >> SWZ) & 7)};
    auto read_a = [&](int buf, int ks, int h, int idx) {
        fah[h][idx] = __builtin_bit_cast(bf16x8, lds[buf * STAGE + a_row + (4 * h + idx) * 16 * CPR + ck[ks]]);
    };
    auto read_b = [&](int buf, int ks, int idx) {
        fbk[ks][idx] = __builtin_bit_cast(bf16x8, lds[buf * STAGE + b_row[idx] + ck[ks]]);
    };
    // substep u = 2 ks + h; `mem(m)` is the memory work behind its m-th MFMA
    auto substep = [&](int u, auto&& mem) {
        const int ks = u >> 1, h = u & 1;
#pragma unroll
        for (int m = 0; m < 16; ++m) {
            const int i = m >> 2, j = m & 3;
            acc[4 * h + i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fbk[ks][j], fah[h][i], acc[4 * h + i][j], 0, 0, 0);
            mem(m);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    int q = xcd * GS + slot_l;                           // first pass over the list
    if (q >= total) return;                              // uniform: nothing for this workgroup
    Tile cur, nxt;
    decode(q, cur);
    int seq = 0;                                         // tiles this workgroup has started; tile n uses slot n % 3
    if (gather) {
        request_rows(cur, 0);
        if (q + 8 * GS < total) {
            decode(q + 8 * GS, nxt);
            request_rows(nxt, 1);
        }
        __builtin_amdgcn_s_waitcnt(waitcnt_imm(0, false));
        __builtin_amdgcn_s_barrier();                    // the indices were fetched by other waves
    }
    finish(cur, 0);
    int g = 0;                                           // global step: buffer g & 1
    for (int t = 0; t < 2; ++t) {                        // KT >= 2 is a launch condition
#pragma unroll
        for (int i = 0; i < NCP; ++i) copy_a(cur.Abase + t * 128, cur.offA[i], t, i);
#pragma unroll
        for (int i = 0; i < NCP; ++i) copy_b(cur.Bbase + t * 128, t, i);
    }
    __builtin_amdgcn_s_waitcnt(waitcnt_imm(2 * NCP, false));             // the first k-tile (copies retire in order)
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int i = 0; i < 4; ++i) { read_a(0, 0, 0, i); read_b(0, 0, i); }
    uint64_t lateB = cur.Bbase + 128;                    // weight rows still owed to the other buffer (none yet:
                                                         // the second k-tile's own once more)
    for (;;) {
        const int qn = q + 8 * GS;                       // same XCD, next round
        const bool has_next = qn < total;
        if (has_next) {
            decode(qn, nxt);
            finish(nxt, (seq + 1) % 3);
            const int qnn = qn + 8 * GS;
            if (gather && qnn < total) {
                Tile t2;
                decode(qnn, t2);
                request_rows(t2, (seq + 2) % 3);
            }
        }
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int v = 0; v < 4; ++v) acc[i][j][v] = 0.f;
        const int KT = cur.KT;
        for (int kt = 0; kt < KT; ++kt, ++g) {
            // k-tile g + 2: of this tile, else of the next one, else (nothing left) this tile's last one again
            const bool in_cur = kt + 2 < KT;
            const bool from_next = !in_cur && has_next;
            const int kf = in_cur ? kt + 2 : (from_next ? kt + 2 - KT : KT - 1);
            const uint64_t baseA = (from_next ? nxt.Abase : cur.Abase) + kf * 128;
            const uint64_t baseB = (from_next ? nxt.Bbase : cur.Bbase) + kf * 128;
            uint32_t offs[NCP];
#pragma unroll
            for (int i = 0; i < NCP; ++i) offs[i] = from_next ? nxt.offA[i] : cur.offA[i];
            const int buf = g & 1;
            __builtin_amdgcn_sched_barrier(0);
            substep(0, [&](int m) {                      // token blocks 4..7 of this k-step, half of the next k-step's weights,
                if (m < 4) read_a(buf, 0, 1, m);         // and the weight rows of k-tile g + 1 into the other buffer
                else if (m < 6) read_b(buf, 1, m - 4);
                if (m < 8 && (m & 1)) copy_b(lateB, buf ^ 1, m >> 1);
            });
            substep(1, [&](int m) {
                if (m < 4) read_a(buf, 1, 0, m);
                else if (m < 6) read_b(buf, 1, m - 2);
            });
            substep(2, [&](int m) {
                if (m < 4) read_a(buf, 1, 1, m);
            });
            // k-tile g + 1 has landed and this wave's reads of buffer buf are done; past the barrier that holds for all
            __builtin_amdgcn_s_waitcnt(waitcnt_imm(0, true));
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);
            substep(3, [&](int m) {                      // the next k-tile's first fragments, and the token rows of k-tile
                if (m < 4) read_a(buf ^ 1, 0, 0, m);     // g + 2 into the buffer just released
                else if (m < 8) read_b(buf ^ 1, 0, m - 4);
                if (m < 8 && (m & 1)) copy_a(baseA, offs[m >> 1], buf, m >> 1);
            });
            lateB = baseB;
        }
        // ---- epilogue of cur (the copies of the next tile are in flight)
        store_blocks_staged16<GLU, DUAL, KEEP>(p, acc, cur.e, cur.m0 + wm * 128, cur.n0 + wn * (GLU ? 32 : 64), cur.count, lane,
                                               stage_all + wave * kStageBytes);
        if (!has_next) break;
        cur = nxt;
        q = qn;
        ++seq;
    }
    __builtin_amdgcn_s_waitcnt(waitcnt_imm(0, false));   // the re-fetched k-tiles of the last two steps
}

// ---------------------------------------------------------------------------------------
// fp32 grouped GEMM, 64x64 tile, 4x4 outputs per thread, plain FMA
// ---------------------------------------------------------------------------------------
template <bool GLU, bool DUAL = false>
__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmParams p) {
    constexpr int BM = 64, BN = 64, BK = 16, LD = BM + 4;
    __shared__ float As[BK][LD];
    __shared__ float Bs[GLU ? 2 : 1][BK][LD];
    int e, mt, nt;
    if (!decode_tile(p, e, mt, nt)) return;
    const int count = group_rows(p, e);
    const int m0 = mt * BM, n0 = nt * BN;
    if (m0 >= count) return;
    const int tid = threadIdx.x, K = group_k(p, e);
    const int LA = p.lda ? p.lda : p.K, LB = p.ldb ? p.ldb : p.K;
    const float* Ag = static_cast<const float*>(p.A) + (p.row_index ? 0 : static_cast<size_t>(e) * p.capacity * LA);
    const float* B0g = static_cast<const float*>(p.B0) + static_cast<size_t>(e) * p.N * LB;
    const float* B1g = GLU ? static_cast<const float*>(p.B1) + static_cast<size_t>(e) * p.N * LB : nullptr;
    const int lr = tid >> 2, lk = (tid & 3) * 4;                  // staging: row, k offset
    int am = min(m0 + lr, p.capacity - 1);
    if (p.row_index) am = min(max(p.row_index[static_cast<size_t>(e) * p.capacity + am], 0), p.a_rows - 1);
    const int bn = min(n0 + lr, p.N - 1);
    const int ty = tid >> 4, tx = tid & 15;
    float acc[GLU ? 2 : 1][4][4] = {};
    for (int k0 = 0; k0 < K; k0 += BK) {
        const bool kin = k0 + lk < K;                             // K % 4 == 0: a float4 is all in or all out
        const float4 z = make_float4(0.f, 0.f, 0.f, 0.f);
        float4 va = kin ? *reinterpret_cast<const float4*>(Ag + static_cast<size_t>(am) * LA + k0 + lk) : z;
        float4 vb = kin ? *reinterpret_cast<const float4*>(B0g + static_cast<size_t>(bn) * LB + k0 + lk) : z;
        As[lk + 0][lr] = va.x; As[lk + 1][lr] = va.y; As[lk + 2][lr] = va.z; As[lk + 3][lr] = va.w;
        Bs[0][lk + 0][lr] = vb.x; Bs[0][lk + 1][lr] = vb.y; Bs[0][lk + 2][lr] = vb.z; Bs[0][lk + 3][lr] = vb.w;
        if constexpr (GLU) {
            float4 vc = kin ? *reinterpret_cast<const float4*>(B1g + static_cast<size_t>(bn) * LB + k0 + lk) : z;
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
        if constexpr (GLU && DUAL) {
            float* C2g = static_cast<float*>(p.C2) + static_cast<size_t>(e) * p.capacity * p.N;
            *reinterpret_cast<float4*>(C2g + static_cast<size_t>(m) * p.N + n) =
                make_float4(acc[1][i][0], acc[1][i][1], acc[1][i][2], acc[1][i][3]);
        }
        if constexpr (GLU && !DUAL) {
            if (p.C3) {                                           // keep the pre-activations (training-mode forward)
                const size_t o = (static_cast<size_t>(e) * p.capacity + m) * p.N + n;
                *reinterpret_cast<float4*>(static_cast<float*>(p.C2) + o) = make_float4(acc[0][i][0], acc[0][i][1], acc[0][i][2], acc[0][i][3]);
                *reinterpret_cast<float4*>(static_cast<float*>(p.C3) + o) = make_float4(acc[1][i][0], acc[1][i][1], acc[1][i][2], acc[1][i][3]);
            }
        }
        float o[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if constexpr (GLU && !DUAL) {
                const float g = acc[0][i][j];
                o[j] = g / (1.0f + expf(-g)) * acc[1][i][j];
            } else {
                o[j] = acc[0][i][j];
            }
        }
        *reinterpret_cast<float4*>(Cg + static_cast<size_t>(m) * p.N + n) = make_float4(o[0], o[1], o[2], o[3]);
    }
}

template <int BM, int BN, int BK, int WGM, int WGN, bool GLU, int SWZ, bool DUAL = false>
hipError_t launch_bf16(GemmParams p, hipStream_t st) {
    constexpr int BROWS = GLU ? 2 * BN : BN;
    constexpr size_t lds = 2ull * (BM + BROWS) * BK * 2;
    const long long blocks = plan_tiles(p, BM, BN);
    auto kern = gemm_bf16_kernel<BM, BN, BK, WGM, WGN, GLU, SWZ, DUAL>;
    hipError_t err = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), lds);
    if (err != hipSuccess) return err;
    hipLaunchKernelGGL(kern, dim3(static_cast<unsigned>(blocks)), dim3(WGM * WGN * 64), lds, st, p);
    return hipGetLastError();
}

template <bool GLU, int WN = 2, bool DUAL = false, int NBUF = 4>
hipError_t launch_bf16_ring(GemmParams p, hipStream_t st) {
    constexpr size_t lds = static_cast<size_t>(NBUF) * 512 * 32 * 2;        // NBUF buffers of 256 + 256 rows x 32 bf16
    const long long blocks = plan_tiles(p, 256, GLU ? 128 : 256);
    auto kern = gemm_bf16_ring_kernel<GLU, WN, DUAL, NBUF>;
    hipError_t err = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), lds);
    if (err != hipSuccess) return err;
    hipLaunchKernelGGL(kern, dim3(static_cast<unsigned>(blocks)), dim3(128 * WN), lds, st, p);
    return hipGetLastError();
}

// Persistent ring kernel: needs every group's contraction length >= 96 (three k-tiles to prefetch)
// and the super-tile prefix to fit in LDS.
template <bool GLU, bool DUAL = false, bool TRA = false, bool TRB = false, int KG = 0>
hipError_t launch_bf16_persist(GemmParams p, hipStream_t st, int n_cu) {
    constexpr size_t lds = 4ull * 512 * 32 * 2 + (KG != 0 ? 16 * 32 * 4 : 0);        // (+ the ring of row numbers)
    plan_tiles(p, 256, GLU ? 128 : 256);
    auto kern = gemm_bf16_persist_kernel<GLU, DUAL, TRA, TRB, KG>;
    hipError_t err = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), lds);
    if (err != hipSuccess) return err;
    hipLaunchKernelGGL(kern, dim3(static_cast<unsigned>(n_cu / 8 * 8)), dim3(512), lds, st, p);
    return hipGetLastError();
}
template <bool GLU, bool DUAL = false, bool KEEP = false>
hipError_t launch_bf16_persistent(GemmParams p, hipStream_t st, int n_cu) {
    constexpr size_t lds = 2ull * 512 * 64 * 2;                             // two buffers of 256 + 256 rows x 64 bf16
    plan_tiles(p, 256, GLU ? 128 : 256, true);
    auto kern = gemm_bf16_persistent_kernel<GLU, DUAL, KEEP>;
    hipError_t err = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), lds);
    if (err != hipSuccess) return err;
    hipLaunchKernelGGL(kern, dim3(static_cast<unsigned>(n_cu / 8 * 8)), dim3(512), lds, st, p);
    return hipGetLastError();
}
// the 64-wide persistent kernel bounds no weight-row address: at least one whole column tile, and 16-byte stores
// (its ragged last tile overlaps the one before)
inline bool whole_column_tiles(const GemmParams& g, bool glu) { return g.N >= (glu ? 128 : 256) && g.N % 8 == 0; }
inline bool persist_ok(const GemmParams& g, bool glu, int max_super = kMaxSuper) {
    GemmParams t = g;
    plan_tiles(t, 256, glu ? 128 : 256, max_super == kMaxSuperWide);
    const long long MG = (t.MT + t.SM - 1) / t.SM, NG = (t.NT + t.SN - 1) / t.SN;
    // (with k_counts the contraction is at least min(128, K) long: four k-tiles)
    return g.K >= 128 && static_cast<long long>(g.E) * MG * NG <= max_super;
}

template <bool GLU, bool DUAL = false>
hipError_t launch_f32(GemmParams p, hipStream_t st) {
    const long long blocks = plan_tiles(p, 64, 64);
    hipLaunchKernelGGL((gemm_f32_kernel<GLU, DUAL>), dim3(static_cast<unsigned>(blocks)), dim3(256), 0, st, p);
    return hipGetLastError();
}

}  // namespace

size_t ffn_ws_bytes(const etr_config& c) {
    return align_up(static_cast<size_t>(c.E) * c.capacity * c.H * elt_bytes(c.dtype));
}

// The pipelined kernels need K % 64 == 0 (copies cannot zero-fill a K tail) and 32-bit byte
// offsets inside one operand; everything else takes the register-staged kernel.
static bool pipelined_ok(const GemmParams& g, size_t a_rows) {
    const size_t a_row_bytes = static_cast<size_t>(g.lda ? g.lda : g.K) * 2, b_row_bytes = static_cast<size_t>(g.ldb ? g.ldb : g.K) * 2;
    return g.K % 64 == 0 && a_row_bytes % 16 == 0 && b_row_bytes % 16 == 0 && a_rows * a_row_bytes < (1ull << 32) &&
           static_cast<size_t>(g.N) * b_row_bytes < (1ull << 32);
}

// General entry for the other stages of the library: grouped "NT" product
//   C[g][m][n] = sum_k A[g][m][k] * B[g][n][k],  g < G, m < m_counts[g] (or M), k < k_counts[g] (or K).
static GemmParams params_of(const GroupedGemm& q) {
    GemmParams g{q.A, q.B0, q.B1, q.C, q.m_counts, q.G, q.M, q.N, q.K, 0, 0, 0, 0, q.row_index, q.a_rows};
    g.lda = q.lda; g.ldb = q.ldb; g.k_counts = q.k_counts; g.C2 = q.C2;
    g.k_index = q.k_index; g.k_index_stride = q.k_index_stride; g.k_rows = q.k_rows; g.k_gather = q.k_gather;
    g.split_m = q.split_m;
    return g;
}

// Operands stored with the contraction index slow run only on the persistent bf16 kernel.
bool grouped_gemm_transposed_ok(const GroupedGemm& q) {
    if (q.dtype != ETR_BF16 || q.epilogue != GEMM_PLAIN || !(q.ta || q.tb)) return false;
    if (q.K < 128 || q.K % 64 != 0 || q.N % 4 != 0) return false;
    if (q.tb && (q.N % 8 != 0 || q.N < 8)) return false;           // 16-byte chunks along the rows of a [K][rows] operand
    if (q.ta && (q.M % 8 != 0 || q.M < 8)) return false;
    const int lda = q.lda ? q.lda : q.K, ldb = q.ldb ? q.ldb : q.K;
    if (lda % 8 != 0 || ldb % 8 != 0) return false;
    if (q.ta && (q.row_index || q.m_counts)) return false;
    if (q.B1 && !(q.tb && q.K % 128 == 0 && !q.k_counts)) return false;          // split B: two halves of whole k-tiles
    // 32-bit per-lane offsets inside one k-tile / one operand
    const size_t a_span = q.ta ? 32ull * lda * 2 : (q.row_index ? static_cast<size_t>(q.a_rows) : static_cast<size_t>(q.M)) * lda * 2;
    const size_t b_span = q.tb ? 32ull * ldb * 2 : static_cast<size_t>(q.N) * ldb * 2;
    if (a_span >= (1ull << 32) || b_span >= (1ull << 32)) return false;
    if (q.split_m && (!q.ta || q.split_m % 32 != 0 || q.M != 2 * q.split_m || !q.C2 || q.m_counts)) return false;
    if (q.k_gather) {
        // gathered contraction rows: both operands transposed, eight k-tiles per group at least, 32-bit row offsets
        if (!(q.ta && q.tb) || (q.k_gather != 1 && q.k_gather != 2) || !q.k_index || q.k_index_stride < 1 || q.k_rows < 1) return false;
        if (q.K < 256 || q.B1) return false;
        if (static_cast<size_t>(q.k_rows) * (q.k_gather == 1 ? lda : ldb) * 2 >= (1ull << 32)) return false;
    }
    return persist_ok(params_of(q), false);
}

hipError_t launch_grouped_gemm(const GroupedGemm& q, hipStream_t st) {
    GemmParams g = params_of(q);
    if (q.N % 4 != 0 || q.K < 0 || q.G < 1 || q.M < 1) return hipErrorInvalidValue;
    if (q.ta || q.tb) {
        if (!grouped_gemm_transposed_ok(q)) return hipErrorInvalidValue;
        const int n_cu = cu_count();
        if (q.k_gather == 1) return launch_bf16_persist<false, false, true, true, 1>(g, st, n_cu);
        if (q.k_gather == 2) return launch_bf16_persist<false, false, true, true, 2>(g, st, n_cu);
        if (q.ta && q.tb) return launch_bf16_persist<false, false, true, true>(g, st, n_cu);
        if (q.tb) return launch_bf16_persist<false, false, false, true>(g, st, n_cu);
        return launch_bf16_persist<false, false, true, false>(g, st, n_cu);
    }
    if (q.dtype == ETR_BF16) {
        if (q.K % 8 != 0 || (q.lda ? q.lda : q.K) % 8 != 0 || (q.ldb ? q.ldb : q.K) % 8 != 0) return hipErrorInvalidValue;
        const bool ring = pipelined_ok(g, q.row_index ? static_cast<size_t>(q.a_rows) : static_cast<size_t>(q.M));
        if (ring && persist_ok(g, q.epilogue != GEMM_PLAIN, kMaxSuperWide) && whole_column_tiles(g, q.epilogue != GEMM_PLAIN)) {
            const int n_cu = cu_count();
            switch (q.epilogue) {
                case GEMM_PLAIN: return launch_bf16_persistent<false>(g, st, n_cu);
                case GEMM_SWIGLU: return launch_bf16_persistent<true>(g, st, n_cu);
                case GEMM_DUAL: return launch_bf16_persistent<true, true>(g, st, n_cu);
            }
        }
        switch (q.epilogue) {
            case GEMM_PLAIN: return ring ? launch_bf16_ring<false, 4>(g, st) : launch_bf16<128, 128, 64, 2, 2, false, 1>(g, st);
            case GEMM_SWIGLU: return ring ? launch_bf16_ring<true, 4>(g, st) : launch_bf16<128, 64, 64, 2, 2, true, 1>(g, st);
            case GEMM_DUAL: return ring ? launch_bf16_ring<true, 4, true>(g, st) : launch_bf16<128, 64, 64, 2, 2, true, 1, true>(g, st);
        }
        return hipErrorInvalidValue;
    }
    if (q.K % 4 != 0 || (q.lda ? q.lda : q.K) % 4 != 0 || (q.ldb ? q.ldb : q.K) % 4 != 0) return hipErrorInvalidValue;
    switch (q.epilogue) {
        case GEMM_PLAIN: return launch_f32<false>(g, st);
        case GEMM_SWIGLU: return launch_f32<true>(g, st);
        case GEMM_DUAL: return launch_f32<true, true>(g, st);
    }
    return hipErrorInvalidValue;
}

bool ffn_can_gather(const etr_config& c) {
    if (c.dtype != ETR_BF16) return false;
    GemmParams g1{nullptr, nullptr, nullptr, nullptr, nullptr, c.E, c.capacity, c.H, c.d, 0, 0, 0, 0, nullptr, c.T};
    return pipelined_ok(g1, static_cast<size_t>(c.T));
}

hipError_t launch_expert_ffn(const etr_config& c, const void* xp, const int32_t* counts, const void* w_gate,
                             const void* w_up, const void* w_down, void* yp, void* hidden, hipStream_t st,
                             hipEvent_t between, const int32_t* gather_rows, void* a_save, void* b_save) {
    // with gather_rows (= slot_token) xp is the token matrix x itself and GEMM-1 fetches row
    // gather_rows[e][s] of it: the rearrangement is folded into the operand load
    GemmParams g1{xp, w_gate, w_up, hidden, counts, c.E, c.capacity, c.H, c.d, 0, 0, 0, 0, gather_rows, c.T};
    GemmParams g2{hidden, w_down, nullptr, yp, counts, c.E, c.capacity, c.d, c.H, 0, 0, 0, 0, nullptr, c.capacity};
    if (a_save && b_save) { g1.C2 = a_save; g1.C3 = b_save; }      // training mode: GEMM-1 also keeps W_gate x and W_up x
    hipError_t err;
    if (c.dtype == ETR_BF16) {
        if (gather_rows && !ffn_can_gather(c)) return hipErrorInvalidValue;
        const bool pipe1 = pipelined_ok(g1, gather_rows ? static_cast<size_t>(c.T) : static_cast<size_t>(c.capacity));
        const int n_cu = cu_count();
        if (pipe1 && persist_ok(g1, true, kMaxSuperWide) && whole_column_tiles(g1, true))
            err = g1.C3 ? launch_bf16_persistent<true, false, true>(g1, st, n_cu) : launch_bf16_persistent<true>(g1, st, n_cu);
        else err = (pipe1 && !g1.C3) ? launch_bf16_ring<true, 4>(g1, st) : launch_bf16<128, 64, 64, 2, 2, true, 1>(g1, st);
        if (err != hipSuccess) return err;
        if (between && (err = hipEventRecord(between, st)) != hipSuccess) return err;
        if (!pipelined_ok(g2, c.capacity)) return launch_bf16<128, 128, 64, 2, 2, false, 1>(g2, st);
        if (persist_ok(g2, false, kMaxSuperWide) && whole_column_tiles(g2, false)) return launch_bf16_persistent<false>(g2, st, n_cu);
        return launch_bf16_ring<false, 4>(g2, st);
    }
    if (gather_rows) return hipErrorInvalidValue;
    err = launch_f32<true>(g1, st);
    if (err != hipSuccess) return err;
    if (between && (err = hipEventRecord(between, st)) != hipSuccess) return err;
    return launch_f32<false>(g2, st);
}

}  // namespace etr
