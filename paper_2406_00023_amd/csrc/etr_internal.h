// Internal launcher interface between the C-ABI layer (api.hip) and the kernel files.
// Everything here takes device pointers that the API layer has already validated.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "etr.h"

namespace etr {

constexpr int kWave = 64;

// ---- select workspace ------------------------------------------------------
// Column-major copy of the per-expert selection keys plus the per-chunk prefix
// counts of the two-level scan.  All offsets are multiples of 256 bytes.
struct SelectWs {
    uint64_t* cmask;     // [T]          bit e set: token listed expert e (Eq. 5)
    uint32_t* keyT;      // [E][Tpad]    order-preserving key of score[t][e]; 0 = not a candidate
    uint32_t* tau;       // [E]          threshold key of expert e
    int32_t*  need_eq;   // [E]          how many candidates with key == tau are kept (lowest token first)
    int32_t*  pre_gt;    // [E][kMaxChunks] kept-for-sure (key > tau) tokens before the chunk
    int32_t*  pre_eq;    // [E][kMaxChunks] key == tau tokens before the chunk
    int32_t*  pre_kept;  // [E][kMaxChunks] strict-intersection variant: surviving tokens before the chunk
    uint32_t* hist1;     // [E][n_slices][2048] first radix digit counted per slice of the column (long columns only)
    int       n_slices;  // 0: no such pre-pass
    int       slice;     // tokens per slice (multiple of 4)
    int       Tpad;      // row stride of keyT
    int       ipt;       // tokens per chunk (= per thread of the per-expert kernel): 4 ... 64 a power of two, else 4 n
};
constexpr int kSelThreads = 1024;       // threads of the per-expert kernel = max chunks
size_t select_ws_bytes(int T, int E);
SelectWs select_ws_carve(void* ws, int T, int E);
// the allocation-free variant keeps this much scratch in a static device array (select.hip)
constexpr size_t kStaticSelectBytes = 8u << 20;
hipError_t static_select_scratch(void** out);    // its device address on the current device

// ---- launchers ---------------------------------------------------------------
// route.hip
hipError_t launch_route(const etr_config& c, const void* x, const float* w_emb, float* score, float* gate,
                        hipStream_t st);
// select.hip
hipError_t launch_select(const etr_config& c, const float* score, int32_t* topk_expert, int32_t* slot_of,
                         int32_t* slot_token, int32_t* counts, const SelectWs& w, hipStream_t st,
                         const int32_t* capacity_dev = nullptr,   // optional device-side bound <= c.capacity
                         long long sum_need = 0);   // > 0: affinity-sum threshold in 2^-30 units (adaptive token count)
// permute.hip
hipError_t launch_dispatch(const etr_config& c, const void* x, const int32_t* slot_token, const int32_t* counts,
                           void* xp, hipStream_t st);
hipError_t launch_combine(const etr_config& c, const void* yp, const float* gate, const int32_t* slot_of,
                          void* out, hipStream_t st);
// ffn.hip
size_t ffn_ws_bytes(const etr_config& c);
hipError_t launch_expert_ffn(const etr_config& c, const void* xp, const int32_t* counts, const void* w_gate,
                             const void* w_up, const void* w_down, void* yp, void* hidden, hipStream_t st,
                             hipEvent_t between = nullptr,    // optional event recorded between the two GEMMs
                             const int32_t* gather_rows = nullptr,    // see ffn_can_gather
                             void* a_save = nullptr, void* b_save = nullptr);   // optional [E][capacity][H]: W_gate x, W_up x
// True when GEMM-1 can read its rows straight from the token matrix through slot_token
// (then xp is never materialised by the fused forward).
bool ffn_can_gather(const etr_config& c);

// General grouped product of ffn.hip, used by the backward pass:
//   C[g][m][n] = sum_k A[g][m][k] * B[g][n][k]   (both operands contiguous along k)
// A is [G][M][lda] (or, with row_index[G][M], row row_index[g][m] of one [a_rows][lda] matrix),
// B0/B1 are [G][N][ldb], C/C2 are [G][M][N], all of the layer's dtype.  m_counts (optional) bounds the
// rows of each group, k_counts (optional) its contraction length: it is rounded up to a multiple of
// 64, at least 128 (at most K), and the operands must hold zeros in that padding.
enum GemmEpilogue { GEMM_PLAIN = 0, GEMM_SWIGLU = 1, GEMM_DUAL = 2 };   // C = A B0^T | SiLU(A B0^T) .* (A B1^T) | both products
struct GroupedGemm {
    const void* A; const void* B0; const void* B1;
    void* C; void* C2;
    const int32_t* m_counts; const int32_t* k_counts; const int32_t* row_index;
    int G, M, N, K, lda, ldb, a_rows;
    int epilogue;
    int dtype;
    // Operands with the contraction index slow (bf16, plain epilogue only; see grouped_gemm_transposed_ok):
    // ta: A is [G][K][lda] holding A[g][m][k] at (k, m); tb: B0 is [G][K][ldb] holding B[g][n][k] at (k, n).
    // With tb and B1 the contraction is split in the middle: B0 and B1 are [G][K/2][ldb] each.
    bool ta = false, tb = false;
    // With ta and tb, the contraction rows of one operand may come through an index (k_gather 1: A, 2: B0): that
    // operand is then one [k_rows][ld] matrix for all groups and row k of group g is its row
    // k_index[g * k_index_stride + min(k, k_index_stride - 1)], clamped into [0, k_rows); the other operand must hold
    // zeros wherever the index does not name the wanted row (empty slots, padding).  Per-group contraction lengths
    // are then rounded up to at least 256.
    const int32_t* k_index = nullptr;
    int k_index_stride = 0, k_rows = 0, k_gather = 0;
    // With ta and the plain epilogue: output rows m < split_m go to C, the others (as rows m - split_m) to C2, both
    // [G][split_m][N]; M = 2 split_m, split_m a multiple of 32.  (Two products that share B in one launch.)
    int split_m = 0;
};
hipError_t launch_grouped_gemm(const GroupedGemm& g, hipStream_t st);
bool grouped_gemm_transposed_ok(const GroupedGemm& g);

// backward.hip
size_t backward_ws_bytes(const etr_config& c);
hipError_t launch_moe_backward(const etr_config& c, const void* x, const float* w_emb, const void* w_gate,
                               const void* w_up, const void* w_down, const float* score, const float* gate,
                               const int32_t* slot_of, const int32_t* slot_token, const int32_t* counts,
                               const void* dout, void* dx, void* dw_gate, void* dw_up, void* dw_down,
                               float* dgate, float* dscore, void* ws, hipStream_t st,
                               const void* a_saved = nullptr, const void* b_saved = nullptr);   // from a training-mode forward

// stats.hip
size_t stats_ws_bytes(int T, int E);
hipError_t launch_route_stats(const etr_config& c, const float* gate, const int32_t* slot_of, const int32_t* counts,
                              const float* target, float* load, float* mean_gate, float* kl, int32_t* n_unrouted,
                              void* ws, hipStream_t st);
hipError_t launch_capacity_lower_bound(const etr_config& c, const float* score, float* dmax, int32_t* capacity,
                                       void* ws, hipStream_t st);

// Host-side launch helpers (api.hip).  Both remember their answer per device, so a steady-state call issues no
// runtime call besides its launches.
//   cu_count            compute units of the current device (256 if the query fails)
//   ensure_dynamic_lds  raises a kernel's dynamic-LDS limit to `bytes` unless a limit at least that large has
//                       already been set for this (device, kernel); limits up to 64 KiB need no call at all
int cu_count();
hipError_t ensure_dynamic_lds(const void* kernel, size_t bytes);

inline size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }
inline size_t elt_bytes(int dtype) { return dtype == ETR_F32 ? 4 : 2; }

}  // namespace etr
