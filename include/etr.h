/* etr.h - C ABI of the MI355X (gfx950) library for the forward pass of one
 * Expert-Token Resonance (ETR) Mixture-of-Experts layer.
 *
 * Notation (paper symbol -> here): tokens s -> T; experts n -> E; hidden size d;
 * GrAP group size D; pooled width P = d/D; token Top-l -> k; expert capacity C
 * (`capacity`); FFN hidden size H; affinity delta_ti -> score[t][e].
 *
 * Conventions shared by every entry point
 *  - Every pointer except the config is a DEVICE pointer owned by the caller.
 *    The library never allocates, frees or keeps device memory and holds no
 *    global state.  All arrays are dense, row-major, innermost index contiguous.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Calls only enqueue work; they never synchronise with the host.
 *  - Stream capture: every entry point may be captured into a HIP graph, with one rule: the FIRST call of an
 *    entry point for a given shape on a device must happen outside capture (it may raise a kernel's
 *    dynamic-LDS limit and query the device once; later calls only launch kernels).
 *  - Arguments are checked on the host before anything is launched; on error
 *    nothing is launched and a status is returned:
 *      ETR_ERR_NULL         a required pointer is NULL
 *      ETR_ERR_SHAPE        a dimension is <= 0, d % D != 0, k < 1 or k > E
 *                           (k is ignored in ECR mode), capacity < 1
 *      ETR_ERR_UNSUPPORTED  E > 64, d % 8 != 0, H % 8 != 0, unknown dtype/mode/cos
 *      ETR_ERR_WORKSPACE    ws_bytes smaller than the matching *_workspace_bytes(cfg)
 *      ETR_ERR_ALIGN        a pointer is not 16-byte aligned
 *      ETR_ERR_HIP          the HIP runtime reported an error at launch
 *      ETR_ERR_TOO_LARGE    (etr_select_noalloc only) the configuration needs more scratch than the
 *                           library's static array holds
 *  - capacity > T is legal: selection keeps min(capacity, #candidates) tokens
 *    and the buffers keep the stride `capacity`.
 *  - Ties are broken towards the lowest index (expert index in the token's
 *    choice, token index in the expert's choice); comparisons are on the fp32
 *    score as stored, -0.0 and +0.0 tie.  NaN or Inf in x or score: undefined
 *    routing.
 *  - dtype is the storage type of x, the FFN weights, xp, yp and out; all
 *    arithmetic accumulates in fp32.  score, gate and w_emb are always fp32.
 */
#ifndef ETR_H
#define ETR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ETR_OK = 0, ETR_ERR_NULL = 1, ETR_ERR_SHAPE = 2, ETR_ERR_UNSUPPORTED = 3,
    ETR_ERR_WORKSPACE = 4, ETR_ERR_ALIGN = 5, ETR_ERR_HIP = 6, ETR_ERR_TOO_LARGE = 7
} etr_status;

typedef enum { ETR_F32 = 0, ETR_BF16 = 1 } etr_dtype;

/* Which half of the bidirectional selection is active; a host-side choice
 * (Sec. Training Strategy: token choice early in training, expert choice late). */
typedef enum {
    ETR_MODE_TCR = 0, ETR_MODE_ECR = 1, ETR_MODE_BIDIR = 2,
    /* variant readings (see etr_select) */
    ETR_MODE_TCR_RANK = 3, ETR_MODE_BIDIR_STRICT = 4
} etr_mode;

/* Norm used in the cosine of Eq. 4 once the pooled width P may differ from E:
 * FULL   cos(x_t, lift(w_e)) in R^d, lift = every pooled coordinate spread evenly
 *        over its D inputs; equals Eqs. 2-4 exactly when P = E and w_emb = I;
 * POOLED cos(GrAP(x_t), w_e) in R^P. */
typedef enum { ETR_COS_FULL = 0, ETR_COS_POOLED = 1 } etr_cos_mode;

typedef struct {
    int32_t T, d, E, D, k, capacity, H;
    int32_t dtype;      /* etr_dtype    */
    int32_t mode;       /* etr_mode     */
    int32_t cos;        /* etr_cos_mode */
    int32_t gate_norm;  /* 0: weights of Eq. 1 = softmax over all experts, as it is;
                           1 (variant): renormalised over the experts that kept the token */
} etr_config;

/* Bytes of device workspace for this config: etr_workspace_bytes is what
 * etr_moe_forward needs (it covers the two stage calls as well; the permuted
 * token buffer is part of it only where the fused call cannot gather the rows
 * inside the first GEMM, i.e. fp32 and odd widths);
 * etr_select_workspace_bytes and etr_ffn_workspace_bytes are the smaller
 * amounts that etr_select and etr_expert_ffn need when called on their own.
 * Each returns 0 for an invalid config. Host-only, launches nothing. */
size_t etr_workspace_bytes(const etr_config* cfg);
size_t etr_select_workspace_bytes(const etr_config* cfg);
size_t etr_ffn_workspace_bytes(const etr_config* cfg);

/* Static, human-readable name of a status code. */
const char* etr_status_string(etr_status s);

/* GrAP + affinity + gate (Sec. Cost-Efficient Sparse Expert-Token Affinity, Eqs. 2-4;
 * gate: the row softmax of Eq. 1's text, without the noise term).
 *   x      [T][d]   dtype   in
 *   w_emb  [E][d/D] fp32    in   expert embeddings (rows should be mutually orthogonal;
 *                                their norm is computed, not assumed)
 *   score  [T][E]   fp32    out  cosine affinity; 0 for a zero-norm token
 *   gate   [T][E]   fp32    out  softmax over e of score[t][.]
 */
etr_status etr_route(const etr_config* cfg, const void* x, const float* w_emb,
                     float* score, float* gate, void* stream);

/* Bidirectional selection under the capacity bound (Sec. Routing Strategy, Eqs. 5-6;
 * keep rules of the pure phases: Proof of the Theorem, parts 1 and 2).
 *   TCR   every token lists its k best experts; expert e keeps the `capacity`
 *         lowest-index tokens among those that listed it
 *   ECR   expert e keeps its min(capacity, T) highest-score tokens of all T; k ignored
 *   BIDIR expert e keeps its `capacity` highest-score tokens among those that listed it
 *   TCR_RANK (variant of TCR for k > 1, where the paper's rule is stated for one choice only):
 *         every token's first choice is served before any second choice, and so on; expert e
 *         keeps the first `capacity` of its choosers in the order (position in the token's list,
 *         token index)
 *   BIDIR_STRICT (variant of BIDIR): the pair survives iff the token lists the expert and is among
 *         the expert's min(capacity, T) highest-score tokens of ALL T: the intersection of the two
 *         pure phases, a subset of BIDIR's keep set
 *   score        [T][E]        fp32  in
 *   topk_expert  [T][k]        int32 out  token's experts by descending score; may be NULL;
 *                                         not written in ECR mode
 *   slot_of      [T][E]        int32 out  slot of token t in expert e's buffer, -1 if not kept;
 *                                         slots of one expert ascend with the token index
 *   slot_token   [E][capacity] int32 out  inverse table; -1 marks an empty slot
 *   counts       [E]           int32 out  kept tokens per expert
 *   ws, ws_bytes               scratch, >= etr_select_workspace_bytes(cfg), 16-byte aligned
 */
etr_status etr_select(const etr_config* cfg, const float* score, int32_t* topk_expert,
                      int32_t* slot_of, int32_t* slot_token, int32_t* counts,
                      void* ws, size_t ws_bytes, void* stream);

/* etr_select for callers that cannot allocate and have no workspace to hand over: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels, same results, bit for bit; the
 * scratch that etr_select takes as `ws` lives in a static device array of the library instead
 * (etr_select_noalloc_max_bytes() = 8 MiB per GPU the library runs on, held until the process ends).
 *  - etr_select_workspace_bytes(cfg) must not exceed that size, else ETR_ERR_TOO_LARGE and nothing is launched
 *    (all five workloads of the benchmark fit: the largest needs 6.7 MiB).
 *  - The call allocates nothing and frees nothing.  Its first call on a device looks the array's address up
 *    (hipGetSymbolAddress), so make that first call outside stream capture; later calls only launch kernels.
 *  - Every call on one GPU uses the same array.  Nothing in it has to start at zero (the kernels write every
 *    word they read), but two calls that overlap in time on one GPU (different streams, or graphs replayed
 *    concurrently) race on it: serialise them.
 * Arguments as etr_select, without ws / ws_bytes. */
size_t etr_select_noalloc_max_bytes(void);
etr_status etr_select_noalloc(const etr_config* cfg, const float* score, int32_t* topk_expert,
                              int32_t* slot_of, int32_t* slot_token, int32_t* counts, void* stream);

/* Token rearrangement into capacity-bounded per-expert buffers (the slot table I_{ki} of Eq. 6).
 *   x [T][d] in; slot_token [E][capacity], counts [E] in
 *   xp [E][capacity][d] dtype out: xp[e][s] = x[slot_token[e][s]] for s < counts[e];
 *   rows s >= counts[e] are left untouched (never read downstream).
 */
etr_status etr_dispatch(const etr_config* cfg, const void* x, const int32_t* slot_token,
                        const int32_t* counts, void* xp, void* stream);

/* Expert networks on the kept rows (Sec. Locality Loss: experts are FFN layers; the
 * Mixtral-style SwiGLU form): yp[e][s] = W_down[e] (SiLU(W_gate[e] xp[e][s]) .* (W_up[e] xp[e][s]))
 * for s < counts[e].  bf16: MFMA grouped GEMM, fp32 accumulate, the hidden activation and
 * yp are rounded to bf16.  fp32: plain FMA kernels.
 *   xp [E][capacity][d] in; counts [E] in (device; the grid is sized for `capacity`)
 *   w_gate, w_up [E][H][d]; w_down [E][d][H]   dtype in
 *   yp [E][capacity][d] dtype out; rows s >= counts[e] are left untouched
 *   ws, ws_bytes: scratch, >= etr_ffn_workspace_bytes(cfg); holds the hidden activation [E][capacity][H]
 */
etr_status etr_expert_ffn(const etr_config* cfg, const void* xp, const int32_t* counts,
                          const void* w_gate, const void* w_up, const void* w_down,
                          void* yp, void* ws, size_t ws_bytes, void* stream);

/* Gate-weighted sum of Eq. 1 over the experts that kept the token, ascending e, fp32
 * accumulation, one rounding to dtype.  A token kept by no expert gives a zero row.
 * With cfg->gate_norm = 1 the weights gate[t][e] of a token are divided by their sum over the
 * experts that kept it.
 *   yp [E][capacity][d] in; gate [T][E], slot_of [T][E] in; out [T][d] dtype out
 */
etr_status etr_combine(const etr_config* cfg, const void* yp, const float* gate,
                       const int32_t* slot_of, void* out, void* stream);

/* The whole layer (Sec. Model Architecture, Eqs. 1-6) on one stream, no host
 * synchronisation: route -> select -> dispatch -> expert FFN -> combine.
 *   x, w_emb, w_gate, w_up, w_down: as above; out [T][d] dtype
 *   score, gate_out [T][E], topk_expert [T][k], slot_of [T][E], slot_token [E][capacity],
 *   counts [E]: optional outputs, each may be NULL (then it lives in ws)
 */
etr_status etr_moe_forward(const etr_config* cfg, const void* x, const float* w_emb,
                           const void* w_gate, const void* w_up, const void* w_down, void* out,
                           float* score, float* gate_out, int32_t* topk_expert, int32_t* slot_of,
                           int32_t* slot_token, int32_t* counts,
                           void* ws, size_t ws_bytes, void* stream);

/* ---- beyond the forward chain: what a trainer reads off the routing ------------------------- */

/* etr_select with the two adaptive bounds of the method:
 *  - capacity_dev (device int32[1], may be NULL): a capacity that lives on the device, e.g. the
 *    output of etr_capacity_lower_bound; the selection uses min(cfg->capacity, max(1, *capacity_dev))
 *    and the buffers keep the stride cfg->capacity, so no host round trip is needed;
 *  - affinity_sum_threshold (host float; <= 0 switches it off): the adaptive token count of
 *    Sec. Routing Strategy ("the expert chooses its Top-l tokens where l is determined by a threshold
 *    of the sum of affinity scores"; the paper gives no value, so it is an argument).  Expert e walks
 *    its candidates from the highest affinity down and stops at the first prefix whose affinity sum
 *    reaches the threshold (all candidates if the positive affinities never get there); it keeps
 *    min(capacity, that prefix length).  Affinities are summed as integers round(clamp(s,-1,1)*2^30),
 *    so the decision does not depend on the order of summation.  Ignored in TCR mode (position
 *    priority, also TCR_RANK); not defined for BIDIR_STRICT (ETR_ERR_UNSUPPORTED); T must be
 *    <= 2^22 when it is on.
 * Everything else as etr_select. */
etr_status etr_select_adaptive(const etr_config* cfg, const float* score, const int32_t* capacity_dev,
                               float affinity_sum_threshold, int32_t* topk_expert, int32_t* slot_of,
                               int32_t* slot_token, int32_t* counts, void* ws, size_t ws_bytes, void* stream);

/* Scratch for the two reductions below. 0 for an invalid config. */
size_t etr_stats_workspace_bytes(const etr_config* cfg);

/* Statistics behind the losses of Sec. Locality Loss (all outputs on the device):
 *   load_frac [E] fp32  D_c: counts[e] / sum(counts), the current distribution of kept
 *                       (token, expert) assignments; all zero if nothing is kept
 *   mean_gate [E] fp32  (1/T) sum_t gate[t][e]
 *   kl        [1] fp32  KL(D_c || D_l) = sum_e D_c(e) ln(D_c(e) / target[e]); terms with D_c(e) = 0
 *                       are 0, target[e] = 0 < D_c(e) gives +inf; L_loc = mu * kl is the caller's
 *   n_unrouted[1] int32 tokens kept by no expert
 *   gate [T][E], slot_of [T][E], counts [E], target [E] (D_l, fp32): in
 * Fixed summation order: results are bit-reproducible. */
etr_status etr_route_stats(const etr_config* cfg, const float* gate, const int32_t* slot_of,
                           const int32_t* counts, const float* target, float* load_frac, float* mean_gate,
                           float* kl, int32_t* n_unrouted, void* ws, size_t ws_bytes, void* stream);

/* Lower bound of the expert capacity, Remark of Sec. Dynamic Lower Bound Module:
 *   C_min = (1/n) exp{ d * dmax^2 / (2 - dmax^2) }, dmax = largest affinity of the batch, n = E.
 *   dmax [1] fp32 out, capacity [1] int32 out = ceil(C_min) clamped into [1, T]; the exponent is
 *   evaluated in fp64 and compared in the log domain (no overflow for real d). */
etr_status etr_capacity_lower_bound(const etr_config* cfg, const float* score, float* dmax,
                                    int32_t* capacity, void* ws, size_t ws_bytes, void* stream);

/* ---- backward of the layer ---------------------------------------------------------------- */

/* Scratch of etr_moe_backward (transposed weights, recomputed pre-activations, transposed
 * per-row gradients, the permuted input gradient). 0 for an invalid config. */
size_t etr_backward_workspace_bytes(const etr_config* cfg);

/* Gradient of the layer of Eqs. 1-6 for an upstream gradient dout, with the routing tables of the
 * forward call held fixed (the kept sets are piecewise constant in x; the gate vectors of Eq. 3 are
 * constants of the method and get no gradient).  With a = Wg x, b = Wu x, h = SiLU(a) .* b,
 * y = Wd h, out[t] = sum_{e kept t} gate[t][e] y_te:
 *   dgate[t][e]  = <dout[t], y_te>  (0 where the pair is not kept)
 *   dscore[t][e] = gate[t][e] (dgate[t][e] - sum_e' dgate[t][e'] gate[t][e'])     (softmax of Eq. 1)
 *   dw_down[e] = sum_t gate dout[t] h^T;  dw_gate[e] = sum_t da x_t^T;  dw_up[e] = sum_t db x_t^T
 *   dx[t] = sum_e (Wg^T da + Wu^T db) + sum_e dscore[t][e] d score[t][e] / d x[t]  (Eq. 4 differentiated,
 *           in the form selected by cfg->cos)
 * The pre-activations a, b are recomputed from x unless the caller hands over the copies that
 * etr_moe_forward_train kept (a_saved, b_saved: both or neither; same results either way, bit for bit).
 *   in : x [T][d], w_emb [E][d/D] fp32, w_gate, w_up [E][H][d], w_down [E][d][H], dout [T][d] (dtype);
 *        score, gate [T][E] fp32, slot_of [T][E], slot_token [E][capacity], counts [E]: outputs of the
 *        forward call (etr_route + etr_select, or etr_moe_forward) for the same x and cfg
 *   out: dx [T][d], dw_gate, dw_up [E][H][d], dw_down [E][d][H] in the layer's dtype, overwritten
 *        (not accumulated); dgate, dscore [T][E] fp32, optional (may be NULL)
 *   a_saved, b_saved [E][capacity][H] dtype in, optional (see above)
 * bf16: products accumulate in fp32; a, b, W_d^T dout and the per-row gradients are rounded to bf16
 * once each between the stages.  E * (d/D) * 4 bytes must fit in 120 KiB (ETR_ERR_UNSUPPORTED). */
etr_status etr_moe_backward(const etr_config* cfg, const void* x, const float* w_emb,
                            const void* w_gate, const void* w_up, const void* w_down,
                            const float* score, const float* gate, const int32_t* slot_of,
                            const int32_t* slot_token, const int32_t* counts, const void* dout,
                            void* dx, void* dw_gate, void* dw_up, void* dw_down,
                            float* dgate, float* dscore, const void* a_saved, const void* b_saved,
                            void* ws, size_t ws_bytes, void* stream);

/* etr_moe_forward in training mode: the same computation and the same `out`, bit for bit, and the
 * FFN pre-activations of the kept rows are kept for etr_moe_backward (which then skips their
 * recomputation, a quarter of its matrix work):
 *   a_save, b_save [E][capacity][H] dtype out: W_gate x and W_up x of buffer row (e, s), s < counts[e]
 * Everything else as etr_moe_forward. */
etr_status etr_moe_forward_train(const etr_config* cfg, const void* x, const float* w_emb,
                                 const void* w_gate, const void* w_up, const void* w_down, void* out,
                                 float* score, float* gate_out, int32_t* topk_expert, int32_t* slot_of,
                                 int32_t* slot_token, int32_t* counts, void* a_save, void* b_save,
                                 void* ws, size_t ws_bytes, void* stream);

/* etr_moe_forward with stage boundaries marked on the stream, for measurement.
 *   events: HOST array of ETR_N_STAGE_EVENTS hipEvent_t handles (as void*), created by the
 *   caller; an entry may be NULL (that boundary is then not marked: each recorded event costs a few
 *   microseconds of stream time); event i is recorded on `stream` at boundary i:
 *     0 start | 1 after route | 2 after select | 3 after dispatch | 4 after FFN GEMM-1
 *     (gate/up + SwiGLU) | 5 after FFN GEMM-2 (down) | 6 after combine
 * Computes exactly what etr_moe_forward computes, with the same kernels. */
#define ETR_N_STAGE_EVENTS 7
etr_status etr_moe_forward_profiled(const etr_config* cfg, const void* x, const float* w_emb,
                                    const void* w_gate, const void* w_up, const void* w_down, void* out,
                                    float* score, float* gate_out, int32_t* topk_expert, int32_t* slot_of,
                                    int32_t* slot_token, int32_t* counts,
                                    void* ws, size_t ws_bytes, void* stream, void* const* events);

#ifdef __cplusplus
}
#endif
#endif /* ETR_H */
