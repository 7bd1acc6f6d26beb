// C-ABI layer: host-side argument validation, workspace carving and the stage chain
// of the whole layer (Sec. Model Architecture, Eqs. 1-6).  Nothing here computes.
#include <cmath>
#include <cstdint>
#include <mutex>
#include <vector>

#include "etr_internal.h"

namespace etr {

namespace {
constexpr int kMaxDevices = 64;
int current_device() {
    int dev = 0;
    return (hipGetDevice(&dev) == hipSuccess && dev >= 0 && dev < kMaxDevices) ? dev : -1;
}
}  // namespace

int cu_count() {
    static std::mutex mu;
    static int cached[kMaxDevices] = {};
    const int dev = current_device();
    if (dev < 0) return 256;
    std::lock_guard<std::mutex> lock(mu);
    if (cached[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 8) n = 256;
        cached[dev] = n;
    }
    return cached[dev];
}

hipError_t ensure_dynamic_lds(const void* kernel, size_t bytes) {
    if (bytes <= 64 * 1024) return hipSuccess;
    struct Entry { const void* kernel; int dev; size_t bytes; };
    static std::mutex mu;
    static std::vector<Entry> set;
    const int dev = current_device();
    std::lock_guard<std::mutex> lock(mu);
    for (Entry& e : set)
        if (e.kernel == kernel && e.dev == dev) {
            if (e.bytes >= bytes) return hipSuccess;
            const hipError_t err = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(bytes));
            if (err == hipSuccess) e.bytes = bytes;
            return err;
        }
    const hipError_t err = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(bytes));
    if (err == hipSuccess && dev >= 0) set.push_back({kernel, dev, bytes});
    return err;
}

}  // namespace etr

namespace {

using namespace etr;

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Checks that apply to every call.
etr_status check_config(const etr_config* c) {
    if (!c) return ETR_ERR_NULL;
    if (c->T <= 0 || c->d <= 0 || c->E <= 0 || c->D <= 0 || c->H <= 0) return ETR_ERR_SHAPE;
    if (c->d % c->D != 0 || c->capacity < 1) return ETR_ERR_SHAPE;
    if (c->mode < ETR_MODE_TCR || c->mode > ETR_MODE_BIDIR_STRICT) return ETR_ERR_UNSUPPORTED;
    if (c->gate_norm != 0 && c->gate_norm != 1) return ETR_ERR_UNSUPPORTED;
    if (c->mode != ETR_MODE_ECR && (c->k < 1 || c->k > c->E)) return ETR_ERR_SHAPE;
    if (c->dtype != ETR_F32 && c->dtype != ETR_BF16) return ETR_ERR_UNSUPPORTED;
    if (c->cos != ETR_COS_FULL && c->cos != ETR_COS_POOLED) return ETR_ERR_UNSUPPORTED;
    if (c->E > 64 || c->d % 8 != 0 || c->H % 8 != 0) return ETR_ERR_UNSUPPORTED;
    // 32-bit index headroom of the row tables and the LDS budget of the route kernel
    if (static_cast<long long>(c->E) * c->capacity > 0x7FFFFFFFll) return ETR_ERR_UNSUPPORTED;
    if (static_cast<long long>(c->T) * c->E > 0x7FFFFFFFll) return ETR_ERR_UNSUPPORTED;
    const long long P = c->d / c->D;
    if (4ll * (c->E * (P + 64) + 64 + 4 * P) > 160ll * 1024) return ETR_ERR_UNSUPPORTED;
    return ETR_OK;
}

// Workspace of etr_moe_forward: optional outputs that the caller did not ask for, the
// select scratch, the permuted buffers and the hidden activation.
struct ForwardWs {
    size_t score, gate, topk, slot_of, slot_token, counts, select, xp, yp, hidden, total;
};

ForwardWs forward_layout(const etr_config& c) {
    ForwardWs w{};
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes); return o; };
    const size_t TE = static_cast<size_t>(c.T) * c.E, EC = static_cast<size_t>(c.E) * c.capacity;
    w.score = take(TE * 4);
    w.gate = take(TE * 4);
    w.topk = take(static_cast<size_t>(c.T) * (c.k > 0 ? c.k : 1) * 4);
    w.slot_of = take(TE * 4);
    w.slot_token = take(EC * 4);
    w.counts = take(static_cast<size_t>(c.E) * 4);
    w.select = take(select_ws_bytes(c.T, c.E));
    // the permuted token buffer exists only where the fused call really dispatches (fp32 / fall-back shapes):
    // with the rows gathered inside GEMM-1 it is never written
    w.xp = take(ffn_can_gather(c) ? 0 : EC * c.d * elt_bytes(c.dtype));
    w.yp = take(EC * c.d * elt_bytes(c.dtype));
    w.hidden = take(ffn_ws_bytes(c));
    w.total = off;
    return w;
}

#define ETR_REQUIRE_PTR(p)            \
    do {                              \
        if (!(p)) return ETR_ERR_NULL; \
        if (!aligned16(p)) return ETR_ERR_ALIGN; \
    } while (0)
#define ETR_OPTIONAL_PTR(p)           \
    do {                              \
        if ((p) && !aligned16(p)) return ETR_ERR_ALIGN; \
    } while (0)
#define ETR_HIP(call)                           \
    do {                                        \
        if ((call) != hipSuccess) return ETR_ERR_HIP; \
    } while (0)

}  // namespace

extern "C" {

const char* etr_status_string(etr_status s) {
    switch (s) {
        case ETR_OK: return "ok";
        case ETR_ERR_NULL: return "a required pointer is NULL";
        case ETR_ERR_SHAPE: return "invalid shape";
        case ETR_ERR_UNSUPPORTED: return "unsupported configuration";
        case ETR_ERR_WORKSPACE: return "workspace too small";
        case ETR_ERR_ALIGN: return "pointer not 16-byte aligned";
        case ETR_ERR_HIP: return "HIP runtime error";
        case ETR_ERR_TOO_LARGE: return "configuration needs more scratch than the allocation-free entry point holds";
    }
    return "unknown status";
}

size_t etr_workspace_bytes(const etr_config* cfg) {
    if (check_config(cfg) != ETR_OK) return 0;
    return forward_layout(*cfg).total;
}

size_t etr_select_workspace_bytes(const etr_config* cfg) {
    if (check_config(cfg) != ETR_OK) return 0;
    return select_ws_bytes(cfg->T, cfg->E);
}

size_t etr_ffn_workspace_bytes(const etr_config* cfg) {
    if (check_config(cfg) != ETR_OK) return 0;
    return ffn_ws_bytes(*cfg);
}

etr_status etr_route(const etr_config* cfg, const void* x, const float* w_emb, float* score, float* gate,
                     void* stream) {
    etr_status s = check_config(cfg);
    if (s != ETR_OK) return s;
    ETR_REQUIRE_PTR(x); ETR_REQUIRE_PTR(w_emb); ETR_REQUIRE_PTR(score); ETR_REQUIRE_PTR(gate);
    ETR_HIP(launch_route(*cfg, x, w_emb, score, gate, static_cast<hipStream_t>(stream)));
    return ETR_OK;
}

etr_status etr_select(const etr_config* cfg, const float* score, int32_t* topk_expert, int32_t* slot_of,
                      int32_t* slot_token, int32_t* counts, void* ws, size_t ws_bytes, void* stream) {
    etr_status s = check_config(cfg);
    if (s != ETR_OK) return s;
    ETR_REQUIRE_PTR(score); ETR_REQUIRE_PTR(slot_of); ETR_REQUIRE_PTR(slot_token); ETR_REQUIRE_PTR(counts);
    ETR_REQUIRE_PTR(ws); ETR_OPTIONAL_PTR(topk_expert);
    if (ws_bytes < select_ws_bytes(cfg->T, cfg->E)) return ETR_ERR_WORKSPACE;
    const SelectWs w = select_ws_carve(ws, cfg->T, cfg->E);
    ETR_HIP(launch_select(*cfg, score, topk_expert, slot_of, slot_token, counts, w, static_cast<hipStream_t>(stream)));
    return ETR_OK;
}

size_t etr_select_noalloc_max_bytes(void) { return kStaticSelectBytes; }

etr_status etr_select_noalloc(const etr_config* cfg, const float* score, int32_t* topk_expert, int32_t* slot_of,
                              int32_t* slot_token, int32_t* counts, void* stream) {
    etr_status s = check_config(cfg);
    if (s != ETR_OK) return s;
    ETR_REQUIRE_PTR(score); ETR_REQUIRE_PTR(slot_of); ETR_REQUIRE_PTR(slot_token); ETR_REQUIRE_PTR(counts);
    ETR_OPTIONAL_PTR(topk_expert);
    if (select_ws_bytes(cfg->T, cfg->E) > kStaticSelectBytes) return ETR_ERR_TOO_LARGE;
    void* ws = nullptr;
    ETR_HIP(static_select_scratch(&ws));
    const SelectWs w = select_ws_carve(ws, cfg->T, cfg->E);
    ETR_HIP(launch_select(*cfg, score, topk_expert, slot_of, slot_token, counts, w, static_cast<hipStream_t>(stream)));
    return ETR_OK;
}

etr_status etr_select_adaptive(const etr_config* cfg, const float* score, const int32_t* capacity_dev,
                               float affinity_sum_threshold, int32_t* topk_expert, int32_t* slot_of,
                               int32_t* slot_token, int32_t* counts, void* ws, size_t ws_bytes, void* stream) {
    etr_status s = check_config(cfg);
    if (s != ETR_OK) return s;
    ETR_REQUIRE_PTR(score); ETR_REQUIRE_PTR(slot_of); ETR_REQUIRE_PTR(slot_token); ETR_REQUIRE_PTR(counts);
    ETR_REQUIRE_PTR(ws); ETR_OPTIONAL_PTR(topk_expert);
    if (capacity_dev && (reinterpret_cast<uintptr_t>(capacity_dev) & 3u)) return ETR_ERR_ALIGN;
    if (!(affinity_sum_threshold == affinity_sum_threshold)) return ETR_ERR_SHAPE;           // NaN
    if (cfg->T > (1 << 22) && affinity_sum_threshold > 0.f) return ETR_ERR_UNSUPPORTED;       // fixed-point sum headroom
    if (cfg->mode == ETR_MODE_BIDIR_STRICT && affinity_sum_threshold > 0.f) return ETR_ERR_UNSUPPORTED;
    if (ws_bytes < select_ws_bytes(cfg->T, cfg->E)) return ETR_ERR_WORKSPACE;
    const SelectWs w = select_ws_carve(ws, cfg->T, cfg->E);
    long long need = 0;
    if (affinity_sum_threshold > 0.f) {
        const double scaled = static_cast<double>(affinity_sum_threshold) * 1073741824.0;
        need = scaled >= 9.0e18 ? 9000000000000000000ll : llrint(scaled);
        if (need < 1) need = 1;
    }
    ETR_HIP(launch_select(*cfg, score, topk_expert, slot_of, slot_token, counts, w, static_cast<hipStream_t>(stream),
                          capacity_dev, need));
    return ETR_OK;
}

size_t etr_stats_workspace_bytes(const etr_config* cfg) {
    if (check_config(cfg) != ETR_OK) return 0;
    return stats_ws_bytes(cfg->T, cfg->E);
}

etr_status etr_route_stats(const etr_config* cfg, const float* gate, const int32_t* slot_of, const int32_t* counts,
                           const float* target, float* load_frac, float* mean_gate, float* kl, int32_t* n_unrouted,
                           void* ws, size_t ws_bytes, void* stream) {
    etr_status s = check_config(cfg);
    if (s != ETR_OK) return s;
    ETR_REQUIRE_PTR(gate); ETR_REQUIRE_PTR(slot_of); ETR_REQUIRE_PTR(counts); ETR_REQUIRE_PTR(target);
    ETR_REQUIRE_PTR(ws);
    if (!load_frac || !mean_gate || !kl || !n_unrouted) return ETR_ERR_NULL;
    if (ws_bytes < stats_ws_bytes(cfg->T, cfg->E)) return ETR_ERR_WORKSPACE;
    ETR_HIP(launch_route_stats(*cfg, gate, slot_of, counts, target, load_frac, mean_gate, kl, n_unrouted, ws,
                               static_cast<hipStream_t>(stream)));
    return ETR_OK;
}

etr_status etr_capacity_lower_bound(const etr_config* cfg, const float* score, float* dmax, int32_t* capacity,
                                    void* ws, size_t ws_bytes, void* stream) {
    etr_status s = check_config(cfg);
    if (s != ETR_OK) return s;
    ETR_REQUIRE_PTR(score); ETR_REQUIRE_PTR(ws);
    if (!dmax || !capacity) return ETR_ERR_NULL;
    if (ws_bytes < stats_ws_bytes(cfg->T, cfg->E)) return ETR_ERR_WORKSPACE;
    ETR_HIP(launch_capacity_lower_bound(*cfg, score, dmax, capacity, ws, static_cast<hipStream_t>(stream)));
    return ETR_OK;
}

size_t etr_backward_workspace_bytes(const etr_config* cfg) {
    if (check_config(cfg) != ETR_OK) return 0;
    return backward_ws_bytes(*cfg);
}

etr_status etr_moe_backward(const etr_config* cfg, const void* x, const float* w_emb, const void* w_gate,
                            const void* w_up, const void* w_down, const float* score, const float* gate,
                            const int32_t* slot_of, const int32_t* slot_token, const int32_t* counts,
                            const void* dout, void* dx, void* dw_gate, void* dw_up, void* dw_down, float* dgate,
                            float* dscore, const void* a_saved, const void* b_saved, void* ws, size_t ws_bytes,
                            void* stream) {
    etr_status s = check_config(cfg);
    if (s != ETR_OK) return s;
    ETR_REQUIRE_PTR(x); ETR_REQUIRE_PTR(w_emb); ETR_REQUIRE_PTR(w_gate); ETR_REQUIRE_PTR(w_up); ETR_REQUIRE_PTR(w_down);
    ETR_REQUIRE_PTR(score); ETR_REQUIRE_PTR(gate); ETR_REQUIRE_PTR(slot_of); ETR_REQUIRE_PTR(slot_token);
    ETR_REQUIRE_PTR(counts); ETR_REQUIRE_PTR(dout); ETR_REQUIRE_PTR(dx); ETR_REQUIRE_PTR(dw_gate);
    ETR_REQUIRE_PTR(dw_up); ETR_REQUIRE_PTR(dw_down); ETR_REQUIRE_PTR(ws);
    ETR_OPTIONAL_PTR(dgate); ETR_OPTIONAL_PTR(dscore); ETR_OPTIONAL_PTR(a_saved); ETR_OPTIONAL_PTR(b_saved);
    if ((a_saved == nullptr) != (b_saved == nullptr)) return ETR_ERR_NULL;      // both or neither
    if (static_cast<size_t>(cfg->E) * (cfg->d / cfg->D) * 4 > 120 * 1024) return ETR_ERR_UNSUPPORTED;
    if (ws_bytes < backward_ws_bytes(*cfg)) return ETR_ERR_WORKSPACE;
    ETR_HIP(launch_moe_backward(*cfg, x, w_emb, w_gate, w_up, w_down, score, gate, slot_of, slot_token, counts, dout, dx,
                                dw_gate, dw_up, dw_down, dgate, dscore, ws, static_cast<hipStream_t>(stream), a_saved,
                                b_saved));
    return ETR_OK;
}

etr_status etr_dispatch(const etr_config* cfg, const void* x, const int32_t* slot_token, const int32_t* counts,
                        void* xp, void* stream) {
    etr_status s = check_config(cfg);
    if (s != ETR_OK) return s;
    ETR_REQUIRE_PTR(x); ETR_REQUIRE_PTR(slot_token); ETR_REQUIRE_PTR(counts); ETR_REQUIRE_PTR(xp);
    ETR_HIP(launch_dispatch(*cfg, x, slot_token, counts, xp, static_cast<hipStream_t>(stream)));
    return ETR_OK;
}

etr_status etr_expert_ffn(const etr_config* cfg, const void* xp, const int32_t* counts, const void* w_gate,
                          const void* w_up, const void* w_down, void* yp, void* ws, size_t ws_bytes, void* stream) {
    etr_status s = check_config(cfg);
    if (s != ETR_OK) return s;
    ETR_REQUIRE_PTR(xp); ETR_REQUIRE_PTR(counts); ETR_REQUIRE_PTR(w_gate); ETR_REQUIRE_PTR(w_up);
    ETR_REQUIRE_PTR(w_down); ETR_REQUIRE_PTR(yp); ETR_REQUIRE_PTR(ws);
    if (ws_bytes < ffn_ws_bytes(*cfg)) return ETR_ERR_WORKSPACE;
    ETR_HIP(launch_expert_ffn(*cfg, xp, counts, w_gate, w_up, w_down, yp, ws, static_cast<hipStream_t>(stream)));
    return ETR_OK;
}

etr_status etr_combine(const etr_config* cfg, const void* yp, const float* gate, const int32_t* slot_of, void* out,
                       void* stream) {
    etr_status s = check_config(cfg);
    if (s != ETR_OK) return s;
    ETR_REQUIRE_PTR(yp); ETR_REQUIRE_PTR(gate); ETR_REQUIRE_PTR(slot_of); ETR_REQUIRE_PTR(out);
    ETR_HIP(launch_combine(*cfg, yp, gate, slot_of, out, static_cast<hipStream_t>(stream)));
    return ETR_OK;
}

static etr_status forward_impl(const etr_config* cfg, const void* x, const float* w_emb, const void* w_gate,
                               const void* w_up, const void* w_down, void* out, float* score, float* gate_out,
                               int32_t* topk_expert, int32_t* slot_of, int32_t* slot_token, int32_t* counts, void* ws,
                               size_t ws_bytes, void* stream, void* const* events, void* a_save = nullptr,
                               void* b_save = nullptr) {
    etr_status s = check_config(cfg);
    if (s != ETR_OK) return s;
    ETR_REQUIRE_PTR(x); ETR_REQUIRE_PTR(w_emb); ETR_REQUIRE_PTR(w_gate); ETR_REQUIRE_PTR(w_up);
    ETR_REQUIRE_PTR(w_down); ETR_REQUIRE_PTR(out); ETR_REQUIRE_PTR(ws);
    ETR_OPTIONAL_PTR(score); ETR_OPTIONAL_PTR(gate_out); ETR_OPTIONAL_PTR(topk_expert); ETR_OPTIONAL_PTR(slot_of);
    ETR_OPTIONAL_PTR(slot_token); ETR_OPTIONAL_PTR(counts);
    const ForwardWs L = forward_layout(*cfg);
    if (ws_bytes < L.total) return ETR_ERR_WORKSPACE;
    char* base = static_cast<char*>(ws);
    float* sc = score ? score : reinterpret_cast<float*>(base + L.score);
    float* gt = gate_out ? gate_out : reinterpret_cast<float*>(base + L.gate);
    int32_t* tk = topk_expert ? topk_expert : reinterpret_cast<int32_t*>(base + L.topk);
    int32_t* so = slot_of ? slot_of : reinterpret_cast<int32_t*>(base + L.slot_of);
    int32_t* stn = slot_token ? slot_token : reinterpret_cast<int32_t*>(base + L.slot_token);
    int32_t* cn = counts ? counts : reinterpret_cast<int32_t*>(base + L.counts);
    void* xp = base + L.xp;
    void* yp = base + L.yp;
    void* hidden = base + L.hidden;
    const SelectWs sw = select_ws_carve(base + L.select, cfg->T, cfg->E);
    hipStream_t st = static_cast<hipStream_t>(stream);

    auto mark = [&](int i) -> hipError_t {
        return (events && events[i]) ? hipEventRecord(static_cast<hipEvent_t>(events[i]), st) : hipSuccess;
    };
    ETR_HIP(mark(0));
    ETR_HIP(launch_route(*cfg, x, w_emb, sc, gt, st));
    ETR_HIP(mark(1));
    ETR_HIP(launch_select(*cfg, sc, tk, so, stn, cn, sw, st));
    ETR_HIP(mark(2));
    // bf16 with the pipelined GEMM: the rearrangement is folded into GEMM-1's operand load
    // (rows are fetched through slot_token), so no permuted copy of the tokens is written
    const bool gather = ffn_can_gather(*cfg);
    if (!gather) ETR_HIP(launch_dispatch(*cfg, x, stn, cn, xp, st));
    ETR_HIP(mark(3));
    ETR_HIP(launch_expert_ffn(*cfg, gather ? x : xp, cn, w_gate, w_up, w_down, yp, hidden, st,
                              events ? static_cast<hipEvent_t>(events[4]) : nullptr, gather ? stn : nullptr, a_save, b_save));
    ETR_HIP(mark(5));
    ETR_HIP(launch_combine(*cfg, yp, gt, so, out, st));
    ETR_HIP(mark(6));
    return ETR_OK;
}

etr_status etr_moe_forward(const etr_config* cfg, const void* x, const float* w_emb, const void* w_gate,
                           const void* w_up, const void* w_down, void* out, float* score, float* gate_out,
                           int32_t* topk_expert, int32_t* slot_of, int32_t* slot_token, int32_t* counts, void* ws,
                           size_t ws_bytes, void* stream) {
    return forward_impl(cfg, x, w_emb, w_gate, w_up, w_down, out, score, gate_out, topk_expert, slot_of, slot_token,
                        counts, ws, ws_bytes, stream, nullptr);
}

etr_status etr_moe_forward_train(const etr_config* cfg, const void* x, const float* w_emb, const void* w_gate,
                                 const void* w_up, const void* w_down, void* out, float* score, float* gate_out,
                                 int32_t* topk_expert, int32_t* slot_of, int32_t* slot_token, int32_t* counts,
                                 void* a_save, void* b_save, void* ws, size_t ws_bytes, void* stream) {
    ETR_REQUIRE_PTR(a_save); ETR_REQUIRE_PTR(b_save);
    return forward_impl(cfg, x, w_emb, w_gate, w_up, w_down, out, score, gate_out, topk_expert, slot_of, slot_token,
                        counts, ws, ws_bytes, stream, nullptr, a_save, b_save);
}

etr_status etr_moe_forward_profiled(const etr_config* cfg, const void* x, const float* w_emb, const void* w_gate,
                                    const void* w_up, const void* w_down, void* out, float* score, float* gate_out,
                                    int32_t* topk_expert, int32_t* slot_of, int32_t* slot_token, int32_t* counts,
                                    void* ws, size_t ws_bytes, void* stream, void* const* events) {
    if (!events) return ETR_ERR_NULL;
    return forward_impl(cfg, x, w_emb, w_gate, w_up, w_down, out, score, gate_out, topk_expert, slot_of, slot_token,
                        counts, ws, ws_bytes, stream, events);
}

}  // extern "C"
