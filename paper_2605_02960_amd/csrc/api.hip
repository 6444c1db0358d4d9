// extern "C" surface of libmoeprefill: argument checks on the host, then the kernel launches.
// Nothing here allocates, synchronises or copies to the host.
#include "common.h"

using namespace moe;

namespace moe {
ProfileSlot g_profile[MOE_KERNEL_COUNT] = {};
}

namespace {

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

int32_t check_config(const moe_config_t* c) {
    if (!c) return MOE_ERR_NULL_PTR;
    if (c->T < 0 || c->H < 1 || c->E < 1 || c->K < 1 || c->I < 1) return MOE_ERR_BAD_SHAPE;
    if (c->K > c->E || c->K > 32 || c->E > 1024) return MOE_ERR_BAD_SHAPE;
    if ((int64_t)c->T * c->K >= (1ll << 31)) return MOE_ERR_BAD_SHAPE;
    if ((int64_t)c->T * c->E >= (1ll << 31)) return MOE_ERR_BAD_SHAPE;
    if (c->x_dtype != MOE_DTYPE_F32 && c->x_dtype != MOE_DTYPE_BF16) return MOE_ERR_BAD_DTYPE;
    if (c->out_dtype != MOE_DTYPE_F32 && c->out_dtype != MOE_DTYPE_BF16) return MOE_ERR_BAD_DTYPE;
    switch (c->w_dtype) {
        case MOE_DTYPE_F32:
            if (c->x_dtype != MOE_DTYPE_F32) return MOE_ERR_BAD_DTYPE;
            break;
        case MOE_DTYPE_BF16:
            if (c->x_dtype != MOE_DTYPE_BF16) return MOE_ERR_BAD_DTYPE;
            if (c->H % 128 != 0 || c->I % 128 != 0) return MOE_ERR_BAD_SHAPE;
            break;
        case MOE_DTYPE_FP8_E4M3:
            if (c->x_dtype != MOE_DTYPE_BF16) return MOE_ERR_BAD_DTYPE;
            if (c->H % 256 != 0 || c->I % 256 != 0) return MOE_ERR_BAD_SHAPE;
            break;
        default:
            return MOE_ERR_BAD_DTYPE;
    }
    if ((c->flags & ~MOE_FLAG_Y_F32) != 0) return MOE_ERR_UNSUPPORTED;
    return MOE_OK;
}

// [logits T*E f32 (used only when the caller passes no logits buffer)][bf16 path: split router weight]
size_t route_logits_ws(const moe_config_t& c) { return align_up((size_t)c.T * c.E * sizeof(float), 256); }
bool route_uses_mfma(const moe_config_t& c) { return c.x_dtype == MOE_DTYPE_BF16; }
size_t route_ws(const moe_config_t& c) {
    return route_logits_ws(c) + (route_uses_mfma(c) ? router_mfma_ws_bytes(c) : 0);
}
size_t ffn_ws(const moe_config_t& c) {
    return c.w_dtype == MOE_DTYPE_F32 ? ffn_f32_ws_bytes(c) : ffn_mfma_ws_bytes(c);
}

// The fused call keeps y in its compact form (16-bit codes + block scales) unless the
// configuration asks for float32 or there is no compact form (F32 path).
bool y_compact(const moe_config_t& c) { return c.w_dtype != MOE_DTYPE_F32 && !(c.flags & MOE_FLAG_Y_F32); }

struct LayerWs {  // carve-up of the fused call's workspace
    size_t logits, idx, w, counts, offsets, perm, inv, y, y_scales, sub, total;
};
LayerWs layer_ws(const moe_config_t& c) {
    const size_t P = (size_t)c.T * c.K;
    LayerWs l{};
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o += align_up(bytes ? bytes : 1, 256); return at; };
    l.logits = take((size_t)c.T * c.E * 4);
    l.idx = take(P * 4);
    l.w = take(P * 4);
    l.counts = take((size_t)c.E * 4);
    l.offsets = take((size_t)(c.E + 1) * 4);
    l.perm = take(P * 4);
    l.inv = take(P * 4);
    if (y_compact(c)) {   // a caller that wants to see y passes its own float32 buffer (taps.y_perm)
        l.y = take(P * c.H * 2);
        l.y_scales = take(P * (c.H / Y_BLOCK_COLS));
    } else {
        l.y = take(P * c.H * 4);
        l.y_scales = l.y;
    }
    size_t sub = permute_ws_bytes(c);
    if (ffn_ws(c) > sub) sub = ffn_ws(c);
    if (route_ws(c) > sub) sub = route_ws(c);
    l.sub = take(sub);
    l.total = o;
    return l;
}

}  // namespace

extern "C" {

int32_t moe_abi_version(void) { return MOE_ABI_VERSION; }

const char* moe_status_string(int32_t st) {
    switch (st) {
        case MOE_OK: return "ok";
        case MOE_ERR_NULL_PTR: return "null pointer";
        case MOE_ERR_BAD_SHAPE: return "bad shape";
        case MOE_ERR_BAD_DTYPE: return "bad dtype";
        case MOE_ERR_UNALIGNED: return "unaligned pointer";
        case MOE_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
        case MOE_ERR_UNSUPPORTED: return "unsupported configuration";
        case MOE_ERR_LAUNCH_FAILED: return "kernel launch failed";
        case MOE_ERR_TOO_LARGE: return "problem too large for the entry point's fixed scratch memory";
        default: return "unknown status";
    }
}

int32_t moe_set_profile_events(int32_t kernel, void* start_event, void* stop_event) {
    if (kernel < 0 || kernel >= MOE_KERNEL_COUNT) return MOE_ERR_UNSUPPORTED;
    if ((start_event == nullptr) != (stop_event == nullptr)) return MOE_ERR_NULL_PTR;
    g_profile[kernel].start = static_cast<hipEvent_t>(start_event);
    g_profile[kernel].stop = static_cast<hipEvent_t>(stop_event);
    return MOE_OK;
}

int32_t moe_workspace_bytes(const moe_config_t* cfg, int32_t call, size_t* bytes_out) {
    int32_t st = check_config(cfg);
    if (st != MOE_OK) return st;
    if (!bytes_out) return MOE_ERR_NULL_PTR;
    switch (call) {
        case MOE_CALL_ROUTE: *bytes_out = route_ws(*cfg); break;
        case MOE_CALL_PERMUTE: *bytes_out = permute_ws_bytes(*cfg); break;
        case MOE_CALL_GROUPED_FFN: *bytes_out = ffn_ws(*cfg); break;
        case MOE_CALL_COMBINE: *bytes_out = 0; break;
        case MOE_CALL_PREFILL_LAYER: *bytes_out = layer_ws(*cfg).total; break;
        default: return MOE_ERR_UNSUPPORTED;
    }
    return MOE_OK;
}

int32_t moe_quantize_rows_e4m3(const void* src_bf16, int64_t rows, int32_t cols, uint8_t* q,
                               float* scale, void* stream) {
    if (!src_bf16 || !q || !scale) return MOE_ERR_NULL_PTR;
    if (rows < 0 || rows >= (1ll << 31) || cols < 8 || cols % 8 != 0) return MOE_ERR_BAD_SHAPE;
    if (!aligned(src_bf16, 16) || !aligned(q, 8)) return MOE_ERR_UNALIGNED;
    return launch_quantize_rows(src_bf16, rows, cols, q, scale, static_cast<hipStream_t>(stream));
}

int32_t moe_route(const moe_config_t* cfg, const void* x, const float* w_router, const float* bias,
                  float* logits_out, int32_t* topk_idx, float* topk_w, void* ws, size_t ws_bytes,
                  void* stream) {
    int32_t st = check_config(cfg);
    if (st != MOE_OK) return st;
    const bool empty = cfg->T == 0;   // buffers with a T dimension may be NULL then
    if (!w_router || (!empty && (!x || !topk_idx || !topk_w))) return MOE_ERR_NULL_PTR;
    if (empty) return MOE_OK;
    float* logits = logits_out;
    const bool mfma = route_uses_mfma(*cfg);
    // with at most 128 experts the matrix-core router selects the top K itself and writes the
    // logits only on request
    const bool fused = mfma && router_mfma_fuses_topk(*cfg);
    if (!logits || mfma) {
        if (!ws) return MOE_ERR_NULL_PTR;
        if (!aligned(ws, 256)) return MOE_ERR_UNALIGNED;
        if (ws_bytes < route_ws(*cfg)) return MOE_ERR_WORKSPACE_TOO_SMALL;
        if (!logits && !fused) logits = static_cast<float*>(ws);
    }
    if (mfma && !aligned(x, 16)) return MOE_ERR_UNALIGNED;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (mfma)
        st = launch_router_logits_mfma(*cfg, x, w_router, bias, logits, topk_idx, topk_w,
                                       static_cast<char*>(ws) + route_logits_ws(*cfg), s);
    else
        st = launch_router_logits(*cfg, x, w_router, bias, logits, s);
    if (st != MOE_OK || fused) return st;
    return launch_topk(*cfg, logits, topk_idx, topk_w, s);
}

int32_t moe_permute(const moe_config_t* cfg, const int32_t* topk_idx, const void* x, int32_t* counts,
                    int32_t* offsets, int32_t* perm, int32_t* inv_perm, void* x_perm, void* ws,
                    size_t ws_bytes, void* stream) {
    int32_t st = check_config(cfg);
    if (st != MOE_OK) return st;
    const bool empty = cfg->T == 0;
    if (!counts || !offsets || !ws || (!empty && (!topk_idx || !perm || !inv_perm))) return MOE_ERR_NULL_PTR;
    if (x_perm && !x) return MOE_ERR_NULL_PTR;
    if (!aligned(ws, 256)) return MOE_ERR_UNALIGNED;
    if (ws_bytes < permute_ws_bytes(*cfg)) return MOE_ERR_WORKSPACE_TOO_SMALL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    st = launch_permute(*cfg, topk_idx, counts, offsets, perm, inv_perm, ws, s);
    if (st != MOE_OK) return st;
    if (x_perm) return launch_gather_rows(*cfg, x, perm, x_perm, s);
    return MOE_OK;
}

}  // extern "C"

namespace {
// moe_grouped_ffn, with y either as float32 (y_perm) or in its compact form (y_codes, y_scales).
int32_t grouped_ffn(const moe_config_t* cfg, const void* x, const int32_t* perm,
                    const int32_t* offsets, const void* w_gate, const void* w_up,
                    const void* w_down, const float* s_gate, const float* s_up,
                    const float* s_down, void* act_tap, uint8_t* act_q_tap,
                    float* act_scale_tap, float* y_perm, int16_t* y_codes, uint8_t* y_scales,
                    void* ws, size_t ws_bytes, void* stream) {
    int32_t st = check_config(cfg);
    if (st != MOE_OK) return st;
    const bool empty = cfg->T == 0;
    if (!offsets || !w_gate || !w_up || !w_down || !ws ||
        (!empty && (!x || !perm || (!y_perm && !(y_codes && y_scales)))))
        return MOE_ERR_NULL_PTR;
    if (cfg->w_dtype == MOE_DTYPE_FP8_E4M3 && (!s_gate || !s_up || !s_down)) return MOE_ERR_NULL_PTR;
    if (!aligned(ws, 256)) return MOE_ERR_UNALIGNED;
    if (cfg->w_dtype != MOE_DTYPE_F32 &&
        (!aligned(x, 16) || !aligned(w_gate, 16) || !aligned(w_up, 16) || !aligned(w_down, 16) ||
         !aligned(y_perm, 16) || !aligned(y_codes, 16) || (act_tap && !aligned(act_tap, 16))))
        return MOE_ERR_UNALIGNED;
    if (ws_bytes < ffn_ws(*cfg)) return MOE_ERR_WORKSPACE_TOO_SMALL;
    if (empty) return MOE_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (cfg->w_dtype == MOE_DTYPE_F32)
        return launch_ffn_f32(*cfg, static_cast<const float*>(x), perm, offsets,
                              static_cast<const float*>(w_gate), static_cast<const float*>(w_up),
                              static_cast<const float*>(w_down), static_cast<float*>(act_tap), y_perm,
                              ws, s);
    return launch_ffn_mfma(*cfg, x, perm, offsets, w_gate, w_up, w_down, s_gate, s_up, s_down,
                           act_tap, act_q_tap, act_scale_tap, y_perm, y_codes, y_scales, ws, s);
}
}  // namespace

extern "C" {

int32_t moe_grouped_ffn(const moe_config_t* cfg, const void* x, const int32_t* perm,
                        const int32_t* offsets, const void* w_gate, const void* w_up,
                        const void* w_down, const float* s_gate, const float* s_up,
                        const float* s_down, void* act_tap, uint8_t* act_q_tap,
                        float* act_scale_tap, float* y_perm, void* ws, size_t ws_bytes,
                        void* stream) {
    if (cfg && cfg->T != 0 && !y_perm) return MOE_ERR_NULL_PTR;
    return grouped_ffn(cfg, x, perm, offsets, w_gate, w_up, w_down, s_gate, s_up, s_down, act_tap,
                       act_q_tap, act_scale_tap, y_perm, nullptr, nullptr, ws, ws_bytes, stream);
}

int32_t moe_combine(const moe_config_t* cfg, const float* y_perm, const int32_t* inv_perm,
                    const float* topk_w, void* out, void* stream) {
    int32_t st = check_config(cfg);
    if (st != MOE_OK) return st;
    if (cfg->T == 0) return MOE_OK;
    if (!y_perm || !inv_perm || !topk_w || !out) return MOE_ERR_NULL_PTR;
    return launch_combine(*cfg, y_perm, inv_perm, topk_w, out, static_cast<hipStream_t>(stream));
}

int32_t moe_prefill_layer(const moe_config_t* cfg, const void* x, const float* w_router,
                          const float* bias, const void* w_gate, const void* w_up,
                          const void* w_down, const float* s_gate, const float* s_up,
                          const float* s_down, void* out, const moe_taps_t* taps, void* ws,
                          size_t ws_bytes, void* stream) {
    int32_t st = check_config(cfg);
    if (st != MOE_OK) return st;
    const bool empty = cfg->T == 0;
    if (!w_router || !w_gate || !w_up || !w_down || !ws || (!empty && (!x || !out))) return MOE_ERR_NULL_PTR;
    if (cfg->w_dtype == MOE_DTYPE_FP8_E4M3 && (!s_gate || !s_up || !s_down)) return MOE_ERR_NULL_PTR;
    if (!aligned(ws, 256)) return MOE_ERR_UNALIGNED;
    const LayerWs l = layer_ws(*cfg);
    if (ws_bytes < l.total) return MOE_ERR_WORKSPACE_TOO_SMALL;
    char* w8 = static_cast<char*>(ws);
    moe_taps_t t{};
    if (taps) t = *taps;
    // the logits are materialised only for a caller that asks for them, or when the selection is a kernel of its own
    float* logits = t.logits ? t.logits
                             : ((route_uses_mfma(*cfg) && router_mfma_fuses_topk(*cfg)) ? nullptr
                                                                                       : reinterpret_cast<float*>(w8 + l.logits));
    int32_t* idx = t.topk_idx ? t.topk_idx : reinterpret_cast<int32_t*>(w8 + l.idx);
    float* tw = t.topk_w ? t.topk_w : reinterpret_cast<float*>(w8 + l.w);
    int32_t* counts = t.counts ? t.counts : reinterpret_cast<int32_t*>(w8 + l.counts);
    int32_t* offsets = t.offsets ? t.offsets : reinterpret_cast<int32_t*>(w8 + l.offsets);
    int32_t* perm = t.perm ? t.perm : reinterpret_cast<int32_t*>(w8 + l.perm);
    int32_t* inv = t.inv_perm ? t.inv_perm : reinterpret_cast<int32_t*>(w8 + l.inv);
    const bool compact = y_compact(*cfg) && !t.y_perm;
    float* y = t.y_perm ? t.y_perm : reinterpret_cast<float*>(w8 + l.y);
    int16_t* y_codes = compact ? reinterpret_cast<int16_t*>(w8 + l.y) : nullptr;
    uint8_t* y_scales = compact ? reinterpret_cast<uint8_t*>(w8 + l.y_scales) : nullptr;
    void* sub = w8 + l.sub;
    const size_t sub_bytes = l.total - l.sub;

    st = moe_route(cfg, x, w_router, bias, logits, idx, tw, sub, sub_bytes, stream);
    if (st != MOE_OK) return st;
    st = moe_permute(cfg, idx, nullptr, counts, offsets, perm, inv, nullptr, sub, sub_bytes, stream);
    if (st != MOE_OK) return st;
    st = grouped_ffn(cfg, x, perm, offsets, w_gate, w_up, w_down, s_gate, s_up, s_down, t.act, t.act_q,
                     t.act_scale, compact ? nullptr : y, y_codes, y_scales, sub, sub_bytes, stream);
    if (st != MOE_OK) return st;
    if (compact) {
        if (empty) return MOE_OK;
        return launch_combine_block16(*cfg, y_codes, y_scales, inv, tw, out, static_cast<hipStream_t>(stream));
    }
    return moe_combine(cfg, y, inv, tw, out, stream);
}

}  // extern "C"
