// One-GPU weight streaming of the expert weights (the single-GPU host-to-device mode of the paper's
// weight streaming engine, App. B.1, and the offloading pipeline of Sec. 6.3): the expert weights
// of all layers live in pinned host memory, the GPU holds a small ring of layer slots, a copy
// stream prefetches the layers ahead while the compute stream runs moe_prefill_layer on the
// current one, and the two meet in a single event wait at each layer's entry.  Also the
// saturation threshold that decides when the transfer is hidden (Eq. 1) and its calibration from
// per-layer timings (App. B.4, Eq. 3).
#include "common.h"

using namespace moe;

namespace {

struct SlotLayout {
    size_t wg, wu, wd, sg, su, sd, total;
    size_t w_bytes, sgu_bytes, sd_bytes;
};

SlotLayout slot_layout(const moe_config_t& c) {
    const size_t esz = c.w_dtype == MOE_DTYPE_FP8_E4M3 ? 1 : (c.w_dtype == MOE_DTYPE_BF16 ? 2 : 4);
    SlotLayout l{};
    l.w_bytes = (size_t)c.E * c.I * c.H * esz;
    const bool fp8 = c.w_dtype == MOE_DTYPE_FP8_E4M3;
    l.sgu_bytes = fp8 ? (size_t)c.E * c.I * 4 : 0;
    l.sd_bytes = fp8 ? (size_t)c.E * c.H * 4 : 0;
    size_t o = 0;
    auto take = [&](size_t b) { size_t at = o; o += align_up(b, 256); return at; };
    l.wg = take(l.w_bytes);
    l.wu = take(l.w_bytes);
    l.wd = take(l.w_bytes);
    l.sg = take(l.sgu_bytes);
    l.su = take(l.sgu_bytes);
    l.sd = take(l.sd_bytes);
    l.total = o;
    return l;
}

int32_t enqueue_layer_copy(const SlotLayout& l, const moe_stream_layer_t& layer, char* slot,
                           hipStream_t copy) {
    auto cp = [&](size_t off, const void* src, size_t bytes) {
        if (bytes == 0) return true;
        return hipMemcpyAsync(slot + off, src, bytes, hipMemcpyHostToDevice, copy) == hipSuccess;
    };
    if (!cp(l.wg, layer.w_gate, l.w_bytes) || !cp(l.wu, layer.w_up, l.w_bytes) ||
        !cp(l.wd, layer.w_down, l.w_bytes) || !cp(l.sg, layer.s_gate, l.sgu_bytes) ||
        !cp(l.su, layer.s_up, l.sgu_bytes) || !cp(l.sd, layer.s_down, l.sd_bytes))
        return MOE_ERR_LAUNCH_FAILED;
    return MOE_OK;
}

}  // namespace

extern "C" {

int32_t moe_layer_weight_bytes(const moe_config_t* cfg, size_t* bytes_out) {
    size_t dummy = 0;
    int32_t st = moe_workspace_bytes(cfg, MOE_CALL_COMBINE, &dummy);   // validates cfg
    if (st != MOE_OK) return st;
    if (!bytes_out) return MOE_ERR_NULL_PTR;
    *bytes_out = slot_layout(*cfg).total;
    return MOE_OK;
}

int32_t moe_prefill_layers_streamed(const moe_config_t* cfg, int32_t n_layers,
                                    const moe_stream_layer_t* layers, const void* x,
                                    void* const* slots, int32_t n_slots, int32_t n_resident,
                                    void* const* slot_events, void* const* layer_events, void* ws,
                                    size_t ws_bytes, void* compute_stream, void* copy_stream) {
    size_t need = 0;
    int32_t st = moe_workspace_bytes(cfg, MOE_CALL_PREFILL_LAYER, &need);
    if (st != MOE_OK) return st;
    if (!layers || !slots || !slot_events || !ws) return MOE_ERR_NULL_PTR;
    if (n_layers < 0 || n_slots < 1 || n_resident < 0 || n_resident > n_slots || n_resident > n_layers)
        return MOE_ERR_BAD_SHAPE;
    if (ws_bytes < need) return MOE_ERR_WORKSPACE_TOO_SMALL;
    if (compute_stream == copy_stream) return MOE_ERR_UNSUPPORTED;   // the two must be able to overlap
    const bool fp8 = cfg->w_dtype == MOE_DTYPE_FP8_E4M3;
    for (int i = 0; i < n_layers; ++i) {
        const moe_stream_layer_t& L = layers[i];
        if (!L.w_gate || !L.w_up || !L.w_down || !L.w_router || (cfg->T > 0 && !L.out)) return MOE_ERR_NULL_PTR;
        if (fp8 && (!L.s_gate || !L.s_up || !L.s_down)) return MOE_ERR_NULL_PTR;
    }
    for (int s = 0; s < n_slots; ++s)
        if (!slots[s] || !slot_events[2 * s] || !slot_events[2 * s + 1]) return MOE_ERR_NULL_PTR;
    for (int s = 0; s < n_slots; ++s)
        if (reinterpret_cast<uintptr_t>(slots[s]) % 256 != 0) return MOE_ERR_UNALIGNED;

    const SlotLayout l = slot_layout(*cfg);
    hipStream_t cs = static_cast<hipStream_t>(compute_stream);
    hipStream_t ps = static_cast<hipStream_t>(copy_stream);
    auto copied = [&](int s) { return static_cast<hipEvent_t>(slot_events[2 * s]); };
    auto freed = [&](int s) { return static_cast<hipEvent_t>(slot_events[2 * s + 1]); };

    // prime the ring: layers that are not resident yet, as far as there are slots
    for (int i = n_resident; i < n_layers && i < n_slots; ++i) {
        st = enqueue_layer_copy(l, layers[i], static_cast<char*>(slots[i]), ps);
        if (st != MOE_OK) return st;
        if (hipEventRecord(copied(i), ps) != hipSuccess) return MOE_ERR_LAUNCH_FAILED;
    }
    for (int i = 0; i < n_layers; ++i) {
        const int s = i % n_slots;
        char* slot = static_cast<char*>(slots[s]);
        if (layer_events && layer_events[2 * i] &&
            hipEventRecord(static_cast<hipEvent_t>(layer_events[2 * i]), cs) != hipSuccess)
            return MOE_ERR_LAUNCH_FAILED;
        // the single wait at the layer's entry: its weights have landed
        if (i >= n_resident && hipStreamWaitEvent(cs, copied(s), 0) != hipSuccess) return MOE_ERR_LAUNCH_FAILED;
        const moe_stream_layer_t& L = layers[i];
        st = moe_prefill_layer(cfg, x, L.w_router, L.bias, slot + l.wg, slot + l.wu, slot + l.wd,
                               fp8 ? reinterpret_cast<const float*>(slot + l.sg) : nullptr,
                               fp8 ? reinterpret_cast<const float*>(slot + l.su) : nullptr,
                               fp8 ? reinterpret_cast<const float*>(slot + l.sd) : nullptr, L.out, nullptr, ws,
                               ws_bytes, compute_stream);
        if (st != MOE_OK) return st;
        if (layer_events && layer_events[2 * i + 1] &&
            hipEventRecord(static_cast<hipEvent_t>(layer_events[2 * i + 1]), cs) != hipSuccess)
            return MOE_ERR_LAUNCH_FAILED;
        // the slot is free once this layer is done: start the transfer of the layer that reuses it
        const int next = i + n_slots;
        if (next < n_layers) {
            if (hipEventRecord(freed(s), cs) != hipSuccess || hipStreamWaitEvent(ps, freed(s), 0) != hipSuccess)
                return MOE_ERR_LAUNCH_FAILED;
            st = enqueue_layer_copy(l, layers[next], slot, ps);
            if (st != MOE_OK) return st;
            if (hipEventRecord(copied(s), ps) != hipSuccess) return MOE_ERR_LAUNCH_FAILED;
        }
    }
    return MOE_OK;
}

double moe_layer_flops_per_token(const moe_config_t* cfg) {
    if (!cfg) return 0.0;
    return (double)cfg->K * 6.0 * cfg->H * cfg->I + 2.0 * (double)cfg->H * cfg->E;
}

double moe_saturation_threshold_flops(double t_ep_seconds, double f_gpu_flops, double gamma) {
    return t_ep_seconds * f_gpu_flops * gamma;
}

double moe_calibrated_threshold_flops(double t_c, double t_e, double c_dummy_flops, double gamma) {
    if (!(t_c > 0.0)) return gamma * c_dummy_flops;              // no calibration: the fallback
    const double ratio = t_e > t_c ? t_e / t_c : 1.0;            // transfers hidden: collapses to gamma * C_dummy
    return gamma * ratio * c_dummy_flops;
}

int32_t moe_resolve_threshold(double pinned, double t_c, double t_e, double f_tok, double n_ref,
                              double gamma, double* threshold_out, int32_t* unit_out) {
    if (!threshold_out || !unit_out) return MOE_ERR_NULL_PTR;
    if (!(gamma > 0.0) || !(n_ref >= 0.0)) return MOE_ERR_BAD_SHAPE;
    const bool have_f_tok = f_tok > 0.0;                  // false also for NaN
    *unit_out = have_f_tok ? MOE_UNIT_FLOPS : MOE_UNIT_TOKENS;
    if (pinned > 0.0) {                                   // the operator's value wins over any calibration
        *threshold_out = pinned;
        return MOE_OK;
    }
    // token-unit accounting is the same arithmetic with one unit of work per token
    const double c_dummy = (have_f_tok ? f_tok : 1.0) * n_ref;
    *threshold_out = moe_calibrated_threshold_flops(t_c, t_e, c_dummy, gamma);
    return MOE_OK;
}

}  // extern "C"
