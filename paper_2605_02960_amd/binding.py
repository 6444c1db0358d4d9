"""ctypes binding of libmoeprefill.so.  Argument marshalling only: every tensor is a torch
tensor on the GPU (torch is used for device memory and streams), every step of the block
runs inside the library's HIP kernels."""
import ctypes
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# MOE_PREFILL_LIB: another build of the same library to load instead (A/B timing of kernel variants)
_LIB_PATH = os.environ.get("MOE_PREFILL_LIB") or os.path.join(_HERE, "libmoeprefill.so")
_lib = None

DTYPE_F32, DTYPE_BF16, DTYPE_FP8_E4M3 = 0, 1, 2
FLAG_Y_F32 = 1
CALL_ROUTE, CALL_PERMUTE, CALL_GROUPED_FFN, CALL_COMBINE, CALL_PREFILL_LAYER = range(5)

KERNEL_ROUTER_GEMM, KERNEL_TOPK, KERNEL_PERMUTE, KERNEL_GATE_UP, KERNEL_DOWN, KERNEL_COMBINE = range(6)
KERNEL_NAMES = ("router_gemm", "topk", "permute", "gate_up", "down", "combine")

EXPORTED_SYMBOLS = (
    "moe_layer_weight_bytes", "moe_prefill_layers_streamed", "moe_layer_flops_per_token",
    "moe_saturation_threshold_flops", "moe_calibrated_threshold_flops", "moe_resolve_threshold",
    "moe_abi_version", "moe_status_string", "moe_init_device", "moe_set_profile_events", "moe_workspace_bytes", "moe_quantize_rows_e4m3",
    "moe_route", "moe_permute", "moe_permute_noalloc", "moe_grouped_ffn", "moe_combine", "moe_prefill_layer",
    "moe_sched_create", "moe_sched_destroy", "moe_sched_hash_blocks", "moe_sched_round",
    "moe_sched_blocks_stored", "moe_sched_blocks_evicted", "moe_sched_table_size",
    "moe_sched_tokens_executed",
)


class MoEError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: {moe_status_string(status)} ({status})")


class MoEConfig(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("T", "H", "E", "K", "I", "x_dtype", "w_dtype", "out_dtype", "flags")]


class MoEStreamLayer(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in
                ("w_gate", "w_up", "w_down", "s_gate", "s_up", "s_down", "w_router", "bias", "out")]


class MoECostModel(ctypes.Structure):
    _fields_ = [("f_tok", ctypes.c_double), ("f_attn", ctypes.c_double)]


class MoETaps(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in
                ("logits", "topk_idx", "topk_w", "counts", "offsets", "perm", "inv_perm", "act",
                 "act_q", "act_scale", "y_perm")]


def lib_path():
    return _LIB_PATH


def lib():
    """The loaded library; raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(f"{_LIB_PATH} is missing: build it with "
                               "`python -m paper_2605_02960_amd.build` (hipcc, gfx950)")
        L = ctypes.CDLL(_LIB_PATH)
        vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
        cfgp = ctypes.POINTER(MoEConfig)
        L.moe_abi_version.restype = i32
        L.moe_abi_version.argtypes = []
        L.moe_status_string.restype = ctypes.c_char_p
        L.moe_status_string.argtypes = [i32]
        L.moe_init_device.restype = i32
        L.moe_init_device.argtypes = []
        L.moe_set_profile_events.restype = i32
        L.moe_set_profile_events.argtypes = [i32, vp, vp]
        L.moe_workspace_bytes.restype = i32
        L.moe_workspace_bytes.argtypes = [cfgp, i32, ctypes.POINTER(sz)]
        L.moe_quantize_rows_e4m3.restype = i32
        L.moe_quantize_rows_e4m3.argtypes = [vp, i64, i32, vp, vp, vp]
        L.moe_route.restype = i32
        L.moe_route.argtypes = [cfgp] + [vp] * 7 + [sz, vp]
        L.moe_permute.restype = i32
        L.moe_permute.argtypes = [cfgp] + [vp] * 8 + [sz, vp]
        L.moe_permute_noalloc.restype = i32
        L.moe_permute_noalloc.argtypes = [cfgp] + [vp] * 8
        L.moe_grouped_ffn.restype = i32
        L.moe_grouped_ffn.argtypes = [cfgp] + [vp] * 14 + [sz, vp]
        L.moe_combine.restype = i32
        L.moe_combine.argtypes = [cfgp] + [vp] * 5
        L.moe_prefill_layer.restype = i32
        L.moe_prefill_layer.argtypes = [cfgp] + [vp] * 10 + [ctypes.POINTER(MoETaps), vp, sz, vp]
        L.moe_layer_weight_bytes.restype = i32
        L.moe_layer_weight_bytes.argtypes = [cfgp, ctypes.POINTER(sz)]
        L.moe_prefill_layers_streamed.restype = i32
        L.moe_prefill_layers_streamed.argtypes = [cfgp, i32, ctypes.POINTER(MoEStreamLayer), vp,
                                                  ctypes.POINTER(vp), i32, i32, ctypes.POINTER(vp),
                                                  ctypes.POINTER(vp), vp, sz, vp, vp]
        f64 = ctypes.c_double
        L.moe_layer_flops_per_token.restype = f64
        L.moe_layer_flops_per_token.argtypes = [cfgp]
        L.moe_saturation_threshold_flops.restype = f64
        L.moe_saturation_threshold_flops.argtypes = [f64, f64, f64]
        L.moe_calibrated_threshold_flops.restype = f64
        L.moe_calibrated_threshold_flops.argtypes = [f64, f64, f64, f64]
        L.moe_resolve_threshold.restype = i32
        L.moe_resolve_threshold.argtypes = [f64] * 6 + [ctypes.POINTER(f64), ctypes.POINTER(i32)]
        L.moe_sched_create.restype = i32
        L.moe_sched_create.argtypes = [i32, i32, ctypes.POINTER(vp)]
        L.moe_sched_destroy.restype = None
        L.moe_sched_destroy.argtypes = [vp]
        L.moe_sched_hash_blocks.restype = i32
        L.moe_sched_hash_blocks.argtypes = [vp, i64, i32, vp]
        L.moe_sched_round.restype = i32
        L.moe_sched_round.argtypes = [vp, ctypes.POINTER(MoECostModel), f64, i64] + [vp] * 8 + [ctypes.POINTER(i64)]
        L.moe_sched_blocks_stored.restype = i32
        L.moe_sched_blocks_stored.argtypes = [vp, i32, vp, i64]
        L.moe_sched_blocks_evicted.restype = i32
        L.moe_sched_blocks_evicted.argtypes = [vp, i32, vp, i64]
        L.moe_sched_tokens_executed.restype = i32
        L.moe_sched_tokens_executed.argtypes = [vp, vp, i32, i64, f64]
        L.moe_sched_table_size.restype = i32
        L.moe_sched_table_size.argtypes = [vp, i32, ctypes.POINTER(i64), ctypes.POINTER(i64)]
        _lib = L
    return _lib


class HipEvents:
    """Raw hipEvent_t handles through the HIP runtime that torch has loaded (plumbing for the
    calls that take events: timing brackets and the streaming ring)."""

    def __init__(self):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]

    def create(self):
        e = ctypes.c_void_p()
        if self.hip.hipEventCreate(ctypes.byref(e)) != 0:
            raise RuntimeError("hipEventCreate failed")
        return e.value

    def elapsed_ms(self, a, b):
        if self.hip.hipEventSynchronize(b) != 0:
            raise RuntimeError("hipEventSynchronize failed")
        ms = ctypes.c_float()
        if self.hip.hipEventElapsedTime(ctypes.byref(ms), a, b) != 0:
            raise RuntimeError("hipEventElapsedTime failed")
        return ms.value

    def destroy(self, e):
        self.hip.hipEventDestroy(e)


# ------------------------------------------------------------------ helpers
def _p(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _check(st, where):
    if st != 0:
        raise MoEError(st, where)


def _ws(cfg, call, device):
    n = moe_workspace_bytes(cfg, call)
    return torch.empty(max(n, 256), dtype=torch.uint8, device=device), n


_TORCH_OF = {DTYPE_F32: torch.float32, DTYPE_BF16: torch.bfloat16}


def make_config(T, H, E, K, I, x_dtype, w_dtype, out_dtype=DTYPE_F32, flags=0):
    return MoEConfig(T, H, E, K, I, x_dtype, w_dtype, out_dtype, flags)


# ------------------------------------------------------------------ entry points
def moe_abi_version():
    return lib().moe_abi_version()


def moe_status_string(status):
    return lib().moe_status_string(status).decode()


def moe_init_device():
    """One-time set-up of the current device (what the first compute call would otherwise do)."""
    _check(lib().moe_init_device(), "moe_init_device")


def moe_set_profile_events(kernel, start_event, stop_event):
    """start_event / stop_event: raw hipEvent_t handles (int) or None to clear."""
    _check(lib().moe_set_profile_events(kernel, ctypes.c_void_p(start_event) if start_event else None,
                                        ctypes.c_void_p(stop_event) if stop_event else None),
           "moe_set_profile_events")


def moe_workspace_bytes(cfg, call):
    n = ctypes.c_size_t(0)
    _check(lib().moe_workspace_bytes(ctypes.byref(cfg), call, ctypes.byref(n)), "moe_workspace_bytes")
    return n.value


def moe_quantize_rows_e4m3(src_bf16, stream=None):
    """src [rows, cols] bf16 -> (codes uint8 [rows, cols], scale float32 [rows])."""
    rows, cols = src_bf16.shape
    q = torch.empty((rows, cols), dtype=torch.uint8, device=src_bf16.device)
    s = torch.empty((rows,), dtype=torch.float32, device=src_bf16.device)
    _check(lib().moe_quantize_rows_e4m3(_p(src_bf16), rows, cols, _p(q), _p(s), _stream(stream)),
           "moe_quantize_rows_e4m3")
    return q, s


def moe_route(cfg, x, w_router, bias=None, want_logits=True, stream=None):
    dev = x.device
    idx = torch.empty((cfg.T, cfg.K), dtype=torch.int32, device=dev)
    w = torch.empty((cfg.T, cfg.K), dtype=torch.float32, device=dev)
    logits = torch.empty((cfg.T, cfg.E), dtype=torch.float32, device=dev) if want_logits else None
    ws, n = _ws(cfg, CALL_ROUTE, dev)
    _check(lib().moe_route(ctypes.byref(cfg), _p(x), _p(w_router), _p(bias), _p(logits), _p(idx), _p(w),
                           _p(ws), n, _stream(stream)), "moe_route")
    return idx, w, logits


def moe_permute(cfg, topk_idx, x=None, want_x_perm=False, stream=None):
    dev = topk_idx.device
    P = cfg.T * cfg.K
    counts = torch.empty((cfg.E,), dtype=torch.int32, device=dev)
    offsets = torch.empty((cfg.E + 1,), dtype=torch.int32, device=dev)
    perm = torch.empty((P,), dtype=torch.int32, device=dev)
    inv = torch.empty((P,), dtype=torch.int32, device=dev)
    xp = torch.empty((P, cfg.H), dtype=x.dtype, device=dev) if want_x_perm else None
    ws, n = _ws(cfg, CALL_PERMUTE, dev)
    _check(lib().moe_permute(ctypes.byref(cfg), _p(topk_idx), _p(x), _p(counts), _p(offsets), _p(perm),
                             _p(inv), _p(xp), _p(ws), n, _stream(stream)), "moe_permute")
    return counts, offsets, perm, inv, xp


def moe_permute_noalloc(cfg, topk_idx, out, stream=None):
    """The allocation-free variant of moe_permute: `out` = (counts, offsets, perm, inv_perm), tensors
    the caller has allocated beforehand; nothing is allocated here or in the library."""
    counts, offsets, perm, inv = out
    _check(lib().moe_permute_noalloc(ctypes.byref(cfg), _p(topk_idx), None, _p(counts), _p(offsets), _p(perm),
                                     _p(inv), None, _stream(stream)), "moe_permute_noalloc")
    return out


def moe_grouped_ffn(cfg, x, perm, offsets, w_gate, w_up, w_down, s_gate=None, s_up=None, s_down=None,
                    want_act=False, y_perm=None, ws=None, stream=None):
    dev = x.device
    P = cfg.T * cfg.K
    fp8 = cfg.w_dtype == DTYPE_FP8_E4M3
    act = act_q = act_s = None
    if want_act:
        act = torch.empty((P, cfg.I), dtype=torch.float32 if cfg.w_dtype == DTYPE_F32 else torch.bfloat16,
                          device=dev)
        if fp8:
            act_q = torch.empty((P, cfg.I), dtype=torch.uint8, device=dev)
            act_s = torch.empty((P,), dtype=torch.float32, device=dev)
    if y_perm is None:
        y_perm = torch.empty((P, cfg.H), dtype=torch.float32, device=dev)
    if ws is None:
        ws, n = _ws(cfg, CALL_GROUPED_FFN, dev)
    else:
        n = ws.numel()
    _check(lib().moe_grouped_ffn(ctypes.byref(cfg), _p(x), _p(perm), _p(offsets), _p(w_gate), _p(w_up),
                                 _p(w_down), _p(s_gate), _p(s_up), _p(s_down), _p(act), _p(act_q),
                                 _p(act_s), _p(y_perm), _p(ws), n, _stream(stream)), "moe_grouped_ffn")
    return y_perm, act, act_q, act_s


def moe_combine(cfg, y_perm, inv_perm, topk_w, out=None, stream=None):
    if out is None:
        out = torch.empty((cfg.T, cfg.H), dtype=_TORCH_OF[cfg.out_dtype], device=y_perm.device)
    _check(lib().moe_combine(ctypes.byref(cfg), _p(y_perm), _p(inv_perm), _p(topk_w), _p(out),
                             _stream(stream)), "moe_combine")
    return out


def moe_layer_weight_bytes(cfg):
    n = ctypes.c_size_t(0)
    _check(lib().moe_layer_weight_bytes(ctypes.byref(cfg), ctypes.byref(n)), "moe_layer_weight_bytes")
    return n.value


def moe_layer_flops_per_token(cfg):
    return lib().moe_layer_flops_per_token(ctypes.byref(cfg))


def moe_saturation_threshold_flops(t_ep_seconds, f_gpu_flops, gamma=1.2):
    return lib().moe_saturation_threshold_flops(t_ep_seconds, f_gpu_flops, gamma)


def moe_calibrated_threshold_flops(t_c, t_e, c_dummy_flops, gamma=1.2):
    return lib().moe_calibrated_threshold_flops(t_c, t_e, c_dummy_flops, gamma)


def moe_resolve_threshold(pinned, t_c, t_e, f_tok, n_ref, gamma=1.2):
    """(threshold, unit) with unit 0 = FLOPs, 1 = tokens (App. B.4, delivery and fallback)."""
    t, u = ctypes.c_double(0.0), ctypes.c_int32(0)
    _check(lib().moe_resolve_threshold(float(pinned), float(t_c), float(t_e), float(f_tok), float(n_ref), float(gamma),
                                       ctypes.byref(t), ctypes.byref(u)), "moe_resolve_threshold")
    return t.value, u.value


def moe_prefill_layers_streamed(cfg, layers, x, slots, n_resident=0, ws=None, compute_stream=None,
                                copy_stream=None, events=None, time_layers=False):
    """layers: list of dicts; w_gate/w_up/w_down (and s_* for fp8) are PINNED HOST tensors, w_router /
    bias / out device tensors.  slots: device uint8 tensors of moe_layer_weight_bytes(cfg).
    Returns the list of (entry, exit) event handles per layer when time_layers, else None."""
    dev = x.device
    n = len(layers)
    arr = (MoEStreamLayer * max(n, 1))()
    for i, l in enumerate(layers):
        for name in ("w_gate", "w_up", "w_down", "s_gate", "s_up", "s_down", "w_router", "bias", "out"):
            ten = l.get(name)
            setattr(arr[i], name, None if ten is None else ten.data_ptr())
    events = events or HipEvents()
    vp = ctypes.c_void_p
    slot_ptrs = (vp * len(slots))(*[s.data_ptr() for s in slots])
    slot_ev = (vp * (2 * len(slots)))(*[events.create() for _ in range(2 * len(slots))])
    layer_ev = None
    pairs = None
    if time_layers:
        handles = [events.create() for _ in range(2 * n)]
        layer_ev = (vp * (2 * n))(*handles)
        pairs = [(handles[2 * i], handles[2 * i + 1]) for i in range(n)]
    if ws is None:
        ws, nb = _ws(cfg, CALL_PREFILL_LAYER, dev)
    else:
        nb = ws.numel()
    cs = torch.cuda.current_stream() if compute_stream is None else compute_stream
    ps = torch.cuda.Stream() if copy_stream is None else copy_stream
    _check(lib().moe_prefill_layers_streamed(ctypes.byref(cfg), n, arr, _p(x), slot_ptrs, len(slots), n_resident,
                                             slot_ev, layer_ev, _p(ws), nb, ctypes.c_void_p(cs.cuda_stream),
                                             ctypes.c_void_p(ps.cuda_stream)), "moe_prefill_layers_streamed")
    return pairs


def moe_prefill_layer(cfg, x, w_router, bias, w_gate, w_up, w_down, s_gate=None, s_up=None, s_down=None,
                      out=None, taps=None, ws=None, stream=None):
    """taps: None, or a dict name -> preallocated tensor for any of the MoETaps members."""
    dev = x.device
    if out is None:
        out = torch.empty((cfg.T, cfg.H), dtype=_TORCH_OF[cfg.out_dtype], device=dev)
    if ws is None:
        ws, n = _ws(cfg, CALL_PREFILL_LAYER, dev)
    else:
        n = ws.numel()
    tp = None
    if taps:
        t = MoETaps()
        for name, ten in taps.items():
            setattr(t, name, ten.data_ptr())
        tp = ctypes.byref(t)
    _check(lib().moe_prefill_layer(ctypes.byref(cfg), _p(x), _p(w_router), _p(bias), _p(w_gate), _p(w_up),
                                   _p(w_down), _p(s_gate), _p(s_up), _p(s_down), _p(out), tp, _p(ws), n,
                                   _stream(stream)), "moe_prefill_layer")
    return out


# ------------------------------------------------------------------ scheduling round (host only; numpy arrays)
def _np(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a, ctypes.c_void_p(a.ctypes.data if a.size else None)


def moe_sched_create(n_workers, block_tokens):
    h = ctypes.c_void_p()
    _check(lib().moe_sched_create(n_workers, block_tokens, ctypes.byref(h)), "moe_sched_create")
    return h


def moe_sched_destroy(handle):
    lib().moe_sched_destroy(handle)


def moe_sched_hash_blocks(tokens, block_tokens):
    tokens, tp = _np(tokens, np.int32)
    out = np.empty(max(tokens.size // block_tokens, 0), dtype=np.uint64)
    _check(lib().moe_sched_hash_blocks(tp, tokens.size, block_tokens,
                                       ctypes.c_void_p(out.ctypes.data if out.size else None)), "moe_sched_hash_blocks")
    return out


def moe_sched_round(handle, f_tok, f_attn, threshold, block_hashes, hash_offsets, prefix_tokens, suffix_tokens, loads):
    """loads (float64 [n_workers]) is updated in place.  Returns (assigned, matched_tokens, delta, n_assigned)."""
    hashes, hp = _np(block_hashes, np.uint64)
    offs, op = _np(hash_offsets, np.int64)
    P, pp = _np(prefix_tokens, np.int64)
    S, sp = _np(suffix_tokens, np.int64)
    if not (isinstance(loads, np.ndarray) and loads.dtype == np.float64 and loads.flags.c_contiguous):
        raise TypeError("loads must be a contiguous float64 numpy array (it is updated in place)")
    n = P.size
    assigned = np.empty(n, dtype=np.int32)
    matched = np.empty(n, dtype=np.int64)
    delta = np.empty(n, dtype=np.float64)
    done = ctypes.c_int64(0)
    cost = MoECostModel(float(f_tok), float(f_attn))
    _check(lib().moe_sched_round(handle, ctypes.byref(cost), float(threshold), n, hp, op, pp, sp,
                                 ctypes.c_void_p(loads.ctypes.data), ctypes.c_void_p(assigned.ctypes.data if n else None),
                                 ctypes.c_void_p(matched.ctypes.data if n else None),
                                 ctypes.c_void_p(delta.ctypes.data if n else None), ctypes.byref(done)), "moe_sched_round")
    return assigned, matched, delta, done.value


def moe_sched_blocks_stored(handle, worker, hashes):
    h, hp = _np(hashes, np.uint64)
    _check(lib().moe_sched_blocks_stored(handle, worker, hp, h.size), "moe_sched_blocks_stored")


def moe_sched_blocks_evicted(handle, worker, hashes):
    h, hp = _np(hashes, np.uint64)
    _check(lib().moe_sched_blocks_evicted(handle, worker, hp, h.size), "moe_sched_blocks_evicted")


def moe_sched_tokens_executed(handle, loads, worker, tokens, f_tok):
    """loads (float64 numpy array) is updated in place."""
    if not (isinstance(loads, np.ndarray) and loads.dtype == np.float64 and loads.flags.c_contiguous):
        raise TypeError("loads must be a contiguous float64 numpy array (it is updated in place)")
    _check(lib().moe_sched_tokens_executed(handle, ctypes.c_void_p(loads.ctypes.data), worker, tokens, float(f_tok)),
           "moe_sched_tokens_executed")


def moe_sched_table_size(handle, worker):
    c, p = ctypes.c_int64(0), ctypes.c_int64(0)
    _check(lib().moe_sched_table_size(handle, worker, ctypes.byref(c), ctypes.byref(p)), "moe_sched_table_size")
    return c.value, p.value
