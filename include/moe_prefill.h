/* moe_prefill.h -- C ABI of the MI355X (gfx950) MoE prefill block.
 *
 * The block is the per-layer Mixture-of-Experts computation that one GPU runs
 * locally when the whole expert set of the current layer is resident on it, as in
 * the paper's asynchronous expert-parallel backend (Sec. 6.2: every GPU evaluates
 * the current MoE layer entirely on-device; Sec. 1: dispatch becomes a local
 * operation).  Sec. 2.3 defines the computation: E experts, each a two-layer MLP;
 * a router sends each token to its top-k experts and their outputs are summed.
 * The token permutation/alignment steps that Sec. 4.3 counts among the small
 * kernels on every layer's critical path are moe_permute here.
 *
 * Conventions (all entry points)
 *   - Every data pointer is DEVICE memory owned by the caller, on the device that
 *     is current when the call is made.  The library allocates nothing, frees
 *     nothing and keeps no pointer after the call's kernels have run.  Scratch
 *     space comes in through (ws, ws_bytes); its minimum size is
 *     moe_workspace_bytes(cfg, call).  ws must be 256-byte aligned.
 *   - Host-side state: per device, the compute-unit count and a one-time kernel
 *     attribute set-up, made under a mutex by the first call on that device (calls
 *     from several host threads are safe); that first call queries the device and
 *     must not fall inside a stream capture: call moe_init_device() once per device
 *     beforehand if it would.  The event pairs of moe_set_profile_events are
 *     process-global and not thread-safe.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Calls
 *     only enqueue work: no host synchronisation and no device-to-host copy.
 *   - Tensors are dense row-major; "[A,B]" lists dimensions slowest first.
 *   - Return value: MOE_OK (0) or a negative moe_status.  Argument errors are
 *     found on the host before anything is enqueued and leave outputs untouched.
 *     MOE_ERR_LAUNCH_FAILED is read from hipGetLastError after each launch, so it
 *     also reports (and clears) an error that an earlier HIP call of the calling
 *     thread left pending.
 *   - Routed rows: P = T*K.  A routed row has a flat id f = t*K + j (token t,
 *     slot j) and a sorted position p in [0,P): rows are sorted by expert id,
 *     and by ascending flat id inside one expert's group.
 *   - NaN/Inf inputs are not supported (results undefined, no fault).
 *   - T = 0 is a valid call: buffers that have a T (or P) dimension may then be NULL; counts
 *     and offsets are still written (all zero).
 */
#ifndef MOE_PREFILL_H
#define MOE_PREFILL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MOE_ABI_VERSION 1

typedef enum moe_status {
    MOE_OK = 0,
    MOE_ERR_NULL_PTR = -1,
    MOE_ERR_BAD_SHAPE = -2,
    MOE_ERR_BAD_DTYPE = -3,
    MOE_ERR_UNALIGNED = -4,
    MOE_ERR_WORKSPACE_TOO_SMALL = -5,
    MOE_ERR_UNSUPPORTED = -6,
    MOE_ERR_LAUNCH_FAILED = -7,
    MOE_ERR_TOO_LARGE = -8 /* the problem needs more than an entry point's fixed scratch memory */
} moe_status;

typedef enum moe_dtype {
    MOE_DTYPE_F32 = 0,
    MOE_DTYPE_BF16 = 1,
    MOE_DTYPE_FP8_E4M3 = 2 /* OCP e4m3 (finite max 448, no infinities) */
} moe_dtype;

enum { /* moe_config.flags */
    MOE_FLAG_NONE = 0,
    /* BF16 / FP8 paths: hand the float32 accumulators of the down projection to the combine as
     * they are.  Without it every 16 adjacent columns of a y row share one power-of-two scale and
     * are rounded to 16-bit codes: with amax the block's largest magnitude, k = biased float32
     * exponent of amax (one higher when amax * 2^(141-k) >= 32767.5; at least 15), code =
     * rint(v * 2^(141-k)), value = 2^(k-141) * code.  That halves the bytes between the two
     * kernels; an element moves by at most 2^(k-142) <= amax/32768 (measured 1e-4 * rms on the
     * layer output, against the 1e-2 * rms that rounding the activations to bf16 contributes).
     * The float32 y that moe_grouped_ffn writes and the y_perm tap hold exactly these values.
     * Non-finite values do not survive this form as themselves: a block that contains +-Inf
     * (an overflowed accumulator) gets exponent byte 255 and reads back as NaN in every one of
     * its 16 elements (so the overflow stays visible in out); a NaN element, which only
     * unsupported NaN input can produce, reads back as 0.
     * No effect on the F32 path. */
    MOE_FLAG_Y_F32 = 1
};

typedef enum moe_call {
    MOE_CALL_ROUTE = 0,
    MOE_CALL_PERMUTE = 1,
    MOE_CALL_GROUPED_FFN = 2,
    MOE_CALL_COMBINE = 3,
    MOE_CALL_PREFILL_LAYER = 4
} moe_call;

/* Shape and types of one layer call.
 *   T tokens, H hidden size, E experts, K experts per token, I expert
 *   intermediate size.  Limits: 1 <= K <= min(E, 32), E <= 1024, T*K < 2^31,
 *   T >= 0 (T = 0 is a valid no-op).
 *   x_dtype   F32 or BF16                       (activations x)
 *   w_dtype   F32 (needs x F32), BF16 (needs x BF16) or FP8_E4M3 (needs x BF16;
 *             weights are e4m3 codes with one float scale per output channel)
 *   out_dtype F32 or BF16 (the bf16 result is the float32 result rounded once)
 *   The BF16 path needs H % 128 == 0 and I % 128 == 0, the FP8 path H % 256 == 0 and
 *   I % 256 == 0; the F32 path takes any size.  The BF16 and FP8 paths also need
 *   T*H*2 < 4 GiB (x is addressed with 32-bit byte offsets), H <= 65536 and I <= 32768;
 *   larger shapes return MOE_ERR_UNSUPPORTED.
 */
typedef struct moe_config {
    int32_t T, H, E, K, I;
    int32_t x_dtype;
    int32_t w_dtype;
    int32_t out_dtype;
    int32_t flags;
} moe_config_t;

/* Optional intermediate outputs of moe_prefill_layer (any member may be NULL).
 * Shapes as in the single calls below. */
typedef struct moe_taps {
    float *logits;       /* [T,E]   */
    int32_t *topk_idx;   /* [T,K]   */
    float *topk_w;       /* [T,K]   */
    int32_t *counts;     /* [E]     */
    int32_t *offsets;    /* [E+1]   */
    int32_t *perm;       /* [P]     */
    int32_t *inv_perm;   /* [P]     */
    void *act;           /* [P,I]   SwiGLU activations in sorted row order: F32 for the F32 path, else BF16 */
    uint8_t *act_q;      /* [P,I]   FP8 path only: e4m3 codes of act            */
    float *act_scale;    /* [P]     FP8 path only: per-row scales of act        */
    float *y_perm;       /* [P,H]   expert outputs in sorted row order, F32 (BF16 / FP8 paths: the
                                    block-scaled values unless MOE_FLAG_Y_F32, see the flag) */
} moe_taps_t;

/* Kernels that moe_set_profile_events can bracket. */
typedef enum moe_kernel {
    MOE_KERNEL_ROUTER_GEMM = 0,
    MOE_KERNEL_TOPK = 1,
    MOE_KERNEL_PERMUTE = 2,   /* histogram + scan + scatter (three launches) */
    MOE_KERNEL_GATE_UP = 3,   /* grouped gate/up GEMM with the SwiGLU epilogue */
    MOE_KERNEL_DOWN = 4,      /* grouped down GEMM */
    MOE_KERNEL_COMBINE = 5,
    MOE_KERNEL_COUNT = 6
} moe_kernel;

int32_t moe_abi_version(void);
const char *moe_status_string(int32_t status);

/* One-time set-up for the device that is current: what the first compute call on a device would
 * otherwise do itself (see "Host-side state" above).  Idempotent, thread-safe, allocates nothing. */
int32_t moe_init_device(void);

/* Minimum workspace, in bytes, of one entry point for this config. */
int32_t moe_workspace_bytes(const moe_config_t *cfg, int32_t call, size_t *bytes_out);

/* Measurement hook (Sec. 8.5 of the paper reports utilisation as achieved over peak FLOP/s;
 * this is how one kernel's share is timed without a profiler).  While a (start, stop) pair of
 * hipEvent_t (passed as void*, created by the caller with timing enabled) is set for a kernel,
 * every launch of that kernel is bracketed by hipEventRecord(start, stream) and
 * hipEventRecord(stop, stream).  Pass NULL, NULL to clear.  Host-side state of the calling
 * process, not thread-safe; costs nothing when unset. */
int32_t moe_set_profile_events(int32_t kernel, void *start_event, void *stop_event);

/* Per-row e4m3 quantiser, the fp8 storage of expert weights (rows = output
 * channels) and of activations (rows = tokens), for the FP8 precision the paper
 * deploys (Sec. 8.1).  All steps in IEEE binary32:
 *   scale[r] = max_c |src[r,c]| / 448  (1 if the row is all zero)
 *   q[r,c]   = e4m3(src[r,c] / scale[r]), round to nearest even, saturating.
 * src is BF16 [rows, cols], cols % 8 == 0; q is [rows, cols] bytes; scale [rows]. */
int32_t moe_quantize_rows_e4m3(const void *src_bf16, int64_t rows, int32_t cols, uint8_t *q,
                               float *scale, void *stream);

/* Router (Sec. 2.3: every token is dispatched to its top-k experts by a small
 * linear router).  logits[t,e] = sum_h x[t,h]*w_router[e,h] (+ bias[e]), accumulated in
 * float32; per token the K largest logits in descending order, equal values
 * ordered by ascending expert index; topk_w = softmax over the selected logits
 * (equal to the full softmax renormalised over the selection).
 *   x [T,H] (x_dtype), w_router [E,H] F32, bias [E] F32 or NULL,
 *   logits_out [T,E] F32 or NULL (then the logits live in ws),
 *   topk_idx [T,K] int32, topk_w [T,K] F32.
 *   ws: moe_workspace_bytes(cfg, MOE_CALL_ROUTE) bytes; it may be NULL only for F32 activations
 *   with logits_out given (BF16 activations keep a bf16 split of w_router there). */
int32_t moe_route(const moe_config_t *cfg, const void *x, const float *w_router, const float *bias,
                  float *logits_out, int32_t *topk_idx, float *topk_w, void *ws, size_t ws_bytes,
                  void *stream);

/* Grouping by expert (the token permutation/alignment step of Sec. 4.3).
 *   counts[e] = number of routed rows of expert e; offsets = exclusive prefix sum,
 *   offsets[E] = P; perm[p] = flat id of sorted row p; inv_perm[f] = sorted position
 *   of flat id f.  Deterministic, independent of scheduling.
 *   x, x_perm: optional; when both are given x_perm[p,:] = x[perm[p]/K,:]
 *   ([P,H], x_dtype).  moe_grouped_ffn does not need x_perm (it gathers rows
 *   itself). */
int32_t moe_permute(const moe_config_t *cfg, const int32_t *topk_idx, const void *x, int32_t *counts,
                    int32_t *offsets, int32_t *perm, int32_t *inv_perm, void *x_perm, void *ws,
                    size_t ws_bytes, void *stream);

/* moe_permute for callers that cannot allocate (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc) and therefore have no workspace to pass: the same
 * kernels and the same results, with the segment counters in a fixed array of
 * MOE_NOALLOC_SCRATCH_BYTES bytes of device memory inside the library (one copy per GPU, held
 * until the process ends).  The call allocates and frees nothing.  Configurations whose
 * moe_workspace_bytes(cfg, MOE_CALL_PERMUTE) = ceil(T*K/2048) * E * 4 exceeds that size return
 * MOE_ERR_TOO_LARGE and enqueue nothing.  All calls on one GPU share the array: calls that may
 * overlap on one GPU (different streams, different host threads) race and must be serialised
 * by the caller.  Nothing in the array has to survive or be cleared between calls.  The first
 * call on a device looks up the array's address (see moe_init_device). */
#define MOE_NOALLOC_SCRATCH_BYTES (1u << 20)
int32_t moe_permute_noalloc(const moe_config_t *cfg, const int32_t *topk_idx, const void *x,
                            int32_t *counts, int32_t *offsets, int32_t *perm, int32_t *inv_perm,
                            void *x_perm, void *stream);

/* Grouped SwiGLU expert FFN over the ragged per-expert row groups (the per-expert
 * GEMMs of Sec. 4.2).  For sorted row p in expert e's group, with
 * x_p = x[perm[p]/K,:]:
 *   g = Wg_e x_p, u = Wu_e x_p, a = g/(1+exp(-g))*u, y_perm[p,:] = Wd_e a.
 * Accumulation is float32; a is rounded once to BF16 between the two GEMMs
 * (kept F32 on the F32 path).  FP8 path: x rows and a rows are quantised per
 * row as in moe_quantize_rows_e4m3 and the float scales are applied to the
 * float32 accumulators.
 *   x [T,H]; perm [P]; offsets [E+1]; w_gate,w_up [E,I,H]; w_down [E,H,I]
 *   (w_dtype; FP8: bytes); s_gate,s_up [E,I], s_down [E,H] F32 (FP8 only, else
 *   NULL); act_tap [P,I] or NULL (BF16, F32 on the F32 path); act_q_tap [P,I],
 *   act_scale_tap [P] or NULL (FP8 only); y_perm [P,H] F32.  On the BF16 / FP8 paths y_perm
 *   holds the block-scaled 16-bit values (exactly representable in F32) unless
 *   MOE_FLAG_Y_F32 is set; moe_prefill_layer keeps y in the compact form itself when no
 *   y_perm tap is asked for, with the same output bits. */
int32_t moe_grouped_ffn(const moe_config_t *cfg, const void *x, const int32_t *perm,
                        const int32_t *offsets, const void *w_gate, const void *w_up,
                        const void *w_down, const float *s_gate, const float *s_up,
                        const float *s_down, void *act_tap, uint8_t *act_q_tap,
                        float *act_scale_tap, float *y_perm, void *ws, size_t ws_bytes,
                        void *stream);

/* Weighted combine back to token order (the sum over a token's k expert outputs, Sec. 2.3):
 *   out[t,:] = sum_{j<K} topk_w[t,j] * y_perm[inv_perm[t*K+j],:], float32 FMA in
 *   slot order, one rounding to out_dtype.  out [T,H]. */
int32_t moe_combine(const moe_config_t *cfg, const float *y_perm, const int32_t *inv_perm,
                    const float *topk_w, void *out, void *stream);

/* The whole block in one call; bit-identical to the four calls above in sequence.
 * taps may be NULL. */
int32_t moe_prefill_layer(const moe_config_t *cfg, const void *x, const float *w_router,
                          const float *bias, const void *w_gate, const void *w_up,
                          const void *w_down, const float *s_gate, const float *s_up,
                          const float *s_down, void *out, const moe_taps_t *taps, void *ws,
                          size_t ws_bytes, void *stream);

/* ---- One-GPU weight streaming (the single-GPU host-to-device mode of the weight streaming engine,
 * App. B.1; offloading pipeline of Sec. 6.3) and the saturation threshold (Eq. 1; App. B.4 Eq. 3).
 *
 * The expert weights of all layers stay in PINNED HOST memory; the GPU holds n_slots layer
 * slots of moe_layer_weight_bytes(cfg) bytes each.  Layer i runs from slot i % n_slots.  The copy
 * stream transfers a layer into its slot as soon as the layer that used the slot before has
 * finished; the compute stream waits once, at the layer's entry, for that transfer.  Layers
 * 0 .. n_resident-1 are taken to be in slots 0 .. n_resident-1 already (the paper keeps the
 * first MoE layer's experts resident), laid out as moe_prefill_layers_streamed lays them out:
 * [w_gate][w_up][w_down][s_gate][s_up][s_down], each part aligned to 256 bytes.
 * Every layer reads the same x and writes its own out (what links two MoE blocks in a model,
 * attention and the residual path, is outside this block).  Nothing is synchronised with the
 * host; the call enqueues all layers and returns. */
typedef struct moe_stream_layer {
    const void *w_gate, *w_up, *w_down;   /* pinned HOST memory, w_dtype, [E,I,H] / [E,H,I] */
    const float *s_gate, *s_up, *s_down;  /* pinned HOST memory, FP8 only, else NULL */
    const float *w_router, *bias;         /* DEVICE memory ([E,H]; [E] or NULL): small, kept resident */
    void *out;                            /* DEVICE memory [T,H], out_dtype */
} moe_stream_layer_t;

int32_t moe_layer_weight_bytes(const moe_config_t *cfg, size_t *bytes_out);

/* slots: n_slots device buffers (256-byte aligned).  slot_events: 2*n_slots hipEvent_t (as
 * void*) owned by the caller, used as "transfer landed" / "slot free" marks.  layer_events: NULL,
 * or 2*n_layers hipEvent_t with timing enabled; [2i] is recorded on the compute stream before
 * layer i's entry wait and [2i+1] after its last kernel, so their distance is the layer's wall
 * time including any stall on the transfer (the t_c / t_e of App. B.4).  compute_stream and
 * copy_stream must differ.  ws: moe_workspace_bytes(cfg, MOE_CALL_PREFILL_LAYER). */
int32_t moe_prefill_layers_streamed(const moe_config_t *cfg, int32_t n_layers,
                                    const moe_stream_layer_t *layers, const void *x,
                                    void *const *slots, int32_t n_slots, int32_t n_resident,
                                    void *const *slot_events, void *const *layer_events, void *ws,
                                    size_t ws_bytes, void *compute_stream, void *copy_stream);

/* f_tok of this block: counted flop per token, K*6*H*I + 2*H*E. */
double moe_layer_flops_per_token(const moe_config_t *cfg);
/* Eq. 1: T = t_EP * F_GPU * gamma (flop a batch must carry for its compute to cover the slowest
 * per-layer transfer). */
double moe_saturation_threshold_flops(double t_ep_seconds, double f_gpu_flops, double gamma);
/* App. B.4, Eq. 3: T = gamma * (t_e / t_c) * C_dummy, with t_c the wall time of the resident
 * first layer, t_e the largest wall time of a later layer and C_dummy = f_tok * n_ref; it
 * collapses to gamma * C_dummy when t_e <= t_c, which is also the fallback when t_c is not
 * positive (no calibration yet). */
double moe_calibrated_threshold_flops(double t_c, double t_e, double c_dummy_flops, double gamma);

/* App. B.4, delivery and fallback: the threshold the frontend installs, and the unit that both it
 * and the work counters L_i are kept in.
 *   pinned > 0          the operator's manual value is used as it is (a calibration result is
 *                       skipped); its unit follows f_tok as below.
 *   f_tok > 0           FLOPs: T = Eq. 3 with C_dummy = f_tok * n_ref (before any calibration,
 *                       t_c <= 0, this is gamma * f_tok * n_ref).
 *   f_tok not positive  (the model configuration lacks what f_tok needs) token-unit accounting:
 *                       the same formula with one unit of work per token, T = gamma *
 *                       max(t_e/t_c, 1) * n_ref tokens; the scheduling round is then run with
 *                       f_tok = 1, f_attn = 0 so that L_i counts uncached tokens.
 * Host arithmetic only.  gamma must be positive and n_ref non-negative (MOE_ERR_BAD_SHAPE). */
enum { MOE_UNIT_FLOPS = 0, MOE_UNIT_TOKENS = 1 };
int32_t moe_resolve_threshold(double pinned, double t_c, double t_e, double f_tok, double n_ref,
                              double gamma, double *threshold_out, int32_t *unit_out);

#ifdef __cplusplus
}
#endif
#endif /* MOE_PREFILL_H */
