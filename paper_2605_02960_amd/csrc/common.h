// Internal declarations shared by the HIP sources of libmoeprefill (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/moe_prefill.h"

namespace moe {

constexpr int WAVE = 64;

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(8))) int i32x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

// bf16 <-> f32 on raw bit patterns (round to nearest even; inputs are finite).
__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) {
    return __uint_as_float(static_cast<uint32_t>(b) << 16);
}
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return static_cast<uint16_t>(u >> 16);
}

// Two float32 -> two bf16 in one dword (lo in the low half), round to nearest even: gfx950's
// packed convert instruction.
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
__device__ __forceinline__ uint32_t pack2_bf16(float lo, float hi) {
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{lo, hi}, bf16x2));
}

__host__ __device__ inline int64_t ceil_div64(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

inline int32_t launch_status() {
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_LAUNCH_FAILED;
}

// ---- device.hip : what the library keeps per device.  Filled once per device, under a mutex,
// by the first call made with that device current (or by moe_init_device): the compute-unit
// count and the kernels' dynamic-LDS attribute.
struct DeviceState {
    int n_cu;
    void* scratch;   // device address of the static scratch array of moe_permute_noalloc on this device
};
int32_t device_state(const DeviceState** out);
// one-time attribute set-up of the kernels that need more than 64 KB of LDS (called by device_state)
int32_t ffn_mfma_set_attributes();
int32_t router_mfma_set_attributes();

// Optional per-kernel event bracket (see moe_set_profile_events).
struct ProfileSlot {
    hipEvent_t start, stop;
};
extern ProfileSlot g_profile[MOE_KERNEL_COUNT];
struct KernelBracket {
    const ProfileSlot& p;
    hipStream_t s;
    KernelBracket(int kernel, hipStream_t stream) : p(g_profile[kernel]), s(stream) {
        if (p.start) (void)hipEventRecord(p.start, s);
    }
    ~KernelBracket() {
        if (p.stop) (void)hipEventRecord(p.stop, s);
    }
};

// ---- route.hip
// logits [T,E] f32 = x [T,H] (f32 or bf16 bits) . w_router[E,H]^T (+bias); then top-k.
int32_t launch_router_logits(const moe_config_t& c, const void* x, const float* w_router,
                             const float* bias, float* logits, hipStream_t s);
// ---- router_mfma.hip : bf16 activations, float32 router weight split into three bf16 parts
size_t router_mfma_ws_bytes(const moe_config_t& c);
// With at most 128 experts the kernel also selects the top K (router_mfma_fuses_topk): logits may
// then be NULL, and topk_idx / topk_w are written by it instead of by launch_topk.
bool router_mfma_fuses_topk(const moe_config_t& c);
int32_t launch_router_logits_mfma(const moe_config_t& c, const void* x, const float* w_router,
                                  const float* bias, float* logits, int32_t* topk_idx, float* topk_w,
                                  void* ws, hipStream_t s);
int32_t launch_topk(const moe_config_t& c, const float* logits, int32_t* topk_idx, float* topk_w,
                    hipStream_t s);

// ---- permute.hip
size_t permute_ws_bytes(const moe_config_t& c);
int32_t launch_permute(const moe_config_t& c, const int32_t* topk_idx, int32_t* counts,
                       int32_t* offsets, int32_t* perm, int32_t* inv_perm, void* ws, hipStream_t s);
int32_t launch_gather_rows(const moe_config_t& c, const void* x, const int32_t* perm, void* x_perm,
                           hipStream_t s);

// ---- tiles.hip : per-expert row tiles of height bm, built on the device from offsets.
// table[0] = number of tiles n; table[1 + 2*i] = expert, table[2 + 2*i] = first sorted row of tile i.
inline int64_t max_row_tiles(const moe_config_t& c, int bm) {
    return ((int64_t)c.T * c.K) / bm + c.E;
}
inline size_t tile_table_bytes(const moe_config_t& c, int bm) {
    return align_up(sizeof(int32_t) * (1 + 2 * (size_t)max_row_tiles(c, bm)), 256);
}
// first_out (optional, [E+1]): index of every expert's first row tile.
int32_t launch_build_tile_table(const moe_config_t& c, const int32_t* offsets, int bm,
                                int32_t* table, int32_t* first_out, hipStream_t s);
// order[L] = (expert, first sorted row, end row, column tile) of launch slot L (nct column tiles
// per row tile): everything a workgroup needs to start a tile, in one 16-byte load.
inline size_t tile_order_bytes(const moe_config_t& c, int bm, int nct) {
    return align_up(sizeof(int4) * (size_t)max_row_tiles(c, bm) * nct, 256);
}
int32_t launch_build_tile_order(const moe_config_t& c, const int32_t* first, const int32_t* offsets, int bm,
                                int nct, int gr, int gc, int4* order, hipStream_t s);

// ---- ffn_f32.hip
size_t ffn_f32_ws_bytes(const moe_config_t& c);
int32_t launch_ffn_f32(const moe_config_t& c, const float* x, const int32_t* perm,
                       const int32_t* offsets, const float* wg, const float* wu, const float* wd,
                       float* act_tap, float* y_perm, void* ws, hipStream_t s);

// ---- ffn_mfma.hip (bf16 and fp8)
size_t ffn_mfma_ws_bytes(const moe_config_t& c);
int32_t launch_ffn_mfma(const moe_config_t& c, const void* x, const int32_t* perm,
                        const int32_t* offsets, const void* wg, const void* wu, const void* wd,
                        const float* s_gate, const float* s_up, const float* s_down, void* act_tap,
                        uint8_t* act_q_tap, float* act_scale_tap, float* y_perm, int16_t* y_codes,
                        uint8_t* y_exps, void* ws, hipStream_t s);
// y in its compact form: 16-column blocks of int16 codes [P,H] with one exponent byte k each
// [P,H/16], value = 2^(k-141) * code.  y_codes != NULL selects it (y_perm is then unused).
constexpr int Y_BLOCK_COLS = 16;

// ---- combine.hip
int32_t launch_combine(const moe_config_t& c, const float* y_perm, const int32_t* inv_perm,
                       const float* topk_w, void* out, hipStream_t s);
int32_t launch_combine_block16(const moe_config_t& c, const int16_t* y_codes, const uint8_t* y_exps,
                               const int32_t* inv_perm, const float* topk_w, void* out,
                               hipStream_t s);

// ---- quant.hip
int32_t launch_quantize_rows(const void* src_bf16, int64_t rows, int32_t cols, uint8_t* q,
                             float* scale, hipStream_t s);

}  // namespace moe
