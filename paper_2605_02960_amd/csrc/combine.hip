// Weighted combine back to token order: out[t,:] = sum_j w[t,j] * y_perm[inv_perm[t*K+j],:]
// (the sum over a token's k expert outputs, Sec. 2.3 of the paper).  HBM-bound gather-reduce: every y_perm row is
// read exactly once, 16 bytes per lane, and the K terms are added in slot order in float32, so
// the result is deterministic.
#include "common.h"

namespace moe {

// KC > 0: K is the compile-time constant KC (slot loop unrolled, all KC row reads of a chunk in
// flight together); KC = 0: any K.  The token's positions and weights are wave-uniform, so they
// are fetched through the scalar path.
template <bool OUT_BF16, int KC>
__global__ __launch_bounds__(256) void combine_kernel(const f32x4* __restrict__ y, int row_vec,
                                                     const int32_t* __restrict__ inv_perm,
                                                     const float* __restrict__ w, int K_any,
                                                     void* __restrict__ out) {
    const int t = blockIdx.x;
    const int K = KC > 0 ? KC : K_any;
    const int32_t* __restrict__ pos = inv_perm + (size_t)t * K;
    const float* __restrict__ wt = w + (size_t)t * K;
    for (int i = threadIdx.x; i < row_vec; i += blockDim.x) {
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
        if constexpr (KC > 0) {
            f32x4 v[KC];
#pragma unroll
            for (int j = 0; j < KC; ++j) v[j] = __builtin_nontemporal_load(y + (size_t)pos[j] * row_vec + i);
#pragma unroll
            for (int j = 0; j < KC; ++j) {
                const float s = wt[j];
                acc.x = fmaf(s, v[j].x, acc.x);
                acc.y = fmaf(s, v[j].y, acc.y);
                acc.z = fmaf(s, v[j].z, acc.z);
                acc.w = fmaf(s, v[j].w, acc.w);
            }
        } else {
            for (int j = 0; j < K; ++j) {
                const f32x4 v = __builtin_nontemporal_load(y + (size_t)pos[j] * row_vec + i);
                const float s = wt[j];
                acc.x = fmaf(s, v.x, acc.x);
                acc.y = fmaf(s, v.y, acc.y);
                acc.z = fmaf(s, v.z, acc.z);
                acc.w = fmaf(s, v.w, acc.w);
            }
        }
        if constexpr (OUT_BF16) {
            uint2 o;
            o.x = pack2_bf16(acc.x, acc.y);
            o.y = pack2_bf16(acc.z, acc.w);
            static_cast<uint2*>(out)[(size_t)t * row_vec + i] = o;
        } else {
            // the output is larger than the caches and is not read again by this block
            __builtin_nontemporal_store(acc, static_cast<f32x4*>(out) + (size_t)t * row_vec + i);
        }
    }
}

// The same sum over y in its compact form (int16 codes in blocks of 16 columns, one exponent byte
// per block): a thread takes 8 adjacent columns, 16 bytes of codes per slot.  Each term is
// 2^(k-141) * code, exact in float32, and then one FMA: the same bits as combine_kernel on the
// float32 copy of the same values.
template <bool OUT_BF16, int KC>
__global__ __launch_bounds__(256) void combine_block16_kernel(const u32x4* __restrict__ yq, int row_vec8,
                                                             const uint8_t* __restrict__ yk, int nblk,
                                                             const int32_t* __restrict__ inv_perm,
                                                             const float* __restrict__ w, int K_any,
                                                             void* __restrict__ out) {
    const int t = blockIdx.x;
    const int K = KC > 0 ? KC : K_any;
    const int32_t* __restrict__ pos = inv_perm + (size_t)t * K;
    const float* __restrict__ wt = w + (size_t)t * K;
    constexpr int KU = KC > 0 ? KC : 1;
    for (int i = threadIdx.x; i < row_vec8; i += blockDim.x) {
        const int blk = i >> 1;
        float acc[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = 0.f;
        for (int j0 = 0; j0 < K; j0 += KU) {
            u32x4 v[KU];
            uint32_t k[KU];
#pragma unroll
            for (int j = 0; j < KU; ++j) {
                v[j] = __builtin_nontemporal_load(yq + (size_t)pos[j0 + j] * row_vec8 + i);
                k[j] = yk[(size_t)pos[j0 + j] * nblk + blk];
            }
#pragma unroll
            for (int j = 0; j < KU; ++j) {
                const float s = wt[j0 + j];
                // exponent byte 255 marks a block that held +-Inf: it reads back as NaN
                const float sc = k[j] == 255u ? __uint_as_float(0x7FC00000u) : __uint_as_float((k[j] - 14u) << 23);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const uint32_t d = v[j][e >> 1];
                    const int code = (e & 1) ? ((int)d >> 16) : (int)(short)(d & 0xFFFFu);
                    acc[e] = fmaf(s, sc * (float)code, acc[e]);
                }
            }
        }
        if constexpr (OUT_BF16) {
            u32x4 o;
#pragma unroll
            for (int e = 0; e < 4; ++e)
                o[e] = pack2_bf16(acc[2 * e], acc[2 * e + 1]);
            static_cast<u32x4*>(out)[(size_t)t * row_vec8 + i] = o;
        } else {
            f32x4* o = static_cast<f32x4*>(out) + ((size_t)t * row_vec8 + i) * 2;
            __builtin_nontemporal_store(f32x4{acc[0], acc[1], acc[2], acc[3]}, o);
            __builtin_nontemporal_store(f32x4{acc[4], acc[5], acc[6], acc[7]}, o + 1);
        }
    }
}

// Any H (no vector width assumption).
template <bool OUT_BF16>
__global__ __launch_bounds__(256) void combine_scalar_kernel(const float* __restrict__ y, int H,
                                                            const int32_t* __restrict__ inv_perm,
                                                            const float* __restrict__ w, int K,
                                                            void* __restrict__ out) {
    const int t = blockIdx.x;
    for (int h = threadIdx.x; h < H; h += blockDim.x) {
        float acc = 0.f;
        for (int j = 0; j < K; ++j)
            acc = fmaf(w[(size_t)t * K + j], y[(size_t)inv_perm[(size_t)t * K + j] * H + h], acc);
        if constexpr (OUT_BF16)
            static_cast<uint16_t*>(out)[(size_t)t * H + h] = f32_to_bf16_bits(acc);
        else
            static_cast<float*>(out)[(size_t)t * H + h] = acc;
    }
}

int32_t launch_combine(const moe_config_t& c, const float* y_perm, const int32_t* inv_perm,
                       const float* topk_w, void* out, hipStream_t s) {
    if (c.T == 0) return MOE_OK;
    const bool bf = c.out_dtype == MOE_DTYPE_BF16;
    KernelBracket kb(MOE_KERNEL_COMBINE, s);
    const bool vec = (c.H % 4 == 0) && ((uintptr_t)y_perm % 16 == 0) && ((uintptr_t)out % 16 == 0);
    if (vec) {
        const f32x4* y = reinterpret_cast<const f32x4*>(y_perm);
#define MOE_COMBINE_LAUNCH(KC_)                                                                      \
    if (bf) combine_kernel<true, KC_><<<c.T, 256, 0, s>>>(y, c.H / 4, inv_perm, topk_w, c.K, out);   \
    else combine_kernel<false, KC_><<<c.T, 256, 0, s>>>(y, c.H / 4, inv_perm, topk_w, c.K, out);
        if (c.K == 8) { MOE_COMBINE_LAUNCH(8) }
        else if (c.K == 4) { MOE_COMBINE_LAUNCH(4) }
        else if (c.K == 2) { MOE_COMBINE_LAUNCH(2) }
        else { MOE_COMBINE_LAUNCH(0) }
#undef MOE_COMBINE_LAUNCH
    } else {
        if (bf) combine_scalar_kernel<true><<<c.T, 256, 0, s>>>(y_perm, c.H, inv_perm, topk_w, c.K, out);
        else combine_scalar_kernel<false><<<c.T, 256, 0, s>>>(y_perm, c.H, inv_perm, topk_w, c.K, out);
    }
    return launch_status();
}

int32_t launch_combine_block16(const moe_config_t& c, const int16_t* y_codes, const uint8_t* y_exps,
                               const int32_t* inv_perm, const float* topk_w, void* out,
                               hipStream_t s) {
    if (c.T == 0) return MOE_OK;
    if (c.H % Y_BLOCK_COLS != 0) return MOE_ERR_BAD_SHAPE;
    const bool bf = c.out_dtype == MOE_DTYPE_BF16;
    KernelBracket kb(MOE_KERNEL_COMBINE, s);
    const u32x4* yq = reinterpret_cast<const u32x4*>(y_codes);
    const int nblk = c.H / Y_BLOCK_COLS;
#define MOE_COMBINE_LAUNCH(KC_)                                                                              \
    if (bf) combine_block16_kernel<true, KC_><<<c.T, 256, 0, s>>>(yq, c.H / 8, y_exps, nblk, inv_perm,       \
                                                                  topk_w, c.K, out);                         \
    else combine_block16_kernel<false, KC_><<<c.T, 256, 0, s>>>(yq, c.H / 8, y_exps, nblk, inv_perm,         \
                                                                topk_w, c.K, out);
    if (c.K == 8) { MOE_COMBINE_LAUNCH(8) }
    else if (c.K == 4) { MOE_COMBINE_LAUNCH(4) }
    else if (c.K == 2) { MOE_COMBINE_LAUNCH(2) }
    else { MOE_COMBINE_LAUNCH(0) }
#undef MOE_COMBINE_LAUNCH
    return launch_status();
}

}  // namespace moe
