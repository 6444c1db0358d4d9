// Router: float32 logits and per-token top-k selection with renormalised softmax weights
// (the router of Sec. 2.3 of the paper).
#include "f32_gemm.h"

namespace moe {

int32_t launch_router_logits(const moe_config_t& c, const void* x, const float* w_router,
                             const float* bias, float* logits, hipStream_t s) {
    if (c.T == 0) return MOE_OK;
    F32GemmArgs a{};
    a.A = x;
    a.lda = c.H;
    a.a_row_index = nullptr;
    a.a_row_div = 1;
    a.B = w_router;
    a.B2 = nullptr;
    a.N = c.E;
    a.K = c.H;
    a.tile_table = nullptr;
    a.offsets = nullptr;
    a.M = c.T;
    a.bias = bias;
    a.C = logits;
    a.ldc = c.E;
    KernelBracket kb(MOE_KERNEL_ROUTER_GEMM, s);
    if (c.E > 64) {
        dim3 grid((unsigned)ceil_div64(c.T, 128), (unsigned)ceil_div64(c.E, 128));
        if (c.x_dtype == MOE_DTYPE_F32)
            f32_gemm_nt_kernel<float, 128, 128, 8, 8, EPI_STORE><<<grid, 256, 0, s>>>(a);
        else
            f32_gemm_nt_kernel<uint16_t, 128, 128, 8, 8, EPI_STORE><<<grid, 256, 0, s>>>(a);
    } else {
        dim3 grid((unsigned)ceil_div64(c.T, 64), (unsigned)ceil_div64(c.E, 64));
        if (c.x_dtype == MOE_DTYPE_F32)
            f32_gemm_nt_kernel<float, 64, 64, 4, 4, EPI_STORE><<<grid, 256, 0, s>>>(a);
        else
            f32_gemm_nt_kernel<uint16_t, 64, 64, 4, 4, EPI_STORE><<<grid, 256, 0, s>>>(a);
    }
    return launch_status();
}

// One wavefront per token.  Lane l holds logits l, l+64, l+128, ... (at most 16 for E <= 1024).
// K rounds: every lane offers its best remaining candidate, a butterfly over the 64 lanes keeps
// the larger value (equal values: the lower expert index), the owner retires it.
// Weights: w_j = exp(l_j - l_0) / sum_i exp(l_i - l_0) over the K selected logits, which equals
// the softmax over all E renormalised over the selection (the common denominator cancels).
template <int PER_LANE>
__global__ __launch_bounds__(256) void topk_kernel(const float* __restrict__ logits, int T, int E,
                                                  int K, int32_t* __restrict__ topk_idx,
                                                  float* __restrict__ topk_w) {
    const int lane = threadIdx.x % WAVE;
    const int t = blockIdx.x * (blockDim.x / WAVE) + threadIdx.x / WAVE;
    if (t >= T) return;
    const float* row = logits + (size_t)t * E;
    float v[PER_LANE];
#pragma unroll
    for (int i = 0; i < PER_LANE; ++i) {
        const int e = i * WAVE + lane;
        float f = (e < E) ? row[e] : -INFINITY;
        v[i] = (f != f) ? -INFINITY : f;   // NaN is unsupported input; keep the search well defined
    }
    uint32_t taken = 0;
#pragma unroll
    for (int i = 0; i < PER_LANE; ++i)
        if (i * WAVE + lane >= E) taken |= 1u << i;

    float my_val = 0.f;   // lane j keeps the j-th selected logit
    int my_idx = 0;
    float top = 0.f;
    for (int j = 0; j < K; ++j) {
        float best = -INFINITY;
        int bidx = 0x7fffffff;
#pragma unroll
        for (int i = 0; i < PER_LANE; ++i) {
            const bool free_slot = !((taken >> i) & 1u);
            const int e = i * WAVE + lane;
            if (free_slot && (v[i] > best || (v[i] == best && e < bidx))) {
                best = v[i];
                bidx = e;
            }
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const float ov = __shfl_xor(best, off, WAVE);
            const int oi = __shfl_xor(bidx, off, WAVE);
            if (ov > best || (ov == best && oi < bidx)) {
                best = ov;
                bidx = oi;
            }
        }
        if ((bidx % WAVE) == lane) taken |= 1u << (bidx / WAVE);
        if (j == 0) top = best;
        if (lane == j) {
            my_val = best;
            my_idx = bidx;
        }
    }
    // K <= 32 lanes hold the selection; sum their exponentials in lane order 0..K-1
    const float ex = (lane < K) ? expf(my_val - top) : 0.f;
    float sum = 0.f;
    for (int j = 0; j < K; ++j) sum += __shfl(ex, j, WAVE);
    if (lane < K) {
        topk_idx[(size_t)t * K + lane] = my_idx;
        topk_w[(size_t)t * K + lane] = ex / sum;
    }
}

int32_t launch_topk(const moe_config_t& c, const float* logits, int32_t* topk_idx, float* topk_w,
                    hipStream_t s) {
    if (c.T == 0) return MOE_OK;
    const int waves_per_block = 4;
    const unsigned grid = (unsigned)ceil_div64(c.T, waves_per_block);
    const int per = (int)ceil_div64(c.E, WAVE);
    KernelBracket kb(MOE_KERNEL_TOPK, s);
#define MOE_TOPK_CASE(P)                                                                          \
    topk_kernel<P><<<grid, waves_per_block * WAVE, 0, s>>>(logits, c.T, c.E, c.K, topk_idx, topk_w)
    if (per <= 1) MOE_TOPK_CASE(1);
    else if (per <= 2) MOE_TOPK_CASE(2);
    else if (per <= 4) MOE_TOPK_CASE(4);
    else if (per <= 8) MOE_TOPK_CASE(8);
    else MOE_TOPK_CASE(16);
#undef MOE_TOPK_CASE
    return launch_status();
}

}  // namespace moe
