// Router logits on the matrix cores for bf16 activations, exact to float32 accumulation.
// The float32 router weight is split into three bf16 parts, w = hi + mid + lo (each the bf16
// rounding of what the previous parts left; three 8-bit parts cover the 24-bit significand), so
// x*w = x*hi + x*mid + x*lo with every product exact in float32.  The three partial GEMMs run
// as one bf16 MFMA GEMM against 3*E weight rows and are added in the epilogue, smallest first.
// This is the router of Sec. 2.3 of the paper at MFMA rate instead of vector-ALU rate.
//
// With at most 128 experts (one expert tile) the selection is made in the same kernel: the 128
// logits of the tile's tokens go from the accumulators to LDS, and 16 lanes per token pick the K
// largest (descending value, equal values by ascending expert index) and form the renormalised
// softmax weights; the logits are written to memory only when the caller asks for them.
//
// Tile: 128 tokens x 128 experts x 3 parts per workgroup (8 waves = 2 along tokens x 4 along
// experts; a wave owns 64 tokens x 32 experts x 3 parts = 6 MFMA 32x32x16 blocks), K step 64,
// two LDS stages of 16 KB (tokens) + 48 KB (weights), global loads staged two K steps ahead in
// registers.  LDS rows are 128 bytes with the same chunk swizzle as the expert GEMMs.
#include "common.h"

namespace moe {

namespace {

constexpr int R_BM = 128, R_BE = 128, R_BK = 64;
constexpr int R_ROW = R_BK * 2;
constexpr int R_A_TILE = R_BM * R_ROW;            // 16 KB
constexpr int R_B_TILE = 3 * R_BE * R_ROW;        // 48 KB
constexpr int R_STAGE = R_A_TILE + R_B_TILE;      // 64 KB
constexpr int R_THREADS = 512;

__global__ __launch_bounds__(256) void split_router_weights_kernel(const float* __restrict__ w,
                                                                  size_t n,
                                                                  uint16_t* __restrict__ w3) {
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n;
         i += (size_t)gridDim.x * blockDim.x) {
        const float v = w[i];
        const uint16_t hi = f32_to_bf16_bits(v);
        const float r1 = v - bf16_bits_to_f32(hi);
        const uint16_t mid = f32_to_bf16_bits(r1);
        const float r2 = r1 - bf16_bits_to_f32(mid);
        w3[i] = hi;
        w3[n + i] = mid;
        w3[2 * n + i] = f32_to_bf16_bits(r2);
    }
}

// 16 lanes (a DPP row) share one token.  The four exchange steps of a reduction over the row, as
// DPP moves (vector ALU speed, no LDS round trip): neighbour in the quad, other pair of the quad,
// mirror inside each half row (pairs quad 0 with 1 and 2 with 3), mirror of the row (pairs the
// halves).  Any pairing of disjoint groups serves, the (value, index) maximum being associative
// and commutative.
template <int STEP>
__device__ __forceinline__ int row_exchange(int v) {
    constexpr int ctrl = STEP == 0 ? 0xB1     // quad_perm [1,0,3,2]
                         : STEP == 1 ? 0x4E   // quad_perm [2,3,0,1]
                         : STEP == 2 ? 0x141  // row_half_mirror
                                     : 0x140; // row_mirror
    return __builtin_amdgcn_update_dpp(v, v, ctrl, 0xF, 0xF, false);
}
template <int STEP>
__device__ __forceinline__ float row_exchange(float v) {
    return __int_as_float(row_exchange<STEP>(__float_as_int(v)));
}

// FUSED: E <= 128 and gridDim.y == 1; topk_idx / topk_w are written, logits only if not NULL.
template <bool FUSED>
__global__ __launch_bounds__(R_THREADS) void router_mfma_kernel(const char* __restrict__ x,
                                                               const char* __restrict__ w3, int T,
                                                               int E, int H,
                                                               const float* __restrict__ bias,
                                                               float* __restrict__ logits, int K,
                                                               int32_t* __restrict__ topk_idx,
                                                               float* __restrict__ topk_w) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave & 1, we = wave >> 1;
    const int t0 = blockIdx.x * R_BM, e0 = blockIdx.y * R_BE;

    // loader: chunk lc of rows lr + 64*i; tokens i = 0,1 (128 rows), weights i = 0..5 (384 rows)
    const int lr = tid >> 3, lc = tid & 7;
    const uint32_t st_off = lr * R_ROW + ((lc ^ ((lr >> 1) & 7)) << 4);
    uint32_t a_off[2], b_off[6];
    const uint32_t row_bytes = (uint32_t)H * 2;
#pragma unroll
    for (int i = 0; i < 2; ++i) a_off[i] = (uint32_t)min(t0 + lr + 64 * i, T - 1) * row_bytes + lc * 16;
#pragma unroll
    for (int i = 0; i < 6; ++i) {
        const int R = lr + 64 * i;              // LDS weight row: part R / 128, expert R % 128
        const int part = R >> 7;
        const int e = min(e0 + (R & 127), E - 1);
        b_off[i] = ((uint32_t)part * E + e) * row_bytes + lc * 16;
    }

    const int fr = lane & 31, fh = lane >> 5;
    const int sw = (fr >> 1) & 7;
    uint32_t frag_off[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) frag_off[kk] = (uint32_t)(((kk * 2 + fh) ^ sw) << 4);
    const uint32_t xa_row = (wm * 64 + fr) * R_ROW;
    const uint32_t wb_row = R_A_TILE + (we * 32 + fr) * R_ROW;       // + part * 128 rows

    f32x16 acc[3][2];
#pragma unroll
    for (int p = 0; p < 3; ++p)
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[p][mi][v] = 0.f;

    u32x4 ra0[2], rb0[6], ra1[2], rb1[6];
#define R_GLOAD(SET_, KT_)                                                                \
    {                                                                                     \
        const uint32_t kb = (uint32_t)(KT_) * R_ROW;                                      \
        _Pragma("unroll") for (int i = 0; i < 2; ++i)                                     \
            ra##SET_[i] = *reinterpret_cast<const u32x4*>(x + (a_off[i] + kb));           \
        _Pragma("unroll") for (int i = 0; i < 6; ++i)                                     \
            rb##SET_[i] = *reinterpret_cast<const u32x4*>(w3 + (b_off[i] + kb));          \
    }
#define R_LSTORE(SET_, STAGE_)                                                            \
    {                                                                                     \
        char* base = smem + (STAGE_) * R_STAGE + st_off;                                  \
        _Pragma("unroll") for (int i = 0; i < 2; ++i)                                     \
            *reinterpret_cast<u32x4*>(base + i * 64 * R_ROW) = ra##SET_[i];               \
        _Pragma("unroll") for (int i = 0; i < 6; ++i)                                     \
            *reinterpret_cast<u32x4*>(base + R_A_TILE + i * 64 * R_ROW) = rb##SET_[i];    \
    }
#define R_COMPUTE(STAGE_)                                                                 \
    {                                                                                     \
        const char* st = smem + (STAGE_) * R_STAGE;                                       \
        _Pragma("unroll") for (int kk = 0; kk < 4; ++kk) {                                \
            bf16x8 xa[2], wb[3];                                                          \
            _Pragma("unroll") for (int mi = 0; mi < 2; ++mi) xa[mi] =                     \
                *reinterpret_cast<const bf16x8*>(st + xa_row + mi * 32 * R_ROW + frag_off[kk]); \
            _Pragma("unroll") for (int p = 0; p < 3; ++p) wb[p] =                         \
                *reinterpret_cast<const bf16x8*>(st + wb_row + p * 128 * R_ROW + frag_off[kk]); \
            _Pragma("unroll") for (int p = 0; p < 3; ++p)                                 \
                _Pragma("unroll") for (int mi = 0; mi < 2; ++mi) acc[p][mi] =             \
                    __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa[mi], wb[p], acc[p][mi], 0, 0, 0); \
        }                                                                                 \
    }

    const int KT = H / R_BK;   // even, >= 2
    R_GLOAD(0, 0);
    R_GLOAD(1, 1);
    R_LSTORE(0, 0);
    __syncthreads();
    for (int kt = 0; kt < KT; kt += 2) {
        R_GLOAD(0, min(kt + 2, KT - 1));
        R_COMPUTE(0);
        R_LSTORE(1, 1);
        __syncthreads();
        R_GLOAD(1, min(kt + 3, KT - 1));
        R_COMPUTE(1);
        R_LSTORE(0, 0);
        __syncthreads();
    }
#undef R_GLOAD
#undef R_LSTORE
#undef R_COMPUTE

    // acc[p][mi][v]: token row mi*32 + (v/4)*8 + fh*4 + v%4 of the wave's 64, expert we*32 + fr
    const int e = e0 + we * 32 + fr;
    const float b = (bias && e < E) ? bias[e] : 0.f;
    float* const lg = reinterpret_cast<float*>(smem);       // FUSED: [128 tokens][128 experts]
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int tr = wm * 64 + mi * 32 + (v >> 2) * 8 + fh * 4 + (v & 3);
            const float l = ((acc[2][mi][v] + acc[1][mi][v]) + acc[0][mi][v]) + b;
            if (e < E && t0 + tr < T && (!FUSED || logits)) logits[(size_t)(t0 + tr) * E + e] = l;
            // the K loop's last barrier lies behind every read of the operand stages
            if (FUSED) lg[tr * R_BE + we * 32 + fr] = l;
        }
    if constexpr (FUSED) {
        __syncthreads();
        // 16 lanes per token, lane q holds experts 8q .. 8q+7; a wave takes 4 tokens at a time
        const int q = lane & 15, grp = lane >> 4;
        for (int it = 0; it < 4; ++it) {
            const int tr = wave * 16 + it * 4 + grp;
            const f32x4 lo = *reinterpret_cast<const f32x4*>(lg + tr * R_BE + q * 8);
            const f32x4 hi = *reinterpret_cast<const f32x4*>(lg + tr * R_BE + q * 8 + 4);
            float val[8] = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
            uint32_t taken = 0;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                if (val[i] != val[i]) val[i] = -INFINITY;   // NaN is unsupported input; keep the search well defined
                if (q * 8 + i >= E) taken |= 1u << i;
            }
            float sel_v[2] = {0.f, 0.f};     // lane j of the row keeps selections j and 16 + j
            int sel_i[2] = {0, 0};
            float top = 0.f;
            for (int j = 0; j < K; ++j) {
                float best = -INFINITY;
                int bidx = 0x7fffffff;
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const bool free_slot = !((taken >> i) & 1u);
                    if (free_slot && (val[i] > best || (val[i] == best && q * 8 + i < bidx))) {
                        best = val[i];
                        bidx = q * 8 + i;
                    }
                }
#define R_BFLY(X_)                                                                        \
    {                                                                                     \
        const float ov = row_exchange<X_>(best);                                          \
        const int oi = row_exchange<X_>(bidx);                                            \
        if (ov > best || (ov == best && oi < bidx)) {                                     \
            best = ov;                                                                    \
            bidx = oi;                                                                    \
        }                                                                                 \
    }
                R_BFLY(0) R_BFLY(1) R_BFLY(2) R_BFLY(3)
#undef R_BFLY
                if ((bidx >> 3) == q) taken |= 1u << (bidx & 7);
                if (j == 0) top = best;
                if (j == q) {
                    sel_v[0] = best;
                    sel_i[0] = bidx;
                }
                if (j == q + 16) {
                    sel_v[1] = best;
                    sel_i[1] = bidx;
                }
            }
            // exponentials of the K selected logits, summed in selection order
            float ex[2];
#pragma unroll
            for (int h2 = 0; h2 < 2; ++h2) ex[h2] = (h2 * 16 + q < K) ? expf(sel_v[h2] - top) : 0.f;
            float sum = 0.f;
            const int row_lane0 = (lane & 48) << 2;          // byte address of the row's first lane
            for (int j = 0; j < min(K, 16); ++j)
                sum += __int_as_float(__builtin_amdgcn_ds_bpermute(row_lane0 + (j << 2), __float_as_int(ex[0])));
            for (int j = 16; j < K; ++j)
                sum += __int_as_float(__builtin_amdgcn_ds_bpermute(row_lane0 + ((j - 16) << 2), __float_as_int(ex[1])));
            const int t = t0 + tr;
            if (t < T) {
#pragma unroll
                for (int h2 = 0; h2 < 2; ++h2) {
                    const int j = h2 * 16 + q;
                    if (j < K) {
                        topk_idx[(size_t)t * K + j] = sel_i[h2];
                        topk_w[(size_t)t * K + j] = ex[h2] / sum;
                    }
                }
            }
        }
    }
}

}  // namespace

int32_t router_mfma_set_attributes() {
    const bool ok = hipFuncSetAttribute(reinterpret_cast<const void*>(&router_mfma_kernel<false>),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, 2 * R_STAGE) == hipSuccess &&
                    hipFuncSetAttribute(reinterpret_cast<const void*>(&router_mfma_kernel<true>),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, 2 * R_STAGE) == hipSuccess;
    return ok ? MOE_OK : MOE_ERR_LAUNCH_FAILED;
}

bool router_mfma_fuses_topk(const moe_config_t& c) { return c.E <= R_BE; }

size_t router_mfma_ws_bytes(const moe_config_t& c) {
    return align_up((size_t)3 * c.E * c.H * 2, 256);
}

// logits may be NULL when the selection is fused (router_mfma_fuses_topk); topk_idx / topk_w are
// written only then.
int32_t launch_router_logits_mfma(const moe_config_t& c, const void* x, const float* w_router,
                                  const float* bias, float* logits, int32_t* topk_idx, float* topk_w,
                                  void* ws, hipStream_t s) {
    if (c.T == 0) return MOE_OK;
    if ((uint64_t)c.T * c.H * 2 > 0xFFFFFFFFull || (uint64_t)3 * c.E * c.H * 2 > 0xFFFFFFFFull)
        return MOE_ERR_UNSUPPORTED;
    const DeviceState* dev_state = nullptr;
    const int32_t st = device_state(&dev_state);     // sets this kernel's LDS attribute once per device
    if (st != MOE_OK) return st;
    uint16_t* w3 = static_cast<uint16_t*>(ws);
    const size_t n = (size_t)c.E * c.H;
    KernelBracket kb(MOE_KERNEL_ROUTER_GEMM, s);
    const size_t split_blocks = (n + 255) / 256;
    split_router_weights_kernel<<<(unsigned)(split_blocks < 1024 ? split_blocks : 1024), 256, 0, s>>>(w_router, n, w3);
    dim3 grid((unsigned)ceil_div64(c.T, R_BM), (unsigned)ceil_div64(c.E, R_BE));
    if (router_mfma_fuses_topk(c))
        router_mfma_kernel<true><<<grid, R_THREADS, 2 * R_STAGE, s>>>(
            static_cast<const char*>(x), reinterpret_cast<const char*>(w3), c.T, c.E, c.H, bias, logits, c.K,
            topk_idx, topk_w);
    else
        router_mfma_kernel<false><<<grid, R_THREADS, 2 * R_STAGE, s>>>(
            static_cast<const char*>(x), reinterpret_cast<const char*>(w3), c.T, c.E, c.H, bias, logits, c.K,
            nullptr, nullptr);
    return launch_status();
}

}  // namespace moe
