// Router logits on the matrix cores for bf16 activations, exact to float32 accumulation.
// The float32 router weight is split into three bf16 parts, w = hi + mid + lo (each the bf16
// rounding of what the previous parts left; three 8-bit parts cover the 24-bit significand), so
// x*w = x*hi + x*mid + x*lo with every product exact in float32.  The three partial GEMMs run
// as one bf16 MFMA GEMM against 3*E weight rows and are added in the epilogue, smallest first.
// This is the router of Sec. 2.3 of the paper at MFMA rate instead of vector-ALU rate.
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

__global__ __launch_bounds__(R_THREADS) void router_mfma_kernel(const char* __restrict__ x,
                                                               const char* __restrict__ w3, int T,
                                                               int E, int H,
                                                               const float* __restrict__ bias,
                                                               float* __restrict__ logits) {
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
    if (e < E) {
        const float b = bias ? bias[e] : 0.f;
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int t = t0 + wm * 64 + mi * 32 + (v >> 2) * 8 + fh * 4 + (v & 3);
                if (t < T) logits[(size_t)t * E + e] = ((acc[2][mi][v] + acc[1][mi][v]) + acc[0][mi][v]) + b;
            }
    }
}

}  // namespace

int32_t router_mfma_set_attributes() {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(&router_mfma_kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize, 2 * R_STAGE) == hipSuccess
               ? MOE_OK
               : MOE_ERR_LAUNCH_FAILED;
}

size_t router_mfma_ws_bytes(const moe_config_t& c) {
    return align_up((size_t)3 * c.E * c.H * 2, 256);
}

int32_t launch_router_logits_mfma(const moe_config_t& c, const void* x, const float* w_router,
                                  const float* bias, float* logits, void* ws, hipStream_t s) {
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
    router_mfma_kernel<<<grid, R_THREADS, 2 * R_STAGE, s>>>(static_cast<const char*>(x),
                                                            reinterpret_cast<const char*>(w3), c.T, c.E,
                                                            c.H, bias, logits);
    return launch_status();
}

}  // namespace moe
