// Float32 vector-ALU tile GEMM, C[m,n] = sum_k A[row(m),k] * B[n,k] ("NT": both operands
// K-contiguous), used where the block computes in float32: the router logits and the
// all-float32 configuration of the expert FFN.  Any M, N, K (bounds are checked); the k loop
// runs in ascending order inside one thread, so results do not depend on the launch shape.
#pragma once

#include "common.h"

namespace moe {

struct F32GemmArgs {
    const void* A;          // rows of K elements (float or bf16 bits), leading dimension lda
    int64_t lda;
    const int32_t* a_row_index;  // optional: source row of sorted row p is a_row_index[p] / a_row_div
    int32_t a_row_div;
    const float* B;         // [groups][N][K]
    const float* B2;        // second B for the SwiGLU epilogue (gate = B, up = B2)
    int32_t N, K;
    const int32_t* tile_table;  // NULL: one group of rows [0, M); else per-expert row tiles
    const int32_t* offsets;     // [E+1] when tile_table is given
    int32_t M;
    const float* bias;      // optional [N]
    float* C;               // [rows][ldc]
    int64_t ldc;
};

enum { EPI_STORE = 0, EPI_SWIGLU = 1 };

template <typename TA>
__device__ __forceinline__ float load_a(const TA* p);
template <>
__device__ __forceinline__ float load_a<float>(const float* p) { return *p; }
template <>
__device__ __forceinline__ float load_a<uint16_t>(const uint16_t* p) { return bf16_bits_to_f32(*p); }

// 256 threads; block tile BM x BN; each thread owns TM x TN outputs split in 4-wide pieces
// (row r of the micro-tile is block row (r/4)*(BM/(TM/4)) + ty*4 + r%4, same for columns).
template <typename TA, int BM, int BN, int TM, int TN, int EPI>
__global__ __launch_bounds__(256) void f32_gemm_nt_kernel(F32GemmArgs a) {
    constexpr int BK = 16;
    constexpr int NTX = BN / TN, NTY = BM / TM;
    static_assert(NTX * NTY == 256, "tile shape");
    constexpr int RM = TM / 4, RN = TN / 4;
    constexpr bool DUAL = (EPI == EPI_SWIGLU);
    __shared__ float As[BK][BM + 4];
    __shared__ float Bs[BK][BN + 4];
    __shared__ float Bs2[DUAL ? BK : 1][DUAL ? BN + 4 : 1];

    int row0, row_end, group;
    if (a.tile_table) {
        const int n_tiles = a.tile_table[0];
        if ((int)blockIdx.x >= n_tiles) return;
        group = a.tile_table[1 + 2 * blockIdx.x];
        row0 = a.tile_table[2 + 2 * blockIdx.x];
        row_end = a.offsets[group + 1];
    } else {
        group = 0;
        row0 = blockIdx.x * BM;
        row_end = a.M;
        if (row0 >= row_end) return;
    }
    const int col0 = blockIdx.y * BN;
    const float* Bg = a.B + (size_t)group * a.N * a.K;
    const float* B2g = DUAL ? a.B2 + (size_t)group * a.N * a.K : nullptr;
    const TA* Ap = static_cast<const TA*>(a.A);

    const int tid = threadIdx.x;
    const int tx = tid % NTX, ty = tid / NTX;

    float acc[TM][TN];
    float acc2[DUAL ? TM : 1][DUAL ? TN : 1];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            acc[i][j] = 0.f;
            if constexpr (DUAL) acc2[i][j] = 0.f;
        }

    // loader mapping: each thread fetches elements (r = e / BK, k = e % BK), e = tid + 256*i
    constexpr int A_PER = BM * BK / 256, B_PER = BN * BK / 256;
    int64_t a_src[A_PER];
#pragma unroll
    for (int i = 0; i < A_PER; ++i) {
        const int r = (tid + 256 * i) / BK;
        const int row = row0 + r;
        if (row < row_end) {
            const int64_t src = a.a_row_index ? (int64_t)(a.a_row_index[row] / a.a_row_div) : (int64_t)row;
            a_src[i] = src * a.lda;
        } else {
            a_src[i] = -1;
        }
    }

    for (int k0 = 0; k0 < a.K; k0 += BK) {
#pragma unroll
        for (int i = 0; i < A_PER; ++i) {
            const int e = tid + 256 * i;
            const int r = e / BK, k = e % BK;
            float v = 0.f;
            if (a_src[i] >= 0 && k0 + k < a.K) v = load_a<TA>(Ap + a_src[i] + k0 + k);
            As[k][r] = v;
        }
#pragma unroll
        for (int i = 0; i < B_PER; ++i) {
            const int e = tid + 256 * i;
            const int r = e / BK, k = e % BK;
            const bool ok = (col0 + r < a.N) && (k0 + k < a.K);
            Bs[k][r] = ok ? Bg[(size_t)(col0 + r) * a.K + k0 + k] : 0.f;
            if constexpr (DUAL) Bs2[k][r] = ok ? B2g[(size_t)(col0 + r) * a.K + k0 + k] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < BK; ++k) {
            float av[TM], bv[TN], bv2[DUAL ? TN : 1];
#pragma unroll
            for (int i = 0; i < RM; ++i)
#pragma unroll
                for (int q = 0; q < 4; ++q) av[i * 4 + q] = As[k][i * (BM / RM) + ty * 4 + q];
#pragma unroll
            for (int j = 0; j < RN; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    bv[j * 4 + q] = Bs[k][j * (BN / RN) + tx * 4 + q];
                    if constexpr (DUAL) bv2[j * 4 + q] = Bs2[k][j * (BN / RN) + tx * 4 + q];
                }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
                    if constexpr (DUAL) acc2[i][j] = fmaf(av[i], bv2[j], acc2[i][j]);
                }
        }
        __syncthreads();
    }

#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int row = row0 + (i / 4) * (BM / RM) + ty * 4 + i % 4;
        if (row >= row_end) continue;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = col0 + (j / 4) * (BN / RN) + tx * 4 + j % 4;
            if (col >= a.N) continue;
            float v;
            if constexpr (DUAL) {
                const float g = acc[i][j];
                v = g / (1.f + expf(-g)) * acc2[i][j];
            } else {
                v = acc[i][j];
                if (a.bias) v += a.bias[col];
            }
            a.C[(size_t)row * a.ldc + col] = v;
        }
    }
}

}  // namespace moe
