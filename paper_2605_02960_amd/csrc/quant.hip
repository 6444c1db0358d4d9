// Per-row dynamic e4m3 quantiser (fp8 storage of expert weights, one scale per output channel,
// and of activations, one scale per token row; the FP8 precision of Sec. 8.1 of the paper).
// All arithmetic is IEEE binary32: scale = amax/448 (1 for an all-zero row), q = e4m3(v/scale)
// with round-to-nearest-even through the hardware converter (OCP e4m3 on gfx950).
#include "common.h"

namespace moe {

__device__ __forceinline__ uint32_t pack4_e4m3(float a, float b, float c, float d) {
    // clamp first: the quotient amax/scale may exceed 448 by an ulp
    a = fminf(fmaxf(a, -448.f), 448.f);
    b = fminf(fmaxf(b, -448.f), 448.f);
    c = fminf(fmaxf(c, -448.f), 448.f);
    d = fminf(fmaxf(d, -448.f), 448.f);
    int r = __builtin_amdgcn_cvt_pk_fp8_f32(a, b, 0, false);
    r = __builtin_amdgcn_cvt_pk_fp8_f32(c, d, r, true);
    return (uint32_t)r;
}

__global__ __launch_bounds__(256) void quantize_rows_kernel(const uint4* __restrict__ src,
                                                           int vec_per_row,
                                                           uint2* __restrict__ q,
                                                           float* __restrict__ scale) {
    __shared__ float red[4];
    const int64_t row = blockIdx.x;
    const uint4* s = src + row * vec_per_row;
    float amax = 0.f;
    for (int i = threadIdx.x; i < vec_per_row; i += blockDim.x) {
        const uint4 v = s[i];
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            amax = fmaxf(amax, fabsf(__uint_as_float(w[k] << 16)));
            amax = fmaxf(amax, fabsf(__uint_as_float(w[k] & 0xFFFF0000u)));
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off, WAVE));
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = amax;
    __syncthreads();
    amax = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    const float sc = (amax == 0.f) ? 1.f : amax / 448.f;
    if (threadIdx.x == 0) scale[row] = sc;
    uint2* d = q + row * vec_per_row;
    for (int i = threadIdx.x; i < vec_per_row; i += blockDim.x) {
        const uint4 v = s[i];
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
        float f[8];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            f[2 * k] = __uint_as_float(w[k] << 16) / sc;
            f[2 * k + 1] = __uint_as_float(w[k] & 0xFFFF0000u) / sc;
        }
        uint2 o;
        o.x = pack4_e4m3(f[0], f[1], f[2], f[3]);
        o.y = pack4_e4m3(f[4], f[5], f[6], f[7]);
        d[i] = o;
    }
}

int32_t launch_quantize_rows(const void* src_bf16, int64_t rows, int32_t cols, uint8_t* q,
                             float* scale, hipStream_t s) {
    if (rows == 0) return MOE_OK;
    quantize_rows_kernel<<<(unsigned)rows, 256, 0, s>>>(static_cast<const uint4*>(src_bf16), cols / 8,
                                                        reinterpret_cast<uint2*>(q), scale);
    return launch_status();
}

}  // namespace moe
