// Device ceilings probe (libmoeceilings.so): what this GPU sustains with nothing in the way.
// Not part of the MoE path and not linked into libmoeprefill.so; `bench.py --ceilings` calls it so
// that roofline fractions quoted against datasheet peaks can be read beside measured ones.
//   [0] matrix pipe, v_mfma_f32_16x16x32_bf16, operands in registers       TFLOP/s
//   [1] matrix pipe, v_mfma_f32_32x32x64_f8f6f4 with e4m3 operands         TFLOP/s
//   [2] streaming read of `bytes` of HBM, 16-byte nontemporal loads         TB/s
//   [3] streaming write of `bytes` of HBM, 16-byte nontemporal stores       TB/s
#include <hip/hip_runtime.h>
#include <cstdint>

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(8))) int i32x8;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

namespace {

constexpr int WG = 512;             // 8 waves, two per SIMD: the occupancy of the FFN kernels
constexpr int POOL = 4096;          // operand pool, 16-byte words

// 32 independent accumulator blocks per wave: the pipe never waits for a result
__global__ __launch_bounds__(WG) void mfma_bf16_loop(const u32x4* in, float* out, int iters) {
    const int tid = threadIdx.x;
    bf16x8 a[4], b[8];
    for (int i = 0; i < 4; ++i) a[i] = __builtin_bit_cast(bf16x8, in[(tid * 12 + i) & (POOL - 1)]);
    for (int i = 0; i < 8; ++i) b[i] = __builtin_bit_cast(bf16x8, in[(tid * 12 + 4 + i) & (POOL - 1)]);
    f32x4 acc[8][4];
    for (int i = 0; i < 8; ++i)
        for (int j = 0; j < 4; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it)
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[j], b[i], acc[i][j], 0, 0, 0);
    float s = 0.f;
    for (int i = 0; i < 8; ++i)
        for (int j = 0; j < 4; ++j) s += acc[i][j][0] + acc[i][j][3];
    out[blockIdx.x * WG + tid] = s;
}

__device__ inline i32x8 e4m3_operand(const u32x4* in, int at) {
    const u32x4 lo = in[at & (POOL - 1)], hi = in[(at + 1) & (POOL - 1)];
    constexpr uint32_t M = 0x77777777u;      // keeps every byte a finite e4m3 value
    return i32x8{(int)(lo[0] & M), (int)(lo[1] & M), (int)(lo[2] & M), (int)(lo[3] & M),
                 (int)(hi[0] & M), (int)(hi[1] & M), (int)(hi[2] & M), (int)(hi[3] & M)};
}

__global__ __launch_bounds__(WG) void mfma_fp8_loop(const u32x4* in, float* out, int iters) {
    const int tid = threadIdx.x;
    i32x8 a[2], b[4];
    for (int i = 0; i < 2; ++i) a[i] = e4m3_operand(in, tid * 12 + 2 * i);
    for (int i = 0; i < 4; ++i) b[i] = e4m3_operand(in, tid * 12 + 4 + 2 * i);
    f32x16 acc[4][2];
    for (int i = 0; i < 4; ++i)
        for (int j = 0; j < 2; ++j)
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    for (int it = 0; it < iters; ++it)
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[j], b[i], acc[i][j], 0, 0, 0, 0, 0, 0);
    float s = 0.f;
    for (int i = 0; i < 4; ++i)
        for (int j = 0; j < 2; ++j) s += acc[i][j][0] + acc[i][j][15];
    out[blockIdx.x * WG + tid] = s;
}

__global__ __launch_bounds__(256) void stream_read(const u32x4* in, size_t n, uint32_t* out) {
    uint32_t s = 0;
    for (size_t i = blockIdx.x * (size_t)256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
        const u32x4 v = __builtin_nontemporal_load(in + i);
        s += v[0] ^ v[1] ^ v[2] ^ v[3];
    }
    if (s == 0x12345678u) out[0] = s;        // keeps the loads; practically never taken
}

__global__ __launch_bounds__(256) void stream_write(u32x4* o, size_t n) {
    for (size_t i = blockIdx.x * (size_t)256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256)
        __builtin_nontemporal_store(u32x4{(uint32_t)i, 1u, 2u, 3u}, o + i);
}

// pairs of bf16 in [0.0078, 2) with pseudo-random mantissas (operand toggling matters for power)
__global__ void fill(uint32_t* p, size_t n) {
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
        uint32_t h = (uint32_t)i * 2654435761u;
        h ^= h >> 15;
        h *= 0x85ebca6bu;
        h ^= h >> 13;
        p[i] = (h & 0x3FFF3FFFu) | 0x3C003C00u;
    }
}

}  // namespace

#define PROBE_CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { rc = (int)e_; goto done; } } while (0)

// Runs the four probes on the current device (default stream), best of `reps` each; the streaming
// kernels run over `stream_bytes` (a multiple of 16) of device memory that the call allocates and
// frees.  Returns 0 or the hipError_t that stopped it.
extern "C" int moe_probe_ceilings(double* result4, unsigned long long stream_bytes, int mfma_iters, int reps) {
    int rc = 0, n_cu = 0, dev = 0;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    uint32_t* pool = nullptr;
    float* sink = nullptr;
    u32x4* big = nullptr;
    const size_t n16 = stream_bytes / 16;
    PROBE_CK(hipGetDevice(&dev));
    PROBE_CK(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev));
    PROBE_CK(hipEventCreate(&e0));
    PROBE_CK(hipEventCreate(&e1));
    PROBE_CK(hipMalloc(&pool, POOL * 16));
    PROBE_CK(hipMalloc(&sink, (size_t)n_cu * WG * sizeof(float)));
    PROBE_CK(hipMalloc(&big, n16 * 16));
    fill<<<16, 256>>>(pool, POOL * 4);
    fill<<<4096, 256>>>((uint32_t*)big, n16 * 4);
    PROBE_CK(hipDeviceSynchronize());
    for (int which = 0; which < 4; ++which) {
        float best = 1e30f;
        const int it = which == 0 ? mfma_iters : mfma_iters / 4;
        for (int r = 0; r < reps; ++r) {
            PROBE_CK(hipEventRecord(e0));
            if (which == 0) mfma_bf16_loop<<<n_cu, WG>>>((const u32x4*)pool, sink, it);
            else if (which == 1) mfma_fp8_loop<<<n_cu, WG>>>((const u32x4*)pool, sink, it);
            else if (which == 2) stream_read<<<n_cu * 16, 256>>>(big, n16, (uint32_t*)sink);
            else stream_write<<<n_cu * 16, 256>>>(big, n16);
            PROBE_CK(hipGetLastError());
            PROBE_CK(hipEventRecord(e1));
            PROBE_CK(hipEventSynchronize(e1));
            float ms = 0.f;
            PROBE_CK(hipEventElapsedTime(&ms, e0, e1));
            if (ms < best) best = ms;
        }
        const double waves = (double)n_cu * (WG / 64);
        if (which == 0) result4[0] = waves * it * 32 * (2.0 * 16 * 16 * 32) / best / 1e9;
        else if (which == 1) result4[1] = waves * it * 8 * (2.0 * 32 * 32 * 64) / best / 1e9;
        else result4[which] = (double)(n16 * 16) / best / 1e9;
    }
done:
    if (big) (void)hipFree(big);
    if (sink) (void)hipFree(sink);
    if (pool) (void)hipFree(pool);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    return rc;
}
