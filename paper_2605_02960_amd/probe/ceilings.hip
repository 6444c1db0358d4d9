// Device ceilings probe (libmoeceilings.so): what this GPU sustains with nothing in the way.
// Not part of the MoE path and not linked into libmoeprefill.so; `bench.py --ceilings` calls it so
// that roofline fractions quoted against datasheet peaks can be read beside measured ones.
//   [0] matrix pipe, v_mfma_f32_16x16x32_bf16, operands in registers       TFLOP/s
//   [1] matrix pipe, v_mfma_f32_32x32x64_f8f6f4 with e4m3 operands         TFLOP/s
//   [2] streaming read of `bytes` of HBM, 16-byte nontemporal loads         TB/s
//   [3] streaming write of `bytes` of HBM, 16-byte nontemporal stores       TB/s
// moe_probe_l2_paths: how fast one CU takes in L2-resident lines,
//   [0] straight into LDS (global_load_lds_dwordx4, the FFN kernels' loader)  TB/s over all CUs
//   [1] into registers (global_load_dwordx4)                                  TB/s over all CUs
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

// Every workgroup of an XCD (workgroup b runs on XCD b % 8) walks the same 2 MB region, each from
// its own offset: the lines miss the 32 KB vector cache of the CU and hit the XCD's L2, as the operand
// panels of the FFN kernels do.  A wave keeps 24 requests of 1 KB in flight.
constexpr int L2_REGION = 2 << 20;

__global__ __launch_bounds__(WG) void l2_to_lds_loop(const char* src, int iters, float* out) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const char* base = src + (size_t)(blockIdx.x & 7) * L2_REGION;
    uint32_t off = (uint32_t)(((blockIdx.x >> 3) * 65536 + wave * 8192 + lane * 16) & (L2_REGION - 1));
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds;
    const uint32_t dst0 = __builtin_amdgcn_readfirstlane(lds_base + wave * 8192);
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                         :
                         : "s"(dst0 + i * 1024), "v"(off + i * 1024), "s"(base)
                         : "memory", "m0");
        }
        asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
        off = (off + 65536) & (L2_REGION - 1);          // the next 64 KB stripe of the region
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    out[blockIdx.x * WG + tid] = reinterpret_cast<const float*>(lds)[tid];
}

__global__ __launch_bounds__(WG) void l2_to_reg_loop(const char* src, int iters, float* out) {
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const char* base = src + (size_t)(blockIdx.x & 7) * L2_REGION;
    uint32_t off = (uint32_t)(((blockIdx.x >> 3) * 65536 + wave * 8192 + lane * 16) & (L2_REGION - 1));
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (int it = 0; it < iters; ++it) {
        u32x4 v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = *reinterpret_cast<const u32x4*>(base + off + i * 1024);
#pragma unroll
        for (int i = 0; i < 8; ++i) acc ^= v[i];
        off = (off + 65536) & (L2_REGION - 1);
    }
    out[blockIdx.x * WG + tid] = __builtin_bit_cast(float, acc[0] ^ acc[1] ^ acc[2] ^ acc[3]);
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

// L2-resident operand delivery on the current device: result2[0] straight into LDS, result2[1] into
// registers, TB/s summed over all CUs (one workgroup of 8 waves per CU, 64 KB per workgroup and
// iteration), best of `reps`.  Returns 0 or the hipError_t that stopped it.
extern "C" int moe_probe_l2_paths(double* result2, int iters, int reps) {
    int rc = 0, n_cu = 0, dev = 0;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    char* src = nullptr;
    float* sink = nullptr;
    PROBE_CK(hipGetDevice(&dev));
    PROBE_CK(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev));
    PROBE_CK(hipEventCreate(&e0));
    PROBE_CK(hipEventCreate(&e1));
    PROBE_CK(hipMalloc(&src, (size_t)8 * L2_REGION + 65536));
    PROBE_CK(hipMalloc(&sink, (size_t)n_cu * WG * sizeof(float)));
    PROBE_CK(hipFuncSetAttribute(reinterpret_cast<const void*>(l2_to_lds_loop),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, 65536));
    fill<<<1024, 256>>>(reinterpret_cast<uint32_t*>(src), ((size_t)8 * L2_REGION + 65536) / 4);
    PROBE_CK(hipDeviceSynchronize());
    for (int which = 0; which < 2; ++which) {
        float best = 1e30f;
        for (int r = 0; r < reps + 1; ++r) {             // the first run warms the L2
            PROBE_CK(hipEventRecord(e0));
            if (which == 0) l2_to_lds_loop<<<n_cu, WG, 65536>>>(src, iters, sink);
            else l2_to_reg_loop<<<n_cu, WG>>>(src, iters, sink);
            PROBE_CK(hipGetLastError());
            PROBE_CK(hipEventRecord(e1));
            PROBE_CK(hipEventSynchronize(e1));
            float ms = 0.f;
            PROBE_CK(hipEventElapsedTime(&ms, e0, e1));
            if (r > 0 && ms < best) best = ms;
        }
        result2[which] = (double)n_cu * iters * 65536.0 / best / 1e9;
    }
done:
    if (src) (void)hipFree(src);
    if (sink) (void)hipFree(sink);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    return rc;
}
