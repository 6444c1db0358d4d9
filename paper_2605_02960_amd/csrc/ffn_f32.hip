// All-float32 grouped SwiGLU expert FFN (the configuration in which every tensor is float32).
// Two launches over the per-expert row tiles: gate/up projection with the SiLU(gate)*up epilogue,
// then the down projection.  Rows of x are gathered through perm while the A tile is loaded.
#include "f32_gemm.h"

namespace moe {

constexpr int F32_BM = 64;

size_t ffn_f32_ws_bytes(const moe_config_t& c) {
    const size_t P = (size_t)c.T * c.K;
    return tile_table_bytes(c, F32_BM) + align_up(P * c.I * sizeof(float), 256);
}

int32_t launch_ffn_f32(const moe_config_t& c, const float* x, const int32_t* perm,
                       const int32_t* offsets, const float* wg, const float* wu, const float* wd,
                       float* act_tap, float* y_perm, void* ws, hipStream_t s) {
    const int64_t P = (int64_t)c.T * c.K;
    if (P == 0) return MOE_OK;
    int32_t* table = static_cast<int32_t*>(ws);
    float* act = act_tap ? act_tap
                         : reinterpret_cast<float*>(static_cast<char*>(ws) + tile_table_bytes(c, F32_BM));
    int32_t st = launch_build_tile_table(c, offsets, F32_BM, table, nullptr, s);
    if (st != MOE_OK) return st;
    const unsigned tiles = (unsigned)max_row_tiles(c, F32_BM);

    F32GemmArgs a{};
    a.A = x;
    a.lda = c.H;
    a.a_row_index = perm;
    a.a_row_div = c.K;
    a.B = wg;
    a.B2 = wu;
    a.N = c.I;
    a.K = c.H;
    a.tile_table = table;
    a.offsets = offsets;
    a.M = (int32_t)P;
    a.bias = nullptr;
    a.C = act;
    a.ldc = c.I;
    {
        KernelBracket kb(MOE_KERNEL_GATE_UP, s);
        f32_gemm_nt_kernel<float, 64, 64, 4, 4, EPI_SWIGLU>
            <<<dim3(tiles, (unsigned)ceil_div64(c.I, 64)), 256, 0, s>>>(a);
    }

    F32GemmArgs b{};
    b.A = act;
    b.lda = c.I;
    b.a_row_index = nullptr;
    b.a_row_div = 1;
    b.B = wd;
    b.B2 = nullptr;
    b.N = c.H;
    b.K = c.I;
    b.tile_table = table;
    b.offsets = offsets;
    b.M = (int32_t)P;
    b.bias = nullptr;
    b.C = y_perm;
    b.ldc = c.H;
    {
        KernelBracket kb(MOE_KERNEL_DOWN, s);
        f32_gemm_nt_kernel<float, 64, 64, 4, 4, EPI_STORE>
            <<<dim3(tiles, (unsigned)ceil_div64(c.H, 64)), 256, 0, s>>>(b);
    }
    return launch_status();
}

}  // namespace moe
