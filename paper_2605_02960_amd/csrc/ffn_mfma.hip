// Grouped SwiGLU expert FFN on the gfx950 matrix cores (bf16 x bf16 -> f32 MFMA): the ragged
// per-expert GEMMs of Sec. 4.2 of the paper, run with every expert of the layer resident
// (Sec. 6.2).  Two launches over the device-built row-tile table:
//   gate/up : act[p, i]  = SiLU(x_p . Wg_e[i,:]) * (x_p . Wu_e[i,:])   rounded once to bf16
//   down    : y[p, h]    = act[p,:] . Wd_e[h,:]                          float32
// Rows of x are gathered through perm while the token tile is loaded (no permuted copy of x).
//
// Tiling.  Workgroup = 512 threads = 8 waves (4 along rows x 2 along columns), tile 256 rows x
// 256 weight rows x 64 (K).  For gate/up the 256 weight rows are 128 rows of Wg and the same
// 128 rows of Wu, so that a lane holds g and u of one output element side by side.  Each wave
// owns 64 rows x 128 weight rows = 2 x 4 MFMA 32x32x16 blocks (128 accumulator registers).
// The weight fragment is the MFMA "A" operand and the token fragment the "B" operand, so a lane
// ends up with 4 consecutive output columns of one row and stores them as one vector.
//
// LDS.  A tile is [256 rows][64 bf16] = 128 bytes per row in 8 chunks of 16 bytes; chunk c of
// row r sits at position c ^ ((r >> 1) & 7), which makes both the 16-byte stores of the loader
// and the 16-byte fragment reads of the MFMA operands free of bank conflicts.  Two stages
// (2 x 64 KB) are double-buffered with one barrier per K step.
#include "common.h"

namespace moe {

namespace {

constexpr int BM = 256;        // rows per tile
constexpr int BNW = 256;       // weight rows per tile
constexpr int BK = 64;         // bf16 per K step
constexpr int ROW_BYTES = BK * 2;
constexpr int TILE_BYTES = 256 * ROW_BYTES;         // 32 KB
constexpr int STAGE_BYTES = 2 * TILE_BYTES;         // tokens + weights
constexpr int THREADS = 512;

enum { MODE_GATE_UP = 0, MODE_DOWN = 1 };

struct MfmaArgs {
    const char* A;          // token-side operand: x [T,H] (gathered) or act [P,I], bf16
    uint32_t lda_bytes;
    const int32_t* perm;    // gate/up: sorted row -> flat id; NULL for down
    int32_t kdiv;
    const char* B0;         // Wg (gate/up) or Wd (down): [E][N][Kd] bf16
    const char* B1;         // Wu (gate/up)
    int32_t N;              // output columns (I or H)
    int32_t Kd;             // contraction length (H or I)
    const int32_t* table;
    const int32_t* offsets;
    char* C;                // act [P,I] bf16 or y [P,H] f32
    int32_t nct;            // column tiles
};

__device__ __forceinline__ float silu_mul(float g, float u) {
    return g * __builtin_amdgcn_rcpf(1.f + __expf(-g)) * u;
}

template <int MODE>
__global__ __launch_bounds__(THREADS) void ffn_mfma_kernel(MfmaArgs a) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    constexpr int NCOLS = (MODE == MODE_GATE_UP) ? 128 : 256;   // output columns per tile

    // XCD-aware tile assignment: workgroups are dealt round-robin to the 8 XCDs, so workgroup b
    // runs on XCD b % 8; give every XCD one contiguous range of tiles (column tile fastest), so
    // that the tiles resident on one XCD at a time share token rows and weight panels in its L2.
    const int n_rt = a.table[0];
    const int total = n_rt * a.nct;
    const int per_xcd = (total + 7) >> 3;
    const int slot = blockIdx.x >> 3;
    if (slot >= per_xcd) return;
    const int L = (blockIdx.x & 7) * per_xcd + slot;
    if (L >= total) return;
    const int rt = L / a.nct, ct = L - rt * a.nct;
    const int e = a.table[1 + 2 * rt];
    const int row0 = a.table[2 + 2 * rt];
    const int row_end = min(a.offsets[e + 1], row0 + BM);
    const int n0 = ct * NCOLS;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave & 3, wn = wave >> 2;

    // ---- loader: thread handles chunk lc of rows lr + 64*i, i = 0..3, of both tiles
    const int lr = tid >> 3, lc = tid & 7;
    const uint32_t st_off = lr * ROW_BYTES + ((lc ^ ((lr >> 1) & 7)) << 4);
    uint32_t a_off[4], b_off[4];
    const char* b0e = a.B0 + (size_t)e * a.N * a.Kd * 2;
    const char* b1e = (MODE == MODE_GATE_UP) ? a.B1 + (size_t)e * a.N * a.Kd * 2 : b0e;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int r = row0 + lr + 64 * i;
        r = min(r, row_end - 1);
        const uint32_t src = a.perm ? (uint32_t)(a.perm[r] / a.kdiv) : (uint32_t)r;
        a_off[i] = src * a.lda_bytes + lc * 16;
        int wr = (MODE == MODE_GATE_UP) ? n0 + lr + 64 * (i & 1) : n0 + lr + 64 * i;
        wr = min(wr, a.N - 1);
        b_off[i] = (uint32_t)wr * (uint32_t)(a.Kd * 2) + lc * 16;
    }

    // ---- fragment read offsets
    const int fr = lane & 31, fh = lane >> 5;
    const int sw = (fr >> 1) & 7;
    uint32_t frag_off[4];   // per kk: byte offset inside a row
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) frag_off[kk] = (uint32_t)(((kk * 2 + fh) ^ sw) << 4);
    const uint32_t xa_row = (wm * 64 + fr) * ROW_BYTES;                    // + mi*32 rows
    uint32_t wb_row[4];
#pragma unroll
    for (int nj = 0; nj < 4; ++nj) {
        int r;
        if (MODE == MODE_GATE_UP) r = (nj >> 1) * 128 + wn * 64 + (nj & 1) * 32 + fr;
        else r = wn * 128 + nj * 32 + fr;
        wb_row[nj] = TILE_BYTES + r * ROW_BYTES;
    }

    f32x16 acc[4][2];
#pragma unroll
    for (int nj = 0; nj < 4; ++nj)
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[nj][mi][v] = 0.f;

    // Two register sets of staged global loads: the tile for K step kt+2 is requested while step
    // kt is being multiplied, so every request has two K steps of MFMA work to hide its latency.
    u32x4 ra0[4], rb0[4], ra1[4], rb1[4];
#define MOE_GLOAD(SET_, KT_)                                                              \
    {                                                                                     \
        const uint32_t kb = (uint32_t)min((KT_), KT - 1) * ROW_BYTES;                     \
        _Pragma("unroll") for (int i = 0; i < 4; ++i) {                                   \
            ra##SET_[i] = *reinterpret_cast<const u32x4*>(a.A + (a_off[i] + kb));         \
            rb##SET_[i] = *reinterpret_cast<const u32x4*>(((i < 2 || MODE == MODE_DOWN) ? b0e : b1e) + (b_off[i] + kb)); \
        }                                                                                 \
    }
#define MOE_LSTORE(SET_, STAGE_)                                                          \
    {                                                                                     \
        char* base = smem + (STAGE_) * STAGE_BYTES + st_off;                              \
        _Pragma("unroll") for (int i = 0; i < 4; ++i) {                                   \
            *reinterpret_cast<u32x4*>(base + i * 64 * ROW_BYTES) = ra##SET_[i];           \
            *reinterpret_cast<u32x4*>(base + TILE_BYTES + i * 64 * ROW_BYTES) = rb##SET_[i]; \
        }                                                                                 \
    }
#define MOE_COMPUTE(STAGE_)                                                               \
    {                                                                                     \
        const char* st = smem + (STAGE_) * STAGE_BYTES;                                   \
        _Pragma("unroll") for (int kk = 0; kk < 4; ++kk) {                                \
            bf16x8 xa[2], wb[4];                                                          \
            _Pragma("unroll") for (int mi = 0; mi < 2; ++mi) xa[mi] =                     \
                *reinterpret_cast<const bf16x8*>(st + xa_row + mi * 32 * ROW_BYTES + frag_off[kk]); \
            _Pragma("unroll") for (int nj = 0; nj < 4; ++nj) wb[nj] =                     \
                *reinterpret_cast<const bf16x8*>(st + wb_row[nj] + frag_off[kk]);         \
            _Pragma("unroll") for (int nj = 0; nj < 4; ++nj)                              \
                _Pragma("unroll") for (int mi = 0; mi < 2; ++mi) acc[nj][mi] =            \
                    __builtin_amdgcn_mfma_f32_32x32x16_bf16(wb[nj], xa[mi], acc[nj][mi], 0, 0, 0); \
        }                                                                                 \
    }

    const int KT = a.Kd / BK;
    MOE_GLOAD(0, 0);
    MOE_GLOAD(1, 1);
    MOE_LSTORE(0, 0);
    __syncthreads();
    int kt = 0;
    for (; kt + 1 < KT; kt += 2) {
        MOE_GLOAD(0, kt + 2);
        MOE_COMPUTE(0);
        MOE_LSTORE(1, 1);
        __syncthreads();
        MOE_GLOAD(1, kt + 3);
        MOE_COMPUTE(1);
        MOE_LSTORE(0, 0);
        __syncthreads();
    }
    if (kt < KT) MOE_COMPUTE(0);
#undef MOE_GLOAD
#undef MOE_LSTORE
#undef MOE_COMPUTE

    // ---- epilogue.  acc[nj][mi][v]: row = mi*32 + fr, column = (v/4)*8 + fh*4 + v%4 of the block
#pragma unroll
    for (int mi = 0; mi < 2; ++mi) {
        const int m = row0 + wm * 64 + mi * 32 + fr;
        if (m >= row_end) continue;
        if (MODE == MODE_GATE_UP) {
            uint16_t* crow = reinterpret_cast<uint16_t*>(a.C) + (size_t)m * a.N;
#pragma unroll
            for (int nj = 0; nj < 2; ++nj)
#pragma unroll
                for (int vg = 0; vg < 4; ++vg) {
                    const int n = n0 + wn * 64 + nj * 32 + vg * 8 + fh * 4;
                    if (n >= a.N) continue;
                    uint16_t h[4];
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        h[q] = f32_to_bf16_bits(silu_mul(acc[nj][mi][vg * 4 + q], acc[nj + 2][mi][vg * 4 + q]));
                    uint2 o;
                    o.x = (uint32_t)h[0] | ((uint32_t)h[1] << 16);
                    o.y = (uint32_t)h[2] | ((uint32_t)h[3] << 16);
                    *reinterpret_cast<uint2*>(crow + n) = o;
                }
        } else {
            float* crow = reinterpret_cast<float*>(a.C) + (size_t)m * a.N;
#pragma unroll
            for (int nj = 0; nj < 4; ++nj)
#pragma unroll
                for (int vg = 0; vg < 4; ++vg) {
                    const int n = n0 + wn * 128 + nj * 32 + vg * 8 + fh * 4;
                    if (n >= a.N) continue;
                    float4 o = make_float4(acc[nj][mi][vg * 4 + 0], acc[nj][mi][vg * 4 + 1],
                                           acc[nj][mi][vg * 4 + 2], acc[nj][mi][vg * 4 + 3]);
                    *reinterpret_cast<float4*>(crow + n) = o;
                }
        }
    }
}

}  // namespace

size_t ffn_mfma_ws_bytes(const moe_config_t& c) {
    const size_t P = (size_t)c.T * c.K;
    return tile_table_bytes(c, BM) + align_up(P * c.I * 2, 256);
}

int32_t launch_ffn_mfma(const moe_config_t& c, const void* x, const int32_t* perm,
                        const int32_t* offsets, const void* wg, const void* wu, const void* wd,
                        const float* s_gate, const float* s_up, const float* s_down, void* act_tap,
                        uint8_t* act_q_tap, float* act_scale_tap, float* y_perm, void* ws,
                        hipStream_t s) {
    (void)s_gate; (void)s_up; (void)s_down; (void)act_q_tap; (void)act_scale_tap;
    if (c.w_dtype != MOE_DTYPE_BF16) return MOE_ERR_UNSUPPORTED;
    const int64_t P = (int64_t)c.T * c.K;
    if (P == 0) return MOE_OK;
    // 32-bit byte offsets are used on the load side
    if ((uint64_t)c.T * c.H * 2 > 0xFFFFFFFFull || (uint64_t)P * c.I * 2 > 0xFFFFFFFFull ||
        (uint64_t)c.I * c.H * 2 > 0xFFFFFFFFull)
        return MOE_ERR_UNSUPPORTED;

    int32_t* table = static_cast<int32_t*>(ws);
    char* act = act_tap ? static_cast<char*>(act_tap)
                        : static_cast<char*>(ws) + tile_table_bytes(c, BM);
    int32_t st = launch_build_tile_table(c, offsets, BM, table, s);
    if (st != MOE_OK) return st;

    static bool attr_done = false;
    if (!attr_done) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(&ffn_mfma_kernel<MODE_GATE_UP>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 2 * STAGE_BYTES) != hipSuccess ||
            hipFuncSetAttribute(reinterpret_cast<const void*>(&ffn_mfma_kernel<MODE_DOWN>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 2 * STAGE_BYTES) != hipSuccess)
            return MOE_ERR_LAUNCH_FAILED;
        attr_done = true;
    }
    const int64_t mrt = max_row_tiles(c, BM);

    MfmaArgs g{};
    g.A = static_cast<const char*>(x);
    g.lda_bytes = (uint32_t)c.H * 2;
    g.perm = perm;
    g.kdiv = c.K;
    g.B0 = static_cast<const char*>(wg);
    g.B1 = static_cast<const char*>(wu);
    g.N = c.I;
    g.Kd = c.H;
    g.table = table;
    g.offsets = offsets;
    g.C = act;
    g.nct = (int32_t)ceil_div64(c.I, 128);
    {
        const int64_t grid = ceil_div64(mrt * g.nct, 8) * 8;
        KernelBracket kb(MOE_KERNEL_GATE_UP, s);
        ffn_mfma_kernel<MODE_GATE_UP><<<(unsigned)grid, THREADS, 2 * STAGE_BYTES, s>>>(g);
    }
    MfmaArgs d{};
    d.A = act;
    d.lda_bytes = (uint32_t)c.I * 2;
    d.perm = nullptr;
    d.kdiv = 1;
    d.B0 = static_cast<const char*>(wd);
    d.B1 = nullptr;
    d.N = c.H;
    d.Kd = c.I;
    d.table = table;
    d.offsets = offsets;
    d.C = reinterpret_cast<char*>(y_perm);
    d.nct = (int32_t)ceil_div64(c.H, 256);
    {
        const int64_t grid = ceil_div64(mrt * d.nct, 8) * 8;
        KernelBracket kb(MOE_KERNEL_DOWN, s);
        ffn_mfma_kernel<MODE_DOWN><<<(unsigned)grid, THREADS, 2 * STAGE_BYTES, s>>>(d);
    }
    return launch_status();
}

}  // namespace moe
