// Grouped SwiGLU expert FFN on the gfx950 matrix cores (bf16 or fp8 operands, f32 accumulate):
// the ragged per-expert GEMMs of Sec. 4.2 of the paper, run with every expert of the layer
// resident (Sec. 6.2).  Two launches over the device-built tile tables:
//   gate/up : act[p, i]  = SiLU(x_p . Wg_e[i,:]) * (x_p . Wu_e[i,:])   rounded once to bf16
//   down    : y[p, h]    = act[p,:] . Wd_e[h,:]                          float32 accumulators, handed
//             on as 16-bit block floating point (16 columns per shared exponent) or as float32
// Rows of x are gathered through perm while the token tile is loaded (no permuted copy of x).
//
// Tiling.  Workgroup = 512 threads = 8 waves (4 along rows x 2 along columns; waves 2j and 2j+1
// share row block j), tile 256 rows x
// 256 weight rows x one K step of 128 bytes per row (64 bf16 or 128 fp8).  For gate/up the 256
// weight rows are 128 rows of Wg and the same 128 rows of Wu, so that a lane holds g and u of one
// output element side by side.  Each wave owns 64 rows x 128 weight rows = 2 x 4 MFMA blocks of
// 32 x 32 (v_mfma_f32_32x32x16_bf16, v_mfma_f32_32x32x64_f8f6f4) or 4 x 8 blocks of 16 x 16
// (v_mfma_f32_16x16x32_bf16); 128 accumulator registers either way.
// The token fragment is the MFMA "A" operand and the weight fragment the "B" operand; the
// wave's weight rows are interleaved over its output columns so that a lane ends up with 2 or 4
// adjacent output columns and the lanes of one block row store whole 128-byte lines.
//
// fp8 (e4m3 codes, float scales per token row and per output channel): the accumulators hold sums
// of code products and the scales are applied in the epilogue (the row scales travel in
// registers, lane j of a wave holding the scale of the wave's row j).
//
// LDS.  A tile is [256 rows][128 bytes] in 8 chunks of 16 bytes per row; chunk c of
// row r sits at position c ^ ((r >> 1) & 7), which makes the 16-byte fragment reads of the MFMA
// operands free of bank conflicts.  Five slots of 32 KB, all of the CU's 160 KB: three for token
// tiles and two for weight tiles; one barrier per K step.
//
// Loader.  The operand tiles go from global memory straight into LDS (global_load_lds_dwordx4:
// 16 bytes per lane, full 128-byte lines per row, no staging registers and no LDS store
// instructions).  The instruction writes lane l at LDS base + 16 l, so the swizzle is applied on
// the global side (the lane that fills position c' of row r fetches chunk c' ^ ((r >> 1) & 7)).
// Rows of x are gathered through the lane offsets.  The top of K step k requests the weight tile
// of step k+1 and then the token tile of step k+2; the step's end waits for all but the four
// youngest requests (requests are served in issue order), so the token tiles, whose rows are
// gathered from all over x, have two steps to arrive (+2.4 % for bf16, +1.3 % for fp8).
//
// MFMA blocks.  bf16 kernels whose tiles have 16 or more K steps multiply 16 x 16 x 32 blocks
// (v_mfma_f32_16x16x32_bf16: half the accumulator writes per flop of the 32 x 32 x 16 form, which
// shows on a part that is limited by power: +3.5 % at 64 K steps per tile, -2 % at 12).
//
// Issue order.  bf16: the fragments of the next K slice (32 x 32 blocks) or of the next group of
// 16 MFMAs (16 x 16 blocks) are read into a second set of fragment registers before the MFMAs of
// the current one are issued, and scheduling group barriers spread those reads between the
// MFMAs, so the matrix pipe never waits for LDS.  fp8 keeps one set.
//
// Pipeline.  The kernel is persistent (one workgroup per CU): the loads that a tile's last K
// steps issue are the first K steps of the workgroup's NEXT tile, so consecutive tiles chain
// without draining the pipeline and the epilogue's stores overlap the next tile's loads.  A
// tile's 16-byte launch-order record is fetched two tiles ahead and moved to scalar registers
// behind a K step's wait, its perm entries one tile ahead: nothing at a tile's start waits for
// memory.
//
// Launch order.  Workgroups are dealt round-robin to the 8 XCDs (workgroup b runs on XCD b % 8).
// The launch-order list (see tiles.hip) walks an expert's output in blocks of 8 x 4 tiles; it is
// dealt to the XCDs in chunks of 32 entries, so the 32 tiles in flight on an XCD share token rows
// and weight rows in that XCD's L2, and the 8 XCDs are on neighbouring blocks of the same expert.
#include <type_traits>

#include "common.h"

namespace moe {

namespace {

constexpr int BM = 256;        // rows per tile
constexpr int BK = 64;         // bf16 per K step
constexpr int ROW_BYTES = BK * 2;
constexpr int TILE_BYTES = 256 * ROW_BYTES;         // 32 KB
constexpr int THREADS = 512;
constexpr int LDS_BYTES = 5 * TILE_BYTES;           // three token-tile slots and two weight-tile slots: all of the CU's 160 KB
#ifndef MOE_GROUP_ROWS
#define MOE_GROUP_ROWS 8
#define MOE_GROUP_COLS 4
#endif
constexpr int GROUP_ROWS = MOE_GROUP_ROWS, GROUP_COLS = MOE_GROUP_COLS;   // tile block one XCD works on at a time

enum { MODE_GATE_UP = 0, MODE_DOWN = 1 };
// How the down kernel hands y to the combine.  A y row is cut into blocks of 16 columns; a block
// is stored as 16 int16 codes and one shared power-of-two scale (its exponent, one byte):
// value = 2^(k - 141) * code.  That halves the bytes the two kernels move through HBM.
enum { Y_EXACT_F32 = 0,      // float32 accumulators as they are
       Y_BLOCK16_AS_F32 = 1, // the block-scaled values, written out as float32 (exactly representable)
       Y_BLOCK16 = 2 };      // codes and exponents
constexpr int Y_BLOCK = 16;

struct MfmaArgs {
    const char* A;          // token-side operand: x [T,H] (gathered) or act [P,I], bf16
    uint32_t lda_bytes;
    const int32_t* perm;    // gate/up: sorted row -> flat id; NULL for down
    int32_t kdiv;
    const char* B0;         // Wg (gate/up) or Wd (down): [E][N][Kd] bf16
    const char* B1;         // Wu (gate/up)
    int32_t N;              // output columns (I or H)
    uint32_t ldb_bytes;     // bytes of one weight row (contraction length x element size)
    int32_t KT;             // K steps of 128 bytes per row (64 bf16 or 128 fp8), even
    const float* sA;        // fp8: scale of sorted row p (of its x row for gate/up, of its act row for down)
    const float* sB0;       // fp8: per-output-channel scales [E][N] of B0
    const float* sB1;       // fp8: same for B1
    const int32_t* table;   // row tiles: [0] = count, then (expert, first row) pairs
    const int4* order;      // launch slot -> (expert, first row, end row, column tile)
    char* C;                // act [P,I] bf16, or y [P,H]: float32 (y_mode 0, 1) or int16 codes (y_mode 2)
    uint8_t* Cs;            // y_mode 2: block exponents [P][N/16]
    int32_t y_mode;         // down only, see Y_* above
    int32_t nct;            // column tiles
};

__device__ __forceinline__ float silu_mul(float g, float u) {
    return g * __builtin_amdgcn_rcpf(1.f + __expf(-g)) * u;
}

// One output tile as seen by one thread's loader and epilogue.
struct TileCtx {
    int row0, row_end, n0;
    uint32_t a_off[4], b_off[4];   // byte offsets of the thread's 4 token rows / 4 weight rows
    const char* b0e;               // expert's Wg / Wd
    const char* b1e;               // expert's Wu
    int e;
};

// How the two operand tiles of a K step get into LDS: global_load_lds_dwordx4 writes 16 bytes per
// lane straight into LDS, lane l of an instruction at LDS position base + 16*l; one instruction
// covers 8 tile rows (8 chunks of 16 bytes each), wave w issues the 4 instructions of rows
// 32w .. 32w+31 of both tiles.  The row swizzle is applied on the global side: the lane that fills
// position c' of row r fetches chunk c' ^ ((r >> 1) & 7).
__device__ __forceinline__ void loader_pos(int tid, int i, int& row, int& chunk) {
    row = (tid >> 6) * 32 + i * 8 + ((tid & 63) >> 3);
    chunk = (tid & 7) ^ ((row >> 1) & 7);
}
// The thread index as a value that the optimiser cannot trace back: the per-tile set-up below
// derives its lane constants from it anew (a few instructions per tile) instead of holding them
// in registers, or in spill slots, across the K loop.
__device__ __forceinline__ int opaque_tid() {
    int x = threadIdx.x;
    asm volatile("" : "+v"(x));
    return x;
}

// A tile's 16-byte launch-order record travels on the scalar path, straight into four scalar
// registers: it occupies no vector registers and no vector-memory wait ever stands for it.  The
// load and the wait for it are one statement, so that the compiler never sees (and never copies)
// registers whose load is still in flight; the wave issues it behind a K step's barrier, where
// the MFMAs it has queued cover the few hundred cycles.  (Scalar loads share the LDS counter;
// the wait also covers the wave's LDS reads in flight.)
typedef __attribute__((ext_vector_type(4))) int i32x4;
__device__ __forceinline__ int4 load_rec(const int4* p) {
    i32x4 r;
    asm volatile("s_load_dwordx4 %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)" : "=s"(r) : "s"(p) : "memory");
    return make_int4(r[0], r[1], r[2], r[3]);
}
// A tile's context from its launch-order record (expert, first row, end row, column tile).  For
// gate/up this issues the loads of the tile's perm entries; their values (and for down the row
// numbers) stay in a_off as they are until fill_a_off turns them into byte offsets, so that no
// wait for them stands between two tiles.
template <int MODE>
__device__ __forceinline__ void ctx_from_rec(TileCtx& t, const MfmaArgs& a, const int4 rec, int) {
    constexpr int NCOLS = (MODE == MODE_GATE_UP) ? 128 : 256;
    const int tid = opaque_tid();
    const int e = rec.x;
    t.e = e;
    t.row0 = rec.y;
    t.row_end = rec.z;
    t.n0 = rec.w * NCOLS;
    const size_t wbytes = (size_t)a.N * a.ldb_bytes;
    t.b0e = a.B0 + (size_t)e * wbytes;
    t.b1e = (MODE == MODE_GATE_UP) ? a.B1 + (size_t)e * wbytes : t.b0e;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int lrow, lchunk;
        loader_pos(tid, i, lrow, lchunk);
        const int r = min(t.row0 + lrow, t.row_end - 1);       // rows past the group's end re-read its last row
        t.a_off[i] = (MODE == MODE_GATE_UP) ? (uint32_t)a.perm[r] : (uint32_t)(r - t.row0);
    }
}
// gate/up gathers rows of x (offsets from x itself, T*H*esz < 4 GiB); down reads the tile's own
// contiguous rows of act, so its offsets are taken from the tile's first row and stay small
// however many routed rows there are.
template <int MODE>
__device__ __forceinline__ void fill_a_off(TileCtx& t, const MfmaArgs& a, int) {
    const int tid = opaque_tid();
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int lrow, lchunk;
        loader_pos(tid, i, lrow, lchunk);
        const uint32_t src = (MODE == MODE_GATE_UP) ? t.a_off[i] / (uint32_t)a.kdiv : t.a_off[i];
        t.a_off[i] = src * a.lda_bytes + lchunk * 16;
    }
}
// MFMA block edge of the bf16 kernels: 32 (v_mfma_f32_32x32x16_bf16) or 16
// (v_mfma_f32_16x16x32_bf16, half the accumulator writes per flop); a template parameter of the
// kernel, chosen at launch from the number of K steps per tile.  fp8 uses
// v_mfma_f32_32x32x64_f8f6f4.
template <bool FP8, int BLK>
struct Blk {
    static constexpr int E = FP8 ? 32 : BLK;     // rows / columns of one MFMA block
    static constexpr int NM = 64 / E;            // blocks along the wave's 64 token rows
    static constexpr int NN = 128 / E;           // blocks along the wave's 128 weight rows
    static constexpr int VLEN = E * E / 64;      // accumulator registers of one block
};

// Weight row held by LDS row R of the weight tile.  A wave's MFMA blocks are interleaved over
// its output columns (block nj, lane row j <-> column NB*j + nj, NB blocks), so that after the
// MFMA one lane holds NB adjacent output columns of a row and a store instruction writes whole
// 128-byte lines (gate/up: NB = 64 / BE columns of act per lane, the gate and the up block of a
// column side by side in the lane; down: NB = 128 / BE).
template <int MODE, int BE>
__device__ __forceinline__ int weight_col_of_lds_row(int R) {
    if (MODE == MODE_GATE_UP) {          // rows 0..127 gate, 128..255 up; 64 columns per wave
        const int w = R & 63;
        return (R & 64) + (64 / BE) * (w % BE) + w / BE;
    }
    const int w = R & 127;               // 128 columns per wave: block nj = w / BE, lane row w % BE
    return (R & 128) + (128 / BE) * (w % BE) + w / BE;
}
template <int MODE, int BE>
__device__ __forceinline__ void fill_b_off(TileCtx& t, const MfmaArgs& a, int) {
    const int tid = opaque_tid();
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int lrow, lchunk;
        loader_pos(tid, i, lrow, lchunk);
        int wr = t.n0 + weight_col_of_lds_row<MODE, BE>(lrow);
        wr = min(wr, a.N - 1);
        t.b_off[i] = (uint32_t)wr * a.ldb_bytes + lchunk * 16;
    }
}

// Epilogue.  The token fragment is the MFMA "A" operand and the weight fragment the "B" operand:
// acc[nj][mi][v] belongs to token row mi*BE + (v/4)*8 + fq*4 + v%4 of the wave's 64 rows (fq =
// lane / BE) and to the output column that weight_col_of_lds_row gives block nj, lane fr.  The BE
// lanes with equal fq write one contiguous run of a row (128 bytes of bf16 act, 256 or 512 bytes
// of f32 y) per store instruction.
// fp8: the accumulators hold sums of code products; the float scales of the row and of the output
// channel are applied here, in float32: value = acc * (s_row * s_channel).  Lane j of a wave
// brings the scale of the wave's row j; the epilogue fetches it across lanes.
// the value that the lane with byte address src_lane4 = 4 * lane index holds (every lane of the
// wave must be active)
__device__ __forceinline__ float from_lane4(float v, int src_lane4) {
    return __int_as_float(__builtin_amdgcn_ds_bpermute(src_lane4, __float_as_int(v)));
}
// 16 * fq, opaque to the optimiser: the lane addresses built from it are then formed where they
// are used (one add each) instead of being kept in registers across the K loop
__device__ __forceinline__ int opaque_fq16(int fq) {
    int x = fq << 4;
    asm volatile("" : "+v"(x));
    return x;
}
// The lane index as a value that the optimiser cannot trace back to the thread index: what an
// epilogue derives from it (lane offsets of its stores) is computed in the epilogue, a few
// instructions per tile, instead of being kept in registers, or spilled, across the K loop
// (a spilled value comes back through a vector memory load, and the wait for it would also wait
// for every tile request in flight).
__device__ __forceinline__ int opaque_lane() {
    int x = threadIdx.x & 63;
    asm volatile("" : "+v"(x));
    return x;
}
// Largest magnitude over the lanes that share a 16-column storage block: LP = 2 (a lane and its
// neighbour lane ^ 1) or LP = 4 (the lanes of a quad), the maximum with the partner lanes taken as
// DPP operands of the max itself (two wait states between writing a register and reading it
// through DPP).  Every lane of the group must be active.
template <int LP>
__device__ __forceinline__ float block_amax(float m) {
    static_assert(LP == 2 || LP == 4, "a storage block is held by 2 or 4 lanes");
    if (LP == 4)
        asm("s_nop 1\n\t"
            "v_max_f32_dpp %0, %0, %0 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
            "s_nop 1\n\t"
            "v_max_f32_dpp %0, %0, %0 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf"
            : "+v"(m));
    else
        asm("s_nop 1\n\t"
            "v_max_f32_dpp %0, %0, %0 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf"
            : "+v"(m));
    return m;
}

// Down projection epilogue.  A lane holds NB = 128 / BE adjacent columns of a row (8 with 16 x 16
// blocks, 4 with 32 x 32 blocks), so a 16-column storage block lies in LP = 16 / NB neighbouring
// lanes.  Block scale: with amax the block's largest magnitude, k = biased exponent of amax (one
// higher if amax * 2^(141-k) would round to 32768), at least 15; code = rint(v * 2^(141-k)),
// |code| <= 32767.  The rounding is the float32 addition of 1.5 * 2^23 (round to nearest even at
// integer spacing), fused with the exact scaling.
// The compact form is written with buffer stores whose range ends at the group's last row: rows
// of the tile beyond it are dropped by the hardware's range check, so the epilogue has no
// branches.  The LP lanes of a block take turns over LP consecutive rows in storing the block's
// exponent byte, so every lane of an exponent store writes one byte.
// Returns the number of vector memory instructions issued when that number is the same for every
// wave that stores (the compact form), else 0: the tile loop lets that many stores stay in flight
// across the next tile's first K step.
template <bool FP8, int y_mode, typename ACC, int NN, int NM>
__device__ __forceinline__ int store_tile_down_as(ACC (&acc)[NN][NM], const MfmaArgs& a,
                                                   const TileCtx& t, int wm, int wn, int fr, int fq,
                                                   float my_scale) {
    constexpr int BE = 64 / NM, VLEN = BE * BE / 64;
    constexpr int NB = NN;                       // adjacent columns per lane
    constexpr int LP = Y_BLOCK / NB;             // lanes per storage block
    static_assert(NB * BE == 128 && (NB == 4 || NB == 8), "a wave covers 128 columns");
    {
        const int lane_o = opaque_lane();
        fr = lane_o % BE;
        fq = lane_o / BE;
    }
    const int fq16 = FP8 ? (fq << 4) : 0;
    const int nb = t.n0 + wn * 128;              // first column of the wave's 128 columns
    if (nb >= a.N) return 0;                     // N is a multiple of 128: the whole wave is in or out
    float sg[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j) sg[j] = FP8 ? a.sB0[(size_t)t.e * a.N + nb + NB * fr + j] : 1.f;
    constexpr uint32_t ESZ = (y_mode == Y_BLOCK16) ? 2 : 4;              // bytes per stored element
    const uint32_t row_bytes = (uint32_t)a.N * ESZ;
    const uint32_t erow_bytes = (uint32_t)a.N / Y_BLOCK;                 // exponent bytes per row
    const int rows_left = t.row_end - t.row0 - wm * 64 - fq * 4;         // rows of the group from this lane's first row on
    // the row of the wave that acc[..][mi][v] belongs to, less the lane's 4 * fq
    auto row_of = [](int mi, int v) { return mi * BE + (v >> 2) * 8 + (v & 3); };

    if constexpr (y_mode != Y_BLOCK16) {
        // float32 y (the staged call and the y tap): plain stores, rows beyond the group skipped
        char* const wave_base = a.C + ((size_t)(t.row0 + wm * 64) * a.N + nb) * ESZ;
        const uint32_t lane_off = (uint32_t)(fq * 4) * row_bytes + (uint32_t)(NB * fr) * ESZ;
#pragma unroll
        for (int mi = 0; mi < NM; ++mi) {
#pragma unroll
            for (int v = 0; v < VLEN; ++v) {
                const int rc = row_of(mi, v);
                const float sr = FP8 ? from_lane4(my_scale, (rc << 2) + fq16) : 1.f;
                float r[NB];
                float m = 0.f;
#pragma unroll
                for (int j = 0; j < NB; ++j) {
                    r[j] = acc[j][mi][v];
                    if (FP8) r[j] *= sr * sg[j];
                    m = fmaxf(m, fabsf(r[j]));
                }
                if (y_mode == Y_BLOCK16_AS_F32) {
                    const float amax = block_amax<LP>(m);
                    uint32_t kf = (__float_as_uint(amax) + 0x100u) & 0x7F800000u;   // k << 23
                    kf = max(kf, 15u << 23);
                    const float inv = __uint_as_float((268u << 23) - kf);           // 2^(141-k)
                    // 2^(k-141); k = 255 (the block held +-Inf) reads back as NaN, as in the combine
                    const float sc = kf == (255u << 23) ? __uint_as_float(0x7FC00000u) : __uint_as_float(kf - (14u << 23));
#pragma unroll
                    for (int j = 0; j < NB; ++j) {
                        const uint32_t c = __float_as_uint(__builtin_fmaf(r[j], inv, 12582912.f));   // low 16 bits: the code
                        r[j] = sc * (float)(int)(short)(c & 0xFFFFu);
                    }
                }
                if (rc >= rows_left) continue;       // the same for all lanes that share a row
                f32x4* const dst = reinterpret_cast<f32x4*>(wave_base + (size_t)rc * row_bytes + lane_off);
#pragma unroll
                for (int j = 0; j < NB; j += 4)
                    // y is read back (by the combine) only after gigabytes more have gone by: streaming store
                    __builtin_nontemporal_store(f32x4{r[j], r[j + 1], r[j + 2], r[j + 3]}, dst + j / 4);
            }
        }
    } else {
        // Buffer ranges: the tile's rows up to the group's end.  Every store gets a descriptor of
        // its own that starts at the wave-uniform row of the store (scalar arithmetic), so that
        // the lane offset is one register for the whole epilogue and the range check still ends
        // at the group's last row.
        const uint32_t tile_rows = (uint32_t)(t.row_end - t.row0);
        char* const codes0 = a.C + (size_t)t.row0 * row_bytes;
        uint8_t* const exps0 = a.Cs + (size_t)t.row0 * erow_bytes;
        const int codes_bytes = (int)(tile_rows * row_bytes), exps_bytes = (int)(tile_rows * erow_bytes);
        const uint32_t lane_row = (uint32_t)(wm * 64 + fq * 4);
        const int lane_off = (int)(lane_row * row_bytes + (uint32_t)(nb + NB * fr) * ESZ);
        // exponent bytes: lane j of a block's LP lanes stores row (first row of the run) + j
        const int lane_eoff = (int)((lane_row + (uint32_t)(fr % LP)) * erow_bytes + (uint32_t)(nb / Y_BLOCK + fr / LP));
#pragma unroll
        for (int mi = 0; mi < NM; ++mi) {
            uint32_t kbits[VLEN];
#pragma unroll
            for (int v = 0; v < VLEN; ++v) {
                const int rc = row_of(mi, v);
                const float sr = FP8 ? from_lane4(my_scale, (rc << 2) + fq16) : 1.f;
                float r[NB];
                float m = 0.f;
#pragma unroll
                for (int j = 0; j < NB; ++j) {
                    r[j] = acc[j][mi][v];
                    if (FP8) r[j] *= sr * sg[j];
                    m = fmaxf(m, fabsf(r[j]));
                }
                const float amax = block_amax<LP>(m);
                uint32_t kf = (__float_as_uint(amax) + 0x100u) & 0x7F800000u;       // k << 23
                kf = max(kf, 15u << 23);
                kbits[v] = kf;
                const float inv = __uint_as_float((268u << 23) - kf);               // 2^(141-k)
                uint32_t c[NB];
#pragma unroll
                for (int j = 0; j < NB; ++j) c[j] = __float_as_uint(__builtin_fmaf(r[j], inv, 12582912.f));   // low 16 bits: the code
                // low halves of two registers side by side (v_perm_b32: bytes 0-3 from the second source, 4-7 from the first)
                const int skip = (int)((uint32_t)rc * row_bytes);         // wave-uniform
                const __amdgpu_buffer_rsrc_t rc_codes = __builtin_amdgcn_make_buffer_rsrc(
                    codes0 + skip, 0, max(codes_bytes - skip, 0), 0x00020000);
                const int voff = lane_off;
                if constexpr (NB == 8) {
                    const u32x4 o = {__builtin_amdgcn_perm(c[1], c[0], 0x05040100u), __builtin_amdgcn_perm(c[3], c[2], 0x05040100u),
                                     __builtin_amdgcn_perm(c[5], c[4], 0x05040100u), __builtin_amdgcn_perm(c[7], c[6], 0x05040100u)};
                    __builtin_amdgcn_raw_buffer_store_b128(o, rc_codes, voff, 0, 2);     // streaming store
                } else {
                    typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
                    const u32x2 o = {__builtin_amdgcn_perm(c[1], c[0], 0x05040100u), __builtin_amdgcn_perm(c[3], c[2], 0x05040100u)};
                    __builtin_amdgcn_raw_buffer_store_b64(o, rc_codes, voff, 0, 2);
                }
                if ((v % LP) == LP - 1) {
                    // rows v-LP+1 .. v are consecutive rows of the wave (LP divides 4)
                    uint32_t k = kbits[v - LP + 1];
#pragma unroll
                    for (int j = 1; j < LP; ++j) k = (fr % LP) == j ? kbits[v - LP + 1 + j] : k;
                    const int eskip = (int)((uint32_t)row_of(mi, v - LP + 1) * erow_bytes);   // wave-uniform
                    const __amdgpu_buffer_rsrc_t rc_exps = __builtin_amdgcn_make_buffer_rsrc(
                        exps0 + eskip, 0, max(exps_bytes - eskip, 0), 0x00020000);
                    __builtin_amdgcn_raw_buffer_store_b8((uint8_t)(k >> 23), rc_exps, lane_eoff, 0, 0);
                }
            }
        }
        return NM * VLEN + NM * VLEN / LP;
    }
    return 0;
}

template <bool FP8, typename ACC, int NN, int NM>
__device__ __forceinline__ int store_tile_down(ACC (&acc)[NN][NM], const MfmaArgs& a,
                                               const TileCtx& t, int wm, int wn, int fr, int fq,
                                               float my_scale) {
    // one copy of the unrolled epilogue per storage form, chosen once per tile
    if (a.y_mode == Y_BLOCK16) return store_tile_down_as<FP8, Y_BLOCK16>(acc, a, t, wm, wn, fr, fq, my_scale);
    if (a.y_mode == Y_BLOCK16_AS_F32) return store_tile_down_as<FP8, Y_BLOCK16_AS_F32>(acc, a, t, wm, wn, fr, fq, my_scale);
    return store_tile_down_as<FP8, Y_EXACT_F32>(acc, a, t, wm, wn, fr, fq, my_scale);
}

template <int MODE, bool FP8, typename ACC, int NN_, int NM_>
__device__ __forceinline__ int store_tile(ACC (&acc)[NN_][NM_], const MfmaArgs& a,
                                          const TileCtx& t, int wm, int wn, int fr, int fq,
                                          float my_scale) {
    if constexpr (MODE == MODE_DOWN) {
        return store_tile_down<FP8>(acc, a, t, wm, wn, fr, fq, my_scale);
    } else {
        constexpr int NM = NM_, BE = 64 / NM, VLEN = BE * BE / 64;
        constexpr int NBG = 64 / BE;              // adjacent output columns per lane
        constexpr int NPER = NBG;                                     // adjacent columns per lane
        {
            const int lane_o = opaque_lane();
            fr = lane_o % BE;
            fq = lane_o / BE;
        }
        const int fq16 = FP8 ? (fq << 4) : 0;
        const int n = t.n0 + wn * 64 + NBG * fr;
        if (n >= a.N) return 0;
        float sg[NPER], su[NPER];   // per-channel scales (fp8): gate or down, and up
#pragma unroll
        for (int q = 0; q < NPER; ++q) {
            sg[q] = FP8 ? a.sB0[(size_t)t.e * a.N + n + q] : 1.f;
            su[q] = FP8 ? a.sB1[(size_t)t.e * a.N + n + q] : 1.f;
        }
        // Buffer stores whose range ends at the group's last row (see the down epilogue): rows of
        // the tile beyond it are dropped by the range check, no branches; every store's descriptor
        // starts at the wave-uniform row of the store, the lane offset is one register.
        const uint32_t row_bytes = (uint32_t)a.N * 2;
        char* const act0 = a.C + (size_t)t.row0 * row_bytes;
        const int act_bytes = (int)((uint32_t)(t.row_end - t.row0) * row_bytes);
        const int lane_off = (int)((uint32_t)(wm * 64 + fq * 4) * row_bytes + (uint32_t)n * 2);
#pragma unroll
        for (int mi = 0; mi < NM; ++mi) {
#pragma unroll
            for (int v = 0; v < VLEN; ++v) {
                const int rc = mi * BE + (v >> 2) * 8 + (v & 3);         // row of the wave, less the lane's 4 * fq
                // lane j of the wave holds the scale of the wave's row j (all lanes take part)
                const float sr = FP8 ? from_lane4(my_scale, (rc << 2) + fq16) : 1.f;
                float h[NPER];
#pragma unroll
                for (int q = 0; q < NPER; ++q) {
                    float g = acc[q][mi][v], u = acc[NBG + q][mi][v];
                    if (FP8) {
                        g *= sr * sg[q];
                        u *= sr * su[q];
                    }
                    h[q] = silu_mul(g, u);
                }
                const int skip = (int)((uint32_t)rc * row_bytes);         // wave-uniform
                const __amdgpu_buffer_rsrc_t rsrc =
                    __builtin_amdgcn_make_buffer_rsrc(act0 + skip, 0, max(act_bytes - skip, 0), 0x00020000);
                if constexpr (NPER == 2) {
                    __builtin_amdgcn_raw_buffer_store_b32(pack2_bf16(h[0], h[1]), rsrc, lane_off, 0, 0);
                } else {
                    typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
                    const u32x2 o = {pack2_bf16(h[0], h[1]), pack2_bf16(h[NPER - 2], h[NPER - 1])};
                    __builtin_amdgcn_raw_buffer_store_b64(o, rsrc, lane_off, 0, 0);
                }
            }
        }
        return NM * VLEN;
    }
}

__device__ __forceinline__ f32x4 mfma_bf16(bf16x8 a, bf16x8 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ f32x16 mfma_bf16(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// 32 bytes of one LDS row (two swizzled 16-byte chunks) as one fp8 MFMA operand
__device__ __forceinline__ i32x8 load_frag8(const char* p0, const char* p1) {
    const u32x4 lo = *reinterpret_cast<const u32x4*>(p0);
    const u32x4 hi = *reinterpret_cast<const u32x4*>(p1);
    return i32x8{(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3], (int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
}

// A pointer that is the same in every lane, moved to scalar registers.
__device__ __forceinline__ const char* uniform_ptr(const char* p) {
    const uint64_t v = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(v));
    const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(v >> 32));
    return reinterpret_cast<const char*>((static_cast<uint64_t>(hi) << 32) | lo);
}

// 16 bytes per lane from global memory (scalar base + 32-bit lane offset) straight into LDS at
// m0 + 16 * lane.  Completion is tracked by vmcnt like any other vector memory load.
__device__ __forceinline__ void dma16(uint32_t lds_addr, uint32_t voff, const char* base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(base)
                 : "memory", "m0");
}

// Ragged tiles.  The four 64-row blocks of a tile are dealt to the SIMDs two by two (waves 2j and
// 2j+1 take block j; wave w runs on SIMD w % 4), and a wave whose block lies entirely beyond the
// group's last row only takes part in loading and in the barriers: in a tile with at most 128
// rows the waves that multiply have their SIMD to themselves and the tile costs half the
// matrix-pipe time (+7-12 % below 256 rows per expert, +3-4 % up to 2048, +1.5 % on the 64K-token
// Zipf batch).
template <int MODE, bool FP8, int BLK>
__global__ __launch_bounds__(THREADS) void ffn_mfma_kernel(MfmaArgs a) {
    extern __shared__ __attribute__((aligned(16))) char smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    // ---- this workgroup's tiles.  The launch-order list is cut into chunks of nslots entries
    // (one per workgroup of an XCD); chunk c goes to XCD c % 8, so the 8 XCDs work on neighbouring
    // stretches of the list (the same expert) at the same time and share it in the memory-side cache.
    const int total = a.table[0] * a.nct;
    const int xcd = blockIdx.x & 7;
    const int nslots = gridDim.x >> 3;
    const int slot = blockIdx.x >> 3;
    const int l_end = total;
    int L = xcd * nslots + slot;
    if (L >= l_end) return;

    // ---- fragment read offsets.  Lane = (fq, fr): fr = row of the MFMA block, fq = which 16-byte
    // (bf16) or 32-byte (fp8) piece of the block's K slice the lane supplies.
    constexpr int BE = Blk<FP8, BLK>::E, NM = Blk<FP8, BLK>::NM, NN = Blk<FP8, BLK>::NN;
    constexpr int NG = 64 / BE;                 // lane groups = pieces per K slice
    const int fr = lane % BE, fq = lane / BE;
    const int sw = (fr >> 1) & 7;
    // bf16: slice kk (8/NG per K step) takes chunk kk*NG + fq;
    // fp8 : slice kk (2 per K step) takes chunks kk*4 + fq*2 and the next one.
    uint32_t frag_off[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        if (FP8) frag_off[c] = (uint32_t)((((c >> 1) * 4 + fq * 2 + (c & 1)) ^ sw) << 4);   // c = kk*2 + half
        else frag_off[c] = (uint32_t)((((c % (8 / NG)) * NG + fq) ^ sw) << 4);               // c = kk
    }
    const uint32_t xa_row = (wm * 64 + fr) * ROW_BYTES;                    // + mi*BE rows
    const uint32_t wb_row = ((MODE == MODE_GATE_UP ? wn * 64 : wn * 128) + fr) * ROW_BYTES;
    // block nj of the wave: gate/up: blocks 0..NN/2-1 are gate rows, the rest the matching up rows
    auto wb_off = [](int nj) -> uint32_t {
        if (MODE == MODE_GATE_UP) return (uint32_t)(((nj / (NN / 2)) * 128 + (nj % (NN / 2)) * BE) * ROW_BYTES);
        return (uint32_t)(nj * BE * ROW_BYTES);
    };

    typedef typename std::conditional<BE == 32, f32x16, f32x4>::type acc_t;
    acc_t acc[NN][NM];

    // ---- LDS slots: three token-tile slots [0, 3) and two weight-tile slots [3, 5) of 32 KB.  The
    // token tile of K step k+2 and the weight tile of step k+1 are requested at the top of step k
    // (weights first), and the step's end waits for all but the last four requests, i.e. for the
    // weight tile of step k+1 (the token tile of step k+1 is a step older).  Requests are served
    // in issue order.
    constexpr int NKK = FP8 ? 4 : 8 / NG;       // distinct fragment offsets per K step
    uint32_t ad_a[NKK], ad_b[NKK];              // byte offsets in LDS of the lane's fragments in the slots being read
    int a_rd = 0, b_rd = 0;                     // slots that hold the current K step
#pragma unroll
    for (int c = 0; c < NKK; ++c) {
        ad_a[c] = xa_row + frag_off[c];
        ad_b[c] = 3 * TILE_BYTES + wb_row + frag_off[c];
    }
#define MOE_A_PTR(KK_) (smem + ad_a[KK_])
#define MOE_B_PTR(KK_) (smem + ad_b[KK_])

    // fp8: a fragment is 32 bytes of a row = two swizzled 16-byte chunks
#define MOE_COMPUTE_FP8()                                                                 \
    {                                                                                     \
        _Pragma("unroll") for (int kk = 0; kk < 2; ++kk) {                                \
            i32x8 xa[NM];                                                                 \
            _Pragma("unroll") for (int mi = 0; mi < NM; ++mi)                             \
                xa[mi] = load_frag8(MOE_A_PTR(kk * 2) + mi * BE * ROW_BYTES,              \
                                    MOE_A_PTR(kk * 2 + 1) + mi * BE * ROW_BYTES);         \
            /* zero scale operands select the unscaled v_mfma_f32_32x32x64_f8f6f4 */       \
            _Pragma("unroll") for (int nj = 0; nj < NN; ++nj) {                           \
                const i32x8 wb = load_frag8(MOE_B_PTR(kk * 2) + wb_off(nj),               \
                                            MOE_B_PTR(kk * 2 + 1) + wb_off(nj));          \
                _Pragma("unroll") for (int mi = 0; mi < NM; ++mi) acc[nj][mi] =           \
                    __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(                      \
                        xa[mi], wb, acc[nj][mi], 0, 0, 0, 0, 0, 0);                       \
            }                                                                             \
        }                                                                                 \
    }

#define MOE_SGB(MASK_, N_) __builtin_amdgcn_sched_group_barrier(MASK_, N_, 0)
    // fp8, rotated loop: a K step is 8 groups of NM MFMAs, group (kk, nj) = K slice kk times
    // weight block nj.  Token fragments of the two slices sit in xaA and xaB, weight fragments
    // alternate between wbP and wbQ: the fragment of group i+1 is read while group i multiplies
    // (-4 % for gate/up, -1 % for down).
    constexpr bool ROT8 = FP8;
    i32x8 xaA[NM], xaB[NM], wbP, wbQ;
#define MOE_F8_RD_A(DST_, KK_)                                                             \
    {                                                                                      \
        _Pragma("unroll") for (int mi = 0; mi < NM; ++mi) DST_[mi] =                       \
            load_frag8(MOE_A_PTR((KK_) * 2) + mi * BE * ROW_BYTES,                         \
                       MOE_A_PTR((KK_) * 2 + 1) + mi * BE * ROW_BYTES);                    \
    }
#define MOE_F8_RD_B(DST_, KK_, NJ_)                                                        \
    DST_ = load_frag8(MOE_B_PTR((KK_) * 2) + wb_off(NJ_), MOE_B_PTR((KK_) * 2 + 1) + wb_off(NJ_));
    /* zero scale operands select the unscaled v_mfma_f32_32x32x64_f8f6f4 */
#define MOE_F8_MM(XA_, WB_, NJ_, Z_)                                                       \
    {                                                                                      \
        _Pragma("unroll") for (int mi = 0; mi < NM; ++mi) {                                \
            if constexpr (Z_) acc[NJ_][mi] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(  \
                XA_[mi], WB_, acc_t{}, 0, 0, 0, 0, 0, 0);                                  \
            else acc[NJ_][mi] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(           \
                XA_[mi], WB_, acc[NJ_][mi], 0, 0, 0, 0, 0, 0);                             \
        }                                                                                  \
    }
    // 16 x 16 blocks: the K loop is rotated by a quarter step.  A step's barrier stands before its
    // last group of 16 MFMAs; behind the barrier the fragments of the NEXT step's first group are
    // read (they are complete in LDS from the barrier on) while those 16 MFMAs, whose operands
    // are in registers already, keep the matrix pipe busy.  The next step then starts multiplying
    // at once instead of waiting for LDS.
    constexpr bool ROT = !FP8 && BE == 16;

    // ---- direct-to-LDS loader: wave w fills rows 32w .. 32w+31 of both operand tiles, 8 rows per
    // instruction; the K offset is added to the lane offsets, the bases are scalar
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem;
    const uint32_t dma_row0 = (uint32_t)(wave_u * 32) * ROW_BYTES;
    // Issue order inside one K step, imposed on the compiler's scheduler (which otherwise gathers
    // the LDS reads in blocks of their own): the loads come first (program order), then the
    // fragments of the first K slice; after that, 32x32 blocks: every MFMA followed by one fragment
    // read of the next slice; 16x16 blocks: three groups of 16 MFMAs with one of the next group's 4
    // fragment reads behind every third MFMA (measured best of six spacings), then the last group.
#define MOE_ISSUE_ORDER()                                                                  \
    if constexpr (!FP8 && BE == 16) {                                                      \
        MOE_SGB(0x100, NM + NN);                                                           \
        _Pragma("unroll") for (int g = 0; g < 3; ++g) {                                    \
            _Pragma("unroll") for (int j = 0; j < NN / 2; ++j) {                           \
                MOE_SGB(0x008, 3);                                                         \
                MOE_SGB(0x100, 1);                                                         \
            }                                                                              \
            MOE_SGB(0x008, NM * NN / 2 - 3 * NN / 2);                                      \
        }                                                                                  \
        MOE_SGB(0x008, NM * NN / 2);                                                       \
    } else if constexpr (BE == 32) {                                                       \
        constexpr int NMF = NM * NN, NKK = FP8 ? 2 : 4, RPF = FP8 ? 2 : 1;                 \
        constexpr int NRS = NM + NN;                                                       \
        MOE_SGB(0x100, NRS * RPF);                                                         \
        _Pragma("unroll") for (int kk = 0; kk < NKK; ++kk) {                               \
            _Pragma("unroll") for (int j = 0; j < NMF; ++j) {                              \
                MOE_SGB(0x008, 1);                                                         \
                if (kk < NKK - 1 && j < NRS) MOE_SGB(0x100, RPF);                          \
            }                                                                              \
        }                                                                                  \
    }
    // bf16: the fragments of K slice k+1 are read (into the other of two fragment sets) before
    // the MFMAs of slice k are issued; the staging registers that the direct-to-LDS loader no
    // longer needs pay for the second set
    bf16x8 fa0[NM], fb0[NN], fa1[NM], fb1[NN];
#define MOE_FREAD(BUF_, KK_)                                                               \
    {                                                                                      \
        _Pragma("unroll") for (int mi = 0; mi < NM; ++mi) fa##BUF_[mi] =                   \
            *reinterpret_cast<const bf16x8*>(MOE_A_PTR(KK_) + mi * BE * ROW_BYTES); \
        _Pragma("unroll") for (int nj = 0; nj < NN; ++nj) fb##BUF_[nj] =                   \
            *reinterpret_cast<const bf16x8*>(MOE_B_PTR(KK_) + wb_off(nj));         \
    }
#define MOE_FMFMA(BUF_)                                                                    \
    {                                                                                      \
        _Pragma("unroll") for (int nj = 0; nj < NN; ++nj)                                  \
            _Pragma("unroll") for (int mi = 0; mi < NM; ++mi)                              \
                acc[nj][mi] = mfma_bf16(fa##BUF_[mi], fb##BUF_[nj], acc[nj][mi]);          \
    }
    // first K slice of a tile: the accumulator input is the constant zero
#define MOE_FMFMA_Z(BUF_)                                                                  \
    {                                                                                      \
        _Pragma("unroll") for (int nj = 0; nj < NN; ++nj)                                  \
            _Pragma("unroll") for (int mi = 0; mi < NM; ++mi)                              \
                acc[nj][mi] = mfma_bf16(fa##BUF_[mi], fb##BUF_[nj], acc_t{});              \
    }
    // 16x16x32 blocks: a K step is two slices; a slice's weight fragments are handled in two
    // halves (blocks 0..NN/2-1 and the rest) so that two half buffers and two token-fragment
    // buffers suffice to keep the reads one group of 16 MFMAs ahead
#define MOE_FREAD_A16(DST_, KK_)                                                           \
    {                                                                                      \
        _Pragma("unroll") for (int mi = 0; mi < NM; ++mi) DST_[mi] =                       \
            *reinterpret_cast<const bf16x8*>(MOE_A_PTR(KK_) + mi * BE * ROW_BYTES); \
    }
#define MOE_FREAD_B16(HALF_, KK_)                                                          \
    {                                                                                      \
        _Pragma("unroll") for (int q = 0; q < NN / 2; ++q) fb0[(HALF_) * (NN / 2) + q] =   \
            *reinterpret_cast<const bf16x8*>(MOE_B_PTR(KK_) + wb_off((HALF_) * (NN / 2) + q)); \
    }
#define MOE_FMFMA16(FA_, HALF_, Z_)                                                        \
    {                                                                                      \
        _Pragma("unroll") for (int q = 0; q < NN / 2; ++q)                                 \
            _Pragma("unroll") for (int mi = 0; mi < NM; ++mi) {                            \
                constexpr int njh = (HALF_) * (NN / 2);                                    \
                if constexpr (Z_) acc[njh + q][mi] = mfma_bf16(FA_[mi], fb0[njh + q], acc_t{}); \
                else acc[njh + q][mi] = mfma_bf16(FA_[mi], fb0[njh + q], acc[njh + q][mi]); \
            }                                                                              \
    }
#define MOE_COMPUTE_STEP(FIRST_)                                                           \
    if constexpr (!FP8 && BE == 32) {                                                      \
        MOE_FREAD(0, 0);                                                                   \
        MOE_FREAD(1, 1);                                                                   \
        if constexpr (FIRST_) MOE_FMFMA_Z(0) else MOE_FMFMA(0);                            \
        MOE_FREAD(0, 2);                                                                   \
        MOE_FMFMA(1);                                                                      \
        MOE_FREAD(1, 3);                                                                   \
        MOE_FMFMA(0);                                                                      \
        MOE_FMFMA(1);                                                                      \
    } else if constexpr (!FP8 && BE == 16) {                                               \
        MOE_FREAD_A16(fa0, 0);                                                             \
        MOE_FREAD_B16(0, 0);                                                               \
        MOE_FREAD_B16(1, 0);                                                               \
        MOE_FMFMA16(fa0, 0, FIRST_);                                                       \
        MOE_FREAD_A16(fa1, 1);                                                             \
        MOE_FREAD_B16(0, 1);                                                               \
        MOE_FMFMA16(fa0, 1, FIRST_);                                                       \
        MOE_FREAD_B16(1, 1);                                                               \
        MOE_FMFMA16(fa1, 0, false);                                                        \
        MOE_FMFMA16(fa1, 1, false);                                                        \
    } else {                                                                               \
        if constexpr (FIRST_) {                                                            \
            _Pragma("unroll") for (int nj = 0; nj < NN; ++nj)                              \
                _Pragma("unroll") for (int mi = 0; mi < NM; ++mi)                          \
                    _Pragma("unroll") for (int v = 0; v < Blk<FP8, BLK>::VLEN; ++v)              \
                        acc[nj][mi][v] = 0.f;                                              \
        }                                                                                  \
        MOE_COMPUTE_FP8();                                                                 \
    }
    // one operand tile of K step KT_ of CTX_ into slot SLOT_ (4 requests per wave)
#define MOE_DMA_A(SLOT_, CTX_, KT_)                                                        \
    {                                                                                      \
        const uint32_t kb = (uint32_t)(KT_) * ROW_BYTES;                                   \
        const char* abase = uniform_ptr(                                                   \
            (MODE == MODE_GATE_UP) ? a.A : a.A + (size_t)CTX_.row0 * a.lda_bytes);         \
        const uint32_t st = __builtin_amdgcn_readfirstlane(                                \
            lds_base + (uint32_t)(SLOT_) * TILE_BYTES + dma_row0);                         \
        _Pragma("unroll") for (int i = 0; i < 4; ++i)                                      \
            dma16(st + i * 8 * ROW_BYTES, CTX_.a_off[i] + kb, abase);                      \
    }
#define MOE_DMA_B(SLOT_, CTX_, KT_)                                                        \
    {                                                                                      \
        const uint32_t kb = (uint32_t)(KT_) * ROW_BYTES;                                   \
        const char* bbase =                                                                \
            uniform_ptr((MODE == MODE_DOWN || wave_u < 4) ? CTX_.b0e : CTX_.b1e);          \
        const uint32_t st = __builtin_amdgcn_readfirstlane(                                \
            lds_base + (uint32_t)(3 + (SLOT_)) * TILE_BYTES + dma_row0);                   \
        _Pragma("unroll") for (int i = 0; i < 4; ++i)                                      \
            dma16(st + i * 8 * ROW_BYTES, CTX_.b_off[i] + kb, bbase);                      \
    }
    // One K step: request the weight tile of step KTB_ of CB_ (the next step) and the token
    // tile of step KTA_ of CA_ (the step after), multiply the current slots, wait for everything
    // but the token tile just requested, move on to the next slots
#define MOE_ADVANCE_SLOTS()                                                                \
    {                                                                                      \
        const uint32_t da = a_rd == 2 ? (uint32_t)(-2 * TILE_BYTES) : (uint32_t)TILE_BYTES; \
        const uint32_t db = b_rd == 1 ? (uint32_t)(-TILE_BYTES) : (uint32_t)TILE_BYTES;    \
        a_rd = a_rd == 2 ? 0 : a_rd + 1;                                                   \
        b_rd ^= 1;                                                                         \
        _Pragma("unroll") for (int c = 0; c < NKK; ++c) {                                  \
            ad_a[c] += da;                                                                 \
            ad_b[c] += db;                                                                 \
        }                                                                                  \
    }
    // rotated loop: the fragments of the current slots' first group (token fragments of K slice 0,
    // weight fragments of its first half)
#define MOE_ROT_HEAD_READS()                                                               \
    {                                                                                      \
        MOE_FREAD_A16(fa0, 0);                                                             \
        MOE_FREAD_B16(0, 0);                                                               \
    }
#define MOE_WAIT_STEP(FIRST_)                                                              \
    {                                                                                      \
        if constexpr (FIRST_) {                                                            \
            /* all but the token tile just requested and the previous epilogue's stores, which \
               were issued after the weight tile that this wait is for (requests and stores    \
               complete in issue order) */                                                     \
            /* 4 + n_stores; the epilogues issue 16 or 32 (gate/up) and 24 or 40 (down) stores */ \
            if (n_stores == 16) asm volatile("s_waitcnt vmcnt(20)" ::: "memory");          \
            else if (n_stores == 24) asm volatile("s_waitcnt vmcnt(28)" ::: "memory");     \
            else if (n_stores == 32) asm volatile("s_waitcnt vmcnt(36)" ::: "memory");     \
            else if (n_stores == 40) asm volatile("s_waitcnt vmcnt(44)" ::: "memory");     \
            else asm volatile("s_waitcnt vmcnt(4)" ::: "memory");                          \
        } else {                                                                           \
            asm volatile("s_waitcnt vmcnt(4)" ::: "memory");                               \
        }                                                                                  \
    }
    // The record of the tile after the current one is fetched (scalar path) in the current tile's
    // first K step, right in front of the barrier: the wave has to wait for its LDS reads there
    // anyway, and most waves wait for the slowest one.
#define MOE_NEXT_REC(FIRST_)                                                               \
    {                                                                                      \
        if constexpr (FIRST_) rec_s = load_rec(a.order + min(L + stride, total - 1));      \
    }
#define MOE_STEP(CB_, KTB_, CA_, KTA_, FIRST_, LAST_)                                     \
    {                                                                                      \
        if constexpr (!(FIRST_)) MOE_DMA_B(b_rd ^ 1, CB_, KTB_);                           \
        MOE_DMA_A(a_rd == 0 ? 2 : a_rd - 1, CA_, KTA_);                                    \
        if constexpr (ROT) {                                                               \
            if constexpr (FIRST_) MOE_ROT_HEAD_READS();                                    \
            MOE_FREAD_B16(1, 0);                                                           \
            MOE_FREAD_A16(fa1, 1);                                                         \
            MOE_FMFMA16(fa0, 0, FIRST_);                                                   \
            MOE_FREAD_B16(0, 1);                                                           \
            MOE_FMFMA16(fa0, 1, FIRST_);                                                   \
            MOE_FREAD_B16(1, 1);                                                           \
            MOE_FMFMA16(fa1, 0, false);                                                    \
            _Pragma("unroll") for (int j = 0; j < NM + NN / 2; ++j) {                      \
                MOE_SGB(0x008, 2);                                                         \
                MOE_SGB(0x100, 1);                                                         \
            }                                                                              \
            _Pragma("unroll") for (int g = 0; g < 2; ++g) {                                \
                _Pragma("unroll") for (int j = 0; j < NN / 2; ++j) {                       \
                    MOE_SGB(0x008, 3);                                                     \
                    MOE_SGB(0x100, 1);                                                     \
                }                                                                          \
                MOE_SGB(0x008, NM * NN / 2 - 3 * NN / 2);                                  \
            }                                                                              \
        } else if constexpr (ROT8) {                                                       \
            static_assert(!FP8 || (NM == 2 && NN == 4), "fp8 step is written for 2 x 4 blocks"); \
            if constexpr (FIRST_) {                                                        \
                MOE_F8_RD_A(xaA, 0);                                                       \
                MOE_F8_RD_B(wbP, 0, 0);                                                    \
            }                                                                              \
            MOE_F8_RD_B(wbQ, 0, 1);                                                        \
            MOE_F8_MM(xaA, wbP, 0, FIRST_);                                                \
            MOE_F8_RD_B(wbP, 0, 2);                                                        \
            MOE_F8_RD_A(xaB, 1);                                                           \
            MOE_F8_MM(xaA, wbQ, 1, FIRST_);                                                \
            MOE_F8_RD_B(wbQ, 0, 3);                                                        \
            MOE_F8_MM(xaA, wbP, 2, FIRST_);                                                \
            MOE_F8_RD_B(wbP, 1, 0);                                                        \
            MOE_F8_MM(xaA, wbQ, 3, FIRST_);                                                \
            MOE_F8_RD_B(wbQ, 1, 1);                                                        \
            MOE_F8_MM(xaB, wbP, 0, false);                                                 \
            MOE_F8_RD_B(wbP, 1, 2);                                                        \
            MOE_F8_MM(xaB, wbQ, 1, false);                                                 \
            MOE_F8_RD_B(wbQ, 1, 3);                                                        \
            MOE_F8_MM(xaB, wbP, 2, false);                                                 \
            if constexpr (FIRST_) MOE_SGB(0x100, 2 * NM + 2);                              \
            MOE_SGB(0x100, 2);                                                             \
            MOE_SGB(0x008, NM);                                                            \
            MOE_SGB(0x100, 2 + 2 * NM);                                                    \
            MOE_SGB(0x008, NM);                                                            \
            _Pragma("unroll") for (int j = 0; j < 5; ++j) {                                \
                MOE_SGB(0x100, 2);                                                         \
                MOE_SGB(0x008, NM);                                                        \
            }                                                                              \
        } else {                                                                           \
            MOE_COMPUTE_STEP(FIRST_);                                                      \
            MOE_ISSUE_ORDER();                                                             \
        }                                                                                  \
        MOE_WAIT_STEP(FIRST_);                                                             \
        MOE_NEXT_REC(FIRST_);                                                              \
        __syncthreads();                                                                   \
        MOE_ADVANCE_SLOTS();                                                               \
        if constexpr (ROT) {                                                               \
            /* a tile's last step leaves the next tile's first fragments to that tile's first  \
               step: they would have to stay in registers across the epilogue */              \
            if constexpr (!(LAST_)) MOE_ROT_HEAD_READS();                                  \
            MOE_FMFMA16(fa1, 1, false);                                                    \
            if constexpr (!(LAST_)) {                                                      \
                _Pragma("unroll") for (int j = 0; j < NM + NN / 2; ++j) {                  \
                    MOE_SGB(0x100, 1);                                                     \
                    MOE_SGB(0x008, 2);                                                     \
                }                                                                          \
            }                                                                              \
        } else if constexpr (ROT8) {                                                       \
            if constexpr (!(LAST_)) {                                                      \
                MOE_F8_RD_A(xaA, 0);                                                       \
                MOE_F8_RD_B(wbP, 0, 0);                                                    \
            }                                                                              \
            MOE_F8_MM(xaB, wbQ, 3, false);                                                 \
            if constexpr (!(LAST_)) {                                                      \
                MOE_SGB(0x100, 2 * NM + 2);                                                \
                MOE_SGB(0x008, NM);                                                        \
            }                                                                              \
        }                                                                                  \
    }

    // the same K step for a wave with nothing to multiply
#define MOE_STEP_IDLE(CB_, KTB_, CA_, KTA_, FIRST_)                                        \
    {                                                                                      \
        if constexpr (!(FIRST_)) MOE_DMA_B(b_rd ^ 1, CB_, KTB_);                           \
        MOE_DMA_A(a_rd == 0 ? 2 : a_rd - 1, CA_, KTA_);                                    \
        MOE_WAIT_STEP(FIRST_);                                                             \
        MOE_NEXT_REC(FIRST_);                                                              \
        __syncthreads();                                                                   \
        MOE_ADVANCE_SLOTS();                                                               \
    }

    const int KT = a.KT;   // even, >= 2
    const int stride = 8 * nslots;
    TileCtx cur, nxt;
    ctx_from_rec<MODE>(cur, a, load_rec(a.order + L), tid);
    fill_a_off<MODE>(cur, a, tid);
    fill_b_off<MODE, BE>(cur, a, tid);
    MOE_DMA_A(0, cur, 0);
    MOE_DMA_B(0, cur, 0);
    MOE_DMA_A(1, cur, 1);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    int4 rec_s = load_rec(a.order + min(L + stride, total - 1));
    __syncthreads();
    MOE_DMA_B(1, cur, 1);
    int n_stores = 0;   // store instructions this wave issued in the previous tile's epilogue (wave-uniform)

    // Invariant at the top of every tile: token slot a_rd holds its K step 0, the next token slot
    // its step 1 (or is receiving it), weight slot b_rd its step 0, and the other weight slot is
    // receiving step 1: that request is made before the previous tile's epilogue, so that the
    // epilogue's stores are younger than everything the tile's first K step waits for and need
    // not have completed by then.  rec_s is the next tile's record.
    for (;;) {
        L += stride;
        const bool has_next = L < l_end;
        // The next tile's context (for gate/up: the loads of its perm entries) is set up behind
        // the first K step, whose fragment prefetch needs the registers; a tile of two K steps
        // needs it at once.
        const int4 rec_n = rec_s;
#define MOE_NEXT_CTX()                                                                     \
    {                                                                                      \
        if (has_next) ctx_from_rec<MODE>(nxt, a, rec_n, tid);                              \
        else nxt = cur; /* nothing follows: the trailing loads re-read this tile (harmless) */ \
    }
        if (KT <= 2) MOE_NEXT_CTX();
        // fp8: lane j of a wave brings the scale of the wave's row j for the epilogue
        float my_scale = 1.f;
        if (FP8) my_scale = a.sA[min(cur.row0 + wm * 64 + lane, cur.row_end - 1)];

        const int wm_u = wave_u >> 1, wn_u = wave_u & 1;
        const bool idle = cur.row0 + wm_u * 64 >= cur.row_end;   // this wave's 64 rows are all padding
        // Invariant at the top of K step k: token slot a_rd holds step k, the next token slot
        // holds (or is receiving) step k+1, weight slot b_rd holds step k.
        if (idle) {
            if (KT > 2) {
                MOE_STEP_IDLE(cur, 1, cur, 2, true);
                MOE_NEXT_CTX();
                for (int kt = 1; kt < KT - 2; ++kt) MOE_STEP_IDLE(cur, kt + 1, cur, kt + 2, false);
                if (has_next) {
                    fill_a_off<MODE>(nxt, a, tid);
                    fill_b_off<MODE, BE>(nxt, a, tid);
                }
                MOE_STEP_IDLE(cur, KT - 1, nxt, 0, false);
                MOE_STEP_IDLE(nxt, 0, nxt, 1, false);
            } else {
                if (has_next) {
                    fill_a_off<MODE>(nxt, a, tid);
                    fill_b_off<MODE, BE>(nxt, a, tid);
                }
                MOE_STEP_IDLE(cur, 1, nxt, 0, true);
                MOE_STEP_IDLE(nxt, 0, nxt, 1, false);
            }
        } else if (KT > 2) {
            MOE_STEP(cur, 1, cur, 2, true, false);
            MOE_NEXT_CTX();
            for (int kt = 1; kt < KT - 2; ++kt) MOE_STEP(cur, kt + 1, cur, kt + 2, false, false);
            if (has_next) {
                fill_a_off<MODE>(nxt, a, tid);
                fill_b_off<MODE, BE>(nxt, a, tid);
            }
            // last two steps of this tile: their requests reach into the next tile
            MOE_STEP(cur, KT - 1, nxt, 0, false, false);
            MOE_STEP(nxt, 0, nxt, 1, false, true);
        } else {
            if (has_next) {
                fill_a_off<MODE>(nxt, a, tid);
                fill_b_off<MODE, BE>(nxt, a, tid);
            }
            MOE_STEP(cur, 1, nxt, 0, true, false);
            MOE_STEP(nxt, 0, nxt, 1, false, true);
        }

        // the next tile's second weight tile, into the slot that the last K step has just left
        MOE_DMA_B(b_rd ^ 1, nxt, 1);
        n_stores = 0;
        if (!idle) n_stores = __builtin_amdgcn_readfirstlane(store_tile<MODE, FP8>(acc, a, cur, wm_u, wn_u, fr, fq, my_scale));
        if (!has_next) {
            // the last step's token-tile requests are still on their way into this workgroup's LDS
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            break;
        }
        cur = nxt;
    }
#undef MOE_COMPUTE_FP8
#undef MOE_ISSUE_ORDER
#undef MOE_STEP
#undef MOE_STEP_IDLE
#undef MOE_WAIT_STEP
#undef MOE_NEXT_REC
#undef MOE_NEXT_CTX
#undef MOE_ADVANCE_SLOTS
#undef MOE_ROT_HEAD_READS
#undef MOE_DMA_A
#undef MOE_DMA_B
#undef MOE_A_PTR
#undef MOE_B_PTR
#undef MOE_COMPUTE_STEP
#undef MOE_FREAD
#undef MOE_FMFMA
#undef MOE_FMFMA_Z
#undef MOE_FREAD_A16
#undef MOE_FREAD_B16
#undef MOE_FMFMA16
#undef MOE_SGB
#undef MOE_F8_RD_A
#undef MOE_F8_RD_B
#undef MOE_F8_MM
}

struct FfnWs {
    size_t table, first, order_gu, order_dn, act, xq, sx, sxp, act_q, sa, total;
};
FfnWs ffn_ws_layout(const moe_config_t& c) {
    const size_t P = (size_t)c.T * c.K;
    const bool fp8 = c.w_dtype == MOE_DTYPE_FP8_E4M3;
    FfnWs w{};
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o += align_up(bytes ? bytes : 1, 256); return at; };
    w.table = take(tile_table_bytes(c, BM));
    w.first = take(sizeof(int32_t) * (c.E + 1));
    w.order_gu = take(tile_order_bytes(c, BM, (int)ceil_div64(c.I, 128)));
    w.order_dn = take(tile_order_bytes(c, BM, (int)ceil_div64(c.H, 256)));
    w.act = take(P * c.I * 2);
    if (fp8) {
        w.xq = take((size_t)c.T * c.H);
        w.sx = take((size_t)c.T * 4);
        w.sxp = take(P * 4);
        w.act_q = take(P * c.I);
        w.sa = take(P * 4);
    }
    w.total = o;
    return w;
}

// sxp[p] = sx[perm[p] / K]: the scale of the x row behind sorted row p
__global__ __launch_bounds__(256) void gather_row_scales_kernel(const float* __restrict__ sx,
                                                               const int32_t* __restrict__ perm,
                                                               int K, int P, float* __restrict__ sxp) {
    const int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p < P) sxp[p] = sx[perm[p] / K];
}

// bf16: 16 x 16 blocks pay when a tile has enough K steps for the K loop to dominate (measured:
// +3.5 % at 64 steps, +2 % at 32, +2.5 % at 24, -2 % at 12)
inline bool use_blk16(int kt) { return kt >= 16; }

template <int MODE>
int32_t launch_kernel(bool fp8, const MfmaArgs& args, dim3 grid, hipStream_t s) {
    if (fp8) ffn_mfma_kernel<MODE, true, 32><<<grid, THREADS, LDS_BYTES, s>>>(args);
    else if (use_blk16(args.KT)) ffn_mfma_kernel<MODE, false, 16><<<grid, THREADS, LDS_BYTES, s>>>(args);
    else ffn_mfma_kernel<MODE, false, 32><<<grid, THREADS, LDS_BYTES, s>>>(args);
    return launch_status();
}

template <int MODE, bool FP8, int BLK>
bool allow_lds() {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(&ffn_mfma_kernel<MODE, FP8, BLK>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES) == hipSuccess;
}
template <bool FP8>
int32_t set_kernel_attributes() {
    bool ok = allow_lds<MODE_GATE_UP, FP8, 32>() && allow_lds<MODE_DOWN, FP8, 32>();
    if (!FP8) ok = ok && allow_lds<MODE_GATE_UP, false, 16>() && allow_lds<MODE_DOWN, false, 16>();
    return ok ? MOE_OK : MOE_ERR_LAUNCH_FAILED;
}

}  // namespace

int32_t ffn_mfma_set_attributes() {
    if (set_kernel_attributes<false>() != MOE_OK || set_kernel_attributes<true>() != MOE_OK)
        return MOE_ERR_LAUNCH_FAILED;
    return MOE_OK;
}

size_t ffn_mfma_ws_bytes(const moe_config_t& c) { return ffn_ws_layout(c).total; }

int32_t launch_ffn_mfma(const moe_config_t& c, const void* x, const int32_t* perm,
                        const int32_t* offsets, const void* wg, const void* wu, const void* wd,
                        const float* s_gate, const float* s_up, const float* s_down, void* act_tap,
                        uint8_t* act_q_tap, float* act_scale_tap, float* y_perm, int16_t* y_codes,
                        uint8_t* y_exps, void* ws, hipStream_t s) {
    const bool fp8 = c.w_dtype == MOE_DTYPE_FP8_E4M3;
    if (!fp8 && c.w_dtype != MOE_DTYPE_BF16) return MOE_ERR_UNSUPPORTED;
    const int64_t P = (int64_t)c.T * c.K;
    if (P == 0) return MOE_OK;
    const int esz = fp8 ? 1 : 2;                // bytes per operand element
    const int kstep = 128 / esz;                // elements per 128-byte K step
    // the K loop runs in pairs of 128-byte steps; 32-bit byte offsets are used on the load side;
    // column tiles are packed in 8 bits
    if (c.H % (2 * kstep) != 0 || c.I % (2 * kstep) != 0) return MOE_ERR_BAD_SHAPE;
    if ((uint64_t)c.T * c.H * esz > 0xFFFFFFFFull || (uint64_t)c.I * c.H * esz > 0xFFFFFFFFull ||
        c.I > 128 * 256 || c.H > 256 * 256)
        return MOE_ERR_UNSUPPORTED;

    const FfnWs w = ffn_ws_layout(c);
    char* ws8 = static_cast<char*>(ws);
    int32_t* table = reinterpret_cast<int32_t*>(ws8 + w.table);
    int32_t* first = reinterpret_cast<int32_t*>(ws8 + w.first);
    int4* order_gu = reinterpret_cast<int4*>(ws8 + w.order_gu);
    int4* order_dn = reinterpret_cast<int4*>(ws8 + w.order_dn);
    char* act = act_tap ? static_cast<char*>(act_tap) : ws8 + w.act;
    const int nct_gu = (int)ceil_div64(c.I, 128), nct_dn = (int)ceil_div64(c.H, 256);
    int32_t st = launch_build_tile_table(c, offsets, BM, table, first, s);
    if (st != MOE_OK) return st;
    st = launch_build_tile_order(c, first, offsets, BM, nct_gu, GROUP_ROWS, GROUP_COLS, order_gu, s);
    if (st != MOE_OK) return st;
    st = launch_build_tile_order(c, first, offsets, BM, nct_dn, GROUP_ROWS, GROUP_COLS, order_dn, s);
    if (st != MOE_OK) return st;

    // one persistent workgroup per compute unit (the kernels use all 160 KB of its LDS)
    const DeviceState* dev_state = nullptr;
    st = device_state(&dev_state);
    if (st != MOE_OK) return st;
    const int n_cu = dev_state->n_cu;
    const unsigned grid = (unsigned)((n_cu + 7) / 8 * 8);

    // fp8: quantise the x rows once per token, and carry each sorted row's scale along
    const char* a_gu = static_cast<const char*>(x);
    uint8_t* act_q = nullptr;
    float *sxp = nullptr, *sa = nullptr;
    if (fp8) {
        uint8_t* xq = reinterpret_cast<uint8_t*>(ws8 + w.xq);
        float* sx = reinterpret_cast<float*>(ws8 + w.sx);
        sxp = reinterpret_cast<float*>(ws8 + w.sxp);
        act_q = act_q_tap ? act_q_tap : reinterpret_cast<uint8_t*>(ws8 + w.act_q);
        sa = act_scale_tap ? act_scale_tap : reinterpret_cast<float*>(ws8 + w.sa);
        st = launch_quantize_rows(x, c.T, c.H, xq, sx, s);
        if (st != MOE_OK) return st;
        gather_row_scales_kernel<<<(unsigned)ceil_div64(P, 256), 256, 0, s>>>(sx, perm, c.K, (int)P, sxp);
        a_gu = reinterpret_cast<const char*>(xq);
    }

    MfmaArgs g{};
    g.A = a_gu;
    g.lda_bytes = (uint32_t)c.H * esz;
    g.perm = perm;
    g.kdiv = c.K;
    g.B0 = static_cast<const char*>(wg);
    g.B1 = static_cast<const char*>(wu);
    g.N = c.I;
    g.ldb_bytes = (uint32_t)c.H * esz;
    g.KT = c.H / kstep;
    g.sA = sxp;
    g.sB0 = s_gate;
    g.sB1 = s_up;
    g.table = table;
    g.order = order_gu;
    g.C = act;
    g.nct = nct_gu;
    {
        KernelBracket kb(MOE_KERNEL_GATE_UP, s);
        st = launch_kernel<MODE_GATE_UP>(fp8, g, grid, s);
    }
    if (st != MOE_OK) return st;
    const char* a_dn = act;
    if (fp8) {   // per-row e4m3 of the bf16 activations
        st = launch_quantize_rows(act, P, c.I, act_q, sa, s);
        if (st != MOE_OK) return st;
        a_dn = reinterpret_cast<const char*>(act_q);
    }
    MfmaArgs d{};
    d.A = a_dn;
    d.lda_bytes = (uint32_t)c.I * esz;
    d.perm = nullptr;
    d.kdiv = 1;
    d.B0 = static_cast<const char*>(wd);
    d.B1 = nullptr;
    d.N = c.H;
    d.ldb_bytes = (uint32_t)c.I * esz;
    d.KT = c.I / kstep;
    d.sA = sa;
    d.sB0 = s_down;
    d.sB1 = nullptr;
    d.table = table;
    d.order = order_dn;
    // y: block-scaled 16-bit codes for the fused call, the same values as float32 for a caller
    // that wants to see y, or the untouched float32 accumulators when the configuration asks
    if (y_codes) {
        d.C = reinterpret_cast<char*>(y_codes);
        d.Cs = y_exps;
        d.y_mode = Y_BLOCK16;
    } else {
        d.C = reinterpret_cast<char*>(y_perm);
        d.Cs = nullptr;
        d.y_mode = (c.flags & MOE_FLAG_Y_F32) ? Y_EXACT_F32 : Y_BLOCK16_AS_F32;
    }
    d.nct = nct_dn;
    {
        KernelBracket kb(MOE_KERNEL_DOWN, s);
        st = launch_kernel<MODE_DOWN>(fp8, d, grid, s);
    }
    return st;
}

}  // namespace moe
