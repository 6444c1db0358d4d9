// Grouping of the T*K routed rows by expert: histogram, exclusive scan and a stable counting
// sort (the token permutation/alignment step that Sec. 4.3 of the paper places on every
// layer's critical path).  No result depends on the order in which waves or atomics run.
//
// The flat ids 0..P-1 are cut into segments of SEG ids, one workgroup each:
//   1. seg_hist[s][e]  = rows of expert e in segment s          (LDS integer histogram)
//   2. seg_base[s][e]  = offsets[e] + sum_{s'<s} seg_hist[s'][e] (one workgroup, columns in
//                        parallel), plus counts and offsets
//   3. every segment ranks its ids stably: wave w of the workgroup owns a contiguous slice,
//      lanes with the same expert find their rank among themselves with ballots, and a
//      per-wave running counter in LDS carries the rank from one 64-id round to the next.
#include "common.h"

namespace moe {

constexpr int SEG = 2048;          // flat ids per workgroup
constexpr int PERM_THREADS = 256;  // 4 waves, 512 ids each
constexpr int PERM_WAVES = PERM_THREADS / WAVE;
constexpr int MAX_E = 1024;

// Expert ids come from the caller; an id outside [0,E) is folded into range so that no index
// derived from it can leave the buffers (the grouping is then meaningless, not unsafe).
__device__ __forceinline__ int safe_expert(int e, int E) { return e < 0 ? 0 : (e >= E ? E - 1 : e); }

size_t permute_ws_bytes(const moe_config_t& c) {
    const int64_t P = (int64_t)c.T * c.K;
    const int64_t nseg = ceil_div64(P, SEG);
    return align_up(sizeof(int32_t) * (size_t)(nseg > 0 ? nseg : 1) * c.E, 256);
}

__global__ __launch_bounds__(PERM_THREADS) void seg_hist_kernel(const int32_t* __restrict__ idx,
                                                               int P, int E,
                                                               int32_t* __restrict__ seg_hist) {
    __shared__ int32_t h[MAX_E];
    for (int e = threadIdx.x; e < E; e += PERM_THREADS) h[e] = 0;
    __syncthreads();
    const int base = blockIdx.x * SEG;
    for (int i = threadIdx.x; i < SEG; i += PERM_THREADS) {
        const int f = base + i;
        if (f < P) atomicAdd(&h[safe_expert(idx[f], E)], 1);
    }
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += PERM_THREADS) seg_hist[(size_t)blockIdx.x * E + e] = h[e];
}

// One workgroup of 1024 threads, C = 1024 / E' of them per expert column (E' = E rounded up to a
// power of two): thread (c, e) owns a contiguous chunk of segments.  Chunk sums -> column totals
// -> offsets over experts -> every thread rewrites its chunk as running positions.  All loads of
// a chunk are independent of each other, so the walk is not a chain of memory latencies.
__global__ __launch_bounds__(1024) void seg_scan_kernel(int32_t* __restrict__ seg_hist, int nseg,
                                                       int E, int32_t* __restrict__ counts,
                                                       int32_t* __restrict__ offsets) {
    __shared__ int32_t part[1024];        // chunk sums, [c][e] with row length EP
    __shared__ int32_t off[MAX_E + 1];
    int EP = 1;
    while (EP < E) EP <<= 1;
    const int C = 1024 / EP;              // chunks per column (>= 1 since E <= 1024)
    const int e = threadIdx.x & (EP - 1), c = threadIdx.x / EP;
    const int per = (nseg + C - 1) / C;
    const int s0 = min(c * per, nseg), s1 = min(s0 + per, nseg);
    int32_t sum = 0;
    if (e < E)
        for (int s = s0; s < s1; ++s) sum += seg_hist[(size_t)s * E + e];
    part[threadIdx.x] = sum;
    __syncthreads();
    // exclusive scan over the chunks of a column (C <= 1024 / 1, short), column total in off[]
    int32_t before = 0, total = 0;
    if (e < E) {
        for (int cc = 0; cc < C; ++cc) {
            const int32_t v = part[cc * EP + e];
            if (cc < c) before += v;
            total += v;
        }
    }
    __syncthreads();
    if (c == 0 && e < E) part[e] = total;   // column totals
    __syncthreads();
    if (threadIdx.x == 0) {
        int32_t acc = 0;
        for (int i = 0; i < E; ++i) {
            off[i] = acc;
            acc += part[i];
        }
        off[E] = acc;
    }
    __syncthreads();
    if (e < E) {
        if (c == 0) {
            counts[e] = part[e];
            offsets[e] = off[e];
        }
        int32_t run = off[e] + before;
        for (int s = s0; s < s1; ++s) {
            const int32_t v = seg_hist[(size_t)s * E + e];
            seg_hist[(size_t)s * E + e] = run;
            run += v;
        }
    }
    if (threadIdx.x == 0) offsets[E] = off[E];
}

__global__ __launch_bounds__(PERM_THREADS) void seg_scatter_kernel(
    const int32_t* __restrict__ idx, int P, int E, const int32_t* __restrict__ seg_base,
    int32_t* __restrict__ perm, int32_t* __restrict__ inv_perm) {
    __shared__ int32_t cur[PERM_WAVES][MAX_E];   // next free position per (wave, expert)
    const int wave = threadIdx.x / WAVE, lane = threadIdx.x % WAVE;
    constexpr int SLICE = SEG / PERM_WAVES;
    const int seg0 = blockIdx.x * SEG;
    const int w0 = seg0 + wave * SLICE;

    for (int e = lane; e < E; e += WAVE) cur[wave][e] = 0;
    __syncthreads();
    // per-wave histogram of its slice
    for (int i = lane; i < SLICE; i += WAVE) {
        const int f = w0 + i;
        if (f < P) atomicAdd(&cur[wave][safe_expert(idx[f], E)], 1);
    }
    __syncthreads();
    // exclusive scan over the waves, on top of the segment's base
    for (int e = threadIdx.x; e < E; e += PERM_THREADS) {
        int32_t run = seg_base[(size_t)blockIdx.x * E + e];
#pragma unroll
        for (int w = 0; w < PERM_WAVES; ++w) {
            const int32_t v = cur[w][e];
            cur[w][e] = run;
            run += v;
        }
    }
    __syncthreads();
    const uint64_t below = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
    for (int r = 0; r < SLICE; r += WAVE) {
        const int f = w0 + r + lane;
        const bool live = f < P;
        const int e = live ? safe_expert(idx[f], E) : 0;
        // lanes that hold the same expert id as this lane
        uint64_t same = __ballot(live);
#pragma unroll
        for (int b = 0; b < 10; ++b) {
            const uint64_t m = __ballot((e >> b) & 1);
            same &= ((e >> b) & 1) ? m : ~m;
        }
        const int rank = __popcll(same & below);
        const int cnt = __popcll(same);
        int pos = 0;
        if (live) {
            pos = cur[wave][e] + rank;
            perm[pos] = f;
            inv_perm[f] = pos;
        }
        __syncthreads();
        if (live && rank == cnt - 1) cur[wave][e] = pos + 1;
        __syncthreads();
    }
}

int32_t launch_permute(const moe_config_t& c, const int32_t* topk_idx, int32_t* counts,
                       int32_t* offsets, int32_t* perm, int32_t* inv_perm, void* ws,
                       hipStream_t s) {
    const int64_t P = (int64_t)c.T * c.K;
    const int nseg = (int)ceil_div64(P, SEG);
    int32_t* seg = static_cast<int32_t*>(ws);
    KernelBracket kb(MOE_KERNEL_PERMUTE, s);
    if (nseg > 0) seg_hist_kernel<<<nseg, PERM_THREADS, 0, s>>>(topk_idx, (int)P, c.E, seg);
    seg_scan_kernel<<<1, 1024, 0, s>>>(seg, nseg, c.E, counts, offsets);
    if (nseg > 0)
        seg_scatter_kernel<<<nseg, PERM_THREADS, 0, s>>>(topk_idx, (int)P, c.E, seg, perm, inv_perm);
    return launch_status();
}

// x_perm[p,:] = x[perm[p]/K,:]; one workgroup per sorted row, 16 bytes per lane and step.
__global__ __launch_bounds__(256) void gather_rows_kernel(const uint4* __restrict__ x,
                                                         const int32_t* __restrict__ perm, int K,
                                                         int row_vec, uint4* __restrict__ xp) {
    const int p = blockIdx.x;
    const int t = perm[p] / K;
    const uint4* src = x + (size_t)t * row_vec;
    uint4* dst = xp + (size_t)p * row_vec;
    for (int i = threadIdx.x; i < row_vec; i += blockDim.x) dst[i] = src[i];
}

__global__ __launch_bounds__(256) void gather_rows_bytes_kernel(const uint8_t* __restrict__ x,
                                                               const int32_t* __restrict__ perm,
                                                               int K, int64_t row_bytes,
                                                               uint8_t* __restrict__ xp) {
    const int p = blockIdx.x;
    const int t = perm[p] / K;
    for (int64_t i = threadIdx.x; i < row_bytes; i += blockDim.x)
        xp[(size_t)p * row_bytes + i] = x[(size_t)t * row_bytes + i];
}

int32_t launch_gather_rows(const moe_config_t& c, const void* x, const int32_t* perm, void* x_perm,
                           hipStream_t s) {
    const int64_t P = (int64_t)c.T * c.K;
    if (P == 0) return MOE_OK;
    const int64_t row_bytes = (int64_t)c.H * (c.x_dtype == MOE_DTYPE_F32 ? 4 : 2);
    const bool vec = (row_bytes % 16 == 0) && ((uintptr_t)x % 16 == 0) && ((uintptr_t)x_perm % 16 == 0);
    if (vec)
        gather_rows_kernel<<<(unsigned)P, 256, 0, s>>>(static_cast<const uint4*>(x), perm, c.K,
                                                      (int)(row_bytes / 16),
                                                      static_cast<uint4*>(x_perm));
    else
        gather_rows_bytes_kernel<<<(unsigned)P, 256, 0, s>>>(static_cast<const uint8_t*>(x), perm,
                                                            c.K, row_bytes,
                                                            static_cast<uint8_t*>(x_perm));
    return launch_status();
}

}  // namespace moe
