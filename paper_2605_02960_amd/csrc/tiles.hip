// Row-tile table of the ragged per-expert groups, built on the device from `offsets` so that
// the host never has to read the routing result.  Expert e with c_e rows contributes
// ceil(c_e / bm) tiles; tiles are listed expert by expert.
#include "common.h"

namespace moe {

__global__ __launch_bounds__(1024) void build_tile_table_kernel(const int32_t* __restrict__ offsets,
                                                               int E, int bm,
                                                               int32_t* __restrict__ table) {
    __shared__ int32_t first[1024 + 1];
    const int e = threadIdx.x;
    int32_t n = 0, o = 0;
    if (e < E) {
        o = offsets[e];
        n = (offsets[e + 1] - o + bm - 1) / bm;
        first[e] = n;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int32_t acc = 0;
        for (int i = 0; i < E; ++i) {
            const int32_t v = first[i];
            first[i] = acc;
            acc += v;
        }
        first[E] = acc;
        table[0] = acc;
    }
    __syncthreads();
    if (e < E) {
        const int32_t t0 = first[e];
        for (int i = 0; i < n; ++i) {
            table[1 + 2 * (t0 + i)] = e;
            table[2 + 2 * (t0 + i)] = o + i * bm;
        }
    }
}

int32_t launch_build_tile_table(const moe_config_t& c, const int32_t* offsets, int bm,
                                int32_t* table, hipStream_t s) {
    build_tile_table_kernel<<<1, 1024, 0, s>>>(offsets, c.E, bm, table);
    return launch_status();
}

}  // namespace moe
