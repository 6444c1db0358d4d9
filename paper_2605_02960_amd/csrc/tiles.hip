// Row-tile table of the ragged per-expert groups, built on the device from `offsets` so that
// the host never has to read the routing result.  Expert e with c_e rows contributes
// ceil(c_e / bm) tiles; tiles are listed expert by expert.
#include "common.h"

namespace moe {

__global__ __launch_bounds__(1024) void build_tile_table_kernel(const int32_t* __restrict__ offsets,
                                                               int E, int bm,
                                                               int32_t* __restrict__ table,
                                                               int32_t* __restrict__ first_out) {
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
    if (first_out) {
        // E + 1 entries; with E = 1024 the block has no thread for the last one
        if (e < E) first_out[e] = first[e];
        if (e == 0) first_out[E] = first[E];
    }
    if (e < E) {
        const int32_t t0 = first[e];
        for (int i = 0; i < n; ++i) {
            table[1 + 2 * (t0 + i)] = e;
            table[2 + 2 * (t0 + i)] = o + i * bm;
        }
    }
}

int32_t launch_build_tile_table(const moe_config_t& c, const int32_t* offsets, int bm,
                                int32_t* table, int32_t* first_out, hipStream_t s) {
    build_tile_table_kernel<<<1, 1024, 0, s>>>(offsets, c.E, bm, table, first_out);
    return launch_status();
}

// Launch order of the output tiles: one record (expert, first sorted row, end row, column tile)
// per launch slot.  Inside one expert, row tiles are taken in groups of `gr` and column tiles in
// groups of `gc`; a group of (up to) gr x gc tiles is listed row by row before the next column
// group starts.  Workgroups that run at the same time on one XCD therefore cover a compact block
// of the expert's output and share its token rows and weight rows in that XCD's L2.  An expert
// with a single row tile degenerates to column-fastest order (all its tiles share the token rows).
__global__ __launch_bounds__(256) void build_tile_order_kernel(const int32_t* __restrict__ first,
                                                              const int32_t* __restrict__ offsets, int bm,
                                                              int nct, int gr, int gc,
                                                              int4* __restrict__ order) {
    const int e = blockIdx.x;
    const int rt0 = first[e];
    const int n = first[e + 1] - rt0;
    const int row_begin = offsets[e], row_end = offsets[e + 1];
    const int total = n * nct;
    int4* out = order + (size_t)rt0 * nct;
    for (int i = threadIdx.x; i < total; i += blockDim.x) {
        const int g = i / (gr * nct);
        const int rem = i - g * gr * nct;
        const int gsz = min(gr, n - g * gr);
        const int cg = rem / (gc * gsz);
        const int rem2 = rem - cg * gc * gsz;
        const int gw = min(gc, nct - cg * gc);
        const int r = rem2 / gw;
        const int c = rem2 - r * gw;
        const int row0 = row_begin + (g * gr + r) * bm;
        out[i] = make_int4(e, row0, min(row_end, row0 + bm), cg * gc + c);
    }
}

int32_t launch_build_tile_order(const moe_config_t& c, const int32_t* first, const int32_t* offsets, int bm,
                                int nct, int gr, int gc, int4* order, hipStream_t s) {
    build_tile_order_kernel<<<c.E, 256, 0, s>>>(first, offsets, bm, nct, gr, gc, order);
    return launch_status();
}

}  // namespace moe
