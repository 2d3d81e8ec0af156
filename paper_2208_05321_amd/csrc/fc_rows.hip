// Row movement: one row-group of lanes per embedding row, 16-byte accesses where dim allows.
// Used for the evict gather, the host-table store of evicted rows, the miss fill and the flush
// (paper Section 4.3, "data transmitter": rows scattered in one memory become a block in the other).
#include "fc_internal.h"

namespace fc {

template <int VEC> struct Vec;
template <> struct Vec<1> { using T = float; };
template <> struct Vec<2> { using T = float2; };
template <> struct Vec<4> { using T = float4; };
__device__ __forceinline__ float nt_load_row(const float* p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ float2 nt_load_row(const float2* p) { return make_float2(__builtin_nontemporal_load(&p->x), __builtin_nontemporal_load(&p->y)); }
__device__ __forceinline__ float4 nt_load_row(const float4* p) {
    typedef float v4f __attribute__((ext_vector_type(4)));
    const v4f t = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(p));
    return make_float4(t.x, t.y, t.z, t.w);
}

// dst[dst_idx ? dst_idx[j] : j] = src[src_idx ? src_idx[j] : j] for j in [0, rows); row length D floats.
// lpr (power of two, <= 64) consecutive lanes own one row; a lane moves VEC floats per access.
// KIND only names the instantiation (profilers then tell the three uses apart): 0 evicted-row gather (HBM -> HBM
// block), 1 evicted-row store (block -> host table), 2 miss fill (host table -> cache slots, or block -> slots).
template <int VEC, int KIND>
__global__ __launch_bounds__(256) void k_copy_rows(float* __restrict__ dst, const int32_t* __restrict__ dst_idx,
                                                   unsigned dst_rows, const float* __restrict__ src,
                                                   const int32_t* __restrict__ src_idx, unsigned src_rows, int rows,
                                                   int D, int lpr_shift) {
    using V = typename Vec<VEC>::T;
    const int lpr = 1 << lpr_shift;
    const int gpb = blockDim.x >> lpr_shift;
    const int gl = threadIdx.x >> lpr_shift, lane = threadIdx.x & (lpr - 1);
    const int nv = D / VEC;
    for (int j = blockIdx.x * gpb + gl; j < rows; j += gridDim.x * gpb) {
        const int di = dst_idx ? dst_idx[j] : j;
        const int si = src_idx ? src_idx[j] : j;
        if ((unsigned)di >= dst_rows || (unsigned)si >= src_rows) continue;   // never true for lists this library builds
        const V* __restrict__ s = reinterpret_cast<const V*>(src + (size_t)si * D);
        V* __restrict__ d = reinterpret_cast<V*>(dst + (size_t)di * D);
        // the evicted rows and the rows of an arrival block are read for the last time here: non-temporal loads keep them
        // from displacing the cached rows in the memory-side cache
        for (int cidx = lane; cidx < nv; cidx += lpr) d[cidx] = KIND == 1 ? s[cidx] : nt_load_row(&s[cidx]);
    }
}

// Flush: every resident slot's row (with a dirty array: every dirty one) goes to its place in the host table.
template <int VEC>
__global__ __launch_bounds__(256) void k_flush_rows(float* __restrict__ host, const float* __restrict__ cache,
                                                    const int32_t* __restrict__ slot_rank, int C, int D, int lpr_shift,
                                                    const uint8_t* __restrict__ dirty) {
    using V = typename Vec<VEC>::T;
    const int lpr = 1 << lpr_shift;
    const int gpb = blockDim.x >> lpr_shift;
    const int gl = threadIdx.x >> lpr_shift, lane = threadIdx.x & (lpr - 1);
    const int nv = D / VEC;
    for (int s = blockIdx.x * gpb + gl; s < C; s += gridDim.x * gpb) {
        const int r = slot_rank[s];
        if (r < 0) continue;
        if (dirty && !dirty[s]) continue;
        const V* __restrict__ src = reinterpret_cast<const V*>(cache + (size_t)s * D);
        V* __restrict__ d = reinterpret_cast<V*>(host + (size_t)r * D);
        for (int cidx = lane; cidx < nv; cidx += lpr) d[cidx] = src[cidx];
    }
}

// Miss fill of the DMA evict transmitter: row j goes to slot fill_slots[j] (to row j if there is no such list); it
// comes from the host table, or, if its newest copy is still in transit (fill_src[j] <= -2), from the evicted-row
// block that holds it.
template <int VEC>
__global__ __launch_bounds__(256) void k_fill_rows(float* __restrict__ cache, const int32_t* __restrict__ fill_slots,
                                                   unsigned C, const float* __restrict__ host,
                                                   const int32_t* __restrict__ miss_ranks, unsigned N,
                                                   const float* __restrict__ blocks, const int32_t* __restrict__ fill_src,
                                                   unsigned block_rows, int rows, int D, int lpr_shift, int only_transit) {
    using V = typename Vec<VEC>::T;
    const int lpr = 1 << lpr_shift;
    const int gpb = blockDim.x >> lpr_shift;
    const int gl = threadIdx.x >> lpr_shift, lane = threadIdx.x & (lpr - 1);
    const int nv = D / VEC;
    // The three list entries of the NEXT row are requested before this row's data: each is a dependent access of a
    // microsecond or so, and a row-group that waits for them has no host read in flight.
    const int stride = gridDim.x * gpb;
    int j = blockIdx.x * gpb + gl;
    int di = 0, code = -1, r = 0;
    if (j < rows) { di = fill_slots ? fill_slots[j] : j; code = fill_src[j]; r = miss_ranks[j]; }
    while (j < rows) {
        const int jn = j + stride;
        int din = 0, coden = -1, rn = 0;
        if (jn < rows) { din = fill_slots ? fill_slots[jn] : jn; coden = fill_src[jn]; rn = miss_ranks[jn]; }
        const float* srow = nullptr;
        if (code <= -2) {
            const unsigned k = (unsigned)(-2 - code);
            if (k < block_rows) srow = blocks + (size_t)k * D;
        } else if (!only_transit && (unsigned)r < N) {
            srow = host + (size_t)r * D;
        }
        if (srow && (unsigned)di < C) {          // never false for lists this library builds
            const V* __restrict__ sv = reinterpret_cast<const V*>(srow);
            V* __restrict__ d = reinterpret_cast<V*>(cache + (size_t)di * D);
            for (int cidx = lane; cidx < nv; cidx += lpr) d[cidx] = sv[cidx];
        }
        j = jn; di = din; code = coden; r = rn;
    }
}

static inline int shift_of(int lpr) { int s = 0; while ((1 << s) < lpr) ++s; return s; }

int launch_copy_rows(fc_cache* c, hipStream_t s, int prof_item, float* dst, const int32_t* dst_idx, int64_t dst_rows,
                     const float* src, const int32_t* src_idx, int64_t src_rows, int64_t rows, int max_blocks) {
    if (rows <= 0) return FC_OK;
    const int sh = shift_of(c->lpr);
    const int gpb = 256 >> sh;
    int64_t blocks = cdiv(rows, gpb);
    if (blocks > max_blocks) blocks = max_blocks;
    ProfScope ps(c, prof_item, s);
#define FC_LAUNCH_ROWS(V, K) \
    k_copy_rows<V, K><<<(unsigned)blocks, 256, 0, s>>>(dst, dst_idx, (unsigned)dst_rows, src, src_idx, (unsigned)src_rows, (int)rows, c->D, sh)
#define FC_LAUNCH_ROWS_V(K) \
    switch (c->vec) { case 4: FC_LAUNCH_ROWS(4, K); break; case 2: FC_LAUNCH_ROWS(2, K); break; default: FC_LAUNCH_ROWS(1, K); break; }
    if (prof_item == P_EVICT_GATHER) { FC_LAUNCH_ROWS_V(0) }
    else if (prof_item == P_EVICT_STORE) { FC_LAUNCH_ROWS_V(1) }
    else { FC_LAUNCH_ROWS_V(2) }
#undef FC_LAUNCH_ROWS_V
#undef FC_LAUNCH_ROWS
    FC_HIP(hipGetLastError());
    return FC_OK;
}

int launch_fill_rows(fc_cache* c, hipStream_t s, int64_t rows, float* dst, int64_t dst_rows, int max_blocks, bool only_transit) {
    if (rows <= 0) return FC_OK;
    const int sh = shift_of(c->lpr);
    const int gpb = 256 >> sh;
    int64_t blocks = cdiv(rows, gpb);
    if (max_blocks <= 0) max_blocks = c->fill_blocks;
    if (blocks > max_blocks) blocks = max_blocks;
    ProfScope ps(c, P_MISS_FILL, s);
#define FC_FILL(V) \
    k_fill_rows<V><<<(unsigned)blocks, 256, 0, s>>>(dst ? dst : c->cache, dst ? nullptr : c->fill_slots, (unsigned)(dst ? dst_rows : c->C), \
                                                    c->host_dev, c->miss_ranks, (unsigned)c->N, \
                                                    c->stage_dev, c->fill_src, (unsigned)(DMA_BLOCKS * c->staging_rows), (int)rows, c->D, sh, only_transit ? 1 : 0)
    switch (c->vec) { case 4: FC_FILL(4); break; case 2: FC_FILL(2); break; default: FC_FILL(1); break; }
#undef FC_FILL
    FC_HIP(hipGetLastError());
    return FC_OK;
}

int launch_flush_rows(fc_cache* c, hipStream_t s) {
    const int sh = shift_of(c->lpr);
    const int gpb = 256 >> sh;
    int64_t blocks = cdiv(c->C, gpb);
    if (blocks > 8192) blocks = 8192;
    ProfScope ps(c, P_FLUSH_ROWS, s);
    switch (c->vec) {
        case 4: k_flush_rows<4><<<(unsigned)blocks, 256, 0, s>>>(c->host_dev, c->cache, c->slot_rank, (int)c->C, c->D, sh, c->dirty); break;
        case 2: k_flush_rows<2><<<(unsigned)blocks, 256, 0, s>>>(c->host_dev, c->cache, c->slot_rank, (int)c->C, c->D, sh, c->dirty); break;
        default: k_flush_rows<1><<<(unsigned)blocks, 256, 0, s>>>(c->host_dev, c->cache, c->slot_rank, (int)c->C, c->D, sh, c->dirty); break;
    }
    FC_HIP(hipGetLastError());
    return FC_OK;
}

}  // namespace fc
