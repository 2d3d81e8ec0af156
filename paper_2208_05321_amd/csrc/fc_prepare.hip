// cache_prepare: Algorithm 1 of the paper (PrepareCache + PrepareCPURowIdxOnGPU, Section 4.3) as a short
// chain of gfx950 kernels.
//
// The paper's prototype strings together framework calls (unique, isin, nonzero, index_fill, argsort,
// index_copy).  Here the same decisions come out of two rank-space bitmaps and popcount scans, with no sort:
//   ubits  rows used by this batch        -> unique() is "which bits are set", ascending for free
//   rbits  rows resident in HBM           -> missing = ubits & ~rbits, evictable = rbits & ~ubits
// and the empty slots are read off the slot->rank map: the i-th missing rank takes the i-th empty slot.
// The victims of Section 4.3 (LFU by static frequency rank: of the rows the batch does not use, the evict_num with
// the largest cpu_row_idx) are the top evict_num set bits of (rbits & ~ubits): a suffix count over bitmap tiles finds the threshold tile.
#include "fc_internal.h"

#include <omp.h>
#include <string.h>

namespace fc {

// ---------------------------------------------------------------------------------------------------------
// K1  ids -> frequency rank (idx_map lookup), mark the rank in ubits, count access-level hits, check offsets.
//
// Frequent ids are by construction the LOW ranks, and they are the ones repeated thousands of times in a
// batch.  Device-scope atomics on one address serialise at the memory side (~100 ns each on this part), so
// the low end of rank space is first marked in a per-workgroup LDS bitmap (fast LDS atomics) and merged into
// the global bitmap once per workgroup; only the long tail of rare ranks goes to global atomics directly.
// At most MARK_MAX_BLOCKS workgroups run, so a hot word sees at most that many global atomics.
// ---------------------------------------------------------------------------------------------------------
constexpr int MARK_THREADS = 1024;
constexpr int MARK_LDS_WORDS = 12288;      // 48 KB: ranks below 393,216
constexpr int MARK_MAX_BLOCKS = 256;

__global__ __launch_bounds__(MARK_THREADS) void k_remap_mark(const int64_t* __restrict__ ids, int n,
                                                             const int64_t* __restrict__ offsets, int num_bags,
                                                             const int32_t* __restrict__ freq_rank, int64_t N,
                                                             uint32_t* ubits, const uint32_t* __restrict__ rbits,
                                                             int32_t* __restrict__ rbuf, Ctl* ctl,
                                                             int32_t* __restrict__ hitpart, int per_block,
                                                             int lds_words) {
    __shared__ uint32_t low[MARK_LDS_WORDS];
    __shared__ int red[MARK_THREADS / 64];
    const int tid = threadIdx.x;
    for (int w = tid; w < lds_words; w += MARK_THREADS) low[w] = 0;
    __syncthreads();
    const int64_t work = n > num_bags + 1 ? n : num_bags + 1;
    const int64_t begin = (int64_t)blockIdx.x * per_block;
    const int64_t end = begin + per_block < work ? begin + per_block : work;
    int hits = 0;
    uint32_t flags = 0;
    // four ids per thread and round: all loads of a stage are issued before any of them is waited for
    for (int64_t i0 = begin + tid; i0 < end; i0 += 4 * MARK_THREADS) {
        int64_t id[4];
        int r[4];
        uint32_t rb[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int64_t i = i0 + (int64_t)k * MARK_THREADS;
            id[k] = (i < end && i < n) ? ids[i] : 0;
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int64_t i = i0 + (int64_t)k * MARK_THREADS;
            r[k] = -1;
            if (i < end && i < n) {
                if (id[k] < 0 || id[k] >= N) flags |= EF_ID_RANGE;
                else r[k] = freq_rank[id[k]];
            }
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) rb[k] = r[k] >= 0 ? rbits[(uint32_t)r[k] >> 5] : 0u;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int64_t i = i0 + (int64_t)k * MARK_THREADS;
            if (i < end && i < n) {
                if (r[k] >= 0) {
                    const uint32_t w = (uint32_t)r[k] >> 5, bit = 1u << (r[k] & 31);
                    if (w < (uint32_t)lds_words) atomicOr(&low[w], bit);
                    // rare ranks: bits are only ever set during this kernel, so a read that sees the bit is final
                    else if (!(ubits[w] & bit)) atomicOr(&ubits[w], bit);
                    hits += (rb[k] & bit) != 0;
                }
                rbuf[i] = r[k];
            }
            if (i < end && i <= num_bags) {
                const int64_t o = offsets[i];
                if (o != i) flags |= EF_NOT_ONE_PER_BAG;
                if (i == 0 && o != 0) flags |= EF_BAD_OFFSETS;
                if (i == num_bags && o != (int64_t)n) flags |= EF_BAD_OFFSETS;
                if (i < num_bags && offsets[i + 1] < o) flags |= EF_BAD_OFFSETS;
            }
        }
    }
    __syncthreads();
    // Merge into the global bitmap: LDS words first, then all global reads at once, then the atomics still needed.
    // Every workgroup holds the hottest words, so each starts at a different word: by the time most of them reach a
    // hot word its bits are already set and the (coherent) read spares the atomic.
    const int rot = (int)(((int64_t)blockIdx.x * lds_words) / gridDim.x);
    constexpr int FL = MARK_LDS_WORDS / MARK_THREADS;
    uint32_t v[FL], g[FL];
    int wi[FL];
#pragma unroll
    for (int k = 0; k < FL; ++k) {
        int w = k * MARK_THREADS + tid;
        v[k] = 0;
        if (w < lds_words) {
            w += rot;
            if (w >= lds_words) w -= lds_words;
            v[k] = low[w];
        }
        wi[k] = w;
    }
#pragma unroll
    for (int k = 0; k < FL; ++k)
        g[k] = v[k] ? __hip_atomic_load(&ubits[wi[k]], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0xFFFFFFFFu;
#pragma unroll
    for (int k = 0; k < FL; ++k)
        if (v[k] & ~g[k]) atomicOr(&ubits[wi[k]], v[k]);
    hits = wave_sum(hits);
    if ((tid & 63) == 0) red[tid >> 6] = hits;
    __syncthreads();
    if (tid == 0) {
        int s = 0;
#pragma unroll
        for (int k = 0; k < MARK_THREADS / 64; ++k) s += red[k];
        hitpart[blockIdx.x] = s;
    }
    if (flags) atomicOr(&ctl->err_flags, flags);
}

// ---------------------------------------------------------------------------------------------------------
// K2a  per rank-space tile: rows used, rows missing, rows evictable.
//      On the way (DMA evict transmitter): the block that this batch's victims will go to has reached the host table, so
//      rows still marked as in transit in it become plain "not resident" (what k_clear_transit does; folded in here
//      because nothing before K3 reads rank_slot, and a launch of its own lengthened the index chain).
// ---------------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(RT_THREADS) void k_rank_count(const uint4* __restrict__ ubits4,
                                                           const uint4* __restrict__ rbits4,
                                                           const uint4* __restrict__ pbits4, int protect_prev,
                                                           int32_t* __restrict__ bsum, int NB,
                                                           const int32_t* __restrict__ landed_ranks, int landed, int landed_base,
                                                           int32_t* rank_slot) {
    __shared__ int lds[3][RT_THREADS / 64];
    for (int j = blockIdx.x * RT_THREADS + threadIdx.x; j < landed; j += gridDim.x * RT_THREADS) {
        const int r = landed_ranks[j];
        if (rank_slot[r] == -2 - (landed_base + j)) rank_slot[r] = -1;
    }
    const size_t idx = (size_t)blockIdx.x * RT_THREADS + threadIdx.x;
    const uint4 u = ubits4[idx];
    uint4 r = rbits4[idx];
    const int cm0 = __popc(u.x & ~r.x) + __popc(u.y & ~r.y) + __popc(u.z & ~r.z) + __popc(u.w & ~r.w);
    if (protect_prev) {        // look-ahead: rows of the previously prepared batch are not evictable either
        const uint4 p = pbits4[idx];
        r.x &= ~p.x; r.y &= ~p.y; r.z &= ~p.z; r.w &= ~p.w;
    }
    int cu = __popc(u.x) + __popc(u.y) + __popc(u.z) + __popc(u.w);
    int cm = cm0;
    int cc = __popc(r.x & ~u.x) + __popc(r.y & ~u.y) + __popc(r.z & ~u.z) + __popc(r.w & ~u.w);
    cu = wave_sum(cu); cm = wave_sum(cm); cc = wave_sum(cc);
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    if (lane == 0) { lds[0][w] = cu; lds[1][w] = cm; lds[2][w] = cc; }
    __syncthreads();
    if (threadIdx.x < 3) {
        int s = 0;
#pragma unroll
        for (int k = 0; k < RT_THREADS / 64; ++k) s += lds[threadIdx.x][k];
        bsum[(size_t)threadIdx.x * NB + blockIdx.x] = s;
    }
}

// ---------------------------------------------------------------------------------------------------------
// K2b  one workgroup: totals, the call's status, evict_num = numel(miss) - empty slots, output offsets of
//      every tile's missing ranks, and which tiles give up how many victims (from the top rank down).
//      (Tried: letting the last workgroup of K2a to finish do this, found by an atomic ticket.  One ticket per tile on
//      one address costs about 100 ns each on this part, 300 us at 3052 tiles: slower than the launch it saves.)
// ---------------------------------------------------------------------------------------------------------
// 256 threads: a workgroup this small finds room on a compute unit at once; a 1024-thread one waited up to 200 us for
// sixteen free wave slots beside the previous batch's forward kernel, with the host waiting for its ticket.
constexpr int PLAN_THREADS = 256;
constexpr int PLAN_ITEMS = 4;
__global__ __launch_bounds__(PLAN_THREADS) void k_rank_plan(const int32_t* __restrict__ bsum, int NB, int C, Ctl* ctl,
                                                    HostCtl* hctl, int32_t* __restrict__ moff,
                                                    int32_t* __restrict__ vtake, int32_t* __restrict__ voff,
                                                    const int32_t* __restrict__ hitpart, int nmark, int ticket) {
    __shared__ int lds[PLAN_THREADS / 64];
    const int tid = threadIdx.x;
    constexpr int CH = PLAN_THREADS * PLAN_ITEMS;          // tiles per round: PLAN_ITEMS consecutive ones per thread
    int hits;
    (void)block_excl_scan<PLAN_THREADS>(tid < nmark ? hitpart[tid] : 0, hits, lds);   // nmark <= 256
    // forward: output offset of every tile's missing ranks; the totals of used and evictable rows on the way
    int carryM = 0, accU = 0, accC = 0;
    for (int base = 0; base < NB; base += CH) {
        const int b0 = base + tid * PLAN_ITEMS;
        int m[PLAN_ITEMS], sum = 0;
#pragma unroll
        for (int k = 0; k < PLAN_ITEMS; ++k) {
            const int b = b0 + k;
            m[k] = b < NB ? bsum[(size_t)NB + b] : 0;
            if (b < NB) { accU += bsum[b]; accC += bsum[(size_t)2 * NB + b]; }
            sum += m[k];
        }
        int tot;
        int run = carryM + block_excl_scan<PLAN_THREADS>(sum, tot, lds);
#pragma unroll
        for (int k = 0; k < PLAN_ITEMS; ++k)
            if (b0 + k < NB) { moff[b0 + k] = run; run += m[k]; }
        carryM += tot;
    }
    int totU, totC;
    (void)block_excl_scan<PLAN_THREADS>(accU, totU, lds);
    (void)block_excl_scan<PLAN_THREADS>(accC, totC, lds);
    const uint32_t ef = ctl->err_flags;
    const int nfree = ctl->nfree;
    int status = FC_OK;
    if (ef & EF_BAD_OFFSETS) status = FC_ERR_BAD_OFFSETS;
    else if (ef & EF_ID_RANGE) status = FC_ERR_ID_OUT_OF_RANGE;
    else if (totU > C) status = FC_ERR_BATCH_EXCEEDS_CACHE;
    const int M = carryM;
    int need = M - nfree;
    if (need < 0) need = 0;
    // enough evictable rows?  (always, unless the look-ahead protects the previous batch as well)
    if (status == FC_OK && need > totC) status = FC_ERR_BATCH_EXCEEDS_CACHE;
    if (status != FC_OK) need = 0;
    // Victims: walk tiles from the highest ranks down; `above` = evictable rows in tiles of larger rank.
    int carry = 0;
    for (int base = 0; base < NB; base += CH) {
        const int r0 = base + tid * PLAN_ITEMS;            // position counted from the top tile
        int cc[PLAN_ITEMS], sum = 0;
#pragma unroll
        for (int k = 0; k < PLAN_ITEMS; ++k) {
            const int b = NB - 1 - (r0 + k);
            cc[k] = b >= 0 ? bsum[(size_t)2 * NB + b] : 0;
            sum += cc[k];
        }
        int tot;
        int above = carry + block_excl_scan<PLAN_THREADS>(sum, tot, lds);
#pragma unroll
        for (int k = 0; k < PLAN_ITEMS; ++k) {
            const int b = NB - 1 - (r0 + k);
            if (b >= 0) {
                int take = 0, off = 0;
                if (above < need && cc[k] > 0) {
                    take = min(cc[k], need - above);
                    off = need - above - take;   // victims are listed in ascending rank
                }
                vtake[b] = take;
                voff[b] = off;
                above += cc[k];
            }
        }
        carry += tot;
    }
    __syncthreads();
    if (tid == 0) {
        ctl->status = status;
        ctl->n_unique = totU;
        ctl->n_miss = M;
        ctl->need = need;
        const int nf = status == FC_OK ? nfree + need - M : nfree;
        ctl->nfree = nf;
        ctl->err_flags = 0;
        hctl->status = status; hctl->n_unique = totU; hctl->n_miss = M; hctl->need = need;
        hctl->hit_ids = hits; hctl->nfree = nf; hctl->async_flags = (int32_t)ctl->async_flags;
        hctl->batch_flags = (int32_t)(ef & EF_NOT_ONE_PER_BAG);
        __threadfence_system();                       // the record first, then the ticket the host is polling for
        *reinterpret_cast<volatile int32_t*>(&hctl->ticket) = ticket;
    }
}

constexpr int FREE_TILE = 1024;

// ---------------------------------------------------------------------------------------------------------
// K2c  per tile: write the missing ranks (ascending), pick and retire the victims, update rbits, clear ubits.
// ---------------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(RT_THREADS) void k_rank_emit(uint4* ubits4, uint4* rbits4, uint4* pbits4, int protect_prev,
                                                          const Ctl* __restrict__ ctl,
                                                          const int32_t* __restrict__ moff,
                                                          const int32_t* __restrict__ vtake,
                                                          const int32_t* __restrict__ voff,
                                                          int32_t* __restrict__ miss_ranks, int32_t* __restrict__ vrank,
                                                          int32_t* __restrict__ vslot, int32_t* rank_slot,
                                                          int32_t* slot_rank, int C, int transit_base,
                                                          int transit_rows, int32_t* __restrict__ fill_src) {
    __shared__ int lds[RT_THREADS / 64];
    const size_t idx = (size_t)blockIdx.x * RT_THREADS + threadIdx.x;
    const uint4 u4 = ubits4[idx];
    const bool anyu = (u4.x | u4.y | u4.z | u4.w) != 0;
    if (ctl->status != FC_OK) {            // failed call: forget the marks, touch nothing else
        if (anyu) ubits4[idx] = make_uint4(0, 0, 0, 0);
        return;
    }
    const uint4 r4 = rbits4[idx];
    const uint4 p4 = pbits4[idx];
    const uint32_t uw[4] = {u4.x, u4.y, u4.z, u4.w};
    const uint32_t rw[4] = {r4.x, r4.y, r4.z, r4.w};
    const uint32_t pw[4] = {protect_prev ? p4.x : 0u, protect_prev ? p4.y : 0u, protect_prev ? p4.z : 0u, protect_prev ? p4.w : 0u};
    uint32_t mw[4], cw[4], vw[4] = {0, 0, 0, 0};
    int cm = 0, cc = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        mw[k] = uw[k] & ~rw[k];
        cw[k] = rw[k] & ~uw[k] & ~pw[k];
        cm += __popc(mw[k]);
        cc += __popc(cw[k]);
    }
    const int rank0 = (int)(idx * 128);
    int totm;
    const int pm = block_excl_scan<RT_THREADS>(cm, totm, lds);
    if (cm) {
        int o = moff[blockIdx.x] + pm;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            uint32_t word = mw[k];
            while (word) {
                const int bit = __ffs(word) - 1;
                const int rank = rank0 + k * 32 + bit;
                // where the row's newest copy is: -1 the host table, <= -2 an evicted-row block (in transit)
                if (fill_src) fill_src[o] = rank_slot[rank];
                miss_ranks[o++] = rank;
                word &= word - 1;
            }
        }
    }
    const int vt = vtake[blockIdx.x];
    if (vt > 0) {
        int totc;
        const int pc = block_excl_scan<RT_THREADS>(cc, totc, lds);
        const bool transit = transit_base >= 0 && ctl->need <= transit_rows;
        const int skip = totc - vt;          // the lowest `skip` evictable ranks of the threshold tile stay
        const int o0 = voff[blockIdx.x];
        int q = pc;
        if (cc && pc + cc > skip) {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                uint32_t word = cw[k];
                while (word) {
                    const int bit = __ffs(word) - 1;
                    if (q >= skip) {
                        const int rank = rank0 + k * 32 + bit;
                        const int slot = rank_slot[rank];
                        const int j = o0 + q - skip;
                        vrank[j] = rank;
                        vslot[j] = slot;
                        // not resident any more; with the DMA evict transmitter the newest copy of the row is
                        // "in transit" in row j of an evicted-row block until the host threads have stored it
                        rank_slot[rank] = transit ? -2 - (transit_base + j) : -1;
                        if ((unsigned)slot < (unsigned)C) slot_rank[slot] = -1;   // always true: the maps are inverse
                        vw[k] |= 1u << bit;
                    }
                    ++q;
                    word &= word - 1;
                }
            }
        }
    }
    if (cm || (vw[0] | vw[1] | vw[2] | vw[3]))
        rbits4[idx] = make_uint4((rw[0] & ~vw[0]) | mw[0], (rw[1] & ~vw[1]) | mw[1], (rw[2] & ~vw[2]) | mw[2],
                                 (rw[3] & ~vw[3]) | mw[3]);
    if (anyu) ubits4[idx] = make_uint4(0, 0, 0, 0);
    if (anyu || (p4.x | p4.y | p4.z | p4.w)) pbits4[idx] = u4;     // this batch is the "previous" one next time
}

// ---------------------------------------------------------------------------------------------------------
// K6  the i-th missing rank takes the i-th lowest empty slot; both index maps are updated.
//     a) empty slots per tile of FREE_TILE slots;  b) each tile ranks its empty slots after the tiles below it.
// ---------------------------------------------------------------------------------------------------------
// 256 threads with 4 consecutive slots each: a workgroup this small finds room on a compute unit at once, also while
// the forward / backward kernels of the previous batch fill the chip (cache_plan_next)
constexpr int FREE_THREADS = 256;
constexpr int FREE_PER = FREE_TILE / FREE_THREADS;

// bit k set: slot s0 + k is empty
__device__ __forceinline__ unsigned empty_mask(const int32_t* __restrict__ slot_rank, int s0, int C) {
    unsigned m = 0;
    if (s0 + FREE_PER <= C) {
        const int4 v = *reinterpret_cast<const int4*>(slot_rank + s0);
        m = (v.x == -1 ? 1u : 0u) | (v.y == -1 ? 2u : 0u) | (v.z == -1 ? 4u : 0u) | (v.w == -1 ? 8u : 0u);
    } else {
        for (int k = 0; k < FREE_PER; ++k) if (s0 + k < C && slot_rank[s0 + k] == -1) m |= 1u << k;
    }
    return m;
}

__global__ __launch_bounds__(FREE_THREADS) void k_free_count(const int32_t* __restrict__ slot_rank, int C,
                                                             int32_t* __restrict__ tcount) {
    static_assert(FREE_PER == 4, "empty_mask reads four slots at a time");
    __shared__ int red[FREE_THREADS / 64];
    const int s0 = blockIdx.x * FREE_TILE + threadIdx.x * FREE_PER;
    const int e = __popc(empty_mask(slot_rank, s0, C));
    const int w = wave_sum(e);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = w;
    __syncthreads();
    if (threadIdx.x == 0) {
        int t = 0;
#pragma unroll
        for (int k = 0; k < FREE_THREADS / 64; ++k) t += red[k];
        tcount[blockIdx.x] = t;
    }
}

__global__ __launch_bounds__(FREE_THREADS) void k_free_assign(int32_t* slot_rank, int C, const int32_t* __restrict__ tcount,
                                                              int M, const int32_t* __restrict__ miss_ranks,
                                                              int32_t* __restrict__ fill_slots, int32_t* rank_slot) {
    __shared__ int lds[FREE_THREADS / 64];
    int part = 0;
    for (int g = threadIdx.x; g < (int)blockIdx.x; g += FREE_THREADS) part += tcount[g];
    int base;
    (void)block_excl_scan<FREE_THREADS>(part, base, lds);
    if (base >= M) return;                                   // all missing rows were placed in lower tiles
    const int s0 = blockIdx.x * FREE_TILE + threadIdx.x * FREE_PER;
    const unsigned m = empty_mask(slot_rank, s0, C);
    int tot;
    int j = base + block_excl_scan<FREE_THREADS>(__popc(m), tot, lds);
    for (int k = 0; k < FREE_PER; ++k) {
        if (!((m >> k) & 1u)) continue;
        if (j >= M) break;
        const int s = s0 + k;
        const int r = miss_ranks[j];
        fill_slots[j] = s;
        slot_rank[s] = r;
        rank_slot[r] = s;
        ++j;
    }
}

// ---------------------------------------------------------------------------------------------------------
// FC_DIRTY_TRACK: of the victims (vrank[j], vslot[j]), j < need, keep those whose slot is dirty, in order.
//     a) dirty victims per tile of DIRTY_TILE victims;  b) each tile writes its dirty victims after those of the
//     tiles before it, clears the dirty flags of all its victims, and (DMA evict transmitter) marks the kept rows as
//     in transit at their place in the block; the last tile reports the total to the host.
// ---------------------------------------------------------------------------------------------------------
constexpr int DIRTY_TILE = 1024;
constexpr int DIRTY_THREADS = 256;
constexpr int DIRTY_PER = DIRTY_TILE / DIRTY_THREADS;

__global__ __launch_bounds__(DIRTY_THREADS) void k_dirty_count(const int32_t* __restrict__ vslot, int need, int C,
                                                              const uint8_t* __restrict__ dirty, int32_t* __restrict__ dcount) {
    __shared__ int red[DIRTY_THREADS / 64];
    const int j0 = blockIdx.x * DIRTY_TILE + threadIdx.x * DIRTY_PER;
    int e = 0;
    for (int k = 0; k < DIRTY_PER; ++k) {
        const int j = j0 + k;
        if (j < need) { const int s = vslot[j]; if ((unsigned)s < (unsigned)C && dirty[s]) ++e; }
    }
    const int w = wave_sum(e);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = w;
    __syncthreads();
    if (threadIdx.x == 0) {
        int t = 0;
#pragma unroll
        for (int k = 0; k < DIRTY_THREADS / 64; ++k) t += red[k];
        dcount[blockIdx.x] = t;
    }
}

__global__ __launch_bounds__(DIRTY_THREADS) void k_dirty_keep(const int32_t* __restrict__ vrank, const int32_t* __restrict__ vslot,
                                                             int need, int C, uint8_t* dirty, const int32_t* __restrict__ dcount,
                                                             int32_t* __restrict__ out_rank, int32_t* __restrict__ out_slot,
                                                             int32_t* rank_slot, int transit_base, int32_t* dctl, int ticket) {
    __shared__ int lds[DIRTY_THREADS / 64];
    int part = 0;
    for (int g = threadIdx.x; g < (int)blockIdx.x; g += DIRTY_THREADS) part += dcount[g];
    int base;
    (void)block_excl_scan<DIRTY_THREADS>(part, base, lds);
    const int j0 = blockIdx.x * DIRTY_TILE + threadIdx.x * DIRTY_PER;
    unsigned m = 0;
    int sl[DIRTY_PER];
    for (int k = 0; k < DIRTY_PER; ++k) {
        const int j = j0 + k;
        sl[k] = -1;
        if (j < need) {
            const int s = vslot[j];
            if ((unsigned)s < (unsigned)C) { sl[k] = s; if (dirty[s]) m |= 1u << k; }
        }
    }
    int tot;
    int o = base + block_excl_scan<DIRTY_THREADS>(__popc(m), tot, lds);
    for (int k = 0; k < DIRTY_PER; ++k) {
        if (sl[k] < 0) continue;
        if ((m >> k) & 1u) {
            const int r = vrank[j0 + k];
            out_rank[o] = r;
            out_slot[o] = sl[k];
            if (transit_base >= 0) rank_slot[r] = -2 - (transit_base + o);
            ++o;
        }
        dirty[sl[k]] = 0;                  // the slot is empty now; whatever is loaded next equals its host copy
    }
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) {
        dctl[0] = base + tot;
        __threadfence_system();
        *reinterpret_cast<volatile int32_t*>(&dctl[1]) = ticket;   // the count first, then the ticket the host polls for
    }
}

// DMA evict transmitter: the host threads have stored block `base / staging_rows`; rows still marked as in transit
// in that block are plain "not resident" again (a row re-fetched or re-evicted meanwhile carries another value).
__global__ __launch_bounds__(256) void k_clear_transit(const int32_t* __restrict__ ranks, int count, int base,
                                                       int32_t* rank_slot) {
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j < count) {
        const int r = ranks[j];
        if (rank_slot[r] == -2 - (base + j)) rank_slot[r] = -1;
    }
}

// K8  gpu_row_idx of every input id.
__global__ __launch_bounds__(256) void k_slots_out(const int32_t* __restrict__ rbuf,
                                                   const int32_t* __restrict__ rank_slot, int32_t* __restrict__ slots,
                                                   int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) slots[i] = rank_slot[rbuf[i]];
}

// ---------------------------------------------------------------------------------------------------------
int ensure_rbuf(fc_cache* c, int64_t n) {
    if (n <= c->n_cap) return FC_OK;
    FC_HIP(hipDeviceSynchronize());
    if (c->rbuf) FC_HIP(hipFree(c->rbuf));
    c->rbuf = nullptr; c->n_cap = 0;
    const int64_t cap = n + n / 4 + 1024;
    FC_HIP(hipMalloc((void**)&c->rbuf, (size_t)cap * 4));
    c->n_cap = cap;
    return FC_OK;
}

// Evicted rows, default transmitter: gather into a device block on the caller's stream (so the slots can be
// refilled at once); the block is stored into the mapped host table by a kernel on the side stream.
// Measured on MI355X: zero-copy stores that saturate the host link stall the other memory operations of the
// compute units they run on and starve reads in the other direction, so such a store must not run under small
// latency-bound kernels (they wait for it to end) nor under the forward / backward kernels (they slow down
// several-fold).  Default schedule (evict_early == 2): the store starts together with the miss fill, once all
// index kernels are done, and the caller's stream waits for it right after the fill; the two then share the
// link (the store finishes first, the fill catches up) and everything after runs undisturbed.
// Blocks before the last are stored at once because the one block buffer must be free again for the next gather.
static int store_block(fc_cache* c, int64_t off, int64_t rows) {
    FC_HIP(hipEventRecord(c->ev_gather_done, c->pst));
    FC_HIP(hipStreamWaitEvent(c->side, c->ev_gather_done, 0));
    FC_TRY(launch_copy_rows(c, c->side, P_EVICT_STORE, c->host_dev, c->out_rank + off, c->N, c->stage_dev, nullptr, c->staging_rows, rows, c->evict_blocks));
    FC_HIP(hipEventRecord(c->ev_evict_done, c->side));
    c->evict_pending = true;
    return FC_OK;
}

static int evict_direct(fc_cache* c, int64_t need, int64_t* last_off, int64_t* last_rows) {
    const int64_t S = c->staging_rows;
    for (int64_t off = 0; off < need; off += S) {
        const int64_t rows = need - off < S ? need - off : S;
        if (off > 0) FC_HIP(hipStreamWaitEvent(c->pst, c->ev_evict_done, 0));   // block buffer is being read
        FC_TRY(launch_copy_rows(c, c->pst, P_EVICT_GATHER, c->stage_dev, nullptr, c->staging_rows, c->cache, c->out_slot + off, c->C, rows, 1 << 20));
        if (off + rows >= need && c->evict_early != 1) { *last_off = off; *last_rows = rows; break; }
        FC_TRY(store_block(c, off, rows));
    }
    return FC_OK;
}

// DMA evict transmitter: wait until every handed-over block is in the host table and drop all transit marks
// (afterwards the host table alone is current for every non-resident row, and all blocks are free).
int dma_quiesce(fc_cache* c, hipStream_t st) {
    if (!c->dma_evict) return FC_OK;
    pool_wait(c, pool_published(c));
    for (int b = 0; b < DMA_BLOCKS; ++b) {
        if (c->blk_rows[b] > 0) {
            k_clear_transit<<<(unsigned)cdiv(c->blk_rows[b], 256), 256, 0, st>>>(c->vrank_buf[b], (int)c->blk_rows[b],
                                                                                       (int)(b * c->staging_rows), c->rank_slot);
            c->blk_rows[b] = 0;
        }
    }
    FC_HIP(hipGetLastError());
    // the index kernels of a later batch read and write the same map entries, possibly on another stream
    FC_HIP(hipEventRecord(c->ev_quiesce, st));
    c->quiesce_stream = st;
    return FC_OK;
}

// DMA evict transmitter: gather into block `buf`, hand the block and its rank list to the DMA engine on the side
// stream, and let the host threads scatter it once it has landed.  Nothing on the caller's stream waits for it.
static int evict_dma(fc_cache* c, int64_t need, int buf) {
    float* blk = c->stage_dev + (size_t)buf * c->staging_rows * c->D;
    FC_TRY(launch_copy_rows(c, c->pst, P_EVICT_GATHER, blk, nullptr, c->staging_rows, c->cache, c->out_slot, c->C, need, 1 << 20));
    FC_HIP(hipEventRecord(c->ev_gather_done, c->pst));
    FC_HIP(hipStreamWaitEvent(c->side, c->ev_gather_done, 0));
    {
        ProfScope ps(c, P_D2H_BLOCK, c->side);
        if (c->ev_copy_a[buf]) FC_HIP(hipEventRecord(c->ev_copy_a[buf], c->side));
        FC_HIP(hipMemcpyAsync(c->vrank_pin[buf], c->out_rank, (size_t)need * 4, hipMemcpyDeviceToHost, c->side));
        FC_HIP(hipMemcpyAsync(c->blk_pin[buf], blk, (size_t)need * c->D * 4, hipMemcpyDeviceToHost, c->side));
        if (c->ev_copy_b[buf]) { FC_HIP(hipEventRecord(c->ev_copy_b[buf], c->side)); c->copy_timed[buf] = true; c->last_copy_buf = buf; }
    }
    FC_HIP(hipEventRecord(c->ev_d2h[buf], c->side));
    c->blk_rows[buf] = need;
    pool_publish(c, buf, need);
    return FC_OK;
}

// The paper's transmitter: block on the source side -> one bulk copy -> scatter on the target side.
static int evict_staged(fc_cache* c, int64_t need, const int32_t* vrank_host) {
    const int64_t S = c->staging_rows;
    const size_t rowb = (size_t)c->D * 4;
    for (int64_t off = 0; off < need; off += S) {
        const int64_t rows = need - off < S ? need - off : S;
        FC_TRY(launch_copy_rows(c, c->pst, P_EVICT_GATHER, c->stage_dev, nullptr, c->staging_rows, c->cache, c->out_slot + off, c->C, rows, 1 << 20));
        {
            ProfScope ps(c, P_D2H_BLOCK, c->pst);
            FC_HIP(hipMemcpyAsync(c->stage_pin, c->stage_dev, rows * rowb, hipMemcpyDeviceToHost, c->pst));
        }
        FC_HIP(hipStreamSynchronize(c->pst));
        float* host = c->host; const float* blk = c->stage_pin; const int32_t* vr = vrank_host + off;
#pragma omp parallel for schedule(static)
        for (int64_t j = 0; j < rows; ++j) memcpy(host + (size_t)vr[j] * c->D, blk + (size_t)j * c->D, rowb);
    }
    return FC_OK;
}

static int fill_staged(fc_cache* c, int64_t M, const int32_t* miss_host) {
    const int64_t S = c->staging_rows;
    const size_t rowb = (size_t)c->D * 4;
    for (int64_t off = 0; off < M; off += S) {
        const int64_t rows = M - off < S ? M - off : S;
        const float* host = c->host; float* blk = c->stage_pin; const int32_t* mr = miss_host + off;
#pragma omp parallel for schedule(static)
        for (int64_t j = 0; j < rows; ++j) memcpy(blk + (size_t)j * c->D, host + (size_t)mr[j] * c->D, rowb);
        {
            ProfScope ps(c, P_H2D_BLOCK, c->pst);
            FC_HIP(hipMemcpyAsync(c->stage_dev2, c->stage_pin, rows * rowb, hipMemcpyHostToDevice, c->pst));
        }
        FC_TRY(launch_copy_rows(c, c->pst, P_MISS_FILL, c->cache, c->fill_slots + off, c->C, c->stage_dev2, nullptr, c->staging_rows, rows, 1 << 20));
        FC_HIP(hipStreamSynchronize(c->pst));   // the pinned block is reused by the next round
    }
    return FC_OK;
}

// A kernel writes a small record into pinned host memory and, last, a ticket; the host polls for the ticket (cheaper
// than an event round trip, and the kernels enqueued behind it keep the GPU busy meanwhile).  Falls back to the
// stream's status so that a failed launch cannot hang the caller.
static int wait_for_ticket(const volatile int32_t* ticket_word, int32_t ticket, hipStream_t st) {
    uint64_t spins = 0;
    while (*ticket_word != ticket) {
        __builtin_ia32_pause();
        if ((++spins & 0x3FFF) == 0) {
            const hipError_t q = hipStreamQuery(st);
            if (q == hipSuccess) break;                          // stream drained: the record is there
            if (q != hipErrorNotReady) { (void)hipGetLastError(); return FC_ERR_HIP; }
        }
    }
    __atomic_thread_fence(__ATOMIC_ACQUIRE);
    return *ticket_word == ticket ? FC_OK : FC_ERR_HIP;
}

// Index half of Algorithm 1: every decision (unique rows, misses, victims, slot assignment, both maps, the slots
// of the batch) and no row movement.  Fills *mv with what prepare_move has to do.
int launch_slots_out(fc_cache* c, hipStream_t st, int32_t* slots, int64_t n) {
    if (n > 0) {
        ProfScope ps(c, P_SLOTS_OUT, st);
        k_slots_out<<<(unsigned)cdiv(n, 256), 256, 0, st>>>(c->rbuf, c->rank_slot, slots, (int)n);
    }
    FC_HIP(hipGetLastError());
    return FC_OK;
}

// before_slots: an event the slot write-out (the first kernel that writes the caller's buffer) has to wait for.
// defer_slots: leave the slot write-out and the ev_index_done record to the caller (who folds the write-out into the sort).
int prepare_index(fc_cache* c, hipStream_t st, bool lookahead, const int64_t* ids, int64_t n, const int64_t* offsets,
                  int64_t num_bags, int32_t* slots, MovePlan* mv, hipEvent_t before_slots, bool defer_slots) {
    const int64_t LIM = ((int64_t)1 << 31) - 65536;
    if (!c || n < 0 || num_bags < 0 || n >= LIM || num_bags >= LIM || !offsets || (n > 0 && (!ids || !slots)))
        return FC_ERR_INVALID_ARG;
    FC_HIP(hipSetDevice(c->device));
    FC_TRY(ensure_rbuf(c, n));
    c->pst = st;
    // the list set this call rewrites (missing ranks, victims, fill slots) was last read by the row movement two
    // batches back, possibly on another stream
    use_list_set(c, c->lset ^ 1);
    c->have_lists = false;
    if (c->move_stream[c->lset] && c->move_stream[c->lset] != st) FC_HIP(hipStreamWaitEvent(st, c->ev_move_done[c->lset], 0));
    if (c->last_index_stream && c->last_index_stream != st) FC_HIP(hipStreamWaitEvent(st, c->ev_index_done, 0));
    if (c->quiesce_stream && c->quiesce_stream != st) FC_HIP(hipStreamWaitEvent(st, c->ev_quiesce, 0));
    c->quiesce_stream = nullptr;
    const int32_t ticket = c->ticket = (c->ticket + 1) & 0x7fffffff;
    const int protect_prev = lookahead ? 1 : 0;
    int transit_base = -1, buf = 0;
    int64_t landed = 0;
    if (c->dma_evict) {
        // the block this call may fill was handed over DMA_BLOCKS blocks ago: its rows must be in the host table by now
        const uint64_t seq = pool_published(c) + 1;
        buf = (int)(seq % DMA_BLOCKS);
        if (seq > DMA_BLOCKS) pool_wait(c, seq - DMA_BLOCKS);
        landed = c->blk_rows[buf];            // cleared by k_rank_count below, before anything reads rank_slot or rewrites the list
        c->blk_rows[buf] = 0;
        if (!c->dirty_track) c->vrank = c->vrank_buf[buf];
        transit_base = (int)(buf * c->staging_rows);
    }
    const int64_t work = n > num_bags + 1 ? n : num_bags + 1;
    int64_t nmark = cdiv(work, (int64_t)c->mark_ids_per_thread * MARK_THREADS);
    if (nmark > MARK_MAX_BLOCKS) nmark = MARK_MAX_BLOCKS;
    const int64_t per_block = cdiv(cdiv(work, nmark), MARK_THREADS) * MARK_THREADS;
    nmark = cdiv(work, per_block);
    const int64_t words = c->NB * RT_WORDS;
    {
        ProfScope ps(c, P_REMAP_MARK, st);
        k_remap_mark<<<(unsigned)nmark, MARK_THREADS, 0, st>>>(ids, (int)n, offsets, (int)num_bags, c->freq_rank, c->N, c->ubits,
                                                              c->rbits, c->rbuf, c->ctl, c->hitpart, (int)per_block,
                                                              (int)(words < MARK_LDS_WORDS ? words : MARK_LDS_WORDS));
    }
    {
        ProfScope ps(c, P_RANK_COUNT, st);
        k_rank_count<<<(unsigned)c->NB, RT_THREADS, 0, st>>>((const uint4*)c->ubits, (const uint4*)c->rbits, (const uint4*)c->pbits,
                                                            protect_prev, c->bsum, (int)c->NB,
                                                            c->dma_evict ? c->vrank_buf[buf] : nullptr, (int)landed,
                                                            (int)(buf * c->staging_rows), c->rank_slot);
    }
    {
        ProfScope ps(c, P_RANK_PLAN, st);
        k_rank_plan<<<1, PLAN_THREADS, 0, st>>>(c->bsum, (int)c->NB, (int)c->C, c->ctl, c->hctl, c->moff, c->vtake, c->voff, c->hitpart, (int)nmark, ticket);
    }
    // Last batch's evicted rows must have reached the host table before the victim lists and the block buffer
    // are reused and before any of those rows could be fetched again; the kernels above do not care.
    if (c->evict_pending) {
        FC_HIP(hipStreamWaitEvent(st, c->ev_evict_done, 0));
        c->evict_pending = false;
    }
    {
        ProfScope ps(c, P_RANK_EMIT, st);
        k_rank_emit<<<(unsigned)c->NB, RT_THREADS, 0, st>>>((uint4*)c->ubits, (uint4*)c->rbits, (uint4*)c->pbits, protect_prev, c->ctl,
                                                           c->moff, c->vtake, c->voff,
                                                           c->miss_ranks, c->vrank, c->vslot, c->rank_slot, c->slot_rank, (int)c->C,
                                                           c->dirty_track ? -1 : transit_base, (int)c->staging_rows,
                                                           c->dma_evict ? c->fill_src : nullptr);
    }
    FC_HIP(hipEventRecord(c->ev_emit_done, st));
    FC_HIP(hipGetLastError());
    // the planning kernel's decision
    HostCtl h;
    {
        const volatile int32_t* hv = reinterpret_cast<const volatile int32_t*>(c->hctl);
        FC_TRY(wait_for_ticket(hv + 8, ticket, st));
        h.status = hv[0]; h.n_unique = hv[1]; h.n_miss = hv[2]; h.need = hv[3]; h.hit_ids = hv[4]; h.nfree = hv[5];
        h.async_flags = hv[6]; h.batch_flags = hv[7]; h.ticket = hv[8];
    }
    if (h.status != FC_OK) return h.status;
    c->last_one_per_bag = n == num_bags && !(h.batch_flags & (int32_t)EF_NOT_ONE_PER_BAG);
    const int64_t M = h.n_miss, need = h.need;
    if (M > 0) {
        {
            const unsigned tiles = (unsigned)cdiv(c->C, FREE_TILE);
            {
                ProfScope ps(c, P_FREE_COUNT, st);
                k_free_count<<<tiles, FREE_THREADS, 0, st>>>(c->slot_rank, (int)c->C, c->tcount);
            }
            ProfScope ps(c, P_FREE_PICK, st);
            k_free_assign<<<tiles, FREE_THREADS, 0, st>>>(c->slot_rank, (int)c->C, c->tcount, (int)M, c->miss_ranks, c->fill_slots,
                                                      c->rank_slot);
        }
    }
    FC_HIP(hipEventRecord(c->ev_assign_done, st));
    // every row of the batch has its slot now: write the slots out (the caller then starts sorting them for the
    // backward pass on a library stream, where the sort runs while the missing rows cross the host link)
    if (before_slots) FC_HIP(hipStreamWaitEvent(st, before_slots, 0));
    if (!defer_slots) {
        FC_TRY(launch_slots_out(c, st, slots, n));
        FC_HIP(hipEventRecord(c->ev_index_done, st));
    }
    c->last_index_stream = st;
    c->aux = (st == c->pre && !lookahead) ? c->pre : c->pf;
    mv->valid = true; mv->M = M; mv->need = need; mv->buf = buf; mv->transit_base = transit_base;
    c->last.n_ids = n;
    c->last.n_unique = h.n_unique;
    c->last.n_hit_unique = h.n_unique - M;
    c->last.n_hit_ids = h.hit_ids;
    c->last.n_miss = M;
    c->last.n_evict = need;
    c->last.bytes_h2d = M * (int64_t)c->D * 4;
    c->last.bytes_d2h = need * (int64_t)c->D * 4;
    c->have_lists = true;
    return FC_OK;
}

// Row-movement half: evicted rows out (gather, then DMA block / kernel store / staged copy), missing rows in.
int prepare_move(fc_cache* c, hipStream_t st, const MovePlan& mv) {
    c->pst = st;
    // the lists this half reads are complete once the last decision is taken; the slot write-out (and, folded into it,
    // the sort) is waited for by whoever hands the batch to the caller
    if (c->last_index_stream != st) FC_HIP(hipStreamWaitEvent(st, c->ev_assign_done, 0));
    const int64_t M = mv.M;
    int64_t need = mv.need;                    // victims to write back
    const bool staged = (c->flags & FC_TRANSMIT_STAGED) != 0;
    c->out_rank = c->vrank; c->out_slot = c->vslot;
    if (c->dirty_track && need > 0) {
        // keep the dirty victims only; their number decides the size of the copies below, so the host waits for it
        const bool dma_block = c->dma_evict && need <= c->staging_rows;
        int32_t* orank = dma_block ? c->vrank_buf[mv.buf] : c->lists[c->lset][5];
        int32_t* oslot = c->lists[c->lset][6];
        const unsigned tiles = (unsigned)cdiv(need, DIRTY_TILE);
        const int32_t ticket = c->dticket = (c->dticket + 1) & 0x7fffffff;
        k_dirty_count<<<tiles, DIRTY_THREADS, 0, st>>>(c->vslot, (int)need, (int)c->C, c->dirty, c->dcount);
        k_dirty_keep<<<tiles, DIRTY_THREADS, 0, st>>>(c->vrank, c->vslot, (int)need, (int)c->C, c->dirty, c->dcount, orank, oslot,
                                                     c->rank_slot, dma_block ? mv.transit_base : -1, c->dctl, ticket);
        FC_HIP(hipGetLastError());
        const volatile int32_t* dv = reinterpret_cast<const volatile int32_t*>(c->dctl);
        FC_TRY(wait_for_ticket(dv + 1, ticket, st));
        need = dv[0];
        c->out_rank = orank; c->out_slot = oslot;
        c->last.bytes_d2h = need * (int64_t)c->D * 4;
    }
    if (staged && (M > 0 || need > 0)) {
        if (M > 0) FC_HIP(hipMemcpyAsync(c->list_pin, c->miss_ranks, (size_t)M * 4, hipMemcpyDeviceToHost, st));
        if (need > 0) FC_HIP(hipMemcpyAsync(c->list_pin + c->C, c->out_rank, (size_t)need * 4, hipMemcpyDeviceToHost, st));
        FC_HIP(hipStreamSynchronize(st));
    }
    int64_t last_off = 0, last_rows = 0;
    // Rows fetched ahead of time (cache_plan_next) were read from the host table and from evicted-row blocks other
    // than the one this batch's victims go to (its marks were dropped before this batch was indexed), so the
    // victims need not wait for them; a kernel-store evict reuses the block buffer from its start and has to.
    bool arrival_waited = !mv.arrived;
    bool dma_path = false;
    // DMA miss path: ev_arrive of this list set is recorded by a gather thread once it has handed the last chunk to the
    // DMA engine; the host waits here until that has happened (the GPU meanwhile works through the current batch)
    const bool via_dma = mv.arrived && c->gather_pending;
    if (via_dma) { FC_TRY(gather_wait(c)); c->gather_pending = false; }
    if (need > 0) {
        if (staged) FC_TRY(evict_staged(c, need, c->list_pin + c->C));
        else if (c->dma_evict && mv.need <= c->staging_rows) { FC_TRY(evict_dma(c, need, mv.buf)); dma_path = true; }
        else {
            // more victims than one block holds (or no DMA transmitter): store by kernel, block by block; the
            // block buffer is reused from its start, so nothing may be in transit in it any more
            if (!arrival_waited) { FC_HIP(hipStreamWaitEvent(st, c->ev_arrive[c->lset], 0)); arrival_waited = true; }
            FC_TRY(dma_quiesce(c, st));
            FC_TRY(evict_direct(c, need, &last_off, &last_rows));
        }
    } else if (c->dma_evict) dma_path = true;
    if (M > 0) {
        if (last_rows > 0 && c->evict_early == 2) {       // store and fill share the link, then the link falls silent
            FC_TRY(store_block(c, last_off, last_rows));
            last_rows = -1;
        }
        if (!arrival_waited) FC_HIP(hipStreamWaitEvent(st, c->ev_arrive[c->lset], 0));
        if (staged) FC_TRY(fill_staged(c, M, c->list_pin));
        else if (mv.arrived) {
            FC_TRY(launch_copy_rows(c, st, P_ROWS_IN, c->cache, c->fill_slots, c->C, c->arrive[c->lset], nullptr, c->staging_rows, M, 1 << 20));
            // DMA miss path: rows in transit did not come over the link; their newest copies are in evicted-row blocks
            // gathered by earlier batches (this stream has run those gathers)
            if (via_dma && c->dma_evict) FC_TRY(launch_fill_rows(c, st, M, nullptr, 0, 0, true));
        }
        else if (c->dma_evict) FC_TRY(launch_fill_rows(c, st, M));
        else FC_TRY(launch_copy_rows(c, st, P_MISS_FILL, c->cache, c->fill_slots, c->C, c->host_dev, c->miss_ranks, c->N, M, c->fill_blocks));
    }
    if (last_rows > 0) FC_TRY(store_block(c, last_off, last_rows));
    if (last_rows < 0) { FC_HIP(hipStreamWaitEvent(st, c->ev_evict_done, 0)); c->evict_pending = false; }
    FC_HIP(hipGetLastError());
    FC_HIP(hipEventRecord(c->ev_move_done[c->lset], st));
    c->move_stream[c->lset] = st;
    // The next early fetch reads evicted-row blocks gathered up to now and host rows stored up to now: with the DMA
    // transmitter the gather just enqueued is the last thing it needs (host rows still on their way carry transit
    // marks); after a kernel store it has to wait for the whole movement.
    if (!dma_path) c->pf_dep = c->ev_move_done[c->lset];
    else if (need > 0) c->pf_dep = c->ev_gather_done;
    return FC_OK;
}

int prepare_impl(fc_cache* c, hipStream_t st, bool lookahead, const int64_t* ids, int64_t n, const int64_t* offsets,
                 int64_t num_bags, int32_t* slots) {
    MovePlan mv;
    FC_TRY(prepare_index(c, st, lookahead, ids, n, offsets, num_bags, slots, &mv));
    // Look-ahead: rows about to be evicted or overwritten may still be in use by work the caller enqueued before
    // this call (the backward pass of the batch before the current one); the index decisions did not care.
    if (n > 0) (void)presort_impl(c, slots, n, offsets, num_bags);   // on failure the backward pass sorts (and reports) itself
    if (lookahead) FC_HIP(hipStreamWaitEvent(st, c->ev_s_now, 0));
    return prepare_move(c, st, mv);
}

}  // namespace fc
