// Stable LSD radix sort of (key, value) int32 pairs, 64-wide wavefronts, tiles of RS_TILE keys per workgroup.
// Used by the backward pass and the slot-order forward (sort lookups by slot, value = bag) and by the static-module
// build (sort ids by descending count).  Keys come from one of four sources, see SortSrc.  A pass is either
// count -> scan -> scatter (up to RS_MAX_BITS bits per digit) or, for batch-sized jobs with many key bits, count -> scatter
// with per-supertile sums in place of the scan (see radix_sort for which is chosen when).
#include "fc_internal.h"

#include <stdlib.h>

namespace fc {

// Jobs of up to FUSE_MAX_TILES tiles run without a scan kernel: k_sort_hist also adds the counts of SS_TILES neighbouring
// tiles up, and k_sort_scatter derives its offsets from those sums (digits of at most FUSE_MAX_BITS bits).
constexpr int SS_TILES = 32, FUSE_MAX_TILES = 2048, FUSE_MAX_BITS = 9;

// First-pass key of lookup i: its slot, or the sentinel C if the slot is out of range.
__device__ __forceinline__ int first_key(const int32_t* __restrict__ slots, int i, int C, bool& bad) {
    const int k = slots[i];
    if ((unsigned)k >= (unsigned)C) { bad = true; return C; }
    return k;
}

// bag of lookup i: the largest b with offsets[b] <= i
__device__ __forceinline__ int bag_of(const int64_t* __restrict__ offsets, int num_bags, int i) {
    int lo = 0, hi = num_bags;
    while (hi - lo > 1) {
        const int mid = (int)(((int64_t)lo + hi) >> 1);
        if (offsets[mid] <= i) lo = mid; else hi = mid;
    }
    return lo;
}

// key of element i by source (SORT_SRC_RANKS is turned into slots by k_sort_hist first)
template <int SRC>
__device__ __forceinline__ int load_key(const int32_t* __restrict__ keys_in, int i, int limit, bool& bad) {
    if (SRC == SORT_SRC_SLOTS) return first_key(keys_in, i, limit, bad);
    if (SRC == SORT_SRC_COUNTS) return limit - keys_in[i];      // limit = largest count: descending counts ascend
    return keys_in[i];
}

template <int SRC, int ITEMS>
__global__ __launch_bounds__(RS_THREADS) void k_sort_hist(const int32_t* __restrict__ keys_in, int n, int limit, int shift,
                                                          int radix_bits, int nblk, int32_t* __restrict__ ghist,
                                                          int32_t* __restrict__ stot,
                                                          uint32_t* flags, const int32_t* __restrict__ rank_slot,
                                                          int32_t* __restrict__ slots_out,
                                                          int32_t* __restrict__ zero_ptr, int zero_words) {
    __shared__ int h[1 << RS_MAX_BITS];
    if (zero_ptr) {     // what the previous sort left in the other set of supertile tables, a slice per workgroup
        const int per = (zero_words + (int)gridDim.x - 1) / (int)gridDim.x;
        const int z1 = min(zero_words, ((int)blockIdx.x + 1) * per);
        for (int i = (int)blockIdx.x * per + (int)threadIdx.x; i < z1; i += RS_THREADS) zero_ptr[i] = 0;
    }
    const int radix = 1 << radix_bits, mask = radix - 1;
    const int tile0 = blockIdx.x * (RS_THREADS * ITEMS);
    // all of the tile's keys are requested before anything waits for one (a lane beyond n rereads the last key)
    int key[ITEMS];
    bool bad = false;
    if (SRC == SORT_SRC_RANKS) {
        // gpu_row_idx of every input id (Algorithm 1's last index_select), written out on the way to becoming sort keys
        int r[ITEMS];
#pragma unroll
        for (int it = 0; it < ITEMS; ++it) r[it] = keys_in[min(tile0 + it * RS_THREADS + (int)threadIdx.x, n - 1)];
#pragma unroll
        for (int it = 0; it < ITEMS; ++it) key[it] = rank_slot[r[it]];
#pragma unroll
        for (int it = 0; it < ITEMS; ++it) {
            const int i = tile0 + it * RS_THREADS + (int)threadIdx.x;
            if (i < n) slots_out[i] = key[it];
            if ((unsigned)key[it] >= (unsigned)limit) { bad = true; key[it] = limit; }
        }
    } else
#pragma unroll
    for (int it = 0; it < ITEMS; ++it)
        key[it] = load_key<SRC>(keys_in, min(tile0 + it * RS_THREADS + (int)threadIdx.x, n - 1), limit, bad);
    for (int d = threadIdx.x; d < radix; d += RS_THREADS) h[d] = 0;
    __syncthreads();
#pragma unroll
    for (int it = 0; it < ITEMS; ++it)
        if (tile0 + it * RS_THREADS + (int)threadIdx.x < n) atomicAdd(&h[(key[it] >> shift) & mask], 1);
    __syncthreads();
    for (int d = threadIdx.x; d < radix; d += RS_THREADS) {
        const int cnt = h[d];
        ghist[(size_t)blockIdx.x * radix + d] = cnt;   // tile-major: one contiguous run per tile
        // counts of SS_TILES neighbouring tiles added up (the table starts at zero): the scatter kernel builds its
        // offsets from these and from the counts of the few tiles before it, and no scan kernel runs in between
        if (stot && cnt) atomicAdd(&stot[(size_t)(blockIdx.x / SS_TILES) * radix + d], cnt);
    }
    if (bad && flags) atomicOr(flags, EF_BAD_SLOT);
}

// Exclusive scan, per digit, of the per-tile counts over the tiles, in place; the digit totals go to dtot.
// The table is tile-major (ghist[tile * radix + digit]): a tile writes its counts, and reads its offsets back, as one
// contiguous run (digit-major, every one of those accesses touched a sector of its own: at 2048 digits x 832 tiles the
// two kernels around this one moved ten times the table).  Here a workgroup takes SC_DIG neighbouring digits, so that
// its reads and writes of one tile's entries are a contiguous 64 bytes, and SC_GROUPS ranges of tiles side by side:
// sums per range first, then each range again with its starting value.
constexpr int SC_DIG = 16, SC_GROUPS = 32, SC_PF = 8;
__global__ __launch_bounds__(SC_DIG * SC_GROUPS) void k_sort_scan(int32_t* ghist, int nblk, int radix, int32_t* __restrict__ dtot) {
    __shared__ int part[SC_GROUPS][SC_DIG];
    const int dl = threadIdx.x % SC_DIG, q = threadIdx.x / SC_DIG;
    const int d = blockIdx.x * SC_DIG + dl;
    const bool live = d < radix;
    const int per = (nblk + SC_GROUPS - 1) / SC_GROUPS;
    const int t0 = q * per, t1 = min(nblk, t0 + per);
    int sum = 0;
    if (live) {
        for (int t = t0; t < t1; t += SC_PF) {
            int v[SC_PF];
#pragma unroll
            for (int k = 0; k < SC_PF; ++k) v[k] = t + k < t1 ? ghist[(size_t)(t + k) * radix + d] : 0;
#pragma unroll
            for (int k = 0; k < SC_PF; ++k) sum += v[k];
        }
    }
    part[q][dl] = sum;
    __syncthreads();
    int run = 0, tot = 0;
#pragma unroll
    for (int g = 0; g < SC_GROUPS; ++g) {
        const int s = part[g][dl];
        if (g < q) run += s;
        tot += s;
    }
    if (live) {
        for (int t = t0; t < t1; t += SC_PF) {
            int v[SC_PF];
#pragma unroll
            for (int k = 0; k < SC_PF; ++k) v[k] = t + k < t1 ? ghist[(size_t)(t + k) * radix + d] : 0;
#pragma unroll
            for (int k = 0; k < SC_PF; ++k) {
                if (t + k < t1) ghist[(size_t)(t + k) * radix + d] = run;
                run += v[k];
            }
        }
        if (q == 0) dtot[d] = tot;
    }
}

// FUSED: `dtot` holds the per-supertile digit counts written by k_sort_hist instead of the digit totals, and `ghist` the
// raw per-tile counts (no scan kernel has run).  OPB (SORT_SRC_SLOTS only): bag b holds exactly lookup b, as checked by
// the caller, so the value of lookup i is i and the offsets are not read.
template <int SRC, int ITEMS, bool FUSED, bool OPB>
__global__ __launch_bounds__(RS_THREADS) void k_sort_scatter(const int32_t* __restrict__ keys_in,
                                                             const int32_t* __restrict__ vals_in,
                                                             const int64_t* __restrict__ offsets, int num_bags, int n,
                                                             int limit, int shift, int radix_bits, int nblk,
                                                             const int32_t* __restrict__ ghist,
                                                             const int32_t* __restrict__ dtot,
                                                             int32_t* __restrict__ keys_out,
                                                             int32_t* __restrict__ vals_out) {
    constexpr int NW = RS_THREADS / 64;
    __shared__ int base[1 << RS_MAX_BITS];     // where this tile's run of each digit starts in the output
    __shared__ int wc[NW][1 << RS_MAX_BITS];   // per-wavefront digit counts, then exclusive offsets
    __shared__ int lds[NW];
    const int radix = 1 << radix_bits, mask = radix - 1;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int tile0 = blockIdx.x * (RS_THREADS * ITEMS) + w * (64 * ITEMS);
    // The tile's keys and values are requested first, all together, so that their latency runs beside the digit
    // bases below.  A lane beyond n rereads element n-1 and is masked out later.
    int key[ITEMS], val[ITEMS];
    int64_t o0[ITEMS], o1[ITEMS];
    bool bad = false;
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
        const int i = min(tile0 + it * 64 + lane, n - 1);
        key[it] = load_key<SRC>(keys_in, i, limit, bad);
        if (SRC == SORT_SRC_SLOTS && OPB) val[it] = i;
        else if (SRC == SORT_SRC_SLOTS) {      // bag of lookup i, first guess: one lookup per bag
            const int g = min(i, num_bags - 1);
            o0[it] = offsets[g];
            o1[it] = offsets[g + 1];
        } else if (SRC == SORT_SRC_COUNTS) val[it] = i;
        else val[it] = vals_in[i];
    }
    if (FUSED) {
        // digit totals = sum over the supertiles; this tile's offset within a digit = the supertiles before its own plus
        // the tiles before it inside its own.  A thread owns `per` <= 2 neighbouring digits (radix <= 512).
        const int nsup = (nblk + SS_TILES - 1) / SS_TILES, mysup = blockIdx.x / SS_TILES;
        const int per = (radix + RS_THREADS - 1) / RS_THREADS;
        const int d0 = tid * per;
        int tot[2] = {0, 0}, bef[2] = {0, 0};
        if (d0 < radix) {
#pragma unroll 8
            for (int s = 0; s < nsup; ++s) {
                const int v0 = dtot[(size_t)s * radix + d0];
                const int v1 = per > 1 ? dtot[(size_t)s * radix + d0 + 1] : 0;
                tot[0] += v0; tot[1] += v1;
                if (s < mysup) { bef[0] += v0; bef[1] += v1; }
            }
#pragma unroll 8
            for (int t = mysup * SS_TILES; t < (int)blockIdx.x; ++t) {
                bef[0] += ghist[(size_t)t * radix + d0];
                if (per > 1) bef[1] += ghist[(size_t)t * radix + d0 + 1];
            }
        }
        int total;
        int run = block_excl_scan<RS_THREADS>(tot[0] + tot[1], total, lds);
        if (d0 < radix) {
            base[d0] = run + bef[0];
            if (per > 1) base[d0 + 1] = run + tot[0] + bef[1];
        }
        for (int d = tid; d < radix; d += RS_THREADS) {
#pragma unroll
            for (int k = 0; k < NW; ++k) wc[k][d] = 0;
        }
    } else {   // digit bases: exclusive scan of the digit totals, plus this tile's offset within the digit
        const int per = (radix + RS_THREADS - 1) / RS_THREADS;
        const int d0 = tid * per;
        int local = 0;
        for (int k = 0; k < per; ++k) if (d0 + k < radix) local += dtot[d0 + k];
        int tot;
        int run = block_excl_scan<RS_THREADS>(local, tot, lds);
        for (int k = 0; k < per; ++k) {
            const int d = d0 + k;
            if (d < radix) {
                base[d] = run + ghist[(size_t)blockIdx.x * radix + d];
                run += dtot[d];
            }
        }
        for (int d = tid; d < radix; d += RS_THREADS) {
#pragma unroll
            for (int k = 0; k < NW; ++k) wc[k][d] = 0;
        }
    }
    __syncthreads();
    if (SRC == SORT_SRC_SLOTS && !OPB) {
#pragma unroll
        for (int it = 0; it < ITEMS; ++it) {
            const int i = min(tile0 + it * 64 + lane, n - 1);
            const int g = min(i, num_bags - 1);
            val[it] = (o0[it] <= i && i < o1[it]) ? g : bag_of(offsets, num_bags, i);
        }
    }
    const uint64_t lt = (1ull << lane) - 1ull;
    int lrank[ITEMS];
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
        const bool valid = tile0 + it * 64 + lane < n;
        const int d = (key[it] >> shift) & mask;
        uint64_t peers = __ballot(valid);
        for (int b = 0; b < radix_bits; ++b) {
            const bool one = (d >> b) & 1;
            const uint64_t bm = __ballot(one);
            peers &= one ? bm : ~bm;
        }
        const int before = __popcll(peers & lt);
        int old = 0;
        if (valid) old = wc[w][d];
        if (valid && before == 0) wc[w][d] = old + __popcll(peers);
        lrank[it] = old + before;
    }
    __syncthreads();
    for (int d = tid; d < radix; d += RS_THREADS) {
        int run = 0;
#pragma unroll
        for (int k = 0; k < NW; ++k) { const int cnt = wc[k][d]; wc[k][d] = run; run += cnt; }
    }
    __syncthreads();
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
        if (tile0 + it * 64 + lane < n) {
            const int d = (key[it] >> shift) & mask;
            const int dest = base[d] + wc[w][d] + lrank[it];
            keys_out[dest] = key[it];
            vals_out[dest] = val[it];
        }
    }
}


template <int SRC, bool FUSED, bool OPB, int ITEMS = RS_ITEMS>
static void launch_pass(const SortJob& j, hipStream_t st, const int32_t* kin, const int32_t* vin, int32_t* kout, int32_t* vout,
                        int shift, int rb, int32_t* stot) {
    const int radix = 1 << rb;
    const int nblk = (int)cdiv(j.n, RS_THREADS * ITEMS);
    {
        ProfScope ps(j.prof, P_SORT_HIST, st);
        const bool first = shift == 0 && j.stot_other && j.other_dirty > 0;
        k_sort_hist<SRC, ITEMS><<<(unsigned)nblk, RS_THREADS, 0, st>>>(kin, j.n, j.limit, shift, rb, nblk, j.ghist, FUSED ? stot : nullptr,
                                                                     j.flags, j.rank_slot, j.slots_out,
                                                                     first ? j.stot_other : nullptr, first ? (int)j.other_dirty : 0);
    }
    if (!FUSED) {
        ProfScope ps(j.prof, P_SORT_SCAN, st);
        k_sort_scan<<<(unsigned)cdiv(radix, SC_DIG), SC_DIG * SC_GROUPS, 0, st>>>(j.ghist, nblk, radix, j.dtot);
    }
    // SORT_SRC_RANKS: the slots are written now, the rest of the pass reads them
    constexpr int SSRC = SRC == SORT_SRC_RANKS ? SORT_SRC_SLOTS : SRC;
    ProfScope ps(j.prof, P_SORT_SCATTER, st);
    k_sort_scatter<SSRC, ITEMS, FUSED, OPB><<<(unsigned)nblk, RS_THREADS, 0, st>>>(SRC == SORT_SRC_RANKS ? j.slots_out : kin, vin, j.offsets, j.num_bags,
                                                                                  j.n, j.limit, shift, rb, nblk, j.ghist, FUSED ? stot : j.dtot, kout, vout);
}

template <bool FUSED, int ITEMS>
static void first_pass(const SortJob& j, hipStream_t st, int32_t* kout, int32_t* vout, int rb, int32_t* stot) {
    const bool opb = j.one_per_bag && j.n == j.num_bags;
    if (j.src == SORT_SRC_PAIRS) launch_pass<SORT_SRC_PAIRS, FUSED, false, ITEMS>(j, st, j.keys_in, j.vals_in, kout, vout, 0, rb, stot);
    else if (j.src == SORT_SRC_COUNTS) launch_pass<SORT_SRC_COUNTS, FUSED, false, ITEMS>(j, st, j.keys_in, j.vals_in, kout, vout, 0, rb, stot);
    else if (j.src == SORT_SRC_SLOTS) {
        if (opb) launch_pass<SORT_SRC_SLOTS, FUSED, true, ITEMS>(j, st, j.keys_in, j.vals_in, kout, vout, 0, rb, stot);
        else launch_pass<SORT_SRC_SLOTS, FUSED, false, ITEMS>(j, st, j.keys_in, j.vals_in, kout, vout, 0, rb, stot);
    } else {
        if (opb) launch_pass<SORT_SRC_RANKS, FUSED, true, ITEMS>(j, st, j.keys_in, j.vals_in, kout, vout, 0, rb, stot);
        else launch_pass<SORT_SRC_RANKS, FUSED, false, ITEMS>(j, st, j.keys_in, j.vals_in, kout, vout, 0, rb, stot);
    }
}

template <bool FUSED, int ITEMS>
static int run_passes(const SortJob& j, hipStream_t st, int passes, int rb, int32_t* stot, size_t stot_pass,
                      const int32_t** kres, const int32_t** vres) {
    const int32_t* kin = j.keys_in; const int32_t* vin = j.vals_in;
    int32_t* kout = j.keysA; int32_t* vout = j.valsA;
    for (int p = 0; p < passes; ++p) {
        int32_t* sp = FUSED ? stot + stot_pass * p : nullptr;
        if (p == 1 && j.tail_stream && j.tail_event && j.tail_stream != st) {
            FC_HIP(hipEventRecord(j.tail_event, st));
            FC_HIP(hipStreamWaitEvent(j.tail_stream, j.tail_event, 0));
            st = j.tail_stream;
        }
        if (p == 0) first_pass<FUSED, ITEMS>(j, st, kout, vout, rb, sp);
        else launch_pass<SORT_SRC_PAIRS, FUSED, false, ITEMS>(j, st, kin, vin, kout, vout, p * rb, rb, sp);
        kin = kout; vin = vout;
        if (kout == j.keysA) { kout = j.keysB; vout = j.valsB; } else { kout = j.keysA; vout = j.valsA; }
    }
    *kres = kin; *vres = vin;
    if (j.last_stream) *j.last_stream = st;
    return FC_OK;
}

int radix_sort(const SortJob& j, hipStream_t st, const int32_t** kres, const int32_t** vres) {
    // Every pass is a chain of short launches bound by latency rather than by bytes.  Batches of up to FUSE_MAX_TILES
    // tiles and more than 18 key bits take passes of at most 9 bits, each two launches (counts, then offsets and scatter in
    // one kernel; the per-supertile counts make the scan in between unnecessary; the caller supplies their table); 7-bit digits leave runs of 16 keys per digit and tile,
    // i.e. whole sectors to write, where 11-bit digits left single keys.  Larger jobs (the static module's ranking) keep
    // the scan kernel: two passes up to 22 key bits, beyond that passes of at most 8 bits.
    // (j.max_bits / j.no_fuse, from FC_SORT_BITS / FC_SORT_FUSED at cache_create, override this for experiments.)
    const int env_bits = (j.max_bits >= 4 && j.max_bits <= RS_TWO_PASS_BITS) ? j.max_bits : 0;
    const bool env_fused = !j.no_fuse;
    const int64_t nblk = cdiv(j.n, RS_TILE);
    int passes, rb;
    // up to 18 key bits two passes with a scan kernel each are the shorter chain (measured at 426 k pairs of 18 bits)
    bool fused = env_fused && j.stot && nblk <= FUSE_MAX_TILES && (env_bits || j.bits > 2 * FUSE_MAX_BITS);
    size_t stot_pass = 0;
    if (fused) {
        const int lim = env_bits ? (env_bits < FUSE_MAX_BITS ? env_bits : FUSE_MAX_BITS) : FUSE_MAX_BITS;
        passes = (j.bits + lim - 1) / lim;
        rb = (j.bits + passes - 1) / passes;
        stot_pass = (size_t)cdiv(nblk, SS_TILES) << rb;
        if ((int64_t)(stot_pass * passes) > j.stot_cap) fused = false;
    }
    if (!fused) {
        const int two = env_bits ? env_bits : RS_TWO_PASS_BITS;
        passes = j.bits <= 2 * two ? (j.bits + two - 1) / two : (j.bits + 7) / 8;
        rb = (j.bits + passes - 1) / passes;
    }
    int32_t* stot = fused ? j.stot : nullptr;
    if (j.dirtied) *j.dirtied = fused ? (int64_t)(stot_pass * passes) : 0;
    if (fused) FC_TRY((run_passes<true, RS_ITEMS>(j, st, passes, rb, stot, stot_pass, kres, vres)));
    else FC_TRY((run_passes<false, RS_ITEMS>(j, st, passes, rb, stot, stot_pass, kres, vres)));
    FC_HIP(hipGetLastError());
    return FC_OK;
}

}  // namespace fc
