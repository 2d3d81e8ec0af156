// Stable LSD radix sort of (key, value) int32 pairs, 64-wide wavefronts, up to 9 bits per pass.
// Used by the backward pass (sort lookups by slot, value = bag) and by the static-module build
// (sort ids by descending count).  Keys come from one of three sources, see SortSrc.
#include "fc_internal.h"

#include <stdlib.h>

namespace fc {

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

// key (and, on the first pass, value) of element i for the three sources
template <int SRC>
__device__ __forceinline__ int load_key(const int32_t* __restrict__ keys_in, int i, int limit, bool& bad) {
    if (SRC == SORT_SRC_SLOTS) return first_key(keys_in, i, limit, bad);
    if (SRC == SORT_SRC_COUNTS) return limit - keys_in[i];      // limit = largest count: descending counts ascend
    return keys_in[i];
}

template <int SRC, int ITEMS>
__global__ __launch_bounds__(RS_THREADS) void k_sort_hist(const int32_t* __restrict__ keys_in, int n, int limit, int shift,
                                                          int radix_bits, int nblk, int32_t* __restrict__ ghist,
                                                          uint32_t* flags, const int32_t* __restrict__ rank_slot,
                                                          int32_t* __restrict__ slots_out) {
    __shared__ int h[1 << RS_MAX_BITS];
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
    for (int d = threadIdx.x; d < radix; d += RS_THREADS) ghist[(size_t)blockIdx.x * radix + d] = h[d];   // tile-major: one contiguous run per tile
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

template <int SRC, int ITEMS>
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
        if (SRC == SORT_SRC_SLOTS) {           // bag of lookup i, first guess: one lookup per bag
            const int g = min(i, num_bags - 1);
            o0[it] = offsets[g];
            o1[it] = offsets[g + 1];
        } else if (SRC == SORT_SRC_COUNTS) val[it] = i;
        else val[it] = vals_in[i];
    }
    {   // digit bases: exclusive scan of the digit totals, plus this tile's offset within the digit
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
    if (SRC == SORT_SRC_SLOTS) {
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


template <int SRC, int ITEMS = RS_ITEMS>
static void launch_pass(const SortJob& j, hipStream_t st, const int32_t* kin, const int32_t* vin, int32_t* kout, int32_t* vout,
                        int shift, int rb) {
    const int radix = 1 << rb;
    const int nblk = (int)cdiv(j.n, RS_THREADS * ITEMS);
    {
        ProfScope ps(j.prof, P_SORT_HIST, st);
        k_sort_hist<SRC, ITEMS><<<(unsigned)nblk, RS_THREADS, 0, st>>>(kin, j.n, j.limit, shift, rb, nblk, j.ghist, j.flags, j.rank_slot, j.slots_out);
    }
    if (SRC == SORT_SRC_RANKS) {        // the slots are written now: the rest of the pass reads them
        ProfScope ps(j.prof, P_SORT_SCAN, st);
        k_sort_scan<<<(unsigned)cdiv(radix, SC_DIG), SC_DIG * SC_GROUPS, 0, st>>>(j.ghist, nblk, radix, j.dtot);
    }
    if (SRC == SORT_SRC_RANKS) {
        ProfScope ps(j.prof, P_SORT_SCATTER, st);
        k_sort_scatter<SORT_SRC_SLOTS, ITEMS><<<(unsigned)nblk, RS_THREADS, 0, st>>>(j.slots_out, vin, j.offsets, j.num_bags, j.n, j.limit, shift, rb,
                                                                                     nblk, j.ghist, j.dtot, kout, vout);
        return;
    }
    {
        ProfScope ps(j.prof, P_SORT_SCAN, st);
        k_sort_scan<<<(unsigned)cdiv(radix, SC_DIG), SC_DIG * SC_GROUPS, 0, st>>>(j.ghist, nblk, radix, j.dtot);
    }
    {
        ProfScope ps(j.prof, P_SORT_SCATTER, st);
        k_sort_scatter<SRC, ITEMS><<<(unsigned)nblk, RS_THREADS, 0, st>>>(kin, vin, j.offsets, j.num_bags, j.n, j.limit, shift, rb,
                                                                         nblk, j.ghist, j.dtot, kout, vout);
    }
}

int radix_sort(const SortJob& j, hipStream_t st, const int32_t** kres, const int32_t** vres) {
    // Two passes up to 22 key bits: every pass is three launches bound by latency rather than by bytes, so a third pass
    // costs more than the larger digit tables of 10- and 11-bit digits do; beyond that, passes of at most 8 bits.
    // (FC_SORT_BITS, read once per process, lowers the two-pass limit per pass for experiments.)
    static const int two_pass_bits = [] {
        const char* e = getenv("FC_SORT_BITS");
        const int v = e ? atoi(e) : 0;
        return (v >= 4 && v <= RS_TWO_PASS_BITS) ? v : RS_TWO_PASS_BITS;
    }();
    const int passes = j.bits <= 2 * two_pass_bits ? (j.bits + two_pass_bits - 1) / two_pass_bits : (j.bits + 7) / 8;
    const int rb = (j.bits + passes - 1) / passes;
    const int32_t* kin = j.keys_in; const int32_t* vin = j.vals_in;
    int32_t* kout = j.keysA; int32_t* vout = j.valsA;
    for (int p = 0; p < passes; ++p) {
        const int shift = p * rb;
        if (p > 0 || j.src == SORT_SRC_PAIRS) launch_pass<SORT_SRC_PAIRS>(j, st, kin, vin, kout, vout, shift, rb);
        else if (j.src == SORT_SRC_SLOTS) launch_pass<SORT_SRC_SLOTS>(j, st, kin, vin, kout, vout, shift, rb);
        else if (j.src == SORT_SRC_RANKS) launch_pass<SORT_SRC_RANKS>(j, st, kin, vin, kout, vout, shift, rb);
        else launch_pass<SORT_SRC_COUNTS>(j, st, kin, vin, kout, vout, shift, rb);
        kin = kout; vin = vout;
        if (kout == j.keysA) { kout = j.keysB; vout = j.valsB; } else { kout = j.keysA; vout = j.valsA; }
    }
    FC_HIP(hipGetLastError());
    *kres = kin; *vres = vin;
    return FC_OK;
}

}  // namespace fc
