// Internal declarations shared by the freqcache HIP sources (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <string>
#include <vector>

#include "../../include/freqcache.h"

namespace fc {

constexpr int WAVE = 64;
// Rank-space bitmaps are scanned in tiles of RT_WORDS 32-bit words (one workgroup each):
// 256 threads x one uint4, i.e. 32768 ranks per tile.
constexpr int RT_THREADS = 256;
constexpr int RT_WORDS = RT_THREADS * 4;
// Radix sort of (slot, bag) pairs for the backward pass.
constexpr int RS_THREADS = 256;
constexpr int RS_ITEMS = 8;                      // keys per thread
constexpr int RS_TILE = RS_THREADS * RS_ITEMS;
constexpr int RS_TWO_PASS_BITS = 11;              // keys of up to 22 bits are sorted in two passes
constexpr int RS_MAX_BITS = RS_TWO_PASS_BITS;     // most bits per pass: sizes the digit tables
// Consecutive sorted lookups reduced by one row-group in the backward pass.
#ifndef FC_BWD_CHUNK
#define FC_BWD_CHUNK 32
#endif
#ifndef FC_BWD_PF
#define FC_BWD_PF 8
#endif
constexpr int BWD_CHUNK = FC_BWD_CHUNK;
// Gradient rows a row-group keeps in flight while it walks its chunk.
constexpr int BWD_PF = FC_BWD_PF;

// Sticky device-side flags.
enum : uint32_t { EF_BAD_OFFSETS = 1u, EF_ID_RANGE = 2u, EF_BAD_SLOT = 4u,
                  EF_NOT_ONE_PER_BAG = 8u };   // not an error: some bag of the batch does not hold exactly its own lookup

// Device-resident control block, read and written by the planning kernels.
struct Ctl {
    uint32_t err_flags;     // EF_* raised by the current cache_prepare
    uint32_t async_flags;   // EF_BAD_SLOT raised by fwd / bwd kernels
    int32_t nfree;          // empty slots
    int32_t status;         // FC_* decision of the current cache_prepare
    int32_t n_unique, n_miss, need;
};

// Host-visible (pinned, mapped) copy of the decision, written by the planning kernel.
struct HostCtl {
    int32_t status, n_unique, n_miss, need, hit_ids, nfree, async_flags;
    int32_t batch_flags; // EF_NOT_ONE_PER_BAG
    int32_t ticket;      // written last: number of the cache_prepare call this record belongs to
};

enum ProfItem {
    P_REMAP_MARK = 0, P_RANK_COUNT, P_RANK_PLAN, P_RANK_EMIT, P_EVICT_GATHER, P_EVICT_STORE, P_FREE_COUNT, P_FREE_PICK,
    P_MISS_FILL, P_SLOTS_OUT, P_BAG_FWD, P_SORT_HIST, P_SORT_SCAN, P_SORT_SCATTER, P_BWD_REDUCE, P_BWD_FIXUP,
    P_H2D_BLOCK, P_D2H_BLOCK, P_FLUSH_ROWS, P_ROWS_IN, P_COUNT
};

struct ProfSpan { int item; hipEvent_t a, b; };

struct ScatterPool;   // host threads that scatter evicted-row blocks into the host table (fc_worker.hip)
struct GatherPool;    // host threads that gather missing rows into a pinned block for the DMA miss path (fc_gather.hip)

// Scratch of one radix sort of a batch's (slot, bag) pairs, and the record of a sort started ahead of time.
struct SortBufs {
    int32_t *keysA = nullptr, *valsA = nullptr, *keysB = nullptr, *valsB = nullptr, *ghist = nullptr, *dtot = nullptr;
    int64_t cap = 0, ghist_cap = 0;
    // Per-supertile digit counts of the scan-free passes (SORT_STOT_WORDS ints each).  They are accumulated with atomics
    // and so have to start at zero: a sort uses set `zset`, which is clean, and its first kernel clears what the sort
    // before it left in the other set (`dirty` words from the start), so no launch is spent on clearing.
    int32_t* stot[2] = {nullptr, nullptr};
    int zset = 0;
    int64_t dirty[2] = {0, 0};
};
constexpr int64_t SORT_STOT_WORDS = 131072;
// What the row-movement half of a cache_prepare has to do (decided by the index half).
// evicted-row blocks of the DMA evict transmitter that may be on their way at once
#ifndef FC_DMA_BLOCKS
#define FC_DMA_BLOCKS 4
#endif
constexpr int DMA_BLOCKS = FC_DMA_BLOCKS;
struct MovePlan { bool valid = false; int64_t M = 0, need = 0; int buf = 0, transit_base = -1; bool arrived = false; };
struct PresortRec {
    bool valid = false;
    int32_t ticket = 0;                 // number of the cache_prepare / _next / plan_next call whose slots it sorted
    bool one_per_bag = false;           // bag b of that batch holds exactly lookup b (the click-log shape)
    const int32_t* slots = nullptr; const int64_t* offsets = nullptr;
    int64_t n = 0, bags = 0;
    const int32_t *keys = nullptr, *vals = nullptr;
    hipEvent_t ev_sorted = nullptr;
    hipStream_t sort_stream = nullptr;  // where ev_sorted was last recorded (null: never)
    bool caller_waited = false;         // the caller's stream already waits for ev_sorted (forward before backward)
};

}  // namespace fc

struct fc_cache {
    int64_t N = 0, C = 0;
    int32_t D = 0;
    int64_t staging_rows = 0;
    int32_t flags = 0;
    int device = 0;
    hipStream_t stream = nullptr, side = nullptr;
    // Look-ahead (cache_prepare_next): the next batch is prepared on `pre` while the caller's stream still trains on
    // the current one.  pst = the stream the cache_prepare / cache_prepare_next in progress enqueues on.
    hipStream_t pre = nullptr, pst = nullptr, last_pst = nullptr;
    hipEvent_t ev_s_now = nullptr, ev_pre_done = nullptr, ev_index_done = nullptr;
    hipEvent_t ev_assign_done = nullptr;   // index half: every decision taken (all but the slot write-out)
    hipEvent_t ev_emit_done = nullptr;     // index half: the missing rows and where their newest copies are: the early fetch may start
    hipEvent_t ev_quiesce = nullptr;       // transit marks dropped by dma_quiesce on another stream than the index stream
    hipStream_t quiesce_stream = nullptr;
    hipStream_t last_index_stream = nullptr;
    // The lists an index half writes and its row-movement half reads exist twice, so that the index half of the next
    // batch can run while the rows of the current one still move: lset = the set of the latest index half.
    int lset = 0;
    int32_t* lists[2][7] = {};      // per set: miss_ranks, vslot, fill_slots, fill_src (DMA evict), vrank (unless it lives
                                    // with the DMA block), and with FC_DIRTY_TRACK the dirty victims' ranks and slots
    hipEvent_t ev_move_done[2] = {nullptr, nullptr};   // the row movement that read set k has finished
    hipStream_t move_stream[2] = {nullptr, nullptr};   // the stream it ran on (nullptr: none yet)
    // cache_plan_next also fetches the planned batch's missing rows ahead of time, on the stream `pf`, into the
    // arrival block of its list set (row j of the block = j-th missing rank); cache_advance then only copies them
    // from HBM into their slots.  Allocated by the first cache_plan_next.
    hipStream_t pf = nullptr;
    float* arrive[2] = {nullptr, nullptr};             // [staging_rows][D] each
    hipEvent_t ev_arrive[2] = {nullptr, nullptr};
    bool next_pending = false;
    fc::MovePlan planned;           // cache_plan_next: row movement still to be done by cache_advance
    uint32_t* pbits = nullptr;      // rank-space bitmap: rows of the previously prepared batch
    hipEvent_t ev_evict_done = nullptr, ev_gather_done = nullptr;
    bool evict_pending = false;
    FILE* timeline = nullptr; std::string timeline_path;   // FC_TIMELINE: where cache_profile_get writes every span's start and end
    int sort_max_bits = 0; bool sort_no_fuse = false;   // tuning: FC_SORT_BITS, FC_SORT_FUSED=0
    float ahead_miss_pct = 2.0f;    // FC_INPUTS_READY: run ahead while the previous batch's misses stay below this share (tuning: FC_AHEAD_MISS_PCT)
    bool ahead_now = false;         // the cache_plan_next in progress runs ahead of the caller's stream
    bool sort_tail_side = true;     // cache_plan_next: the sort's passes after the first run on the side stream (tuning: FC_SORT_TAIL=0)
    hipEvent_t ev_sort_tail = nullptr;
    bool fwd_sorted = true;         // one-lookup-per-bag batches: forward in slot order when the pairs are sorted ahead of time (tuning: FC_FWD_SORTED=0)
    bool last_one_per_bag = false;  // the batch of the latest index half has that shape
    int fwd_bags = 4;               // bags per row-group of the forward kernel for one-lookup-per-bag batches: 1, 2 or 4 (tuning: FC_FWD_BAGS)
    int mark_ids_per_thread = 2;    // ids per thread of the marking kernel (tuning: FC_MARK_IPT)
    int fill_blocks = 1024;         // cap on the workgroups of the miss fill (tuning: FC_FILL_BLOCKS); 40 with FC_EVICT_DMA:
                                    // ~200 KB of reads in flight fill the link and still let the DMA engine's writes through
    int fill_blocks_early = 32;     // the same for rows fetched ahead of time by cache_plan_next (tuning: FC_FILL_BLOCKS_EARLY)
    int evict_blocks = 1024;        // workgroups of the host-table store kernel (tuning: FC_EVICT_BLOCKS)
    int evict_early = 2;            // when that kernel starts (tuning: FC_EVICT_EARLY): 0 after the miss fill, under
                                    // forward/backward; 1 right after the gather; 2 together with the miss fill

    // row geometry: VEC floats per lane access, LPR lanes per row
    int vec = 1, lpr = 1;

    // device state
    int32_t* freq_rank = nullptr;   // [N]  idx_map
    int32_t* rank_slot = nullptr;   // [N]  cpu_row_idx -> gpu_row_idx, -1 = not resident
    int32_t* slot_rank = nullptr;   // [C]  gpu_row_idx -> cpu_row_idx, -1 = empty
    float* cache = nullptr;         // [C][D]
    uint32_t* ubits = nullptr;      // rank-space bitmap: rows used by the current batch (zero between calls)
    uint32_t* rbits = nullptr;      // rank-space bitmap: resident rows
    int32_t* tcount = nullptr;      // empty slots per tile of 1024 slots
    int32_t* hitpart = nullptr;     // [256] per-workgroup access-level hit counts of the marking kernel
    int64_t NB = 0;                 // rank-space tiles
    int32_t* bsum = nullptr;        // [3][NB] per-tile counts: used, missing, evictable
    int32_t* moff = nullptr;        // [NB] output offset of a tile's missing ranks
    int32_t* vtake = nullptr;       // [NB] victims taken from a tile
    int32_t* voff = nullptr;        // [NB] output offset of a tile's victims
    int32_t* miss_ranks = nullptr;  // [C]  these five point into lists[lset] (vrank into vrank_buf with FC_EVICT_DMA)
    int32_t* vrank = nullptr;       // [C]
    int32_t* vslot = nullptr;       // [C]
    int32_t* fill_slots = nullptr;  // [C]
    int32_t* fill_src = nullptr;    // [C]  FC_EVICT_DMA: where each missing row is read from (-1 host, <= -2 transit)
    int32_t* rbuf = nullptr;        // [n_cap] rank of every input id
    int64_t n_cap = 0;
    fc::Ctl* ctl = nullptr;
    fc::HostCtl* hctl = nullptr;    // pinned
    int32_t ticket = 0;             // cache_prepare calls issued so far
    float* stage_dev = nullptr;     // [staging_rows][D] evicted-row block
    float* stage_dev2 = nullptr;    // staged mode: H2D block
    float* stage_pin = nullptr;     // staged mode: pinned block (both directions)
    int32_t* list_pin = nullptr;    // staged mode: pinned copies of miss / victim rank lists [2*C]

    // FC_DIRTY_TRACK: dirty[s] = 1 once the backward pass has updated slot s since it was loaded.  out_rank / out_slot:
    // the victims that are written back (all of them without the flag).
    bool dirty_track = false;
    uint8_t* dirty = nullptr;       // [C]
    int32_t* dcount = nullptr;      // dirty victims per tile of 1024 victims
    int32_t* dctl = nullptr;        // pinned: {dirty victims in all, ticket}
    int32_t dticket = 0;
    const int32_t* out_rank = nullptr;
    const int32_t* out_slot = nullptr;

    // DMA evict transmitter (FC_EVICT_DMA): evicted-row blocks leave HBM by hipMemcpyAsync on the side stream and
    // are scattered into the host table by worker threads; up to DMA_BLOCKS blocks in flight.  While a row's newest copy is
    // still on its way, rank_slot[rank] = -2 - (block * staging_rows + row in block) ("in transit") and a miss
    // on it is served from the device-side block instead of the host table.
    bool dma_evict = false;
    fc::ScatterPool* pool = nullptr;
    float* blk_pin[fc::DMA_BLOCKS] = {};          // pinned landing blocks
    int32_t* vrank_pin[fc::DMA_BLOCKS] = {};      // pinned copies of the evicted ranks
    int32_t* vrank_buf[fc::DMA_BLOCKS] = {};      // device lists of the evicted ranks, one per block
    int64_t blk_rows[fc::DMA_BLOCKS] = {};        // rows whose transit marks are still set, per block
    hipEvent_t ev_d2h[fc::DMA_BLOCKS] = {};
    hipEvent_t pf_dep = nullptr;                  // what the next early fetch of missing rows has to wait for
    // DMA miss path (FC_MISS_DMA): cache_plan_next's missing rows are gathered by host threads into a pinned block and
    // copied into the arrival block by hipMemcpyAsync on the fetch stream, instead of being read by a kernel.
    bool miss_dma = false;
    fc::GatherPool* gpool = nullptr;
    float* arrive_pin[2] = {nullptr, nullptr};    // [staging_rows][D], pinned
    int32_t* miss_pin[2] = {nullptr, nullptr};    // [staging_rows] pinned copies of the missing ranks
    int32_t* src_pin[2] = {nullptr, nullptr};     // ... and of where each row's newest copy is (-1: host table)
    hipEvent_t ev_list[2] = {nullptr, nullptr};   // those copies have landed
    bool gather_pending = false;                  // a job was started for the planned batch
    // The early fetch (zero-copy reads) and the evicted-row block copy (DMA writes) share the host link all the time in
    // the pipelined schedule; how they split it depends on the fetch's workgroup count, and a step gets longer, not
    // shorter, once the block copy is the slower one (more fetch workgroups also slow the index kernels of the batch
    // after next, which the following fetch waits for).  Unless FC_FILL_BLOCKS_EARLY pins it, that
    // count follows the measured durations: timing events around both, a smoothed ratio fetch / copy, one workgroup
    // fewer every few steps while the copy is the slower one, one more (up to the default, which suits steps that are
    // not bound by the link) while the fetch is clearly the slower one.
    bool tune_early = true;
    int fill_blocks_early_max = 32;
    hipEvent_t ev_fetch_a[2] = {nullptr, nullptr}, ev_fetch_b[2] = {nullptr, nullptr};
    hipEvent_t ev_copy_a[fc::DMA_BLOCKS] = {}, ev_copy_b[fc::DMA_BLOCKS] = {};
    bool fetch_timed[2] = {false, false}, copy_timed[fc::DMA_BLOCKS] = {};
    int last_copy_buf = -1;
    float tune_ratio = 0.f;
    int tune_count = 0;
    uint64_t dma_seq = 0;                         // blocks handed to the pool so far

    float* host = nullptr;          // pinned, rank-ordered table
    float* host_dev = nullptr;      // its device-side address
    bool own_host = false;

    // backward-pass scratch
    fc::SortBufs sb[3];             // [0], [1]: sorts started by cache_prepare (alternating); [2]: sorts inside the backward call
    float* part = nullptr;          // [groups][2][D] partial sums of slots spanning chunk borders
    int32_t* pmeta = nullptr;       // [groups][4]
    int64_t part_groups = 0;

    // sort of the (slot, bag) pairs started by cache_prepare / cache_plan_next on the stream `aux` (one of the two above)
    bool presort = true;            // FC_NO_PRESORT clears it
    hipStream_t aux = nullptr;      // = pf, or pre when cache_plan_next indexes there (pf then fetches rows): the device
                                    // offers four hardware queues, so the library keeps to three streams of its own
    hipEvent_t ev_slots = nullptr;
    fc::PresortRec rec[2];
    int rec_next = 0;
    // A record serves the backward pass of the batch it was made for and no other: cur_ticket = the call that prepared
    // the current batch (the one forward / backward run on), pending_ticket = the call that prepared the batch
    // cache_advance will make current.
    int32_t cur_ticket = 0, pending_ticket = 0;

    // last prepare
    fc_stats last = {};
    bool have_lists = false;

    // profiling
    bool prof_on = false;
    std::vector<fc::ProfSpan> spans;
    std::vector<hipEvent_t> ev_pool;
    double prof_ms[fc::P_COUNT] = {};
    int64_t prof_n[fc::P_COUNT] = {};
};

namespace fc {

// make list set k the current one (with FC_EVICT_DMA the victim ranks live with their block, not with the set)
inline void use_list_set(fc_cache* c, int k) {
    c->lset = k;
    c->miss_ranks = c->lists[k][0]; c->vslot = c->lists[k][1]; c->fill_slots = c->lists[k][2]; c->fill_src = c->lists[k][3];
    if (c->lists[k][4]) c->vrank = c->lists[k][4];
}

// ---- error plumbing ----
#define FC_HIP(expr)                                   \
    do {                                               \
        hipError_t _e = (expr);                        \
        if (_e != hipSuccess) {                        \
            (void)hipGetLastError();                   \
            return (_e == hipErrorOutOfMemory) ? FC_ERR_OOM_DEVICE : FC_ERR_HIP; \
        }                                              \
    } while (0)

#define FC_TRY(expr)                  \
    do {                              \
        int _rc = (expr);             \
        if (_rc != FC_OK) return _rc; \
    } while (0)

// Optional event bracket around one launch / copy on stream `s`.
struct ProfScope {
    fc_cache* c; hipStream_t s; int item; hipEvent_t a = nullptr, b = nullptr;
    ProfScope(fc_cache* c_, int item_, hipStream_t s_);
    ~ProfScope();
};
void prof_collect(fc_cache* c);

inline int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }

// entry points implemented across the sources
int prepare_index(fc_cache* c, hipStream_t st, bool lookahead, const int64_t* ids, int64_t n, const int64_t* offsets,
                  int64_t num_bags, int32_t* slots, MovePlan* mv, hipEvent_t before_slots = nullptr, bool defer_slots = false);
int launch_slots_out(fc_cache* c, hipStream_t st, int32_t* slots, int64_t n);
int prepare_move(fc_cache* c, hipStream_t st, const MovePlan& mv);
int prepare_impl(fc_cache* c, hipStream_t st, bool lookahead, const int64_t* ids, int64_t n, const int64_t* offsets,
                 int64_t num_bags, int32_t* slots);
int fwd_impl(fc_cache* c, const int32_t* slots, int64_t n, const int64_t* offsets, int64_t num_bags, float* out);
int dma_quiesce(fc_cache* c, hipStream_t st);
// from_ranks: the slots are not written yet; the sort's first kernel derives them from the per-id ranks and writes them
// to `slots_out` on its way (the slot write-out folded into the sort)
int presort_impl(fc_cache* c, const int32_t* slots, int64_t n, const int64_t* offsets, int64_t num_bags, int32_t* slots_out = nullptr);
int ensure_rbuf(fc_cache* c, int64_t n);  // per-id rank buffer for batches of n ids
int reserve_bwd(fc_cache* c, int64_t n);   // sort scratch of all three sets and the partial rows for batches of n lookups
int bwd_impl(fc_cache* c, const int32_t* slots, int64_t n, const int64_t* offsets, int64_t num_bags,
             const float* grad, float lr);
int bwd_noalloc_impl(fc_cache* c, const int32_t* slots, int64_t n, const int64_t* offsets, int64_t num_bags,
                     const float* grad, float lr);
int noalloc_setup(int device);

// row movement (fc_rows.hip).  dst_idx / src_idx: per-row index lists in device memory, or nullptr for row j.
// dst_rows / src_rows bound the row indices on either side (rows with an index outside are skipped).
int launch_copy_rows(fc_cache* c, hipStream_t s, int prof_item, float* dst, const int32_t* dst_idx, int64_t dst_rows,
                     const float* src, const int32_t* src_idx, int64_t src_rows, int64_t rows, int max_blocks);
// host[slot_rank[s]] = cache[s] for every resident slot, written straight into the mapped host table.
int launch_flush_rows(fc_cache* c, hipStream_t s);   // FC_DIRTY_TRACK: dirty rows only
// miss fill that honours transit marks: row j comes from the host table or from a device-side evicted-row block
// dst == nullptr: into the cache slots fill_slots[j]; else into row j of the block dst (of dst_rows rows)
// only_transit: rows whose newest copy is in the host table are skipped (the DMA miss path has brought them)
int launch_fill_rows(fc_cache* c, hipStream_t s, int64_t rows, float* dst = nullptr, int64_t dst_rows = 0, int max_blocks = 0,
                     bool only_transit = false);

// gather pool of the DMA miss path (fc_gather.hip)
int gather_create(fc_cache* c, int threads);
void gather_destroy(fc_cache* c);
int gather_start(fc_cache* c, int64_t M);
int gather_wait(fc_cache* c);

// scatter pool (fc_worker.hip)
int pool_create(fc_cache* c, int threads);
void pool_destroy(fc_cache* c);
void pool_publish(fc_cache* c, int buf, int64_t rows);   // block `buf` holds `rows` rows once ev_d2h[buf] fires
void pool_wait(fc_cache* c, uint64_t seq);               // until block number `seq` (1-based) is in the host table
uint64_t pool_published(fc_cache* c);

// ---- radix sort (fc_sort.hip) ----
enum SortSrc {
    SORT_SRC_PAIRS = 0,   // keys_in / vals_in as given
    SORT_SRC_SLOTS = 1,   // keys_in = slots of a batch (out-of-range -> sentinel `limit`, flag raised), value = bag of lookup i
    SORT_SRC_COUNTS = 2,  // keys_in = occurrence counts, key = limit - count (limit = largest count), value = i
    SORT_SRC_RANKS = 3    // keys_in = frequency ranks of a batch's ids: the first kernel looks their slots up in rank_slot and
                          // writes them to slots_out; from then on as SORT_SRC_SLOTS with keys_in = slots_out
};
struct SortJob {
    int src = SORT_SRC_PAIRS;
    const int32_t* keys_in = nullptr; const int32_t* vals_in = nullptr;
    const int64_t* offsets = nullptr; int num_bags = 0;
    bool one_per_bag = false;                  // SORT_SRC_SLOTS / _RANKS: the caller knows that offsets[b] == b for every bag
    const int32_t* rank_slot = nullptr; int32_t* slots_out = nullptr;     // SORT_SRC_RANKS
    int n = 0, limit = 0, bits = 1;
    int max_bits = 0; bool no_fuse = false;    // experiments: most bits per pass (0 = the default policy), never skip the scan kernel
    uint32_t* flags = nullptr;                 // device word for EF_BAD_SLOT, may be null
    int32_t *keysA = nullptr, *valsA = nullptr, *keysB = nullptr, *valsB = nullptr;   // n ints each
    int32_t *ghist = nullptr, *dtot = nullptr; // (tiles << RS_MAX_BITS) ints, (1 << RS_MAX_BITS) ints
    // scan-free passes (optional): a clean table of stot_cap ints to accumulate into; the first kernel also clears the first
    // other_dirty ints of stot_other; *dirtied receives how many ints of stot this sort has written to
    int32_t *stot = nullptr, *stot_other = nullptr;
    int64_t stot_cap = 0, other_dirty = 0;
    int64_t* dirtied = nullptr;
    // optional: the passes after the first run on tail_stream (ordered behind the first by tail_event), so that the stream
    // of the first pass is free again sooner; *last_stream receives the stream the last pass ran on
    hipStream_t tail_stream = nullptr; hipEvent_t tail_event = nullptr; hipStream_t* last_stream = nullptr;
    fc_cache* prof = nullptr;                  // where to book per-kernel times, may be null
};
int radix_sort(const SortJob& j, hipStream_t st, const int32_t** kres, const int32_t** vres);

// ---- device helpers ----
template <int NT>
__device__ __forceinline__ int block_excl_scan(int v, int& total, int* lds /* NT/64 ints */) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    int x = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        int y = __shfl_up(x, o);
        if (lane >= o) x += y;
    }
    if (lane == 63) lds[w] = x;
    __syncthreads();
    int wbase = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < NT / 64; ++i) {
        int s = lds[i];
        if (i < w) wbase += s;
        tot += s;
    }
    __syncthreads();
    total = tot;
    return wbase + x - v;
}

__device__ __forceinline__ int wave_sum(int x) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_down(x, o);
    return x;  // valid in lane 0
}

}  // namespace fc
