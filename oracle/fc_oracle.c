/* CPU ORACLE -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, single-threaded statement of what the frequency-aware
 * software cache of arXiv:2208.05321 computes per training iteration.  It is
 * used only by the tests, by the smoke check and by the benchmark's CPU
 * baseline; the GPU library never calls it and shares no code with it.
 *
 * Two layers of definition (paper Section 2.2 on synchronous embedding updates,
 * Section 4.3, Algorithm 1):
 *   - VALUES (pooled outputs, updated rows, flushed table): with synchronous
 *     updates the cache is invisible; results equal EmbeddingBag-sum + SGD run
 *     on the whole table.  Pinned by tests against a no-cache computation.
 *   - CACHE BEHAVIOUR (hit/miss sets, victims, slot assignment, bytes moved):
 *     the policy of Algorithm 1, taken step by step below.  Pinned by tests
 *     against a brute-force set-based statement of Algorithm 1 on tiny tables, a
 *     hand-worked trace, and invariants.
 *   - parity unpinned: absolute hit-ratio values (the paper prints none).
 *
 * Notation (paper Section 4.1): ids -> cpu_row_idx through idx_map (here
 * `rank`, the frequency rank, Section 4.2); the CPU Weight `host` holds row
 * cpu_row_idx; the CUDA Cached Weight `cache` holds `C` rows; cache_idx_map is
 * kept as two mutually inverse arrays, slot_rank[gpu_row_idx] = cpu_row_idx
 * (-1 = empty slot, the marker Algorithm 1 uses for a row that is not on the GPU) and
 * rank_slot[cpu_row_idx] = gpu_row_idx (-1 = not resident), because the
 * algorithm indexes the map in both directions.
 *
 * Readings where the listing is silent or garbled:
 *   - "cache_capacity" in evict_num = numel(miss) - cache_capacity is the number
 *     of currently empty slots (otherwise nothing would ever be evicted).
 *   - evicted rows are always written back (the paper tracks no dirty state),
 *     after which both map entries are reset to -1.  Optional variant, not in
 *     the paper (fco_set_dirty_tracking): a resident row is dirty once a
 *     backward pass has updated it since it was loaded; only dirty victims
 *     are written back (a clean row equals its copy in the CPU Weight), and
 *     bytes_d2h counts those alone.  Values never differ between the two.
 *   - the j-th smallest missing cpu_row_idx goes to the j-th smallest empty
 *     slot (unique() returns ascending values, nonzero() ascending indices).
 *   - victims: the evict_num resident rows with the largest cpu_row_idx among
 *     rows the current batch does not use; equal keys (impossible when `rank`
 *     is a permutation) would evict the lower slot first.
 *   - a batch with more distinct rows than slots is an error; state unchanged.
 *   - one slot index is returned per input id (EmbeddingBag needs that).
 *   - pooling is sum; the optimizer is plain SGD: row <- row - lr * grad_sum,
 *     the product rounded to fp32 before the subtraction.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum {
    FCO_OK = 0,
    FCO_INVALID_ARG = 1,
    FCO_ID_OUT_OF_RANGE = 2,
    FCO_BAD_OFFSETS = 3,
    FCO_BATCH_EXCEEDS_CACHE = 4,
    FCO_NOT_PERMUTATION = 5,
    FCO_OOM = 6
};

typedef struct fco {
    int64_t N, C;
    int32_t D;
    int32_t* rank;       /* [N] id -> cpu_row_idx                          */
    float* host;         /* [N][D] CPU Weight, rank-ordered; caller-owned  */
    float* cache;        /* [C][D] cached weight                           */
    int32_t* slot_rank;  /* [C]                                            */
    int32_t* rank_slot;  /* [N]                                            */
    /* observables of the last prepare */
    int64_t n_ids, n_unique, n_hit_unique, n_hit_ids, n_miss, n_evict, bytes_h2d, bytes_d2h;
    int32_t* miss_ranks;   /* [C] ascending                                */
    int32_t* evict_ranks;  /* [C] ascending cpu_row_idx                    */
    int32_t* evict_slots;  /* [C] slot of evict_ranks[j]                   */
    int32_t* fill_slots;   /* [C] fill_slots[j] receives miss_ranks[j]     */
    /* look-ahead variant: rows of the previously prepared batch (ascending), also protected from eviction */
    int32_t* prev_U;       /* [C]                                          */
    int64_t n_prev;
    /* dirty-tracking variant: dirty[s] = 1 once slot s was updated after it was loaded */
    int32_t dirty_track;
    unsigned char* dirty;  /* [C]                                          */
} fco;

static int cmp_i32(const void* a, const void* b) {
    int32_t x = *(const int32_t*)a, y = *(const int32_t*)b;
    return (x > y) - (x < y);
}

typedef struct { int32_t rank, slot; } cand_t;

/* larger cpu_row_idx first; equal keys: lower slot first */
static int cmp_cand(const void* a, const void* b) {
    const cand_t* x = (const cand_t*)a; const cand_t* y = (const cand_t*)b;
    if (x->rank != y->rank) return (x->rank < y->rank) - (x->rank > y->rank);
    return (x->slot > y->slot) - (x->slot < y->slot);
}

static int contains_sorted(const int32_t* a, int64_t n, int32_t v) {
    return bsearch(&v, a, (size_t)n, sizeof(int32_t), cmp_i32) != NULL;
}

void fco_destroy(fco* o) {
    if (!o) return;
    free(o->rank); free(o->cache); free(o->slot_rank); free(o->rank_slot);
    free(o->miss_ranks); free(o->evict_ranks); free(o->evict_slots); free(o->fill_slots); free(o->prev_U); free(o->dirty);
    free(o);
}

/* Section 4.2 (static module) + Section 4.3 last paragraph (warm-up). */
int fco_create(int64_t N, int32_t D, int64_t C, const int32_t* freq_rank, float* host, int32_t warm, fco** out) {
    if (!out || !freq_rank || !host || N <= 0 || D <= 0 || C <= 0 || C > N) return FCO_INVALID_ARG;
    /* idx_map must be a permutation of [0, N): the CPU Weight is the original table re-ordered */
    unsigned char* seen = (unsigned char*)calloc((size_t)N, 1);
    if (!seen) return FCO_OOM;
    for (int64_t i = 0; i < N; ++i) {
        int32_t r = freq_rank[i];
        if (r < 0 || r >= N || seen[r]) { free(seen); return FCO_NOT_PERMUTATION; }
        seen[r] = 1;
    }
    free(seen);
    fco* o = (fco*)calloc(1, sizeof(fco));
    if (!o) return FCO_OOM;
    o->N = N; o->C = C; o->D = D; o->host = host;
    o->rank = (int32_t*)malloc((size_t)N * 4);
    o->cache = (float*)calloc((size_t)C * D, 4);
    o->slot_rank = (int32_t*)malloc((size_t)C * 4);
    o->rank_slot = (int32_t*)malloc((size_t)N * 4);
    o->miss_ranks = (int32_t*)malloc((size_t)C * 4);
    o->evict_ranks = (int32_t*)malloc((size_t)C * 4);
    o->evict_slots = (int32_t*)malloc((size_t)C * 4);
    o->fill_slots = (int32_t*)malloc((size_t)C * 4);
    o->prev_U = (int32_t*)malloc((size_t)C * 4);
    o->n_prev = 0;
    o->dirty = (unsigned char*)calloc((size_t)C, 1);
    if (!o->prev_U || !o->dirty ||  !o->rank || !o->cache || !o->slot_rank || !o->rank_slot || !o->miss_ranks || !o->evict_ranks ||
        !o->evict_slots || !o->fill_slots) { fco_destroy(o); return FCO_OOM; }
    memcpy(o->rank, freq_rank, (size_t)N * 4);
    for (int64_t r = 0; r < N; ++r) o->rank_slot[r] = -1;
    for (int64_t s = 0; s < C; ++s) o->slot_rank[s] = -1;
    if (warm) {
        /* fill the cached weight with the highest-frequency rows: slot s <- cpu_row_idx s */
        for (int64_t s = 0; s < C; ++s) {
            o->slot_rank[s] = (int32_t)s;
            o->rank_slot[s] = (int32_t)s;
            memcpy(o->cache + (size_t)s * D, host + (size_t)s * D, (size_t)D * 4);
        }
    }
    *out = o;
    return FCO_OK;
}

/* Algorithm 1: PrepareCache + PrepareCPURowIdxOnGPU. slots_out[n] receives gpu_row_idx per input id.
 * protect_prev = 0: the algorithm as printed (the backlist is the current batch).
 * protect_prev = 1: look-ahead variant (the paper's Future Work section proposes prefetching on the ids of coming
 *   batches): this batch is prepared while the previously prepared batch is still being trained on, so the
 *   backlist is the union of both batches' rows.  If that leaves fewer evictable rows than needed the call fails
 *   with BATCH_EXCEEDS_CACHE and changes nothing. */
static int prepare_core(fco* o, const int64_t* ids, int64_t n, const int64_t* offsets, int64_t num_bags, int32_t* slots_out,
                        int protect_prev) {
    if (!o || n < 0 || num_bags < 0 || (n > 0 && (!ids || !slots_out)) || !offsets) return FCO_INVALID_ARG;
    const int64_t N = o->N, C = o->C; const int32_t D = o->D;
    /* bag boundaries must tile [0, n) */
    if (offsets[0] != 0 || offsets[num_bags] != n) return FCO_BAD_OFFSETS;
    for (int64_t b = 0; b < num_bags; ++b) if (offsets[b] > offsets[b + 1]) return FCO_BAD_OFFSETS;
    for (int64_t i = 0; i < n; ++i) if (ids[i] < 0 || ids[i] >= N) return FCO_ID_OUT_OF_RANGE;

    /* cpu_row_idxs = unique(index_select(idx_map, ids)) */
    int32_t* r = (int32_t*)malloc((size_t)(n > 0 ? n : 1) * 4);
    int32_t* U = (int32_t*)malloc((size_t)(n > 0 ? n : 1) * 4);
    if (!r || !U) { free(r); free(U); return FCO_OOM; }
    for (int64_t i = 0; i < n; ++i) r[i] = o->rank[ids[i]];
    memcpy(U, r, (size_t)n * 4);
    qsort(U, (size_t)n, 4, cmp_i32);
    int64_t nU = 0;
    for (int64_t i = 0; i < n; ++i) if (i == 0 || U[i] != U[i - 1]) U[nU++] = U[i];
    if (nU > C) { free(r); free(U); return FCO_BATCH_EXCEEDS_CACHE; }

    /* comm_cpu_row_idxs = cpu_row_idxs not present in the cached map (ascending) */
    int64_t nM = 0, nH = 0;
    for (int64_t j = 0; j < nU; ++j) {
        if (o->rank_slot[U[j]] >= 0) ++nH; else o->miss_ranks[nM++] = U[j];
    }
    int64_t hit_ids = 0;
    for (int64_t i = 0; i < n; ++i) if (o->rank_slot[r[i]] >= 0) ++hit_ids;

    /* evict_num = numel(miss) - (empty slots) */
    int64_t empty = 0;
    for (int64_t s = 0; s < C; ++s) if (o->slot_rank[s] == -1) ++empty;
    int64_t evict_num = nM - empty;
    int64_t nV = 0, n_written = 0;
    if (evict_num > 0) {
        /* rows of the current batch (the "backlist") are protected; among the other resident rows
           take the evict_num largest cpu_row_idx (LFU by static frequency rank, Section 4.3) */
        cand_t* cand = (cand_t*)malloc((size_t)C * sizeof(cand_t));
        if (!cand) { free(r); free(U); return FCO_OOM; }
        int64_t nc = 0;
        for (int64_t s = 0; s < C; ++s) {
            int32_t k = o->slot_rank[s];
            if (k < 0 || contains_sorted(U, nU, k)) continue;
            if (protect_prev && contains_sorted(o->prev_U, o->n_prev, k)) continue;
            cand[nc].rank = k; cand[nc].slot = (int32_t)s; ++nc;
        }
        /* without look-ahead this cannot happen when nU <= C */
        if (nc < evict_num) { free(cand); free(r); free(U); return protect_prev ? FCO_BATCH_EXCEEDS_CACHE : FCO_INVALID_ARG; }
        qsort(cand, (size_t)nc, sizeof(cand_t), cmp_cand);
        nV = evict_num;
        /* report victims in ascending cpu_row_idx order */
        for (int64_t j = 0; j < nV; ++j) {
            o->evict_ranks[j] = cand[nV - 1 - j].rank;
            o->evict_slots[j] = cand[nV - 1 - j].slot;
        }
        free(cand);
        /* data_transmitter.move_to_cpu, then the slots become empty */
        for (int64_t j = 0; j < nV; ++j) {
            int32_t s = o->evict_slots[j], k = o->evict_ranks[j];
            if (!o->dirty_track || o->dirty[s]) {
                memcpy(o->host + (size_t)k * D, o->cache + (size_t)s * D, (size_t)D * 4);
                ++n_written;
            }
            o->dirty[s] = 0;                   /* the slot is empty; whatever is loaded next equals its CPU copy */
            o->rank_slot[k] = -1;
            o->slot_rank[s] = -1;
        }
    }
    /* target_gpu_row_idxs = first numel(miss) empty slots; data_transmitter.move_to_gpu; map update */
    int64_t j = 0;
    for (int64_t s = 0; s < C && j < nM; ++s) {
        if (o->slot_rank[s] == -1) {
            int32_t k = o->miss_ranks[j];
            o->fill_slots[j] = (int32_t)s;
            memcpy(o->cache + (size_t)s * D, o->host + (size_t)k * D, (size_t)D * 4);
            o->slot_rank[s] = k;
            o->rank_slot[k] = (int32_t)s;
            ++j;
        }
    }
    /* gpu_row_idxs = index_select(cached map, cpu_row_idx of every input id) */
    for (int64_t i = 0; i < n; ++i) slots_out[i] = o->rank_slot[r[i]];

    o->n_ids = n; o->n_unique = nU; o->n_hit_unique = nH; o->n_hit_ids = hit_ids;
    o->n_miss = nM; o->n_evict = nV;
    o->bytes_h2d = nM * (int64_t)D * 4; o->bytes_d2h = n_written * (int64_t)D * 4;
    memcpy(o->prev_U, U, (size_t)nU * 4);     /* this batch is the "previous" one of the next call */
    o->n_prev = nU;
    free(r); free(U);
    return FCO_OK;
}

int fco_prepare(fco* o, const int64_t* ids, int64_t n, const int64_t* offsets, int64_t num_bags, int32_t* slots_out) {
    return prepare_core(o, ids, n, offsets, num_bags, slots_out, 0);
}

int fco_prepare_lookahead(fco* o, const int64_t* ids, int64_t n, const int64_t* offsets, int64_t num_bags,
                          int32_t* slots_out) {
    return prepare_core(o, ids, n, offsets, num_bags, slots_out, 1);
}

/* EmbeddingBag, mode=sum, on the cached weight: out[b] = sum over the bag, in position order. */
/* The bag sum itself, on any weight array of `rows` rows: out[b] = rows of bag b added one by one in position order. */
int fco_bag_sum(const float* weight, int64_t rows, int32_t D, const int32_t* slots, int64_t n, const int64_t* offsets,
                int64_t num_bags, float* out) {
    if (!weight || !offsets || !out) return FCO_INVALID_ARG;
    for (int64_t b = 0; b < num_bags; ++b) {
        float* ob = out + (size_t)b * D;
        for (int32_t c = 0; c < D; ++c) ob[c] = 0.0f;
        for (int64_t i = offsets[b]; i < offsets[b + 1]; ++i) {
            if (i >= n || slots[i] < 0 || slots[i] >= rows) return FCO_INVALID_ARG;
            const float* row = weight + (size_t)slots[i] * D;
            for (int32_t c = 0; c < D; ++c) ob[c] = ob[c] + row[c];
        }
    }
    return FCO_OK;
}

int fco_embedding_bag_fwd(const fco* o, const int32_t* slots, int64_t n, const int64_t* offsets, int64_t num_bags, float* out) {
    if (!o) return FCO_INVALID_ARG;
    return fco_bag_sum(o->cache, o->C, o->D, slots, n, offsets, num_bags, out);
}

/* Backward of the sum-bag + SGD step: each lookup of a row receives its bag's output gradient;
   g[slot] accumulates them in position order; row <- row - lr * g. */
int fco_embedding_bag_bwd_sgd(fco* o, const int32_t* slots, int64_t n, const int64_t* offsets, int64_t num_bags,
                              const float* grad_out, float lr) {
    if (!o || !offsets || !grad_out) return FCO_INVALID_ARG;
    const int32_t D = o->D; const int64_t C = o->C;
    float* g = (float*)calloc((size_t)C * D, 4);
    unsigned char* touched = (unsigned char*)calloc((size_t)C, 1);
    if (!g || !touched) { free(g); free(touched); return FCO_OOM; }
    for (int64_t b = 0; b < num_bags; ++b) {
        const float* gb = grad_out + (size_t)b * D;
        for (int64_t i = offsets[b]; i < offsets[b + 1]; ++i) {
            if (i >= n || slots[i] < 0 || slots[i] >= C) { free(g); free(touched); return FCO_INVALID_ARG; }
            float* gs = g + (size_t)slots[i] * D;
            for (int32_t c = 0; c < D; ++c) gs[c] = gs[c] + gb[c];
            touched[slots[i]] = 1;
        }
    }
    for (int64_t s = 0; s < C; ++s) {
        if (!touched[s]) continue;
        float* row = o->cache + (size_t)s * D; const float* gs = g + (size_t)s * D;
        for (int32_t c = 0; c < D; ++c) {
            float step = lr * gs[c];            /* rounded product (no contraction), then the subtraction */
            row[c] = row[c] - step;
        }
        o->dirty[s] = 1;
    }
    free(g); free(touched);
    return FCO_OK;
}

/* Write every resident row back to the CPU Weight (the store of record, Section 3); residency unchanged. */
int fco_flush(fco* o) {
    if (!o) return FCO_INVALID_ARG;
    for (int64_t s = 0; s < o->C; ++s) {
        int32_t k = o->slot_rank[s];
        if (k >= 0 && (!o->dirty_track || o->dirty[s]))
            memcpy(o->host + (size_t)k * o->D, o->cache + (size_t)s * o->D, (size_t)o->D * 4);
        o->dirty[s] = 0;                       /* the CPU Weight is current for every resident row now */
    }
    return FCO_OK;
}

/* Variant beyond the paper: write back only victims that a backward pass has updated since they were loaded. */
int fco_set_dirty_tracking(fco* o, int32_t on) {
    if (!o) return FCO_INVALID_ARG;
    o->dirty_track = on ? 1 : 0;
    return FCO_OK;
}
const unsigned char* fco_dirty(const fco* o) { return o->dirty; }

/* ---- accessors for the tests ---- */
void fco_stats(const fco* o, int64_t out[8]) {
    out[0] = o->n_ids; out[1] = o->n_unique; out[2] = o->n_hit_unique; out[3] = o->n_hit_ids;
    out[4] = o->n_miss; out[5] = o->n_evict; out[6] = o->bytes_h2d; out[7] = o->bytes_d2h;
}
const int32_t* fco_slot_rank(const fco* o) { return o->slot_rank; }
const int32_t* fco_rank_slot(const fco* o) { return o->rank_slot; }
const float* fco_cache(const fco* o) { return o->cache; }
const int32_t* fco_miss_ranks(const fco* o) { return o->miss_ranks; }
const int32_t* fco_evict_ranks(const fco* o) { return o->evict_ranks; }
const int32_t* fco_evict_slots(const fco* o) { return o->evict_slots; }
const int32_t* fco_fill_slots(const fco* o) { return o->fill_slots; }
