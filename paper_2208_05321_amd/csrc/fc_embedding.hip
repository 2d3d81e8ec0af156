// EmbeddingBag-sum forward and the fused backward + SGD step on the cached weight
// (paper Section 4.3: after the cache step the embedding op and the optimizer run on the cached rows;
//  Section 2.2: the update is synchronous).
//
// Forward: one row-group of lanes per bag, rows added in position order.
// Backward: lookups are stably radix-sorted by slot (payload = bag index), so each slot's gradients form
// one contiguous, position-ordered run; fixed chunks of BWD_CHUNK consecutive sorted lookups are reduced by
// one row-group each (perfectly balanced however skewed the ids are), runs that cross chunk borders are
// finished by a second small kernel in chunk order.  No floating-point atomics: results are reproducible.
#include "fc_internal.h"

// Scratch of embedding_bag_bwd_sgd_noalloc: sort buffers, radix histograms and the partial rows of the reduction for
// batches of up to FC_NOALLOC_MAX_IDS lookups live here instead of in memory the library allocates.  Every GPU the
// library runs on holds its own copy of the array, at its own address, until the process ends.  In host code the name
// is only a handle for hipGetSymbolAddress: the address kernels and copies use is the one that call returns.
static __device__ __align__(256) unsigned char scratch[FC_NOALLOC_SCRATCH_BYTES];

namespace fc {

constexpr int NOALLOC_MAX_DEVICES = 64;
static unsigned char* scratch_ptr[NOALLOC_MAX_DEVICES] = {};   // per device: where `scratch` lives there

// Called by cache_create with the handle's device current: look the array's address on this device up once.
int noalloc_setup(int device) {
    if (device < 0 || device >= NOALLOC_MAX_DEVICES) return FC_OK;          // the entry point then reports the failure
    if (scratch_ptr[device]) return FC_OK;
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) { (void)hipGetLastError(); return FC_ERR_HIP; }
    scratch_ptr[device] = static_cast<unsigned char*>(p);
    return FC_OK;
}

template <int VEC> struct Vec;
template <> struct Vec<1> { using T = float; };
template <> struct Vec<2> { using T = float2; };
template <> struct Vec<4> { using T = float4; };

__device__ __forceinline__ float vzero(float) { return 0.f; }
__device__ __forceinline__ float2 vzero(float2) { return make_float2(0.f, 0.f); }
__device__ __forceinline__ float4 vzero(float4) { return make_float4(0.f, 0.f, 0.f, 0.f); }
__device__ __forceinline__ float vadd(float a, float b) { return a + b; }
__device__ __forceinline__ float2 vadd(float2 a, float2 b) { return make_float2(a.x + b.x, a.y + b.y); }
__device__ __forceinline__ float4 vadd(float4 a, float4 b) { return make_float4(a.x + b.x, a.y + b.y, a.z + b.z, a.w + b.w); }
// Streaming accesses (data touched once per step: pooled outputs, output gradients) are marked non-temporal so that
// they do not push the cached rows, which forward and backward both touch, out of the memory-side cache.
__device__ __forceinline__ void nt_store(float* p, float v) { __builtin_nontemporal_store(v, p); }
__device__ __forceinline__ void nt_store(float2* p, float2 v) { __builtin_nontemporal_store(v.x, &p->x); __builtin_nontemporal_store(v.y, &p->y); }
__device__ __forceinline__ void nt_store(float4* p, float4 v) {
    typedef float v4f __attribute__((ext_vector_type(4)));
    v4f t = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(t, reinterpret_cast<v4f*>(p));
}
__device__ __forceinline__ float nt_load(const float* p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ float2 nt_load(const float2* p) { return make_float2(__builtin_nontemporal_load(&p->x), __builtin_nontemporal_load(&p->y)); }
__device__ __forceinline__ float4 nt_load(const float4* p) {
    typedef float v4f __attribute__((ext_vector_type(4)));
    const v4f t = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(p));
    return make_float4(t.x, t.y, t.z, t.w);
}
// row - lr * g with the product rounded before the subtraction (no fused multiply-add)
__device__ __forceinline__ float sgd1(float w, float g, float lr) { return __fsub_rn(w, __fmul_rn(lr, g)); }
__device__ __forceinline__ float vsgd(float w, float g, float lr) { return sgd1(w, g, lr); }
__device__ __forceinline__ float2 vsgd(float2 w, float2 g, float lr) { return make_float2(sgd1(w.x, g.x, lr), sgd1(w.y, g.y, lr)); }
__device__ __forceinline__ float4 vsgd(float4 w, float4 g, float lr) {
    return make_float4(sgd1(w.x, g.x, lr), sgd1(w.y, g.y, lr), sgd1(w.z, g.z, lr), sgd1(w.w, g.w, lr));
}

// ---------------------------------------------------------------------------------------------------------
// forward
// ---------------------------------------------------------------------------------------------------------
// A row-group takes FWD_BAGS consecutive bags.  When each of them holds exactly one lookup (the click-log shape: one id
// per feature) their rows are independent loads in flight together; otherwise the bags are summed one after the other,
// four lookups in flight.  The host picks FWD_BAGS = 4 for batches with as many lookups as bags, else 1.

template <int VEC>
__device__ __forceinline__ bool bag_sum(const float* __restrict__ cache, const int32_t* __restrict__ slots, int64_t beg,
                                        int64_t end, int n, int C, int D, int lane, int lpr, int nv,
                                        typename Vec<VEC>::T* __restrict__ o) {
    using V = typename Vec<VEC>::T;
    bool bad = false;
    if (beg < 0) beg = 0;
    if (end > n) end = n;
    for (int cidx = lane; cidx < nv; cidx += lpr) {
        V acc = vzero(V());
        int64_t i = beg;
        for (; i + 4 <= end; i += 4) {
            const int s0 = slots[i], s1 = slots[i + 1], s2 = slots[i + 2], s3 = slots[i + 3];
            const bool k0 = (unsigned)s0 < (unsigned)C, k1 = (unsigned)s1 < (unsigned)C,
                       k2 = (unsigned)s2 < (unsigned)C, k3 = (unsigned)s3 < (unsigned)C;
            bad |= !(k0 && k1 && k2 && k3);
            const V v0 = k0 ? reinterpret_cast<const V*>(cache + (size_t)s0 * D)[cidx] : vzero(V());
            const V v1 = k1 ? reinterpret_cast<const V*>(cache + (size_t)s1 * D)[cidx] : vzero(V());
            const V v2 = k2 ? reinterpret_cast<const V*>(cache + (size_t)s2 * D)[cidx] : vzero(V());
            const V v3 = k3 ? reinterpret_cast<const V*>(cache + (size_t)s3 * D)[cidx] : vzero(V());
            acc = vadd(acc, v0); acc = vadd(acc, v1); acc = vadd(acc, v2); acc = vadd(acc, v3);
        }
        for (; i < end; ++i) {
            const int s0 = slots[i];
            const bool k0 = (unsigned)s0 < (unsigned)C;
            bad |= !k0;
            if (k0) acc = vadd(acc, reinterpret_cast<const V*>(cache + (size_t)s0 * D)[cidx]);
        }
        nt_store(&o[cidx], acc);
    }
    return bad;
}

template <int VEC, int FWD_BAGS>
__global__ __launch_bounds__(256) void k_bag_fwd(const float* __restrict__ cache, const int32_t* __restrict__ slots,
                                                 const int64_t* __restrict__ offsets, int num_bags, int n, int C, int D,
                                                 int lpr_shift, float* __restrict__ out, Ctl* ctl) {
    using V = typename Vec<VEC>::T;
    const int lpr = 1 << lpr_shift;
    const int gpb = blockDim.x >> lpr_shift;
    const int gl = threadIdx.x >> lpr_shift, lane = threadIdx.x & (lpr - 1);
    const int nv = D / VEC;
    bool bad = false;
    for (int64_t b0 = (int64_t)(blockIdx.x * gpb + gl) * FWD_BAGS; b0 < num_bags; b0 += (int64_t)gridDim.x * gpb * FWD_BAGS) {
        const int nb = num_bags - b0 < FWD_BAGS ? (int)(num_bags - b0) : FWD_BAGS;
        int64_t off[FWD_BAGS + 1];
#pragma unroll
        for (int k = 0; k <= FWD_BAGS; ++k) off[k] = k <= nb ? offsets[b0 + k] : 0;
        bool single = nb == FWD_BAGS && off[0] >= 0 && off[FWD_BAGS] <= n;
#pragma unroll
        for (int k = 0; k < FWD_BAGS; ++k) single = single && off[k + 1] - off[k] == 1;
        if (single) {
            int sl[FWD_BAGS];
#pragma unroll
            for (int k = 0; k < FWD_BAGS; ++k) sl[k] = slots[off[0] + k];
            for (int cidx = lane; cidx < nv; cidx += lpr) {
                V v[FWD_BAGS];
#pragma unroll
                for (int k = 0; k < FWD_BAGS; ++k)
                    v[k] = (unsigned)sl[k] < (unsigned)C ? reinterpret_cast<const V*>(cache + (size_t)sl[k] * D)[cidx] : vzero(V());
#pragma unroll
                for (int k = 0; k < FWD_BAGS; ++k) nt_store(&reinterpret_cast<V*>(out + (size_t)(b0 + k) * D)[cidx], vadd(vzero(V()), v[k]));
            }
#pragma unroll
            for (int k = 0; k < FWD_BAGS; ++k) bad |= (unsigned)sl[k] >= (unsigned)C;
        } else {
            for (int k = 0; k < nb; ++k)
                bad |= bag_sum<VEC>(cache, slots, off[k], off[k + 1], n, C, D, lane, lpr, nv, reinterpret_cast<V*>(out + (size_t)(b0 + k) * D));
        }
    }
    if (bad) atomicOr(&ctl->async_flags, EF_BAD_SLOT);
}

// Forward for batches with one lookup per bag whose (slot, bag) pairs are already sorted by slot (the sort the backward
// pass needs, started by cache_prepare): out[bag] = row of slot, walked in SLOT order.  In bag order every compute-unit
// cluster meets every popular row and fetches its own copy through its own L2 (config 4: 286 MB fetched for 96 MB of
// distinct rows); in slot order a row's lookups sit next to each other, so each row crosses the fabric once and the
// kernel is left with writing the pooled output.  FWD_ROWS lookups per row-group are in flight together; a repeated
// slot is simply loaded again (it hits the L1 / L2 of the same compute unit).
constexpr int FWD_ROWS = 8;      // measured at config 4: 4 and 8 alike (188 us), 16 slower (203 us); ordinary stores instead of non-temporal ones 239 us
template <int VEC>
__global__ __launch_bounds__(256) void k_bag_fwd_sorted(const float* __restrict__ cache, const int32_t* __restrict__ keys,
                                                        const int32_t* __restrict__ vals, int n, int num_bags, int C, int D,
                                                        int lpr_shift, float* __restrict__ out) {
    using V = typename Vec<VEC>::T;
    const int lpr = 1 << lpr_shift;
    const int gpb = blockDim.x >> lpr_shift;
    const int gl = threadIdx.x >> lpr_shift, lane = threadIdx.x & (lpr - 1);
    const int nv = D / VEC;
    for (int64_t i0 = (int64_t)(blockIdx.x * gpb + gl) * FWD_ROWS; i0 < n; i0 += (int64_t)gridDim.x * gpb * FWD_ROWS) {
        int k[FWD_ROWS], b[FWD_ROWS];
#pragma unroll
        for (int j = 0; j < FWD_ROWS; ++j) {
            const int64_t i = i0 + j < n ? i0 + j : n - 1;      // the tail repeats the last lookup (same value stored twice)
            k[j] = keys[i];
            b[j] = vals[i];
        }
        for (int cidx = lane; cidx < nv; cidx += lpr) {
            V v[FWD_ROWS];
#pragma unroll
            for (int j = 0; j < FWD_ROWS; ++j)     // a slot out of range was sorted under the key C: its bag reads as zeros
                v[j] = (unsigned)k[j] < (unsigned)C ? reinterpret_cast<const V*>(cache + (size_t)k[j] * D)[cidx] : vzero(V());
#pragma unroll
            for (int j = 0; j < FWD_ROWS; ++j)
                if ((unsigned)b[j] < (unsigned)num_bags) nt_store(&reinterpret_cast<V*>(out + (size_t)b[j] * D)[cidx], vadd(vzero(V()), v[j]));
        }
    }
}

static inline int shift_of(int lpr) { int s = 0; while ((1 << s) < lpr) ++s; return s; }

int fwd_impl(fc_cache* c, const int32_t* slots, int64_t n, const int64_t* offsets, int64_t num_bags, float* out) {
    const int64_t LIM = ((int64_t)1 << 31) - 65536;
    if (!c || n < 0 || num_bags < 0 || n >= LIM || num_bags >= LIM || !offsets || (n > 0 && !slots) || (num_bags > 0 && !out))
        return FC_ERR_INVALID_ARG;
    if (num_bags == 0) return FC_OK;
    FC_HIP(hipSetDevice(c->device));
    const int sh = shift_of(c->lpr);
    const int gpb = 256 >> sh;
    // One lookup per bag and the batch's pairs sorted ahead of time by the call that prepared it: walk them in slot order.
    // (Offsets are not consulted: the record was made from these very buffers, and with as many lookups as bags the
    // sort found bag i for lookup i or, for offsets that do not say so, whatever bag holds lookup i.)
    if (n == num_bags && c->fwd_sorted) {
        for (PresortRec& r : c->rec) {
            if (r.valid && r.one_per_bag && r.ticket == c->cur_ticket && r.slots == slots && r.n == n && r.offsets == offsets && r.bags == num_bags) {
                if (!r.caller_waited) { FC_HIP(hipStreamWaitEvent(c->stream, r.ev_sorted, 0)); r.caller_waited = true; }
                int64_t blocks = cdiv(n, (int64_t)gpb * FWD_ROWS);
                if (blocks > (1 << 20)) blocks = 1 << 20;
                ProfScope ps(c, P_BAG_FWD, c->stream);
                switch (c->vec) {
                    case 4: k_bag_fwd_sorted<4><<<(unsigned)blocks, 256, 0, c->stream>>>(c->cache, r.keys, r.vals, (int)n, (int)num_bags, (int)c->C, c->D, sh, out); break;
                    case 2: k_bag_fwd_sorted<2><<<(unsigned)blocks, 256, 0, c->stream>>>(c->cache, r.keys, r.vals, (int)n, (int)num_bags, (int)c->C, c->D, sh, out); break;
                    default: k_bag_fwd_sorted<1><<<(unsigned)blocks, 256, 0, c->stream>>>(c->cache, r.keys, r.vals, (int)n, (int)num_bags, (int)c->C, c->D, sh, out); break;
                }
                FC_HIP(hipGetLastError());
                return FC_OK;
            }
        }
    }
    const int bags_per_group = (n == num_bags && c->fwd_bags > 1) ? c->fwd_bags : 1;
    int64_t blocks = cdiv(num_bags, (int64_t)gpb * bags_per_group);
    if (blocks > (1 << 20)) blocks = 1 << 20;
    ProfScope ps(c, P_BAG_FWD, c->stream);
#define FC_FWD(V, B) \
    k_bag_fwd<V, B><<<(unsigned)blocks, 256, 0, c->stream>>>(c->cache, slots, offsets, (int)num_bags, (int)n, (int)c->C, c->D, sh, out, c->ctl)
#define FC_FWD_V(B) \
    switch (c->vec) { case 4: FC_FWD(4, B); break; case 2: FC_FWD(2, B); break; default: FC_FWD(1, B); break; }
    if (bags_per_group == 4) { FC_FWD_V(4) }
    else if (bags_per_group == 2) { FC_FWD_V(2) }
    else { FC_FWD_V(1) }
#undef FC_FWD_V
#undef FC_FWD
    FC_HIP(hipGetLastError());
    return FC_OK;
}

// ---------------------------------------------------------------------------------------------------------
// backward, step 2: chunked segmented reduction + SGD
// ---------------------------------------------------------------------------------------------------------
// A row-group owns BWD_CHUNK consecutive sorted lookups; a workgroup owns gpb such chunks in a row.
// Runs (lookups of one slot) that lie inside a chunk are applied to the cached row at once.  Pieces of runs that
// cross chunk borders meet in LDS and are joined in chunk order by the group where the run starts inside the
// workgroup; only pieces of runs that cross WORKGROUP borders go to global memory (two rows per workgroup) and are
// joined by k_bwd_fixup.  kinds of a chunk's / workgroup's first piece: 0 none, 1 = ends a run begun earlier,
// 2 = lies wholly inside a longer run.
struct BwdMeta { int first_kind, has_head, head_slot, pad; };

// STREAM: every gradient row is read exactly once (one lookup per bag) -> non-temporal loads
template <int VEC, bool STREAM>
__global__ __launch_bounds__(256) void k_bwd_reduce(const int32_t* __restrict__ keys, const int32_t* __restrict__ vals,
                                                    int n, int C, const float* __restrict__ grad, float* cache, int D,
                                                    int lpr_shift, float lr, float* __restrict__ part,
                                                    BwdMeta* __restrict__ bmeta) {
    using V = typename Vec<VEC>::T;
    extern __shared__ __align__(16) unsigned char smem[];
    const int lpr = 1 << lpr_shift;
    const int gpb = blockDim.x >> lpr_shift;
    const int gl = threadIdx.x >> lpr_shift, lane = threadIdx.x & (lpr - 1);
    const int nv = D / VEC;
    // LDS: keys[gpb*CHUNK], vals[gpb*CHUNK], meta[gpb], pieces[gpb][2][D]
    int* skeys = reinterpret_cast<int*>(smem);
    int* svals = skeys + gpb * BWD_CHUNK;
    BwdMeta* smeta = reinterpret_cast<BwdMeta*>(svals + gpb * BWD_CHUNK);
    float* spiece = reinterpret_cast<float*>(smeta + gpb);
    __shared__ BwdMeta blockmeta;

    const int64_t blk0 = (int64_t)blockIdx.x * gpb * BWD_CHUNK;
    for (int t = threadIdx.x; t < gpb * BWD_CHUNK; t += blockDim.x) {
        const int64_t e = blk0 + t;
        skeys[t] = e < n ? keys[e] : -1;
        svals[t] = e < n ? vals[e] : 0;
    }
    if (threadIdx.x == 0) blockmeta = BwdMeta{0, 0, -1, 0};
    __syncthreads();

    const int64_t beg = blk0 + (int64_t)gl * BWD_CHUNK;
    const int cnt = beg >= n ? 0 : (int)(beg + BWD_CHUNK <= n ? BWD_CHUNK : n - beg);
    const int* mk = skeys + gl * BWD_CHUNK;
    const int* mv = svals + gl * BWD_CHUNK;
    V* __restrict__ pfirst = reinterpret_cast<V*>(spiece + (size_t)(gl * 2) * D);
    V* __restrict__ plast = reinterpret_cast<V*>(spiece + (size_t)(gl * 2 + 1) * D);
    int first_kind = 0, has_head = 0, head_slot = -1;
    if (cnt > 0) {
        const int prevk = gl > 0 ? mk[-1] : (beg > 0 ? keys[beg - 1] : -1);
        const int nextk = beg + cnt < n ? (gl + 1 < gpb ? mk[BWD_CHUNK] : keys[beg + cnt]) : -2;
        for (int cidx = lane; cidx < nv; cidx += lpr) {
            bool open_left = prevk == mk[0];
            first_kind = 0; has_head = 0; head_slot = -1;
            V acc = vzero(V());
            for (int e0 = 0; e0 < cnt; e0 += BWD_PF) {
                // BWD_PF independent gradient rows in flight, and with them the cached row of every run that ends
                // among these lookups (known from the keys): the update below then finds its operand loaded
                V g[BWD_PF], w[BWD_PF];
                bool ends[BWD_PF];
#pragma unroll
                for (int k = 0; k < BWD_PF; ++k) {
                    const int e = e0 + k;
                    ends[k] = false;
                    g[k] = vzero(V()); w[k] = vzero(V());
                    if (e < cnt) {
                        const V* gp = &reinterpret_cast<const V*>(grad + (size_t)mv[e] * D)[cidx];
                        g[k] = STREAM ? nt_load(gp) : *gp;
                        const int kk = mk[e];
                        ends[k] = (e + 1 < cnt ? mk[e + 1] : nextk) != kk;
                        if (ends[k] && kk < C) w[k] = reinterpret_cast<const V*>(cache + (size_t)kk * D)[cidx];
                    }
                }
#pragma unroll
                for (int k = 0; k < BWD_PF; ++k) {
                    if (e0 + k < cnt) {
                        acc = vadd(acc, g[k]);
                        if (ends[k]) {                // the run of mk[e0 + k] ends here
                            const int kk = mk[e0 + k];
                            if (open_left) { pfirst[cidx] = acc; first_kind = 1; }
                            else if (kk < C) reinterpret_cast<V*>(cache + (size_t)kk * D)[cidx] = vsgd(w[k], acc, lr);
                            open_left = false;
                            acc = vzero(V());
                        }
                    }
                }
            }
            if (nextk == mk[cnt - 1]) {               // the last run goes on in the next chunk
                if (open_left) { pfirst[cidx] = acc; first_kind = 2; }
                else { plast[cidx] = acc; has_head = 1; head_slot = mk[cnt - 1]; }
            }
        }
    }
    if (lane == 0) smeta[gl] = BwdMeta{first_kind, has_head, head_slot, 0};
    __syncthreads();
    // join the pieces inside the workgroup, in chunk order (chunks past the end of the batch have no pieces)
    if (gl == 0 && first_kind != 0) {          // a run that entered from the previous workgroup
        int kind = first_kind, j = 0;
        while (kind == 2 && j + 1 < gpb && smeta[j + 1].first_kind != 0) { ++j; kind = smeta[j].first_kind; }
        // chunks 0..j carry pieces of that run; kind says whether it ended (1) or leaves the workgroup (2)
        V* __restrict__ out = reinterpret_cast<V*>(part + (size_t)(blockIdx.x * 2) * D);
        for (int cidx = lane; cidx < nv; cidx += lpr) {
            V acc = pfirst[cidx];
            for (int q = 1; q <= j; ++q) acc = vadd(acc, reinterpret_cast<const V*>(spiece + (size_t)(q * 2) * D)[cidx]);
            out[cidx] = acc;
        }
        if (lane == 0) blockmeta.first_kind = kind;
    }
    if (has_head) {                             // a run that starts in this chunk and continues to the right
        int j = gl, kind = 2;
        while (kind == 2 && j + 1 < gpb && smeta[j + 1].first_kind != 0) { ++j; kind = smeta[j].first_kind; }
        const bool closed = kind == 1;          // ended inside the workgroup
        V* __restrict__ out = reinterpret_cast<V*>(part + (size_t)(blockIdx.x * 2 + 1) * D);
        for (int cidx = lane; cidx < nv; cidx += lpr) {
            V acc = plast[cidx];
            for (int q = gl + 1; q <= j; ++q) acc = vadd(acc, reinterpret_cast<const V*>(spiece + (size_t)(q * 2) * D)[cidx]);
            if (!closed) out[cidx] = acc;
            else if (head_slot < C) {
                V* row = reinterpret_cast<V*>(cache + (size_t)head_slot * D);
                row[cidx] = vsgd(row[cidx], acc, lr);
            }
        }
        if (!closed && lane == 0) { blockmeta.has_head = 1; blockmeta.head_slot = head_slot; }
    }
    __syncthreads();
    if (threadIdx.x == 0) bmeta[blockIdx.x] = blockmeta;
}

// FC_DIRTY_TRACK: every slot the backward pass updates differs from its host copy from now on.
__global__ __launch_bounds__(256) void k_mark_dirty(const int32_t* __restrict__ slots, int n, int C, uint8_t* __restrict__ dirty) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) {
        const int s = slots[i];
        if ((unsigned)s < (unsigned)C) dirty[s] = 1;
    }
}

// Runs that cross workgroup borders: the workgroup where the run starts adds the later workgroups' pieces in order.
template <int VEC>
__global__ __launch_bounds__(256) void k_bwd_fixup(int C, float* cache, int D, int lpr_shift, float lr,
                                                   const float* __restrict__ part, const BwdMeta* __restrict__ bmeta,
                                                   int nblocks) {
    using V = typename Vec<VEC>::T;
    const int lpr = 1 << lpr_shift;
    const int gpb = blockDim.x >> lpr_shift;
    const int gl = threadIdx.x >> lpr_shift, lane = threadIdx.x & (lpr - 1);
    const int nv = D / VEC;
    const int b = blockIdx.x * gpb + gl;
    if (b >= nblocks || !bmeta[b].has_head) return;
    const int slot = bmeta[b].head_slot;
    if (slot >= C) return;
    // The pieces are added in workgroup order, FIX_PF of them requested together (a popular row's run spans hundreds of
    // workgroups; one dependent load per piece made this kernel as long as that chain).  Pieces past the end of the run
    // are loaded and ignored.
    constexpr int FIX_PF = 8;
    for (int cidx = lane; cidx < nv; cidx += lpr) {
        V acc = reinterpret_cast<const V*>(part + (size_t)(b * 2 + 1) * D)[cidx];
        bool done = false;
        for (int h = b + 1; h < nblocks && !done; h += FIX_PF) {
            V p[FIX_PF];
            int kind[FIX_PF];
#pragma unroll
            for (int j = 0; j < FIX_PF; ++j) {
                const int hh = h + j < nblocks ? h + j : nblocks - 1;
                p[j] = reinterpret_cast<const V*>(part + (size_t)(hh * 2) * D)[cidx];
                kind[j] = bmeta[hh].first_kind;
            }
#pragma unroll
            for (int j = 0; j < FIX_PF; ++j) {
                if (!done && h + j < nblocks) {
                    acc = vadd(acc, p[j]);
                    done = kind[j] != 2;
                }
            }
        }
        V* row = reinterpret_cast<V*>(cache + (size_t)slot * D);
        row[cidx] = vsgd(row[cidx], acc, lr);
    }
}

// threads per workgroup of the reduction: at most 64 chunks per workgroup
static inline int bwd_threads(int lpr) { int t = 32 * lpr; if (t > 256) t = 256; if (t < 64) t = 64; return t; }

// (Re)allocation of sort scratch and of the reduction's partial rows; growth is rare and waits for the whole device.
static int ensure_sort(SortBufs& sb, int64_t n) {
    const int64_t nblk = cdiv(n, RS_TILE);
    if (n > sb.cap) {
        FC_HIP(hipDeviceSynchronize());
        for (int32_t** p : {&sb.keysA, &sb.valsA, &sb.keysB, &sb.valsB}) { if (*p) FC_HIP(hipFree(*p)); *p = nullptr; }
        sb.cap = 0;
        const int64_t cap = n + n / 4 + 1024;
        for (int32_t** p : {&sb.keysA, &sb.valsA, &sb.keysB, &sb.valsB}) FC_HIP(hipMalloc((void**)p, (size_t)cap * 4));
        sb.cap = cap;
    }
    const int64_t gh = nblk << RS_MAX_BITS;
    if (gh > sb.ghist_cap) {
        FC_HIP(hipDeviceSynchronize());
        if (sb.ghist) FC_HIP(hipFree(sb.ghist));
        sb.ghist = nullptr; sb.ghist_cap = 0;
        FC_HIP(hipMalloc((void**)&sb.ghist, (size_t)(gh + gh / 4) * 4));
        sb.ghist_cap = gh + gh / 4;
    }
    if (!sb.dtot) FC_HIP(hipMalloc((void**)&sb.dtot, (size_t)(1 << RS_MAX_BITS) * 4));
    for (int k = 0; k < 2; ++k)
        if (!sb.stot[k]) {
            FC_HIP(hipMalloc((void**)&sb.stot[k], (size_t)SORT_STOT_WORDS * 4));
            FC_HIP(hipMemset(sb.stot[k], 0, (size_t)SORT_STOT_WORDS * 4));
            sb.dirty[k] = 0;
        }
    return FC_OK;
}

// radix_sort with the buffers of sb, keeping track of which of its two supertile tables is clean
static int sort_in(SortJob& j, SortBufs& sb, hipStream_t st, const int32_t** kres, const int32_t** vres) {
    j.keysA = sb.keysA; j.valsA = sb.valsA; j.keysB = sb.keysB; j.valsB = sb.valsB; j.ghist = sb.ghist; j.dtot = sb.dtot;
    int64_t dirtied = 0;
    if (sb.stot[0] && sb.stot[1] && sb.dirty[sb.zset] > 0) {     // only after a failed sort: the table to use is not known to be clean
        FC_HIP(hipMemsetAsync(sb.stot[sb.zset], 0, (size_t)SORT_STOT_WORDS * 4, st));
        sb.dirty[sb.zset] = 0;
    }
    if (sb.stot[0] && sb.stot[1]) {
        j.stot = sb.stot[sb.zset]; j.stot_cap = SORT_STOT_WORDS;
        j.stot_other = sb.stot[sb.zset ^ 1]; j.other_dirty = sb.dirty[sb.zset ^ 1];
        j.dirtied = &dirtied;
    }
    const int rc = radix_sort(j, st, kres, vres);
    if (j.stot) {
        // after a failed launch nothing is known about either table: both count as written to in full
        sb.dirty[sb.zset] = rc == FC_OK ? dirtied : SORT_STOT_WORDS;
        sb.dirty[sb.zset ^ 1] = rc == FC_OK ? 0 : SORT_STOT_WORDS;
        sb.zset ^= 1;
    }
    return rc;
}

static int ensure_part(fc_cache* c, int64_t groups);
static inline void bwd_geometry(const fc_cache* c, int64_t n, int* rthreads, int64_t* rblocks, size_t* lds);

int reserve_bwd(fc_cache* c, int64_t n) {
    if (n <= 0) return FC_OK;
    for (SortBufs& sb : c->sb) FC_TRY(ensure_sort(sb, n));
    int rthreads; int64_t rblocks; size_t lds;
    bwd_geometry(c, n, &rthreads, &rblocks, &lds);
    return ensure_part(c, rblocks);
}

static int ensure_part(fc_cache* c, int64_t groups) {
    if (groups > c->part_groups) {
        FC_HIP(hipDeviceSynchronize());
        if (c->part) FC_HIP(hipFree(c->part));
        if (c->pmeta) FC_HIP(hipFree(c->pmeta));
        c->part = nullptr; c->pmeta = nullptr; c->part_groups = 0;
        const int64_t cap = groups + groups / 4 + 64;
        FC_HIP(hipMalloc((void**)&c->part, (size_t)cap * 2 * c->D * 4));
        FC_HIP(hipMalloc((void**)&c->pmeta, (size_t)cap * sizeof(BwdMeta)));
        c->part_groups = cap;
    }
    return FC_OK;
}

// Stable sort of the batch's (slot, bag) pairs by slot on stream `st`; *kres / *vres receive the sorted arrays.
static int sort_pairs(fc_cache* c, SortBufs& sb, hipStream_t st, const int32_t* slots, int64_t n, const int64_t* offsets,
                      int64_t num_bags, const int32_t** kres, const int32_t** vres, int32_t* slots_out = nullptr,
                      hipStream_t tail = nullptr, hipStream_t* last = nullptr) {
    int bits = 1;
    while (((int64_t)1 << bits) <= c->C) ++bits;           // keys lie in [0, C] (C = out-of-range sentinel)
    SortJob j;
    j.src = SORT_SRC_SLOTS; j.keys_in = slots; j.offsets = offsets; j.num_bags = (int)num_bags; j.n = (int)n;
    if (slots_out) { j.src = SORT_SRC_RANKS; j.keys_in = c->rbuf; j.rank_slot = c->rank_slot; j.slots_out = slots_out; }
    j.limit = (int)c->C; j.bits = bits; j.flags = &c->ctl->async_flags;
    j.one_per_bag = c->last_one_per_bag;      // sort_pairs serves the batch the last index half looked at
    j.tail_stream = tail; j.tail_event = c->ev_sort_tail; j.last_stream = last;
    j.max_bits = c->sort_max_bits; j.no_fuse = c->sort_no_fuse;
    j.prof = c;
    return sort_in(j, sb, st, kres, vres);
}

static inline void bwd_geometry(const fc_cache* c, int64_t n, int* rthreads, int64_t* rblocks, size_t* lds) {
    *rthreads = bwd_threads(c->lpr);
    const int rgpb = *rthreads / c->lpr;                      // chunks per workgroup of the reduction
    *rblocks = cdiv(n, (int64_t)rgpb * BWD_CHUNK);
    *lds = (size_t)rgpb * BWD_CHUNK * 8 + (size_t)rgpb * sizeof(BwdMeta) + (size_t)rgpb * 2 * c->D * 4;
}

// Called by cache_prepare / cache_prepare_next / cache_plan_next once the slots of the batch are on their way: the
// sort needs nothing but the slots and the bag offsets, so it runs on a library stream (c->aux) while the missing
// rows are still crossing the host link.  Two records alternate, so that the sort of the next batch does not
// disturb the current one's.
int presort_impl(fc_cache* c, const int32_t* slots, int64_t n, const int64_t* offsets, int64_t num_bags, int32_t* slots_out) {
    const int k = c->rec_next;
    c->rec_next ^= 1;
    PresortRec& r = c->rec[k];
    r.valid = false;
    // the other record stays only if it belongs to the current batch (look-ahead / pipelined schedules: its backward pass
    // may still be to come); a batch that was prepared and never trained on leaves nothing behind
    if (c->rec[k ^ 1].valid && c->rec[k ^ 1].ticket != c->cur_ticket) c->rec[k ^ 1].valid = false;
    if (!c->presort || n <= 0 || num_bags <= 0) return slots_out ? FC_ERR_INVALID_ARG : FC_OK;   // the caller then writes the slots out itself
    FC_TRY(ensure_sort(c->sb[k], n));
    FC_HIP(hipEventRecord(c->ev_slots, c->pst));
    FC_HIP(hipStreamWaitEvent(c->aux, c->ev_slots, 0));
    // the record's previous sort was read by a backward pass on the caller's stream, enqueued before this call
    if (c->pst != c->stream) FC_HIP(hipStreamWaitEvent(c->aux, c->ev_s_now, 0));
    // the record's buffers were last written by a sort that may have run on another library stream (the schedule changed)
    // (a record the caller's stream has consumed is covered by the wait for that stream above)
    if (r.sort_stream && r.sort_stream != c->aux && !r.caller_waited) FC_HIP(hipStreamWaitEvent(c->aux, r.ev_sorted, 0));
    // cache_plan_next running ahead (FC_INPUTS_READY while HBM rather than the host link binds the step):
    // the index stream is then the busiest of the schedule, and the next batch's index kernels queue behind this sort; its
    // passes after the first move to the side stream, which only carries the evicted-row block.  Where the host link binds
    // the step, that block copy fills the side stream and the sort must not delay it: measured 7% slower there, 8% faster
    // where HBM binds.
    hipStream_t last = c->aux;
    const bool split = slots_out && c->sort_tail_side && c->ahead_now && c->aux == c->pre &&
                       c->side && c->side != c->aux;
    FC_TRY(sort_pairs(c, c->sb[k], c->aux, slots, n, offsets, num_bags, &r.keys, &r.vals, slots_out, split ? c->side : nullptr, &last));
    FC_HIP(hipEventRecord(r.ev_sorted, last));
    r.sort_stream = last;
    r.caller_waited = false;
    r.slots = slots; r.n = n; r.offsets = offsets; r.bags = num_bags;
    r.ticket = c->ticket;
    r.one_per_bag = c->last_one_per_bag;
    r.valid = true;
    return FC_OK;
}

// The backward pass on stream st with the given scratch: kin / vin = the batch's (slot, bag) pairs sorted by slot, or
// null to sort here into sb; part / pmeta hold 2 rows and one record per workgroup of the reduction.
static int bwd_run(fc_cache* c, hipStream_t st, const int32_t* slots, int64_t n, const int64_t* offsets, int64_t num_bags,
                   const float* grad, float lr, const int32_t* kin, const int32_t* vin, SortBufs& sb, float* part,
                   int32_t* pmeta, fc_cache* prof) {
    int rthreads; int64_t rblocks; size_t lds;
    bwd_geometry(c, n, &rthreads, &rblocks, &lds);
    if (!kin) {
        int bits = 1;
        while (((int64_t)1 << bits) <= c->C) ++bits;           // keys lie in [0, C] (C = out-of-range sentinel)
        SortJob j;
        j.src = SORT_SRC_SLOTS; j.keys_in = slots; j.offsets = offsets; j.num_bags = (int)num_bags; j.n = (int)n;
        j.limit = (int)c->C; j.bits = bits; j.flags = &c->ctl->async_flags;
        j.max_bits = c->sort_max_bits; j.no_fuse = c->sort_no_fuse;
        j.prof = prof;
        FC_TRY(sort_in(j, sb, st, &kin, &vin));      // the scratch of the entry point that allocates nothing has no supertile tables: scan kernels there
    }
    const int sh = shift_of(c->lpr);
    if (c->dirty) k_mark_dirty<<<(unsigned)cdiv(n, 256), 256, 0, st>>>(slots, (int)n, (int)c->C, c->dirty);
    {
        ProfScope ps(prof, P_BWD_REDUCE, st);
        BwdMeta* bm = reinterpret_cast<BwdMeta*>(pmeta);
#define FC_BWD(V, S) \
        k_bwd_reduce<V, S><<<(unsigned)rblocks, rthreads, lds, st>>>(kin, vin, (int)n, (int)c->C, grad, c->cache, c->D, sh, lr, part, bm)
#define FC_BWD_V(S) \
        switch (c->vec) { case 4: FC_BWD(4, S); break; case 2: FC_BWD(2, S); break; default: FC_BWD(1, S); break; }
        if (n == num_bags) { FC_BWD_V(true) } else { FC_BWD_V(false) }
#undef FC_BWD_V
#undef FC_BWD
    }
    {
        ProfScope ps(prof, P_BWD_FIXUP, st);
        const BwdMeta* bm = reinterpret_cast<const BwdMeta*>(pmeta);
        const unsigned fb = (unsigned)cdiv(rblocks, 256 >> sh);
        switch (c->vec) {
            case 4: k_bwd_fixup<4><<<fb, 256, 0, st>>>((int)c->C, c->cache, c->D, sh, lr, part, bm, (int)rblocks); break;
            case 2: k_bwd_fixup<2><<<fb, 256, 0, st>>>((int)c->C, c->cache, c->D, sh, lr, part, bm, (int)rblocks); break;
            default: k_bwd_fixup<1><<<fb, 256, 0, st>>>((int)c->C, c->cache, c->D, sh, lr, part, bm, (int)rblocks); break;
        }
    }
    FC_HIP(hipGetLastError());
    return FC_OK;
}

static int bwd_check_args(fc_cache* c, const int32_t* slots, int64_t n, const int64_t* offsets, int64_t num_bags, const float* grad) {
    const int64_t LIM = ((int64_t)1 << 31) - 65536;
    if (!c || n < 0 || num_bags < 0 || n >= LIM || num_bags >= LIM || !offsets || (n > 0 && (!slots || !grad || num_bags == 0)))
        return FC_ERR_INVALID_ARG;
    return FC_OK;
}

int bwd_impl(fc_cache* c, const int32_t* slots, int64_t n, const int64_t* offsets, int64_t num_bags,
             const float* grad, float lr) {
    FC_TRY(bwd_check_args(c, slots, n, offsets, num_bags, grad));
    if (n == 0) return FC_OK;
    FC_HIP(hipSetDevice(c->device));
    hipStream_t st = c->stream;
    int rthreads; int64_t rblocks; size_t lds;
    bwd_geometry(c, n, &rthreads, &rblocks, &lds);
    FC_TRY(ensure_part(c, rblocks));
    const int32_t* kin = nullptr; const int32_t* vin = nullptr;
    for (PresortRec& r : c->rec) {
        // sorted ahead of time by the call that prepared the current batch, from these very buffers
        if (r.valid && r.ticket == c->cur_ticket && r.slots == slots && r.n == n && r.offsets == offsets && r.bags == num_bags) {
            if (!r.caller_waited) FC_HIP(hipStreamWaitEvent(st, r.ev_sorted, 0));      // sorted ahead of time
            kin = r.keys; vin = r.vals;
            r.valid = false;
            break;
        }
    }
    if (!kin) FC_TRY(ensure_sort(c->sb[2], n));
    return bwd_run(c, st, slots, n, offsets, num_bags, grad, lr, kin, vin, c->sb[2], c->part, c->pmeta, c);
}

// embedding_bag_bwd_sgd for callers that cannot allocate: the same kernels, with the file-scope array `scratch` in
// place of the buffers bwd_impl allocates.  Nothing in the array has to start at zero: the sort's histograms, the digit
// totals and the reduction's per-workgroup records are all written in full before they are read, and a partial row is
// read only where such a record says it was written.
int bwd_noalloc_impl(fc_cache* c, const int32_t* slots, int64_t n, const int64_t* offsets, int64_t num_bags,
                     const float* grad, float lr) {
    FC_TRY(bwd_check_args(c, slots, n, offsets, num_bags, grad));
    if (n > FC_NOALLOC_MAX_IDS) return FC_ERR_SCRATCH_EXCEEDED;
    int rthreads; int64_t rblocks; size_t lds;
    bwd_geometry(c, n > 0 ? n : 1, &rthreads, &rblocks, &lds);
    const size_t a256 = 255;
    const size_t pair_bytes = ((size_t)FC_NOALLOC_MAX_IDS * 4 + a256) & ~a256;
    const size_t ghist_bytes = ((size_t)(cdiv(FC_NOALLOC_MAX_IDS, RS_TILE) << RS_MAX_BITS) * 4 + a256) & ~a256;
    const size_t dtot_bytes = ((size_t)(1 << RS_MAX_BITS) * 4 + a256) & ~a256;
    const size_t fixed = 4 * pair_bytes + ghist_bytes + dtot_bytes;
    const size_t meta_bytes = ((size_t)rblocks * sizeof(BwdMeta) + a256) & ~a256;
    const size_t part_bytes = (size_t)rblocks * 2 * c->D * 4;
    static_assert(4 * (((size_t)FC_NOALLOC_MAX_IDS * 4 + 255) & ~(size_t)255) + (1 << 20) <= FC_NOALLOC_SCRATCH_BYTES, "scratch too small for the sort");
    if (fixed + meta_bytes + part_bytes > (size_t)FC_NOALLOC_SCRATCH_BYTES) return FC_ERR_SCRATCH_EXCEEDED;   // wide rows: fewer lookups fit
    if (n == 0) return FC_OK;
    FC_HIP(hipSetDevice(c->device));
    unsigned char* base = (c->device >= 0 && c->device < NOALLOC_MAX_DEVICES) ? scratch_ptr[c->device] : nullptr;
    if (!base) return FC_ERR_HIP;                    // the array's address on this device was never found
    SortBufs sb;
    unsigned char* p = base;
    sb.keysA = reinterpret_cast<int32_t*>(p); p += pair_bytes;
    sb.valsA = reinterpret_cast<int32_t*>(p); p += pair_bytes;
    sb.keysB = reinterpret_cast<int32_t*>(p); p += pair_bytes;
    sb.valsB = reinterpret_cast<int32_t*>(p); p += pair_bytes;
    sb.ghist = reinterpret_cast<int32_t*>(p); p += ghist_bytes;
    sb.dtot = reinterpret_cast<int32_t*>(p); p += dtot_bytes;
    int32_t* pmeta = reinterpret_cast<int32_t*>(p); p += meta_bytes;
    float* part = reinterpret_cast<float*>(p);
    // no ahead-of-time record is used (its buffers are the library's own allocations) and nothing is timed (timing
    // events are created on demand)
    return bwd_run(c, c->stream, slots, n, offsets, num_bags, grad, lr, nullptr, nullptr, sb, part, pmeta, nullptr);
}

}  // namespace fc
