// Static module of the cache (paper Section 4.2), built on the GPU: count how often every id occurs in (a sample
// of) the dataset, order the rows by descending count (ties: lower id first) -> idx_map ("freq_rank"), and
// re-order the embedding table accordingly.
#include "fc_internal.h"

#include <limits.h>

#include <new>
#include <vector>

struct fc_freq {
    int64_t N = 0;
    int device = 0;
    hipStream_t stream = nullptr;
    int32_t* counts = nullptr;     // [N]
    int64_t total = 0;             // ids counted so far: no single counter can exceed it
    uint32_t* flags = nullptr;     // EF_ID_RANGE
    int32_t* maxc = nullptr;
};

namespace fc {

constexpr int FQ_THREADS = 256;
constexpr int FQ_ITEMS = 8;
constexpr int FQ_HASH = 4096;      // twice the ids of a workgroup: open addressing always finds a free entry

// counts[id] += occurrences.  Popular ids repeat thousands of times and same-address device atomics serialise,
// so each workgroup first aggregates its 2048 ids in an LDS hash table and sends one atomic per distinct id.
__global__ __launch_bounds__(FQ_THREADS) void k_freq_count(const int64_t* __restrict__ ids, int64_t n, int64_t N,
                                                           int32_t* counts, uint32_t* flags) {
    __shared__ int hkey[FQ_HASH];
    __shared__ int hcnt[FQ_HASH];
    for (int e = threadIdx.x; e < FQ_HASH; e += FQ_THREADS) { hkey[e] = -1; hcnt[e] = 0; }
    __syncthreads();
    const int64_t base = (int64_t)blockIdx.x * FQ_THREADS * FQ_ITEMS;
    bool bad = false;
#pragma unroll
    for (int it = 0; it < FQ_ITEMS; ++it) {
        const int64_t i = base + it * FQ_THREADS + threadIdx.x;
        if (i < n) {
            const int64_t id = ids[i];
            if (id < 0 || id >= N) { bad = true; continue; }
            const int k = (int)id;
            unsigned h = ((unsigned)k * 2654435761u) >> 20;          // 12 bits
            for (;;) {
                const int prev = atomicCAS(&hkey[h], -1, k);
                if (prev == -1 || prev == k) { atomicAdd(&hcnt[h], 1); break; }
                h = (h + 1) & (FQ_HASH - 1);
            }
        }
    }
    __syncthreads();
    for (int e = threadIdx.x; e < FQ_HASH; e += FQ_THREADS)
        if (hkey[e] >= 0) atomicAdd(&counts[hkey[e]], hcnt[e]);
    if (bad) atomicOr(flags, EF_ID_RANGE);
}

__global__ __launch_bounds__(256) void k_max_i32(const int32_t* __restrict__ x, int64_t n, int32_t* out) {
    __shared__ int red[4];
    int m = 0;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) m = max(m, x[i]);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) m = max(m, __shfl_down(m, o));
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) atomicMax(out, max(max(red[0], red[1]), max(red[2], red[3])));
}

// sorted position r holds id inv[r]; the id's rank is r
__global__ __launch_bounds__(256) void k_rank_of(const int32_t* __restrict__ inv, int64_t n, int32_t* __restrict__ rank) {
    const int64_t r = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (r < n) rank[inv[r]] = (int32_t)r;
}

// dst[r, :] = src[inv[r], :]; both tables may be mapped host memory
__global__ __launch_bounds__(256) void k_reorder_rows(float* __restrict__ dst, const float* __restrict__ src,
                                                      const int32_t* __restrict__ inv, int64_t rows, int D, int vec4) {
    const int lane = threadIdx.x & 63;
    const int64_t w0 = ((int64_t)blockIdx.x * 256 + threadIdx.x) >> 6, nw = ((int64_t)gridDim.x * 256) >> 6;
    for (int64_t r = w0; r < rows; r += nw) {
        const float* s = src + (size_t)inv[r] * D;
        float* d = dst + (size_t)r * D;
        if (vec4) { for (int c = lane; c < D / 4; c += 64) reinterpret_cast<float4*>(d)[c] = reinterpret_cast<const float4*>(s)[c]; }
        else { for (int c = lane; c < D; c += 64) d[c] = s[c]; }
    }
}

static void freq_free(fc_freq* f) {
    if (!f) return;
    (void)hipSetDevice(f->device);
    if (f->counts) (void)hipFree(f->counts);
    if (f->flags) (void)hipFree(f->flags);
    if (f->maxc) (void)hipFree(f->maxc);
    delete f;
}

static int freq_init(fc_freq* f, int64_t N, void* stream) {
    FC_HIP(hipGetDevice(&f->device));
    f->N = N; f->stream = (hipStream_t)stream;
    FC_HIP(hipMalloc((void**)&f->counts, (size_t)N * 4));
    FC_HIP(hipMalloc((void**)&f->flags, 4));
    FC_HIP(hipMalloc((void**)&f->maxc, 4));
    FC_HIP(hipMemsetAsync(f->counts, 0, (size_t)N * 4, f->stream));
    FC_HIP(hipMemsetAsync(f->flags, 0, 4, f->stream));
    FC_HIP(hipStreamSynchronize(f->stream));
    return FC_OK;
}

static int freq_build_impl(fc_freq* f, int32_t* freq_rank_host, int32_t* inv_rank_host, int32_t* counts_host) {
    const int64_t N = f->N;
    hipStream_t st = f->stream;
    uint32_t flags = 0;
    FC_HIP(hipMemsetAsync(f->maxc, 0, 4, st));
    k_max_i32<<<1024, 256, 0, st>>>(f->counts, N, f->maxc);
    int32_t maxc = 0;
    FC_HIP(hipMemcpyAsync(&maxc, f->maxc, 4, hipMemcpyDeviceToHost, st));
    FC_HIP(hipMemcpyAsync(&flags, f->flags, 4, hipMemcpyDeviceToHost, st));
    FC_HIP(hipStreamSynchronize(st));
    if (flags & EF_ID_RANGE) return FC_ERR_ID_OUT_OF_RANGE;
    int bits = 1;
    while (((int64_t)1 << bits) <= maxc) ++bits;
    const int64_t nblk = cdiv(N, RS_TILE);
    int32_t* buf[4] = {nullptr, nullptr, nullptr, nullptr};
    int32_t *ghist = nullptr, *dtot = nullptr, *rank = nullptr;
    int rc = FC_OK;
    auto cleanup = [&]() {
        for (int32_t* p : buf) if (p) (void)hipFree(p);
        if (ghist) (void)hipFree(ghist);
        if (dtot) (void)hipFree(dtot);
        if (rank) (void)hipFree(rank);
    };
    auto body = [&]() -> int {
        for (int k = 0; k < 4; ++k) FC_HIP(hipMalloc((void**)&buf[k], (size_t)N * 4));
        FC_HIP(hipMalloc((void**)&ghist, (size_t)(nblk << RS_MAX_BITS) * 4));
        FC_HIP(hipMalloc((void**)&dtot, (size_t)(1 << RS_MAX_BITS) * 4));
        FC_HIP(hipMalloc((void**)&rank, (size_t)N * 4));
        SortJob j;
        j.src = SORT_SRC_COUNTS; j.keys_in = f->counts; j.n = (int)N; j.limit = maxc; j.bits = bits;
        j.keysA = buf[0]; j.valsA = buf[1]; j.keysB = buf[2]; j.valsB = buf[3]; j.ghist = ghist; j.dtot = dtot;
        const int32_t *ks, *vs;
        FC_TRY(radix_sort(j, st, &ks, &vs));       // stable: equal counts keep ascending id order
        k_rank_of<<<(unsigned)cdiv(N, 256), 256, 0, st>>>(vs, N, rank);
        FC_HIP(hipGetLastError());
        if (freq_rank_host) FC_HIP(hipMemcpyAsync(freq_rank_host, rank, (size_t)N * 4, hipMemcpyDeviceToHost, st));
        if (inv_rank_host) FC_HIP(hipMemcpyAsync(inv_rank_host, vs, (size_t)N * 4, hipMemcpyDeviceToHost, st));
        if (counts_host) FC_HIP(hipMemcpyAsync(counts_host, f->counts, (size_t)N * 4, hipMemcpyDeviceToHost, st));
        FC_HIP(hipStreamSynchronize(st));
        return FC_OK;
    };
    rc = body();
    cleanup();
    return rc;
}

static bool pinned_dev_ptr(const void* host, void** dev) {
    hipPointerAttribute_t attr;
    if (hipPointerGetAttributes(&attr, host) != hipSuccess || attr.type != hipMemoryTypeHost) { (void)hipGetLastError(); return false; }
    if (hipHostGetDevicePointer(dev, const_cast<void*>(host), 0) != hipSuccess) { (void)hipGetLastError(); return false; }
    return true;
}

}  // namespace fc

using namespace fc;

extern "C" {

int freq_create(int64_t num_rows, void* hip_stream, fc_freq** out) {
    const int64_t LIM = ((int64_t)1 << 31) - 65536;
    if (!out) return FC_ERR_INVALID_ARG;
    *out = nullptr;
    if (num_rows <= 0 || num_rows >= LIM) return FC_ERR_INVALID_ARG;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev <= 0) { (void)hipGetLastError(); return FC_ERR_HIP; }
    fc_freq* f = new (std::nothrow) fc_freq();
    if (!f) return FC_ERR_INVALID_ARG;
    const int rc = freq_init(f, num_rows, hip_stream);
    if (rc != FC_OK) { freq_free(f); return rc; }
    *out = f;
    return FC_OK;
}

int freq_add(fc_freq* f, const int64_t* ids_dev, int64_t n) {
    if (!f || n < 0 || (n > 0 && !ids_dev)) return FC_ERR_INVALID_ARG;
    if (n == 0) return FC_OK;
    // counters are 32 bits wide: an id that occurred more than 2^31 - 1 times would wrap around unnoticed, so the
    // accumulator takes at most that many ids in all (larger datasets are sampled, as Section 4.2 suggests)
    if (f->total + n > (int64_t)INT32_MAX) return FC_ERR_COUNT_OVERFLOW;
    f->total += n;
    FC_HIP(hipSetDevice(f->device));
    k_freq_count<<<(unsigned)cdiv(n, FQ_THREADS * FQ_ITEMS), FQ_THREADS, 0, f->stream>>>(ids_dev, n, f->N, f->counts, f->flags);
    FC_HIP(hipGetLastError());
    return FC_OK;
}

int freq_build(fc_freq* f, int32_t* freq_rank_host, int32_t* inv_rank_host, int32_t* counts_host) {
    if (!f) return FC_ERR_INVALID_ARG;
    FC_HIP(hipSetDevice(f->device));
    return freq_build_impl(f, freq_rank_host, inv_rank_host, counts_host);
}

int freq_destroy(fc_freq* f) {
    if (!f) return FC_ERR_INVALID_ARG;
    (void)hipSetDevice(f->device);
    (void)hipStreamSynchronize(f->stream);
    freq_free(f);
    return FC_OK;
}

int table_reorder(const float* src_pinned, float* dst_pinned, const int32_t* inv_rank_host, int64_t num_rows, int32_t dim,
                  void* hip_stream) {
    const int64_t LIM = ((int64_t)1 << 31) - 65536;
    if (!src_pinned || !dst_pinned || !inv_rank_host || num_rows <= 0 || num_rows >= LIM || dim <= 0 || src_pinned == dst_pinned)
        return FC_ERR_INVALID_ARG;
    for (int64_t r = 0; r < num_rows; ++r) if (inv_rank_host[r] < 0 || inv_rank_host[r] >= num_rows) return FC_ERR_NOT_PERMUTATION;
    void *sd = nullptr, *dd = nullptr;
    if (!pinned_dev_ptr(src_pinned, &sd) || !pinned_dev_ptr(dst_pinned, &dd)) return FC_ERR_NOT_PINNED;
    hipStream_t st = (hipStream_t)hip_stream;
    int32_t* inv = nullptr;
    FC_HIP(hipMalloc((void**)&inv, (size_t)num_rows * 4));
    int rc = FC_OK;
    auto body = [&]() -> int {
        FC_HIP(hipMemcpyAsync(inv, inv_rank_host, (size_t)num_rows * 4, hipMemcpyHostToDevice, st));
        k_reorder_rows<<<4096, 256, 0, st>>>((float*)dd, (const float*)sd, inv, num_rows, dim, dim % 4 == 0);
        FC_HIP(hipGetLastError());
        FC_HIP(hipStreamSynchronize(st));
        return FC_OK;
    };
    rc = body();
    (void)hipFree(inv);
    return rc;
}

}  // extern "C"
