// Software-managed feature cache in GPU memory in front of a slower feature store (Section 6.5 of the
// paper: an LRU cache of node-feature rows).  Set-associative, updated once per mini-batch in three
// phases (look-ups, per-set replacement in batch order, row copies), so the outcome does not depend on
// the order in which waves run.
#include "cr_common.h"

namespace cr {

constexpr int CNT_QUERIES = 0, CNT_MISSES = 1, CNT_UNCACHED = 2, CNT_STATUS = 3, CNT_DIRTY = 4, CNT_FILL = 5, CNT_OVER = 6;

struct CacheArgs {
    cr_feature_cache c;
    const char *store;
    int64_t store_ld;
    const int32_t *ids;
    const int32_t *n_ptr;
    int32_t max_n;
    int32_t stamp;
    int32_t *slot_out;
    int32_t *dirty;       // [max_n] sets that took a miss in this batch
    int32_t *fill_src;    // [max_n] node id of every row to copy
    int32_t *fill_dst;    // [max_n] its destination row
};

__global__ void cache_begin_kernel(CacheArgs a)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        const int n = min(max(*a.n_ptr, 0), a.max_n);
        a.c.counters[CNT_QUERIES] += n;
        a.c.counters[CNT_DIRTY] = 0;
        a.c.counters[CNT_FILL] = 0;
        a.c.counters[CNT_OVER] = 0;
    }
}

// GW lanes (a power of two >= ways) look one node up: lane w compares way w
template <int GW>
__global__ __launch_bounds__(256) void cache_lookup_kernel(CacheArgs a)
{
    const int n = min(max(*a.n_ptr, 0), a.max_n);
    const int i = (int)(blockIdx.x * (256 / GW) + threadIdx.x / GW);
    if (i >= n) return;
    const int w = threadIdx.x % GW, lane = lane_id();
    const int32_t id = a.ids[i];
    const int set = (int)((uint32_t)id % (uint32_t)a.c.n_sets);
    const int64_t s0 = (int64_t)set * a.c.ways;
    const bool match = w < a.c.ways && a.c.keys[s0 + w] == id;
    const uint64_t all = __ballot(match);
    const uint64_t mine = GW == 64 ? all : (all >> (lane & ~(GW - 1))) & ((1ull << GW) - 1ull);
    if (mine) {
        if (match) {
            a.c.stamps[s0 + w] = a.stamp;
            a.slot_out[i] = (int32_t)(s0 + w);
        }
    } else if (w == 0) {
        const int r = atomicAdd(&a.c.set_count[set], 1);
        if (r < CR_CACHE_LIST_CAP) a.c.set_list[(int64_t)set * CR_CACHE_LIST_CAP + r] = i;
        else atomicOr(&a.c.counters[CNT_STATUS], 1);
        if (r == 0) a.dirty[atomicAdd(&a.c.counters[CNT_DIRTY], 1)] = set;
    }
}

// One wave per set that took misses: the misses in batch order take the set's rows in (stamp, way) order,
// except rows used in this batch; what is left over goes to the overflow area.
__global__ __launch_bounds__(256) void cache_resolve_kernel(CacheArgs a)
{
    __shared__ int way_of_rank[4][WAVE];
    const int d = (int)(blockIdx.x * 4 + threadIdx.x / WAVE);
    if (d >= a.c.counters[CNT_DIRTY]) return;
    const int lane = lane_id(), wv = threadIdx.x / WAVE;
    const int set = a.dirty[d];
    const int m_all = a.c.set_count[set];
    const int m = min(m_all, (int)CR_CACHE_LIST_CAP);
    const int64_t s0 = (int64_t)set * a.c.ways;

    const int pos = lane < m ? a.c.set_list[(int64_t)set * CR_CACHE_LIST_CAP + lane] : 0x7FFFFFFF;
    int miss_rank = 0;
    for (int j = 0; j < m; ++j) miss_rank += __builtin_amdgcn_readlane(pos, j) < pos ? 1 : 0;

    const int st = lane < a.c.ways ? a.c.stamps[s0 + lane] : a.stamp;
    const bool elig = lane < a.c.ways && st != a.stamp;
    int way_rank = 0;
    for (int j = 0; j < a.c.ways; ++j) {
        const int sj = __builtin_amdgcn_readlane(st, j);
        way_rank += (sj != a.stamp && (sj < st || (sj == st && j < lane))) ? 1 : 0;
    }
    const int n_avail = __popcll(__ballot(elig));
    if (elig) way_of_rank[wv][way_rank] = lane;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");

    if (lane < m) {
        const int32_t id = a.ids[pos];
        int32_t slot;
        if (miss_rank < n_avail) {
            slot = (int32_t)(s0 + way_of_rank[wv][miss_rank]);
            a.c.keys[slot] = id;
            a.c.stamps[slot] = a.stamp;
        } else {
            const int o = atomicAdd(&a.c.counters[CNT_OVER], 1);
            if (o >= a.c.n_overflow) atomicOr(&a.c.counters[CNT_STATUS], 2);
            slot = a.c.n_sets * a.c.ways + min(o, a.c.n_overflow - 1);
        }
        a.slot_out[pos] = slot;
        const int f = atomicAdd(&a.c.counters[CNT_FILL], 1);
        a.fill_src[f] = id;
        a.fill_dst[f] = slot;
    }
    if (lane == 0) {
        a.c.set_count[set] = 0;
        atomicAdd(&a.c.counters[CNT_MISSES], m_all);
    }
}

// copies the missing rows from the store, 16 bytes per thread
__global__ __launch_bounds__(256) void cache_fill_kernel(CacheArgs a)
{
    const int chunks = a.c.row_bytes / 16;
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t f = gid / chunks;
    const int c = (int)(gid % chunks);
    const int n_fill = a.c.counters[CNT_FILL];
    if (gid == 0) a.c.counters[CNT_UNCACHED] += a.c.counters[CNT_OVER];
    if (f >= n_fill) return;
    const uint4 v = *reinterpret_cast<const uint4 *>(a.store + (int64_t)a.fill_src[f] * a.store_ld + (int64_t)c * 16);
    *reinterpret_cast<uint4 *>(static_cast<char *>(a.c.rows) + (int64_t)a.fill_dst[f] * a.c.row_bytes + (int64_t)c * 16) = v;
}

__global__ __launch_bounds__(256) void stage_rows_kernel(const char *__restrict__ store, int64_t store_ld, const int32_t *__restrict__ ids,
                                                        const int32_t *__restrict__ n_ptr, int max_n, char *__restrict__ out, int row_bytes)
{
    const int chunks = row_bytes / 16;
    const int n = min(max(*n_ptr, 0), max_n);
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t i = gid / chunks;
    const int c = (int)(gid % chunks);
    if (i >= n) return;
    const uint4 v = *reinterpret_cast<const uint4 *>(store + (int64_t)ids[i] * store_ld + (int64_t)c * 16);
    *reinterpret_cast<uint4 *>(out + i * row_bytes + (int64_t)c * 16) = v;
}

__global__ __launch_bounds__(256) void cache_reset_kernel(cr_feature_cache c)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t slots = (int64_t)c.n_sets * c.ways;
    if (i < slots) { c.keys[i] = -1; c.stamps[i] = -1; }
    if (i < c.n_sets) c.set_count[i] = 0;
    if (i < 8) c.counters[i] = 0;
}

}  // namespace cr

using namespace cr;

static cr_status check_cache(const cr_feature_cache *c)
{
    CR_REQUIRE(c != nullptr, CR_ERR_INVALID_ARG, "cache is NULL");
    CR_REQUIRE(c->n_sets >= 1 && c->ways >= 1 && c->ways <= CR_CACHE_MAX_WAYS, CR_ERR_INVALID_ARG,
               "cache of %d sets x %d ways: need n_sets >= 1 and 1 <= ways <= %d", c->n_sets, c->ways, CR_CACHE_MAX_WAYS);
    CR_REQUIRE((int64_t)c->n_sets * c->ways + c->n_overflow <= 0x7FFFFFFFll, CR_ERR_UNSUPPORTED, "cache rows exceed 2^31");
    CR_REQUIRE(c->row_bytes >= 16 && c->row_bytes % 16 == 0, CR_ERR_INVALID_ARG, "row_bytes = %d must be a positive multiple of 16", c->row_bytes);
    CR_REQUIRE(c->n_overflow >= 1, CR_ERR_INVALID_ARG, "n_overflow must be positive");
    CR_REQUIRE(c->keys && c->stamps && c->rows && c->set_count && c->set_list && c->counters, CR_ERR_INVALID_ARG, "cache has a NULL array");
    CR_REQUIRE(aligned16(c->rows), CR_ERR_INVALID_ARG, "cache rows must be 16-byte aligned");
    return CR_OK;
}

extern "C" cr_status cr_cache_reset(const cr_feature_cache *cache, void *stream)
{
    cr_status st = check_cache(cache);
    if (st != CR_OK) return st;
    if (dry_run()) return CR_OK;
    int64_t n = (int64_t)cache->n_sets * cache->ways;
    if (n < 8) n = 8;
    hipLaunchKernelGGL(cache_reset_kernel, dim3((unsigned)ceil_div(n, 256)), dim3(256), 0, static_cast<hipStream_t>(stream), *cache);
    CR_LAUNCH_CHECK();
    return CR_OK;
}

extern "C" cr_status cr_cache_fetch_workspace_bytes(int32_t max_n, size_t *bytes)
{
    CR_REQUIRE(bytes != nullptr && max_n >= 1, CR_ERR_INVALID_ARG, "bytes must not be NULL and max_n must be positive");
    Carver c(nullptr);
    c.take<int32_t>((size_t)max_n);
    c.take<int32_t>((size_t)max_n);
    c.take<int32_t>((size_t)max_n);
    *bytes = c.bytes();
    return CR_OK;
}

extern "C" cr_status cr_cache_fetch(const cr_feature_cache *cache, const void *store, int64_t store_ld_bytes,
                                    const int32_t *ids, const int32_t *hdr, int32_t hdr_word, int32_t max_n,
                                    int32_t stamp, int32_t *slot_out, void *ws, size_t ws_bytes, void *stream)
{
    cr_status st = check_cache(cache);
    if (st != CR_OK) return st;
    CR_REQUIRE(store != nullptr && aligned16(store), CR_ERR_INVALID_ARG, "store must be a 16-byte aligned pointer the GPU can read");
    CR_REQUIRE(store_ld_bytes >= cache->row_bytes && store_ld_bytes % 16 == 0, CR_ERR_INVALID_ARG,
               "store_ld_bytes = %lld must be a multiple of 16 covering row_bytes = %d", (long long)store_ld_bytes, cache->row_bytes);
    CR_REQUIRE(ids && hdr && slot_out, CR_ERR_INVALID_ARG, "ids / hdr / slot_out must not be NULL");
    CR_REQUIRE(hdr_word >= 0 && hdr_word < CR_HDR_WORDS, CR_ERR_INVALID_ARG, "hdr_word outside 0..%d", CR_HDR_WORDS - 1);
    CR_REQUIRE(max_n >= 1 && stamp >= 0, CR_ERR_INVALID_ARG, "max_n must be positive and stamp non-negative");
    CR_REQUIRE(cache->n_overflow >= max_n, CR_ERR_CAPACITY, "overflow area of %d rows, %d needed (max_n)", cache->n_overflow, max_n);
    Carver c(ws);
    CacheArgs a;
    a.c = *cache; a.store = static_cast<const char *>(store); a.store_ld = store_ld_bytes; a.ids = ids; a.n_ptr = hdr + hdr_word;
    a.max_n = max_n; a.stamp = stamp; a.slot_out = slot_out;
    a.dirty = c.take<int32_t>((size_t)max_n);
    a.fill_src = c.take<int32_t>((size_t)max_n);
    a.fill_dst = c.take<int32_t>((size_t)max_n);
    CR_REQUIRE(ws != nullptr && aligned16(ws), CR_ERR_INVALID_ARG, "workspace must be a 16-byte aligned device pointer");
    CR_REQUIRE(ws_bytes >= c.bytes(), CR_ERR_CAPACITY, "workspace of %zu bytes, %zu needed", ws_bytes, c.bytes());
    if (dry_run()) return CR_OK;

    hipStream_t s = static_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(cache_begin_kernel, dim3(1), dim3(64), 0, s, a);
    if (cache->ways <= 16) hipLaunchKernelGGL(cache_lookup_kernel<16>, dim3((unsigned)ceil_div(max_n, 16)), dim3(256), 0, s, a);
    else if (cache->ways <= 32) hipLaunchKernelGGL(cache_lookup_kernel<32>, dim3((unsigned)ceil_div(max_n, 8)), dim3(256), 0, s, a);
    else hipLaunchKernelGGL(cache_lookup_kernel<64>, dim3((unsigned)ceil_div(max_n, 4)), dim3(256), 0, s, a);
    const int64_t max_dirty = max_n < cache->n_sets ? max_n : cache->n_sets;
    hipLaunchKernelGGL(cache_resolve_kernel, dim3((unsigned)ceil_div(max_dirty, 4)), dim3(256), 0, s, a);
    hipLaunchKernelGGL(cache_fill_kernel, dim3((unsigned)ceil_div((int64_t)max_n * (cache->row_bytes / 16), 256)), dim3(256), 0, s, a);
    CR_LAUNCH_CHECK();
    return CR_OK;
}

extern "C" cr_status cr_stage_rows(const void *store, int64_t store_ld_bytes, const int32_t *ids, const int32_t *hdr,
                                   int32_t hdr_word, int32_t max_n, void *rows_out, int32_t row_bytes, void *stream)
{
    CR_REQUIRE(store != nullptr && aligned16(store), CR_ERR_INVALID_ARG, "store must be a 16-byte aligned pointer the GPU can read");
    CR_REQUIRE(row_bytes >= 16 && row_bytes % 16 == 0, CR_ERR_INVALID_ARG, "row_bytes = %d must be a positive multiple of 16", row_bytes);
    CR_REQUIRE(store_ld_bytes >= row_bytes && store_ld_bytes % 16 == 0, CR_ERR_INVALID_ARG,
               "store_ld_bytes = %lld must be a multiple of 16 covering row_bytes = %d", (long long)store_ld_bytes, row_bytes);
    CR_REQUIRE(ids && hdr && rows_out && aligned16(rows_out), CR_ERR_INVALID_ARG, "ids / hdr / rows_out must not be NULL (rows_out 16-byte aligned)");
    CR_REQUIRE(hdr_word >= 0 && hdr_word < CR_HDR_WORDS, CR_ERR_INVALID_ARG, "hdr_word outside 0..%d", CR_HDR_WORDS - 1);
    CR_REQUIRE(max_n >= 1, CR_ERR_INVALID_ARG, "max_n must be positive");
    if (dry_run()) return CR_OK;
    hipLaunchKernelGGL(stage_rows_kernel, dim3((unsigned)ceil_div((int64_t)max_n * (row_bytes / 16), 256)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), static_cast<const char *>(store), store_ld_bytes, ids, hdr + hdr_word, max_n,
                       static_cast<char *>(rows_out), row_bytes);
    CR_LAUNCH_CHECK();
    return CR_OK;
}

extern "C" cr_status cr_host_alloc(size_t bytes, void **host_ptr, void **device_ptr)
{
    CR_REQUIRE(host_ptr != nullptr && device_ptr != nullptr && bytes >= 1, CR_ERR_INVALID_ARG, "host_ptr / device_ptr must not be NULL and bytes must be positive");
    *host_ptr = nullptr;
    *device_ptr = nullptr;
    if (dry_run()) return CR_OK;
    void *h = nullptr, *d = nullptr;
    CR_HIP_CHECK(hipHostMalloc(&h, bytes, hipHostMallocMapped));
    hipError_t e = hipHostGetDevicePointer(&d, h, 0);
    if (e != hipSuccess) {
        (void)hipHostFree(h);
        set_error("hipHostGetDevicePointer failed: %s", hipGetErrorString(e));
        return CR_ERR_HIP;
    }
    *host_ptr = h;
    *device_ptr = d;
    return CR_OK;
}

extern "C" cr_status cr_host_free(void *host_ptr)
{
    if (host_ptr == nullptr || dry_run()) return CR_OK;
    CR_HIP_CHECK(hipHostFree(host_ptr));
    return CR_OK;
}
