// Software-managed feature cache in GPU memory in front of a slower feature store (Section 6.5 of the
// paper: an LRU cache of node-feature rows).  Set-associative, updated once per mini-batch in three
// phases (look-ups, per-set replacement in batch order, row copies), so the outcome does not depend on
// the order in which waves run.
#include "cr_common.h"

namespace cr {

constexpr int CNT_QUERIES = 0, CNT_MISSES = 1, CNT_UNCACHED = 2;

struct CacheArgs {
    cr_feature_cache c;
    const char *store;
    int64_t store_ld;
    const int32_t *ids;
    const int32_t *n_ptr;
    int32_t max_n;
    int32_t stamp;
    int32_t *slot_out;
};

constexpr int32_t NO_POS = 0x7FFFFFFF;       // an empty entry of a set's list

// copies one feature row from the store into row `slot` of the cache's row array, by the GW lanes of a group
template <int GW>
__device__ __forceinline__ void copy_row(const CacheArgs &a, int32_t id, int32_t slot, int w)
{
    const int chunks = a.c.row_bytes / 16;
    for (int c = w; c < chunks; c += GW) {
        const uint4 v = *reinterpret_cast<const uint4 *>(a.store + (int64_t)id * a.store_ld + (int64_t)c * 16);
        *reinterpret_cast<uint4 *>(static_cast<char *>(a.c.rows) + (int64_t)slot * a.c.row_bytes + (int64_t)c * 16) = v;
    }
}

// GW lanes (a power of two >= ways) look one node up: lane w compares way w.  A set can give at most `ways` rows to the
// misses of one batch, and by the replacement rule they go to the misses that come FIRST in the batch, so a set's list
// keeps the `ways` smallest batch positions among its misses, whatever order the waves run in: a miss replaces the
// list's largest entry if it is smaller (compare-and-swap on that entry; entries only ever decrease, so the entry that
// was the largest when it was read still is when the swap succeeds).  A miss that cannot enter the list, or is pushed out
// of it, is served from the overflow area: the group that finds this out writes its slot and copies its row right away.
template <int GW>
__global__ __launch_bounds__(256) void cache_lookup_kernel(CacheArgs a)
{
    const int n = min(max(*a.n_ptr, 0), a.max_n);
    if (blockIdx.x == 0 && threadIdx.x == 0) a.c.counters[CNT_QUERIES] += n;
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
        return;
    }
    // a miss (the whole group takes this path together)
    if (w == 0) atomicAdd(&a.c.set_count[set], 1);
    int32_t *list = a.c.set_list + (int64_t)set * CR_CACHE_LIST_CAP;
    int32_t out_pos = -1;                                   // batch position that goes to the overflow area, if any
    for (;;) {
        int32_t vmax = w < a.c.ways ? __hip_atomic_load(&list[w], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : -1;
        int smax = w;
#pragma unroll
        for (int off = GW / 2; off; off >>= 1) {
            const int32_t ov = __shfl_xor(vmax, off, GW);
            const int os = __shfl_xor(smax, off, GW);
            if (ov > vmax || (ov == vmax && os < smax)) { vmax = ov; smax = os; }
        }
        if (i > vmax) { out_pos = i; break; }               // `ways` earlier misses are listed already
        int ok = 0;
        if (w == 0) ok = atomicCAS(&list[smax], vmax, (int32_t)i) == vmax ? 1 : 0;
        ok = __shfl(ok, 0, GW);
        if (ok) { out_pos = vmax == NO_POS ? -1 : vmax; break; }
    }
    if (out_pos >= 0) {
        const int32_t slot = a.c.n_sets * a.c.ways + out_pos;
        if (w == 0) a.slot_out[out_pos] = slot;
        copy_row<GW>(a, a.ids[out_pos], slot, w);
    }
}

// Replacement and row copies.  A fixed grid of waves walks the sets, 64 set counters per load; for a set that took
// misses, the listed misses (the earliest `ways` of the batch) in batch order take the set's rows in (stamp, way) order,
// except rows used in this batch; what is left over goes to the overflow area at the node's position in the batch.  The wave then copies its sets'
// missing rows from the store, 16 bytes per lane.  Counters are accumulated per wave and added once.
__global__ __launch_bounds__(256) void cache_resolve_kernel(CacheArgs a)
{
    __shared__ int way_of_rank[4][WAVE];
    const int lane = lane_id(), wv = threadIdx.x / WAVE;
    const int n_waves = gridDim.x * 4;
    const int wave_id = blockIdx.x * 4 + wv;
    const int chunks = a.c.row_bytes / 16;
    const int n_slots = a.c.n_sets * a.c.ways;
    int misses = 0, uncached = 0;
    for (int base = wave_id * WAVE; base < a.c.n_sets; base += n_waves * WAVE) {
        const int my_cnt = base + lane < a.c.n_sets ? a.c.set_count[base + lane] : 0;
        uint64_t dirty = __ballot(my_cnt > 0);
        while (dirty) {
            const int j = __ffsll((long long)dirty) - 1;
            dirty &= dirty - 1;
            const int set = base + j;
            const int m_all = __builtin_amdgcn_readlane(my_cnt, j);
            const int m = min(m_all, a.c.ways);              // the list holds the set's earliest misses, in its first m entries
            const int64_t s0 = (int64_t)set * a.c.ways;

            const int pos = lane < m ? a.c.set_list[(int64_t)set * CR_CACHE_LIST_CAP + lane] : NO_POS;
            int miss_rank = 0;
            for (int t = 0; t < m; ++t) miss_rank += __builtin_amdgcn_readlane(pos, t) < pos ? 1 : 0;

            const int st = lane < a.c.ways ? a.c.stamps[s0 + lane] : a.stamp;
            const bool elig = lane < a.c.ways && st != a.stamp;
            int way_rank = 0;
            for (int t = 0; t < a.c.ways; ++t) {
                const int sj = __builtin_amdgcn_readlane(st, t);
                way_rank += (sj != a.stamp && (sj < st || (sj == st && t < lane))) ? 1 : 0;
            }
            const int n_avail = __popcll(__ballot(elig));
            if (elig) way_of_rank[wv][way_rank] = lane;
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");

            int32_t id = 0, slot = 0;
            if (lane < m) {
                id = a.ids[pos];
                if (miss_rank < n_avail) {
                    slot = (int32_t)(s0 + way_of_rank[wv][miss_rank]);
                    a.c.keys[slot] = id;
                    a.c.stamps[slot] = a.stamp;
                } else {
                    slot = n_slots + pos;                 // overflow area: one row per batch position
                }
                a.slot_out[pos] = slot;
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // way_of_rank is reused for the next set
            if (lane == 0) a.c.set_count[set] = 0;
            if (lane < m) a.c.set_list[(int64_t)set * CR_CACHE_LIST_CAP + lane] = NO_POS;
            misses += m_all;
            uncached += m_all - min(m, n_avail);

            // copy the m rows: 64 / chunks rows per step when a row is at most 64 lanes wide
            if (chunks <= WAVE) {
                const int per = WAVE / chunks;
                for (int r0 = 0; r0 < m; r0 += per) {
                    const int r = r0 + lane / chunks, c = lane % chunks;
                    const int32_t rid = __shfl(id, r), rslot = __shfl(slot, r);
                    if (lane < per * chunks && r < m) {
                        const uint4 v = *reinterpret_cast<const uint4 *>(a.store + (int64_t)rid * a.store_ld + (int64_t)c * 16);
                        *reinterpret_cast<uint4 *>(static_cast<char *>(a.c.rows) + (int64_t)rslot * a.c.row_bytes + (int64_t)c * 16) = v;
                    }
                }
            } else {
                for (int r = 0; r < m; ++r) {
                    const int32_t rid = __builtin_amdgcn_readlane(id, r), rslot = __builtin_amdgcn_readlane(slot, r);
                    for (int c = lane; c < chunks; c += WAVE) {
                        const uint4 v = *reinterpret_cast<const uint4 *>(a.store + (int64_t)rid * a.store_ld + (int64_t)c * 16);
                        *reinterpret_cast<uint4 *>(static_cast<char *>(a.c.rows) + (int64_t)rslot * a.c.row_bytes + (int64_t)c * 16) = v;
                    }
                }
            }
        }
    }
    if (lane == 0 && misses) {
        atomicAdd(&a.c.counters[CNT_MISSES], misses);
        if (uncached) atomicAdd(&a.c.counters[CNT_UNCACHED], uncached);
    }
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
    if (i < (int64_t)c.n_sets * CR_CACHE_LIST_CAP) c.set_list[i] = NO_POS;
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
    int64_t n = (int64_t)cache->n_sets * CR_CACHE_LIST_CAP;       // >= n_sets * ways, the list array is the longest
    if (n < 8) n = 8;
    hipLaunchKernelGGL(cache_reset_kernel, dim3((unsigned)ceil_div(n, 256)), dim3(256), 0, static_cast<hipStream_t>(stream), *cache);
    CR_LAUNCH_CHECK();
    return CR_OK;
}

extern "C" cr_status cr_cache_fetch(const cr_feature_cache *cache, const void *store, int64_t store_ld_bytes,
                                    const int32_t *ids, const int32_t *hdr, int32_t hdr_word, int32_t max_n,
                                    int32_t stamp, int32_t *slot_out, void *stream)
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
    CacheArgs a;
    a.c = *cache; a.store = static_cast<const char *>(store); a.store_ld = store_ld_bytes; a.ids = ids; a.n_ptr = hdr + hdr_word;
    a.max_n = max_n; a.stamp = stamp; a.slot_out = slot_out;
    if (dry_run()) return CR_OK;

    hipStream_t s = static_cast<hipStream_t>(stream);
    if (cache->ways <= 16) hipLaunchKernelGGL(cache_lookup_kernel<16>, dim3((unsigned)ceil_div(max_n, 16)), dim3(256), 0, s, a);
    else if (cache->ways <= 32) hipLaunchKernelGGL(cache_lookup_kernel<32>, dim3((unsigned)ceil_div(max_n, 8)), dim3(256), 0, s, a);
    else hipLaunchKernelGGL(cache_lookup_kernel<64>, dim3((unsigned)ceil_div(max_n, 4)), dim3(256), 0, s, a);
    int64_t blocks = ceil_div(cache->n_sets, 4 * WAVE);
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(cache_resolve_kernel, dim3((unsigned)blocks), dim3(256), 0, s, a);
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
