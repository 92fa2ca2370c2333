// Root node partitioning (Algorithm 1 Step-1; Section 4.1; Table 1): the epoch's permutation of the
// training set under NORAND-ROOTS, COMM-RAND-MIX and RAND-ROOTS.  Every shuffle is a stable
// least-significant-digit radix sort by a Philox key, started from ascending ids, so equal keys
// keep the smaller id first and the result does not depend on scheduling.
#include <mutex>

#include "cr_common.h"

namespace cr {

constexpr int SORT_TILE = 2048;   // keys per single-wave workgroup

// digit histogram of one tile -> hist[digit * nblk + block]
__global__ __launch_bounds__(64) void radix_hist_kernel(const uint64_t *__restrict__ keys, int n, int shift, int nblk,
                                                        int32_t *__restrict__ hist)
{
    __shared__ int cnt[256];
    for (int i = threadIdx.x; i < 256; i += 64) cnt[i] = 0;
    __syncthreads();
    const int start = blockIdx.x * SORT_TILE;
    const int stop = min(n, start + SORT_TILE);
    for (int i = start + threadIdx.x; i < stop; i += 64) atomicAdd(&cnt[(int)((keys[i] >> shift) & 255u)], 1);
    __syncthreads();
    for (int d = threadIdx.x; d < 256; d += 64) hist[d * nblk + blockIdx.x] = cnt[d];
}

// in-place exclusive scan of the histogram table (one workgroup)
__global__ __launch_bounds__(1024) void radix_scan_kernel(int32_t *hist, int n)
{
    __shared__ int lds[17];
    scan_chunked(hist, hist, nullptr, n, lds);
}

// stable scatter: the wave walks its tile 64 keys at a time; within a chunk a key's rank among the
// keys with the same digit comes from eight ballots
__global__ __launch_bounds__(64) void radix_scatter_kernel(const uint64_t *__restrict__ keys_in,
                                                           const uint32_t *__restrict__ vals_in, int n, int shift, int nblk,
                                                           const int32_t *__restrict__ offs, uint64_t *__restrict__ keys_out,
                                                           uint32_t *__restrict__ vals_out)
{
    __shared__ int cursor[256];
    for (int d = threadIdx.x; d < 256; d += 64) cursor[d] = offs[d * nblk + blockIdx.x];
    __syncthreads();
    const int start = blockIdx.x * SORT_TILE;
    const int stop = min(n, start + SORT_TILE);
    const int lane = lane_id();
    for (int c = start; c < stop; c += 64) {
        const int i = c + lane;
        const bool have = i < stop;
        uint64_t key = 0;
        uint32_t val = 0;
        if (have) { key = keys_in[i]; val = vals_in[i]; }
        const uint32_t d = (uint32_t)((key >> shift) & 255u);
        uint64_t peers = __ballot(have);
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const uint64_t m = __ballot(have && ((d >> b) & 1u));
            peers &= ((d >> b) & 1u) ? m : ~m;
        }
        const uint64_t below = peers & ((1ull << lane) - 1ull);
        int pos = 0;
        if (have) pos = cursor[d] + __popcll(below);
        __syncthreads();
        if (have && below == 0) cursor[d] += __popcll(peers);
        __syncthreads();
        if (have) { keys_out[pos] = key; vals_out[pos] = val; }
    }
}

__global__ __launch_bounds__(256) void zero_i32_kernel(int32_t *p, int64_t n)
{
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) p[i] = 0;
}

__global__ __launch_bounds__(256) void mark_present_kernel(const int32_t *__restrict__ train, int n_train,
                                                           const int32_t *__restrict__ comm, int32_t *present)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n_train) present[comm[train[i]]] = 1;
}

// communities: key = Philox key of the community; absent ones sort behind every present one
__global__ __launch_bounds__(256) void community_keys_kernel(const int32_t *__restrict__ present, int n_comm, uint64_t seed,
                                                             uint32_t epoch, uint64_t *keys, uint64_t *absent, uint32_t *vals)
{
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c >= n_comm) return;
    keys[c] = shuffle_key(seed, epoch, DOMAIN_COMMUNITY, (uint32_t)c);
    absent[c] = present[c] ? 0ull : 1ull;
    vals[c] = (uint32_t)c;
}

// carry a one-bit key through an earlier permutation
__global__ __launch_bounds__(256) void gather_flag_kernel(const uint32_t *__restrict__ vals, int n,
                                                          const uint64_t *__restrict__ flag_by_id, uint64_t *keys)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) keys[i] = flag_by_id[vals[i]];
}

__global__ __launch_bounds__(256) void block_of_kernel(const uint32_t *__restrict__ sorted_comm, int n_comm, int mix,
                                                       int32_t *block_of)
{
    const int r = blockIdx.x * 256 + threadIdx.x;
    if (r < n_comm) block_of[sorted_comm[r]] = r / mix;
}

__global__ __launch_bounds__(256) void node_keys_kernel(const int32_t *__restrict__ train, int n, uint64_t seed, uint32_t epoch,
                                                        uint64_t *keys, uint32_t *vals)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const uint32_t v = (uint32_t)train[i];
    keys[i] = shuffle_key(seed, epoch, DOMAIN_NODE, v);
    vals[i] = v;
}

__global__ __launch_bounds__(256) void super_block_keys_kernel(const uint32_t *__restrict__ vals, int n,
                                                               const int32_t *__restrict__ comm,
                                                               const int32_t *__restrict__ block_of, uint64_t *keys)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) keys[i] = (uint64_t)(uint32_t)block_of[comm[vals[i]]];
}

__global__ __launch_bounds__(256) void copy_i32_kernel(const int32_t *__restrict__ in, int n, int32_t *out)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) out[i] = in[i];
}

struct SortBuffers {
    uint64_t *keys[2];
    uint32_t *vals[2];
    int32_t *hist;
    int cur = 0;
};

// sorts (keys[cur], vals[cur]) by bits [0, bits) of the key; the result ends up in [cur]
static void radix_sort(SortBuffers &b, int n, int bits, hipStream_t s)
{
    if (n <= 0) return;
    const int nblk = (int)ceil_div(n, SORT_TILE);
    for (int shift = 0; shift < bits; shift += 8) {
        const int o = b.cur ^ 1;
        hipLaunchKernelGGL(radix_hist_kernel, dim3(nblk), dim3(64), 0, s, b.keys[b.cur], n, shift, nblk, b.hist);
        hipLaunchKernelGGL(radix_scan_kernel, dim3(1), dim3(1024), 0, s, b.hist, 256 * nblk);
        hipLaunchKernelGGL(radix_scatter_kernel, dim3(nblk), dim3(64), 0, s, b.keys[b.cur], b.vals[b.cur], n, shift, nblk,
                           b.hist, b.keys[o], b.vals[o]);
        b.cur = o;
    }
}

struct BatchPlan {
    uint64_t *keys[2];
    uint32_t *vals[2];
    int32_t *hist;
    int32_t *present;
    uint64_t *absent;
    int32_t *block_of;
    size_t bytes;
};

static void plan_batches(int64_t n_train, int32_t n_comm, void *ws, BatchPlan &p)
{
    const size_t n = (size_t)(n_train > n_comm ? n_train : n_comm) + 1;
    Carver c(ws);
    p.keys[0] = c.take<uint64_t>(n);
    p.keys[1] = c.take<uint64_t>(n);
    p.vals[0] = c.take<uint32_t>(n);
    p.vals[1] = c.take<uint32_t>(n);
    p.hist = c.take<int32_t>(256 * (size_t)ceil_div((int64_t)n, SORT_TILE) + 1);
    p.present = c.take<int32_t>((size_t)n_comm);
    p.absent = c.take<uint64_t>((size_t)n_comm);
    p.block_of = c.take<int32_t>((size_t)n_comm);
    p.bytes = c.bytes();
}

}  // namespace cr

using namespace cr;

extern "C" cr_status cr_build_batches_workspace_bytes(int64_t n_train, int32_t n_comm, size_t *bytes)
{
    CR_REQUIRE(n_train >= 0 && n_train < 0x7FFFFFFF, CR_ERR_INVALID_ARG, "n_train must be in 0..2^31-2");
    CR_REQUIRE(n_comm >= 1, CR_ERR_INVALID_ARG, "n_comm must be positive");
    CR_REQUIRE(bytes != nullptr, CR_ERR_INVALID_ARG, "bytes is NULL");
    BatchPlan p;
    plan_batches(n_train, n_comm, nullptr, p);
    *bytes = p.bytes;
    return CR_OK;
}

static cr_status build_batches_impl(const cr_batch_cfg *cfg, const int32_t *train_ids, int64_t n_train,
                                    const int32_t *comm, int32_t n_comm, void *ws, size_t ws_bytes,
                                    int32_t *out_perm, int64_t *out_n_batches, void *stream)
{
    BatchPlan p;
    plan_batches(n_train, n_comm, ws, p);
    CR_REQUIRE(ws != nullptr && aligned16(ws), CR_ERR_INVALID_ARG, "workspace must be a 16-byte aligned device pointer");
    CR_REQUIRE(ws_bytes >= p.bytes, CR_ERR_CAPACITY, "workspace of %zu bytes, %zu needed", ws_bytes, p.bytes);
    if (out_n_batches) *out_n_batches = ceil_div(n_train, cfg->batch_size);
    if (dry_run() || n_train == 0) return CR_OK;

    hipStream_t s = static_cast<hipStream_t>(stream);
    const int n = (int)n_train;
    const dim3 blk(256);
    const dim3 grid_n((unsigned)ceil_div(n, 256)), grid_c((unsigned)ceil_div(n_comm, 256));
    if (cfg->policy == CR_ROOTS_NORAND) {
        hipLaunchKernelGGL(copy_i32_kernel, grid_n, blk, 0, s, train_ids, n, out_perm);
        CR_LAUNCH_CHECK();
        return CR_OK;
    }
    SortBuffers b;
    b.keys[0] = p.keys[0]; b.keys[1] = p.keys[1]; b.vals[0] = p.vals[0]; b.vals[1] = p.vals[1]; b.hist = p.hist;
    const bool comm_rand = cfg->policy == CR_ROOTS_COMM_RAND && cfg->mix_count < n_comm;
    if (comm_rand) {
        // order of the communities present in the training set: by (key, id), absent ones last
        hipLaunchKernelGGL(zero_i32_kernel, grid_c, blk, 0, s, p.present, (int64_t)n_comm);
        hipLaunchKernelGGL(mark_present_kernel, grid_n, blk, 0, s, train_ids, n, comm, p.present);
        b.cur = 0;
        hipLaunchKernelGGL(community_keys_kernel, grid_c, blk, 0, s, p.present, n_comm, cfg->seed, cfg->epoch, b.keys[0], p.absent, b.vals[0]);
        radix_sort(b, n_comm, 64, s);
        hipLaunchKernelGGL(gather_flag_kernel, grid_c, blk, 0, s, b.vals[b.cur], n_comm, p.absent, b.keys[b.cur]);
        radix_sort(b, n_comm, 1, s);
        hipLaunchKernelGGL(block_of_kernel, grid_c, blk, 0, s, b.vals[b.cur], n_comm, cfg->mix_count, p.block_of);
    }
    // shuffle inside the super-blocks: sort by node key, then stably by super-block number
    b.cur = 0;
    hipLaunchKernelGGL(node_keys_kernel, grid_n, blk, 0, s, train_ids, n, cfg->seed, cfg->epoch, b.keys[0], b.vals[0]);
    radix_sort(b, n, 64, s);
    if (comm_rand) {
        hipLaunchKernelGGL(super_block_keys_kernel, grid_n, blk, 0, s, b.vals[b.cur], n, comm, p.block_of, b.keys[b.cur]);
        int bits = 1;
        const int64_t n_blocks = ceil_div(n_comm, cfg->mix_count);
        while ((1ll << bits) < n_blocks) ++bits;
        radix_sort(b, n, bits, s);
    }
    hipLaunchKernelGGL(copy_i32_kernel, grid_n, blk, 0, s, reinterpret_cast<const int32_t *>(b.vals[b.cur]), n, out_perm);
    CR_LAUNCH_CHECK();
    return CR_OK;
}

static cr_status check_batch_args(const cr_batch_cfg *cfg, const int32_t *train_ids, int64_t n_train, const int32_t *comm,
                                  int32_t n_comm, const int32_t *out_perm)
{
    CR_REQUIRE(cfg != nullptr, CR_ERR_INVALID_ARG, "cfg is NULL");
    CR_REQUIRE(cfg->policy >= CR_ROOTS_NORAND && cfg->policy <= CR_ROOTS_RAND, CR_ERR_INVALID_ARG, "unknown root policy %d", cfg->policy);
    CR_REQUIRE(cfg->policy != CR_ROOTS_COMM_RAND || cfg->mix_count >= 1, CR_ERR_INVALID_ARG, "mix_count must be >= 1");
    CR_REQUIRE(cfg->batch_size >= 1, CR_ERR_INVALID_ARG, "batch_size must be positive");
    CR_REQUIRE(cfg->epoch < (1u << 24), CR_ERR_INVALID_ARG, "epoch must be below 2^24");
    CR_REQUIRE(n_train >= 0 && n_train < 0x7FFFFFFF, CR_ERR_INVALID_ARG, "n_train must be in 0..2^31-2");
    CR_REQUIRE(n_comm >= 1, CR_ERR_INVALID_ARG, "n_comm must be positive");
    CR_REQUIRE(n_train == 0 || (train_ids && out_perm), CR_ERR_INVALID_ARG, "train_ids / out_perm must not be NULL");
    CR_REQUIRE(comm != nullptr, CR_ERR_INVALID_ARG, "comm is NULL");
    return CR_OK;
}

extern "C" cr_status cr_build_batches(const cr_batch_cfg *cfg, const int32_t *train_ids, int64_t n_train,
                                      const int32_t *comm, int32_t n_comm, void *ws, size_t ws_bytes,
                                      int32_t *out_perm, int64_t *out_n_batches, void *stream)
{
    cr_status st = check_batch_args(cfg, train_ids, n_train, comm, n_comm, out_perm);
    if (st != CR_OK) return st;
    return build_batches_impl(cfg, train_ids, n_train, comm, n_comm, ws, ws_bytes, out_perm, out_n_batches, stream);
}

// ---------------------------------------------------------------------------------------------
// The same without a caller workspace: sort buffers, histograms and community tables live in a fixed device array of
// this library.  Host code never uses the array's name as an address: the array's device address is looked up once
// per device and kept.
// ---------------------------------------------------------------------------------------------
constexpr size_t STATIC_SCRATCH_BYTES = 8u << 20;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
std::mutex scratch_mutex;
void *scratch_ptr[MAX_DEVICES] = {};
}  // namespace

extern "C" cr_status cr_build_batches_static(const cr_batch_cfg *cfg, const int32_t *train_ids, int64_t n_train,
                                             const int32_t *comm, int32_t n_comm, int32_t *out_perm,
                                             int64_t *out_n_batches, void *stream)
{
    cr_status st = check_batch_args(cfg, train_ids, n_train, comm, n_comm, out_perm);
    if (st != CR_OK) return st;
    CR_REQUIRE(n_train <= CR_STATIC_MAX_TRAIN, CR_ERR_CAPACITY,
               "n_train = %lld exceeds what the library's fixed scratch array holds (%d training nodes); use cr_build_batches with a workspace",
               (long long)n_train, CR_STATIC_MAX_TRAIN);
    CR_REQUIRE(n_comm <= CR_STATIC_MAX_COMM, CR_ERR_CAPACITY,
               "n_comm = %d exceeds what the library's fixed scratch array holds (%d communities); use cr_build_batches with a workspace",
               n_comm, CR_STATIC_MAX_COMM);
    BatchPlan p;
    plan_batches(n_train, n_comm, nullptr, p);
    CR_REQUIRE(p.bytes <= STATIC_SCRATCH_BYTES, CR_ERR_CAPACITY, "scratch of %zu bytes, %zu needed", STATIC_SCRATCH_BYTES, p.bytes);
    if (dry_run()) {
        if (out_n_batches) *out_n_batches = ceil_div(n_train, cfg->batch_size);
        return CR_OK;
    }
    int dev = 0;
    CR_HIP_CHECK(hipGetDevice(&dev));
    CR_REQUIRE(dev >= 0 && dev < MAX_DEVICES, CR_ERR_UNSUPPORTED, "device index %d outside 0..%d", dev, MAX_DEVICES - 1);
    void *ws = nullptr;
    {
        std::lock_guard<std::mutex> lock(scratch_mutex);
        if (!scratch_ptr[dev]) {
            void *ptr = nullptr;
            CR_HIP_CHECK(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
            CR_REQUIRE(ptr != nullptr, CR_ERR_HIP, "the scratch array has no device address");
            scratch_ptr[dev] = ptr;
        }
        ws = scratch_ptr[dev];
    }
    return build_batches_impl(cfg, train_ids, n_train, comm, n_comm, ws, STATIC_SCRATCH_BYTES, out_perm, out_n_batches, stream);
}
