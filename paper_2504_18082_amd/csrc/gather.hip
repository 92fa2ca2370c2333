// Feature-row gather with GraphSAGE-mean aggregation (forward) and its atomic-free backward over
// the transposed block.  HBM-bound: every lane moves 16 bytes per load, a sub-wave group of LPR
// lanes owns one output row and keeps several independent row loads in flight.
#include <type_traits>

#include "cr_common.h"
#include "linear_bwd.h"

namespace cr {

// load_raw / unpack split a row-chunk load from its conversion: inside the edge loops the loads sit under a
// condition, and a conversion in the same branch would make every load wait for its data before the next is issued.
template <typename T> struct Vec16;
template <> struct Vec16<float> {
    static constexpr int N = 4;
    using Raw = float4;
    __device__ static __forceinline__ Raw load_raw(const float *p) { return *reinterpret_cast<const float4 *>(p); }
    __device__ static __forceinline__ void unpack(const Raw &x, float (&v)[4]) { v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w; }
    __device__ static __forceinline__ void load(const float *p, float (&v)[4])
    {
        const float4 x = *reinterpret_cast<const float4 *>(p);
        v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w;
    }
};
template <> struct Vec16<uint16_t> {
    static constexpr int N = 8;
    using Raw = uint4;
    __device__ static __forceinline__ Raw load_raw(const uint16_t *p) { return *reinterpret_cast<const uint4 *>(p); }
    __device__ static __forceinline__ void unpack(const Raw &x, float (&v)[8])
    {
        v[0] = __uint_as_float(x.x << 16); v[1] = __uint_as_float(x.x & 0xFFFF0000u);
        v[2] = __uint_as_float(x.y << 16); v[3] = __uint_as_float(x.y & 0xFFFF0000u);
        v[4] = __uint_as_float(x.z << 16); v[5] = __uint_as_float(x.z & 0xFFFF0000u);
        v[6] = __uint_as_float(x.w << 16); v[7] = __uint_as_float(x.w & 0xFFFF0000u);
    }
    __device__ static __forceinline__ void load(const uint16_t *p, float (&v)[8])
    {
        const uint4 x = *reinterpret_cast<const uint4 *>(p);
        v[0] = __uint_as_float(x.x << 16); v[1] = __uint_as_float(x.x & 0xFFFF0000u);
        v[2] = __uint_as_float(x.y << 16); v[3] = __uint_as_float(x.y & 0xFFFF0000u);
        v[4] = __uint_as_float(x.z << 16); v[5] = __uint_as_float(x.z & 0xFFFF0000u);
        v[6] = __uint_as_float(x.w << 16); v[7] = __uint_as_float(x.w & 0xFFFF0000u);
    }
};

template <int N>
__device__ __forceinline__ void store_bf16_row(uint16_t *dst, const float (&v)[N], int col, int F)
{
    // dst points at column `col` of a zero-padded bf16 row; columns >= F are written as zero
    uint32_t packed[N / 2];
#pragma unroll
    for (int i = 0; i < N; i += 2) {
        const uint32_t both = pack_bf16x2(v[i], v[i + 1]);
        packed[i / 2] = (col + i + 1 < F) ? both : ((col + i < F) ? (both & 0xFFFFu) : 0u);
    }
    if constexpr (N == 4) {
        *reinterpret_cast<uint2 *>(dst) = make_uint2(packed[0], packed[1]);
    } else {
        *reinterpret_cast<uint4 *>(dst) = make_uint4(packed[0], packed[1], packed[2], packed[3]);
    }
}

// ------------------------------------------------------------------------------------------------
// forward
//   ids[e]      : per-edge source row (through edge_map when it is given)
//   self_map[v] : table row of destination v (identity when NULL)
// A workgroup owns a contiguous range of destination rows (XCD-aware), its sub-wave groups walk the
// range interleaved.  The walk is software pipelined: while the feature rows of the current
// destination are in flight, the neighbour ids of the next destination and the row pointers of the
// one after are already being fetched, so a destination costs one memory round trip instead of a
// chain of four.  Look-ahead loads are unconditional (clamped to valid addresses).
// ------------------------------------------------------------------------------------------------
// GCN == true turns the mean into the GCN propagation of a sampled block: every gathered row is weighted by
// 1/sqrt(d~_u) (gcn.edge_w: by local source position, or gcn.node_norm[2u] by global id), the sum is scaled by the
// destination's (deg_v / |N_s(v)|) / sqrt(d~_v) (gcn.dst_scale) and the destination's own row enters with 1/d~_v
// (gcn.dst_self); d~ = degree in the full graph + 1.
struct GcnFwd {
    const float *edge_w;      // [n_src] or NULL
    const float *node_norm;   // [2 * n_nodes] (1/sqrt(d~), degree) or NULL
    const float *dst_scale;   // [n_dst]
    const float *dst_self;    // [n_dst]
};

// GROUPED == true walks the rows of a whole group of batches in one launch: `order` then holds entries
// batch * cap_dst + row followed (at index n_batches * cap_dst) by their number, the per-batch arrays are the group's
// (batch g's slice at g times its capacity) and batch g's outputs start at row g * out_stride.
struct GroupInfo {
    int32_t n_batches, cap_dst, cap_src, cap_nnz;
    int64_t out_stride;       // output rows per batch
    int32_t out_cols;         // bf16 output columns this launch writes (payload + zero padding); 0 = the whole row stride
};

template <typename T, int LPR, int NCHUNK, bool GCN = false, bool GROUPED = false>
__global__ __launch_bounds__(256) void gather_mean_fwd_kernel(
    const int32_t *__restrict__ hdr, const int32_t *__restrict__ indptr,
    const int32_t *__restrict__ ids, const int32_t *__restrict__ edge_map,
    const int32_t *__restrict__ self_map, const T *__restrict__ table, int64_t ld, int F,
    float *__restrict__ agg, uint16_t *__restrict__ agg_bf16, uint16_t *__restrict__ self_bf16, int64_t ld_bf16,
    GcnFwd gcn = GcnFwd{nullptr, nullptr, nullptr, nullptr}, const int32_t *__restrict__ order = nullptr,
    GroupInfo grp = GroupInfo{0, 0, 0, 0, 0, 0})
{
    constexpr int VEC = Vec16<T>::N;
    constexpr int U = NCHUNK == 1 ? 8 : (NCHUNK <= 3 ? 4 : 2);   // independent row loads in flight per lane
    constexpr int GPB = 256 / LPR;                                // groups (rows in progress) per workgroup
    const int n_dst = GROUPED ? min(order[(int64_t)grp.n_batches * grp.cap_dst], grp.n_batches * grp.cap_dst) : hdr[CR_HDR_N_DST];
    const int n_src = GROUPED ? grp.cap_src : hdr[CR_HDR_N_SRC];
    if (n_dst <= 0) return;
    // Each XCD (the workgroups with the same blockIdx.x mod 8; the grid is a multiple of 8) owns one contiguous eighth
    // of the rows and its workgroups sweep it together: workgroup j of the XCD takes rows j*GPB.., then steps by the
    // XCD's whole front.  The rows in flight on an XCD at any time are then neighbours, which is what makes a
    // processing order by community pay: their sources meet in that XCD's L2.
    const int per_xcd = (int)(gridDim.x / 8);
    const int xcd_rows = ((n_dst + 7) / 8 + GPB - 1) / GPB * GPB;
    const int block_first = (int)(blockIdx.x % 8) * xcd_rows + (int)(blockIdx.x / 8) * GPB;
    const int block_end = min(n_dst, (int)(blockIdx.x % 8 + 1) * xcd_rows);
    const int STEP = per_xcd * GPB;
    const int gl = (int)(threadIdx.x % LPR);
    int row = block_first + (int)(threadIdx.x / LPR);
    if (row >= block_end) return;

    // `order` (optional) is a permutation of the destination rows: position i of the walk handles row order[i].  It only
    // changes which workgroup computes a row and when (rows that share sources next to each other hit in L1/L2); the
    // row ids are fetched one more stage ahead of the pointers.
    auto load_row = [&](int r) -> int {
        const int rc = min(r, n_dst - 1);
        return order ? order[rc] : rc;
    };
    float sc0 = 0.f, sf0 = 0.f, sc1 = 0.f, sf1 = 0.f, sc2 = 0.f, sf2 = 0.f;     // GCN: destination scale / self weight
    auto load_ptrs = [&](int r, int &rc, int &s, int &e, int &self_row, float &sc, float &sf) {
        if constexpr (GROUPED) {
            // rc comes in as batch * cap_dst + row and goes out as the output row
            const int g = min(max(rc, 0) / grp.cap_dst, grp.n_batches - 1), rr = max(rc, 0) - g * grp.cap_dst;
            const int32_t *ip = indptr + (int64_t)g * (grp.cap_dst + 1);
            const int a = ip[rr] + g * grp.cap_nnz, b = ip[rr + 1] + g * grp.cap_nnz;
            self_row = self_map[(int64_t)g * grp.cap_src + rr];
            if constexpr (GCN) {
                // the destination's scale and self weight, as cr_gcn_block_norm computes them, from the per-node
                // normalisation of the graph (self_row is the destination's node id here)
                const float isd = gcn.node_norm[2 * (int64_t)self_row], dg = gcn.node_norm[2 * (int64_t)self_row + 1];
                const int n_s = b - a;
                sc = n_s > 0 ? dg / (float)n_s * isd : 0.0f;
                sf = 1.0f / (dg + 1.0f);
            }
            rc = (int)(g * grp.out_stride + rr);
            s = r < block_end ? a : 0;
            e = r < block_end ? b : 0;
        } else {
            const int a = indptr[rc], b = indptr[rc + 1];
            const int sr = self_map ? self_map[rc] : rc;
            if constexpr (GCN) { sc = gcn.dst_scale[rc]; sf = gcn.dst_self[rc]; }
            s = r < block_end ? a : 0;
            e = r < block_end ? b : 0;
            self_row = sr;
        }
    };
    auto load_ids = [&](int first, int e, float &w) -> int {
        const int idx = max(min(first + gl, e - 1), 0);
        int x = ids[idx];
        if constexpr (GCN) {
            // ids are local source positions (weights by position) or, through gather_ids, global ids (weights by node)
            w = gcn.edge_w ? gcn.edge_w[min(max(x, 0), max(n_src, 1) - 1)] : gcn.node_norm[2 * (int64_t)max(x, 0)];
        }
        if (edge_map) x = edge_map[min(max(x, 0), n_src - 1)];   // (a lane past the row's end may have read a stale entry)
        return x;
    };

    int s0, e0, self0, s1, e1, self1;
    float w0 = 1.f, w1 = 1.f;
    int out0 = load_row(row), out1 = load_row(row + STEP), out2 = load_row(row + 2 * STEP);   // rows handled now, next, after next
    load_ptrs(row, out0, s0, e0, self0, sc0, sf0);
    int rid0 = load_ids(s0, e0, w0);
    load_ptrs(row + STEP, out1, s1, e1, self1, sc1, sf1);

    for (; row < block_end; row += STEP) {
        // look ahead: ids of the next destination, pointers of the one after
        const int rid1 = load_ids(s1, e1, w1);
        int s2, e2, self2;
        load_ptrs(row + 2 * STEP, out2, s2, e2, self2, sc2, sf2);
        const int out3 = load_row(row + 3 * STEP);

        float acc[NCHUNK][VEC];
#pragma unroll
        for (int c = 0; c < NCHUNK; ++c)
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[c][i] = 0.f;

        int rid = rid0;
        float wgt = w0;
        for (int base = s0; base < e0; base += LPR) {
            if (base > s0) rid = load_ids(base, e0, wgt);       // rows longer than the group width
            const int cnt = min(LPR, e0 - base);
            for (int t = 0; t < cnt; t += U) {
                typename Vec16<T>::Raw v[U][NCHUNK];
                float wu[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int r = __shfl(rid, t + u, LPR);
                    if constexpr (GCN) wu[u] = __shfl(wgt, t + u, LPR);
                    const T *p = table + (int64_t)r * ld;
#pragma unroll
                    for (int c = 0; c < NCHUNK; ++c) {
                        const int col = (c * LPR + gl) * VEC;
                        if (col < F && t + u < cnt) v[u][c] = Vec16<T>::load_raw(p + col);
                    }
                }
#pragma unroll
                for (int u = 0; u < U; ++u)
#pragma unroll
                    for (int c = 0; c < NCHUNK; ++c) {
                        const int col = (c * LPR + gl) * VEC;
                        if (col < F && t + u < cnt) {
                            float f[VEC];
                            Vec16<T>::unpack(v[u][c], f);
#pragma unroll
                            for (int i = 0; i < VEC; ++i) {
                                if constexpr (GCN) acc[c][i] = __builtin_fmaf(wu[u], f[i], acc[c][i]);
                                else acc[c][i] += f[i];
                            }
                        }
                    }
            }
        }

        const int deg = e0 - s0;
        const float fdeg = (float)(deg > 0 ? deg : 1);
        const int64_t wcols = (GROUPED && grp.out_cols) ? (int64_t)grp.out_cols : ld_bf16;     // a column panel writes its own columns only
#pragma unroll
        for (int c = 0; c < NCHUNK; ++c) {
            const int col = (c * LPR + gl) * VEC;
            if constexpr (GCN) {
                float sv[VEC];
#pragma unroll
                for (int i = 0; i < VEC; ++i) sv[i] = 0.f;
                if (col < F) Vec16<T>::load(table + (int64_t)self0 * ld + col, sv);
#pragma unroll
                for (int i = 0; i < VEC; ++i) {
                    // (spelled out so that every instantiation rounds the same way: the self term first, then one fused step)
                    const float self_term = sv[i] * sf0;
                    acc[c][i] = __builtin_fmaf(acc[c][i], sc0, self_term);
                }
            } else {
#pragma unroll
                for (int i = 0; i < VEC; ++i) acc[c][i] = acc[c][i] / fdeg;
            }
            if (agg && col < F) {
                float *o = agg + (int64_t)out0 * F + col;
                if ((F & 3) == 0) {
#pragma unroll
                    for (int i = 0; i < VEC; i += 4)
                        *reinterpret_cast<float4 *>(o + i) = make_float4(acc[c][i], acc[c][i + 1], acc[c][i + 2], acc[c][i + 3]);
                } else {
#pragma unroll
                    for (int i = 0; i < VEC; ++i)
                        if (col + i < F) o[i] = acc[c][i];
                }
            }
            if (agg_bf16 && col < wcols) store_bf16_row<VEC>(agg_bf16 + (int64_t)out0 * ld_bf16 + col, acc[c], col, F);
        }

        if (self_bf16) {
            const T *p = table + (int64_t)self0 * ld;
#pragma unroll
            for (int c = 0; c < NCHUNK; ++c) {
                const int col = (c * LPR + gl) * VEC;
                if (col < wcols) {
                    float v[VEC];
#pragma unroll
                    for (int i = 0; i < VEC; ++i) v[i] = 0.f;
                    if (col < F) Vec16<T>::load(p + col, v);
                    store_bf16_row<VEC>(self_bf16 + (int64_t)out0 * ld_bf16 + col, v, col, F);
                }
            }
        }

        s0 = s1; e0 = e1; self0 = self1; rid0 = rid1; w0 = w1; sc0 = sc1; sf0 = sf1; out0 = out1;
        s1 = s2; e1 = e2; self1 = self2; sc1 = sc2; sf1 = sf2; out1 = out2; out2 = out3;
    }
}

template <typename T, int LPR, int NCHUNK>
static void launch_fwd(int cap_dst, const int32_t *hdr, const int32_t *indptr, const int32_t *ids,
                       const int32_t *edge_map, const int32_t *self_map, const void *table, int64_t ld, int F,
                       float *agg, uint16_t *agg_bf16, uint16_t *self_bf16, int64_t ld_bf16, hipStream_t st,
                       const GcnFwd *gcn = nullptr, const int32_t *order = nullptr)
{
    constexpr int GPB = 256 / LPR;
    int64_t grid = round_up(ceil_div(cap_dst, GPB), 8);
    if (grid > 1024) grid = 1024;          // 4 workgroups per CU; each group then walks several rows
    if (gcn)
        hipLaunchKernelGGL((gather_mean_fwd_kernel<T, LPR, NCHUNK, true>), dim3((unsigned)grid), dim3(256), 0, st, hdr, indptr,
                           ids, edge_map, self_map, static_cast<const T *>(table), ld, F, agg, agg_bf16, self_bf16, ld_bf16, *gcn, order);
    else
        hipLaunchKernelGGL((gather_mean_fwd_kernel<T, LPR, NCHUNK, false>), dim3((unsigned)grid), dim3(256), 0, st, hdr, indptr,
                           ids, edge_map, self_map, static_cast<const T *>(table), ld, F, agg, agg_bf16, self_bf16, ld_bf16,
                           GcnFwd{nullptr, nullptr, nullptr, nullptr}, order);
}

constexpr int GROUP_PANEL_BYTES = 512;             // column panel of the grouped gather
constexpr int GROUP_PANEL_MIN_ROW_BYTES = 1024;    // rows wider than this are gathered in panels

template <typename T, int LPR, int NCHUNK, bool GCN = false>
static void launch_fwd_group(const cr_block_set *b, const void *table, int64_t ld, int F, uint16_t *agg_bf16, uint16_t *self_bf16,
                             int64_t out_stride, int64_t ld_bf16, hipStream_t st, int out_cols = 0, const float *node_norm = nullptr)
{
    constexpr int GPB = 256 / LPR;
    int64_t grid = round_up(ceil_div((int64_t)b->n_batches * b->cap_dst, GPB), 8);
    if (grid > 1024) grid = 1024;
    const GroupInfo gi{b->n_batches, b->cap_dst, b->cap_src, b->cap_nnz, out_stride, out_cols};
    hipLaunchKernelGGL((gather_mean_fwd_kernel<T, LPR, NCHUNK, GCN, true>), dim3((unsigned)grid), dim3(256), 0, st, b->hdr, b->indptr,
                       b->gather_ids, (const int32_t *)nullptr, b->src_ids, static_cast<const T *>(table), ld, F, (float *)nullptr, agg_bf16,
                       self_bf16, ld_bf16, GcnFwd{nullptr, node_norm, nullptr, nullptr}, b->group_order, gi);
}

// ------------------------------------------------------------------------------------------------
// backward: one sub-wave group per source row pulls from the destination rows that used it
// ------------------------------------------------------------------------------------------------
// GCN == true is the transpose of the GCN forward: destination v contributes with gcn.dst_scale[v], the sum is
// scaled by the source's 1/sqrt(d~) (gcn.edge_w), and a source that is also a destination adds gcn.dst_self * its own
// gradient row (d_self is then the same array as d_agg).
// `bid` of `nblk` workgroups (a multiple of eight) share the rows.
template <typename T, int LPR, int NCHUNK, bool GCN>
__device__ __forceinline__ void gather_mean_bwd_body(
    uint32_t bid, uint32_t nblk, const int32_t *__restrict__ hdr, const int32_t *__restrict__ indptr,
    const int32_t *__restrict__ t_indptr, const int32_t *__restrict__ t_indices,
    const T *__restrict__ d_agg, const T *__restrict__ d_self, int64_t ld_in, int F,
    const void *__restrict__ relu_out, int relu_is_bf16, int64_t ld_relu, float *__restrict__ d_src,
    uint16_t *__restrict__ d_src_bf16, int64_t ld_bf16, const GcnFwd &gcn)
{
    constexpr int VEC = Vec16<T>::N;
    constexpr int U = NCHUNK == 1 ? 4 : 2;       // slots per pass after the first (few rows get that far)
    constexpr int GPB = 256 / LPR;
    const int n_dst = hdr[CR_HDR_N_DST], n_src = hdr[CR_HDR_N_SRC];
    if (n_src <= 0) return;
    // the same walk as in the forward kernel: an eighth of the rows per XCD, swept by its workgroups together
    const int per_xcd = (int)(nblk / 8);
    const int xcd_rows = ((n_src + 7) / 8 + GPB - 1) / GPB * GPB;
    const int block_first = (int)(bid % 8) * xcd_rows + (int)(bid / 8) * GPB;
    const int block_end = min(n_src, (int)(bid % 8 + 1) * xcd_rows);
    const int STEP = per_xcd * GPB;
    const int gl = (int)(threadIdx.x % LPR);
    int s = block_first + (int)(threadIdx.x / LPR);
    if (s >= block_end) return;

    // same pipelining as the forward kernel: destination ids and their 1/degree weights of the next
    // source row, and the segment pointers of the one after, are fetched while the current rows stream in
    auto load_ptrs = [&](int r, int &b, int &e) {
        const int rc = min(r, n_src - 1);
        const int x = t_indptr[rc], y = t_indptr[rc + 1];
        b = r < block_end ? x : 0;
        e = r < block_end ? y : 0;
    };
    auto load_ids = [&](int first, int e, int &v, float &w) {
        const int idx = max(min(first + gl, e - 1), 0);
        v = min(max(t_indices[idx], 0), n_dst - 1);               // (a lane past the segment's end may have read a stale entry)
        if constexpr (GCN) {
            w = gcn.dst_scale[v];
        } else {
            const int deg = indptr[v + 1] - indptr[v];
            w = 1.0f / (float)(deg > 0 ? deg : 1);
        }
    };

    int b0, e0, b1, e1, v0, v1;
    float w0, w1;
    load_ptrs(s, b0, e0);
    load_ids(b0, e0, v0, w0);
    load_ptrs(s + STEP, b1, e1);

    for (; s < block_end; s += STEP) {
        load_ids(b1, e1, v1, w1);
        int b2, e2;
        load_ptrs(s + 2 * STEP, b2, e2);

        float acc[NCHUNK][VEC];
#pragma unroll
        for (int c = 0; c < NCHUNK; ++c)
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[c][i] = 0.f;

        // bf16 gradients: the row's own d_self chunk and its ReLU mask are requested here, branch-free (a stand-in
        // address when there is none, applied with weight 0 / ignored), so that they travel while the edge loop runs
        // instead of costing two more round trips after it
        constexpr bool PRE = VEC == 8;
        const bool mask_bf16 = relu_out != nullptr && relu_is_bf16 != 0;
        uint4 self_raw[NCHUNK], mask_raw[NCHUNK];
        if constexpr (PRE) {
            const int sd = max(min(s, n_dst - 1), 0);
            const uint16_t *sp = reinterpret_cast<const uint16_t *>(d_self ? d_self : d_agg) + (int64_t)sd * ld_in;
            const uint16_t *mp = mask_bf16 ? static_cast<const uint16_t *>(relu_out) + (int64_t)s * ld_relu
                                           : reinterpret_cast<const uint16_t *>(d_agg) + (int64_t)sd * ld_in;
#pragma unroll
            for (int c = 0; c < NCHUNK; ++c) {
                const int col = (c * LPR + gl) * VEC;
                const int colc = col < F ? col : 0;
                self_raw[c] = *reinterpret_cast<const uint4 *>(sp + colc);
                mask_raw[c] = *reinterpret_cast<const uint4 *>(mp + colc);
            }
        }

        int v = v0;
        float w = w0;
        for (int base = b0; base < e0; base += LPR) {
            if (base > b0) load_ids(base, e0, v, w);
            const int cnt = min(LPR, e0 - base);
            // branch-free: a slot past the segment's end re-reads the segment's last row with weight 0, a lane past
            // the row's end reads column 0; so the loads of one pass are issued back to back.  Most source rows of a
            // sampled block are used by one or two destinations, so the first pass takes two slots and only longer
            // segments go on in passes of U (a pass costs its loads whether the slots exist or not).
            auto pass = [&](auto width, int t) {
                constexpr int UU = decltype(width)::value;
                typename Vec16<T>::Raw x[UU][NCHUNK];
                float ww[UU];
#pragma unroll
                for (int u = 0; u < UU; ++u) {
                    const int src = min(t + u, cnt - 1);
                    const int vv = __shfl(v, src, LPR);
                    const float wv = __shfl(w, src, LPR);
                    ww[u] = t + u < cnt ? wv : 0.f;
                    const T *p = d_agg + (int64_t)vv * ld_in;
#pragma unroll
                    for (int c = 0; c < NCHUNK; ++c) {
                        const int col = (c * LPR + gl) * VEC;
                        x[u][c] = Vec16<T>::load_raw(p + (col < F ? col : 0));
                    }
                }
#pragma unroll
                for (int u = 0; u < UU; ++u)
#pragma unroll
                    for (int c = 0; c < NCHUNK; ++c) {
                        float f[VEC];
                        Vec16<T>::unpack(x[u][c], f);
#pragma unroll
                        for (int i = 0; i < VEC; ++i) acc[c][i] += f[i] * ww[u];
                    }
            };
            pass(std::integral_constant<int, 2>{}, 0);
            for (int t = 2; t < cnt; t += U) pass(std::integral_constant<int, U>{}, t);
        }
#pragma unroll
        for (int c = 0; c < NCHUNK; ++c) {
            const int col = (c * LPR + gl) * VEC;
            if (col < F) {
                if constexpr (GCN) {
                    const float ws = gcn.edge_w[s];
#pragma unroll
                    for (int i = 0; i < VEC; ++i) acc[c][i] *= ws;
                }
                if constexpr (PRE) {
                    if (d_self && s < n_dst) {
                        float x[8];
                        Vec16<uint16_t>::unpack(self_raw[c], x);
                        const float wself = GCN ? gcn.dst_self[s] : 1.0f;
#pragma unroll
                        for (int i = 0; i < VEC; ++i) acc[c][i] += wself * x[i];
                    }
                } else if (d_self && s < n_dst) {
                    float x[VEC];
                    Vec16<T>::load(d_self + (int64_t)s * ld_in + col, x);
                    const float wself = GCN ? gcn.dst_self[s] : 1.0f;
#pragma unroll
                    for (int i = 0; i < VEC; ++i) acc[c][i] += wself * x[i];
                }
                if (PRE && mask_bf16) {
                    float y[8];
                    Vec16<uint16_t>::unpack(mask_raw[c], y);
#pragma unroll
                    for (int i = 0; i < VEC; ++i)
                        if (!(y[i] > 0.f)) acc[c][i] = 0.f;
                } else if (relu_out) {
                    float y[VEC];
                    if (relu_is_bf16) {
                        const uint16_t *r = static_cast<const uint16_t *>(relu_out) + (int64_t)s * ld_relu + col;
                        if constexpr (VEC == 8) {
                            Vec16<uint16_t>::load(r, y);
                        } else {
                            const uint2 h = *reinterpret_cast<const uint2 *>(r);
                            y[0] = __uint_as_float(h.x << 16); y[1] = __uint_as_float(h.x & 0xFFFF0000u);
                            y[2] = __uint_as_float(h.y << 16); y[3] = __uint_as_float(h.y & 0xFFFF0000u);
                        }
                    } else {
                        const float *r = static_cast<const float *>(relu_out) + (int64_t)s * ld_relu + col;
#pragma unroll
                        for (int i = 0; i < VEC; i += 4) {
                            float4 q = make_float4(1.f, 1.f, 1.f, 1.f);
                            if (col + i < F) q = *reinterpret_cast<const float4 *>(r + i);     // stays inside the row's stride
                            y[i] = q.x; y[i + 1] = q.y; y[i + 2] = q.z; y[i + 3] = q.w;
                        }
                    }
#pragma unroll
                    for (int i = 0; i < VEC; ++i)
                        if (!(y[i] > 0.f)) acc[c][i] = 0.f;
                }
                if (d_src) {
                    float *o = d_src + (int64_t)s * F + col;
                    if ((F & 3) == 0) {
#pragma unroll
                        for (int i = 0; i < VEC; i += 4)
                            if (col + i < F) *reinterpret_cast<float4 *>(o + i) = make_float4(acc[c][i], acc[c][i + 1], acc[c][i + 2], acc[c][i + 3]);
                    } else {
#pragma unroll
                        for (int i = 0; i < VEC; ++i)
                            if (col + i < F) o[i] = acc[c][i];
                    }
                }
            }
            if (d_src_bf16 && col < ld_bf16) store_bf16_row<VEC>(d_src_bf16 + (int64_t)s * ld_bf16 + col, acc[c], col, F);
        }

        b0 = b1; e0 = e1; v0 = v1; w0 = w1;
        b1 = b2; e1 = e2;
    }
}

template <typename T, int LPR, int NCHUNK, bool GCN = false>
__global__ __launch_bounds__(256) void gather_mean_bwd_kernel(
    const int32_t *__restrict__ hdr, const int32_t *__restrict__ indptr,
    const int32_t *__restrict__ t_indptr, const int32_t *__restrict__ t_indices,
    const T *__restrict__ d_agg, const T *__restrict__ d_self, int64_t ld_in, int F,
    const void *__restrict__ relu_out, int relu_is_bf16, int64_t ld_relu, float *__restrict__ d_src,
    uint16_t *__restrict__ d_src_bf16, int64_t ld_bf16, GcnFwd gcn = GcnFwd{nullptr, nullptr, nullptr, nullptr})
{
    gather_mean_bwd_body<T, LPR, NCHUNK, GCN>(blockIdx.x, gridDim.x, hdr, indptr, t_indptr, t_indices, d_agg, d_self, ld_in, F, relu_out,
                                              relu_is_bf16, ld_relu, d_src, d_src_bf16, ld_bf16, gcn);
}

// The aggregation's backward pass and the weight update of the same layer in one launch: neither needs anything
// from the other (the update reads the weight-gradient partials, the aggregation the input gradients, both written
// by the launch before), and both are short and bound by memory round trips.  The first `agg_blocks` workgroups
// (a multiple of eight) walk the source rows, the rest reduce the partials and apply the SGD step.
template <int LPR, int NCHUNK>
__global__ __launch_bounds__(256) void gather_bwd_sgd_kernel(
    uint32_t agg_blocks, SgdArgs sgd, const int32_t *__restrict__ hdr, const int32_t *__restrict__ indptr,
    const int32_t *__restrict__ t_indptr, const int32_t *__restrict__ t_indices,
    const uint16_t *__restrict__ d_agg, const uint16_t *__restrict__ d_self, int64_t ld_in, int F,
    const void *__restrict__ relu_out, int relu_is_bf16, int64_t ld_relu, uint16_t *__restrict__ d_src_bf16, int64_t ld_bf16)
{
    __shared__ float4 red[4][64];
    if (blockIdx.x < agg_blocks) {
        gather_mean_bwd_body<uint16_t, LPR, NCHUNK, false>(blockIdx.x, agg_blocks, hdr, indptr, t_indptr, t_indices, d_agg, d_self, ld_in, F,
                                                           relu_out, relu_is_bf16, ld_relu, nullptr, d_src_bf16, ld_bf16,
                                                           GcnFwd{nullptr, nullptr, nullptr, nullptr});
    } else {
        sgd_reduce_body(sgd, blockIdx.x - agg_blocks, red);
    }
}

// six workgroups per compute unit: what the backward kernels' registers allow (the rows in flight are what hides
// the chain of dependent loads behind a source row)
constexpr int64_t BWD_MAX_BLOCKS = 1536;

template <int LPR, int NCHUNK>
static void launch_bwd_sgd(const SgdArgs &sgd, unsigned sgd_blocks, int cap_src, const int32_t *hdr, const int32_t *indptr,
                           const int32_t *t_indptr, const int32_t *t_indices, const uint16_t *d_agg, const uint16_t *d_self,
                           int64_t ld_in, int F, const void *relu_out, int relu_is_bf16, int64_t ld_relu, uint16_t *d_src_bf16,
                           int64_t ld_bf16, hipStream_t st)
{
    int64_t grid = round_up(ceil_div(cap_src, 256 / LPR), 8);
    if (grid > BWD_MAX_BLOCKS) grid = BWD_MAX_BLOCKS;
    hipLaunchKernelGGL((gather_bwd_sgd_kernel<LPR, NCHUNK>), dim3((unsigned)grid + sgd_blocks), dim3(256), 0, st, (uint32_t)grid, sgd, hdr,
                       indptr, t_indptr, t_indices, d_agg, d_self, ld_in, F, relu_out, relu_is_bf16, ld_relu, d_src_bf16, ld_bf16);
}

template <typename T, int LPR, int NCHUNK>
static void launch_bwd(int cap_src, const int32_t *hdr, const int32_t *indptr, const int32_t *t_indptr,
                       const int32_t *t_indices, const void *d_agg, const void *d_self, int64_t ld_in, int F,
                       const void *relu_out, int relu_is_bf16, int64_t ld_relu, float *d_src, uint16_t *d_src_bf16,
                       int64_t ld_bf16, hipStream_t st, const GcnFwd *gcn = nullptr)
{
    int64_t grid = round_up(ceil_div(cap_src, 256 / LPR), 8);
    if (grid > BWD_MAX_BLOCKS) grid = BWD_MAX_BLOCKS;
    if (gcn)
        hipLaunchKernelGGL((gather_mean_bwd_kernel<T, LPR, NCHUNK, true>), dim3((unsigned)grid), dim3(256), 0, st, hdr, indptr, t_indptr,
                           t_indices, static_cast<const T *>(d_agg), static_cast<const T *>(d_self), ld_in, F, relu_out, relu_is_bf16,
                           ld_relu, d_src, d_src_bf16, ld_bf16, *gcn);
    else
        hipLaunchKernelGGL((gather_mean_bwd_kernel<T, LPR, NCHUNK, false>), dim3((unsigned)grid), dim3(256), 0, st, hdr, indptr, t_indptr,
                           t_indices, static_cast<const T *>(d_agg), static_cast<const T *>(d_self), ld_in, F, relu_out, relu_is_bf16,
                           ld_relu, d_src, d_src_bf16, ld_bf16, GcnFwd{nullptr, nullptr, nullptr, nullptr});
}

// per-node normalisation of the full graph: norm[2v] = 1/sqrt(deg_v + 1), norm[2v + 1] = deg_v
__global__ __launch_bounds__(256) void gcn_node_norm_kernel(const int64_t *__restrict__ indptr, int64_t n_nodes, float *__restrict__ norm)
{
    const int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (v >= n_nodes) return;
    const float deg = (float)(indptr[v + 1] - indptr[v]);
    norm[2 * v] = 1.0f / sqrtf(deg + 1.0f);
    norm[2 * v + 1] = deg;
}

// per-block normalisation of one batch: source weights, destination scales and self weights (see GcnFwd)
__global__ __launch_bounds__(256) void gcn_block_norm_kernel(const int32_t *__restrict__ hdr, const int32_t *__restrict__ indptr,
                                                             const int32_t *__restrict__ node_ids, const float *__restrict__ norm,
                                                             float *__restrict__ edge_w, float *__restrict__ dst_scale,
                                                             float *__restrict__ dst_self)
{
    const int n_dst = hdr[CR_HDR_N_DST], n_src = hdr[CR_HDR_N_SRC];
    const int i = (int)(blockIdx.x * 256 + threadIdx.x);
    if (i < n_src) edge_w[i] = norm[2 * (int64_t)node_ids[i]];
    if (i < n_dst) {
        const int64_t v = node_ids[i];
        const float isd = norm[2 * v], deg = norm[2 * v + 1];
        const int n_s = indptr[i + 1] - indptr[i];
        dst_scale[i] = n_s > 0 ? deg / (float)n_s * isd : 0.0f;
        dst_self[i] = 1.0f / (deg + 1.0f);
    }
}

}  // namespace cr

using namespace cr;

static cr_status check_block_set(const cr_block_set *b, int32_t g, bool need_t)
{
    CR_REQUIRE(b != nullptr, CR_ERR_INVALID_ARG, "blocks is NULL");
    CR_REQUIRE(b->n_batches > 0 && g >= 0 && g < b->n_batches, CR_ERR_INVALID_ARG,
               "batch index %d outside the block set's %d batches", g, b->n_batches);
    CR_REQUIRE(b->cap_dst > 0 && b->cap_src >= b->cap_dst && b->cap_nnz > 0, CR_ERR_INVALID_ARG,
               "block set capacities must be positive with cap_src >= cap_dst");
    CR_REQUIRE(b->hdr && b->src_ids && b->indptr && b->indices, CR_ERR_INVALID_ARG, "block set has a NULL array");
    if (need_t) CR_REQUIRE(b->t_indptr && b->t_indices, CR_ERR_INVALID_ARG, "block set carries no transposed block");
    return CR_OK;
}

static void run_fwd(const cr_block_set *blocks, int32_t g, const void *H_src, int32_t dtype, int64_t ld_src, int32_t F,
                    int32_t indirect, float *agg, uint16_t *agg_bf16, uint16_t *self_bf16, int64_t ld_bf16, hipStream_t s,
                    const GcnFwd *gcn)
{
    const int32_t *hdr = blocks->hdr + (int64_t)g * CR_HDR_WORDS;
    const int32_t *indptr = blocks->indptr + (int64_t)g * (blocks->cap_dst + 1);
    const int32_t *src_ids = blocks->src_ids + (int64_t)g * blocks->cap_src;
    const int32_t *ids = blocks->indices + (int64_t)g * blocks->cap_nnz;
    const int32_t *edge_map = nullptr, *self_map = nullptr;
    if (indirect) {
        self_map = src_ids;
        if (blocks->gather_ids) ids = blocks->gather_ids + (int64_t)g * blocks->cap_nnz;   // per-edge table rows, one level less
        else edge_map = src_ids;
    }
    const int cap = blocks->cap_dst;
    const int32_t *order = blocks->row_order ? blocks->row_order + (int64_t)g * blocks->cap_dst : nullptr;
#define CR_FWD(T, LPR, NC) launch_fwd<T, LPR, NC>(cap, hdr, indptr, ids, edge_map, self_map, H_src, ld_src, F, agg, agg_bf16, self_bf16, ld_bf16, s, gcn, order)
    if (dtype == CR_F32) {
        if (F <= 64) CR_FWD(float, 16, 1);
        else if (F <= 128) CR_FWD(float, 32, 1);
        else if (F <= 256) CR_FWD(float, 64, 1);
        else if (F <= 512) CR_FWD(float, 64, 2);
        else if (F <= 768) CR_FWD(float, 64, 3);
        else CR_FWD(float, 64, 4);
    } else {
        if (F <= 128) CR_FWD(uint16_t, 16, 1);
        else if (F <= 256) CR_FWD(uint16_t, 32, 1);
        else if (F <= 512) CR_FWD(uint16_t, 64, 1);
        else CR_FWD(uint16_t, 64, 2);
    }
#undef CR_FWD
}

extern "C" cr_status cr_gather_aggregate_fwd(const cr_block_set *blocks, int32_t g, const void *H_src,
                                             int32_t dtype, int64_t ld_src, int32_t F, int32_t indirect,
                                             float *agg, uint16_t *agg_bf16, uint16_t *self_bf16,
                                             int64_t ld_bf16, void *stream)
{
    cr_status st = check_block_set(blocks, g, false);
    if (st != CR_OK) return st;
    CR_REQUIRE(H_src != nullptr && aligned16(H_src), CR_ERR_INVALID_ARG, "H_src must be a 16-byte aligned device pointer");
    CR_REQUIRE(dtype == CR_F32 || dtype == CR_BF16, CR_ERR_INVALID_ARG, "dtype must be CR_F32 or CR_BF16");
    const int vec = dtype == CR_F32 ? 4 : 8;
    CR_REQUIRE(F >= 1 && F <= 1024, CR_ERR_UNSUPPORTED, "F = %d outside 1..1024", F);
    CR_REQUIRE(ld_src >= round_up(F, vec) && ld_src % vec == 0, CR_ERR_INVALID_ARG,
               "ld_src = %lld must be a multiple of %d and cover F rounded up to it", (long long)ld_src, vec);
    CR_REQUIRE(agg || agg_bf16 || self_bf16, CR_ERR_INVALID_ARG, "no output requested");
    CR_REQUIRE(aligned16(agg) && aligned16(agg_bf16) && aligned16(self_bf16), CR_ERR_INVALID_ARG, "outputs must be 16-byte aligned");
    if (agg_bf16 || self_bf16)
        CR_REQUIRE(ld_bf16 % 32 == 0 && ld_bf16 >= F && ld_bf16 <= round_up(F, 64), CR_ERR_INVALID_ARG,
                   "ld_bf16 = %lld must be a multiple of 32 in [F, F rounded up to 64]", (long long)ld_bf16);
    if (dry_run()) return CR_OK;

    run_fwd(blocks, g, H_src, dtype, ld_src, F, indirect, agg, agg_bf16, self_bf16, ld_bf16, static_cast<hipStream_t>(stream), nullptr);
    CR_LAUNCH_CHECK();
    return CR_OK;
}

static void run_bwd(const cr_block_set *blocks, int32_t g, const void *d_agg, const void *d_self, int32_t in_dtype, int64_t ld_in,
                    int32_t F, const void *relu_out, int32_t relu_dtype, int64_t ld_relu, float *d_src, uint16_t *d_src_bf16,
                    int64_t ld_bf16, hipStream_t s, const GcnFwd *gcn)
{
    const int32_t *hdr = blocks->hdr + (int64_t)g * CR_HDR_WORDS;
    const int32_t *indptr = blocks->indptr + (int64_t)g * (blocks->cap_dst + 1);
    const int32_t *t_indptr = blocks->t_indptr + (int64_t)g * (blocks->cap_src + 1);
    const int32_t *t_indices = blocks->t_indices + (int64_t)g * blocks->cap_nnz;
    const int cap = blocks->cap_src;
#define CR_BWD(T, LPR, NC) launch_bwd<T, LPR, NC>(cap, hdr, indptr, t_indptr, t_indices, d_agg, d_self, ld_in, F, relu_out, relu_dtype == CR_BF16 ? 1 : 0, ld_relu, d_src, d_src_bf16, ld_bf16, s, gcn)
    if (in_dtype == CR_F32) {
        if (F <= 64) CR_BWD(float, 16, 1);
        else if (F <= 128) CR_BWD(float, 32, 1);
        else if (F <= 256) CR_BWD(float, 64, 1);
        else if (F <= 512) CR_BWD(float, 64, 2);
        else if (F <= 768) CR_BWD(float, 64, 3);
        else CR_BWD(float, 64, 4);
    } else {
        if (F <= 128) CR_BWD(uint16_t, 16, 1);
        else if (F <= 256) CR_BWD(uint16_t, 32, 1);
        else if (F <= 512) CR_BWD(uint16_t, 64, 1);
        else CR_BWD(uint16_t, 64, 2);
    }
#undef CR_BWD
}

// the grouped gather of GraphSAGE (GCN == false: aggregate and self rows) and of GCN (GCN == true: the normalised sum, node_norm given)
template <bool GCN>
static cr_status gather_group(const cr_block_set *blocks, const void *H_src, int32_t dtype, int64_t ld_src, int32_t F, uint16_t *agg_bf16,
                              uint16_t *self_bf16, int64_t batch_stride_rows, int64_t ld_bf16, void *stream, const float *node_norm)
{
    CR_REQUIRE(blocks != nullptr, CR_ERR_INVALID_ARG, "blocks is NULL");
    CR_REQUIRE(blocks->n_batches >= 1 && blocks->cap_dst >= 1 && blocks->cap_src >= blocks->cap_dst && blocks->cap_nnz >= 1,
               CR_ERR_INVALID_ARG, "blocks capacities are not positive");
    CR_REQUIRE(blocks->hdr && blocks->indptr && blocks->src_ids, CR_ERR_INVALID_ARG, "blocks has a NULL array");
    CR_REQUIRE(blocks->gather_ids && blocks->group_order, CR_ERR_INVALID_ARG, "the grouped gather needs blocks->gather_ids and blocks->group_order");
    CR_REQUIRE((int64_t)blocks->n_batches * blocks->cap_dst < 0x7FFFFFFF && (int64_t)blocks->n_batches * blocks->cap_nnz < 0x7FFFFFFF,
               CR_ERR_UNSUPPORTED, "the group's rows or edges do not fit 31 bits");
    CR_REQUIRE(H_src != nullptr && aligned16(H_src), CR_ERR_INVALID_ARG, "H_src must be a 16-byte aligned device pointer");
    CR_REQUIRE(dtype == CR_F32 || dtype == CR_BF16, CR_ERR_INVALID_ARG, "dtype must be CR_F32 or CR_BF16");
    const int vec = dtype == CR_F32 ? 4 : 8;
    CR_REQUIRE(F >= 1 && F <= 1024, CR_ERR_INVALID_ARG, "F = %d outside 1..1024", F);
    CR_REQUIRE(ld_src >= round_up(F, vec) && ld_src % vec == 0, CR_ERR_INVALID_ARG,
               "ld_src = %lld must be a multiple of %d and >= F rounded up to it", (long long)ld_src, vec);
    CR_REQUIRE(agg_bf16 && aligned16(agg_bf16) && aligned16(self_bf16) && (GCN || self_bf16), CR_ERR_INVALID_ARG,
               "agg_bf16 / self_bf16 must be 16-byte aligned device pointers");
    CR_REQUIRE(!GCN || node_norm, CR_ERR_INVALID_ARG, "norm must not be NULL");
    CR_REQUIRE(ld_bf16 % 32 == 0 && ld_bf16 >= F && ld_bf16 <= round_up(F, 64), CR_ERR_INVALID_ARG,
               "ld_bf16 = %lld must be a multiple of 32 in [F, F rounded up to 64]", (long long)ld_bf16);
    CR_REQUIRE(batch_stride_rows >= blocks->cap_dst, CR_ERR_INVALID_ARG, "batch_stride_rows = %lld below cap_dst = %d",
               (long long)batch_stride_rows, blocks->cap_dst);
    CR_REQUIRE(batch_stride_rows * blocks->n_batches < 0x7FFFFFFF, CR_ERR_UNSUPPORTED, "output rows do not fit 31 bits");
    if (dry_run()) return CR_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    // Rows wider than 1 KB go in column panels of 512 bytes, one sweep over the group's rows per panel: with the rows in
    // community order a sweep then keeps one community's panel (nodes x 512 B) in an XCD's L2 where whole rows of a
    // large community do not fit (233 K-node reddit-like graph: 4660 nodes x 2408 B = 11 MB per community, 2.4 MB per
    // panel).  The row pointers and ids are read once per panel, a small price beside the rows themselves.
    const int elem = dtype == CR_F32 ? 4 : 2;
    if ((int64_t)F * elem > GROUP_PANEL_MIN_ROW_BYTES) {
        const int pw = GROUP_PANEL_BYTES / elem;                  // panel width in elements
        for (int c0 = 0; c0 < F; c0 += pw) {
            const int Fk = F - c0 < pw ? F - c0 : pw;
            const bool last = c0 + pw >= F;
            const int out_cols = last ? (int)(ld_bf16 - c0) : pw;
            const void *tab = static_cast<const char *>(H_src) + (int64_t)c0 * elem;
            uint16_t *self_k = self_bf16 ? self_bf16 + c0 : nullptr;
            if (dtype == CR_F32) launch_fwd_group<float, 32, 1, GCN>(blocks, tab, ld_src, Fk, agg_bf16 + c0, self_k, batch_stride_rows, ld_bf16, s, out_cols, node_norm);
            else launch_fwd_group<uint16_t, 32, 1, GCN>(blocks, tab, ld_src, Fk, agg_bf16 + c0, self_k, batch_stride_rows, ld_bf16, s, out_cols, node_norm);
        }
        CR_LAUNCH_CHECK();
        return CR_OK;
    }
#define CR_FWDG(T, LPR, NC) launch_fwd_group<T, LPR, NC, GCN>(blocks, H_src, ld_src, F, agg_bf16, self_bf16, batch_stride_rows, ld_bf16, s, 0, node_norm)
    if (dtype == CR_F32) {
        if (F <= 64) CR_FWDG(float, 16, 1);
        else if (F <= 128) CR_FWDG(float, 32, 1);
        else if (F <= 256) CR_FWDG(float, 64, 1);
        else if (F <= 512) CR_FWDG(float, 64, 2);
        else if (F <= 768) CR_FWDG(float, 64, 3);
        else CR_FWDG(float, 64, 4);
    } else {
        if (F <= 128) CR_FWDG(uint16_t, 16, 1);
        else if (F <= 256) CR_FWDG(uint16_t, 32, 1);
        else if (F <= 512) CR_FWDG(uint16_t, 64, 1);
        else CR_FWDG(uint16_t, 64, 2);
    }
#undef CR_FWDG
    CR_LAUNCH_CHECK();
    return CR_OK;
}

extern "C" cr_status cr_gather_aggregate_fwd_group(const cr_block_set *blocks, const void *H_src, int32_t dtype, int64_t ld_src,
                                                   int32_t F, uint16_t *agg_bf16, uint16_t *self_bf16, int64_t batch_stride_rows,
                                                   int64_t ld_bf16, void *stream)
{
    return gather_group<false>(blocks, H_src, dtype, ld_src, F, agg_bf16, self_bf16, batch_stride_rows, ld_bf16, stream, nullptr);
}

extern "C" cr_status cr_gcn_aggregate_fwd_group(const cr_block_set *blocks, const float *norm, const void *H_src, int32_t dtype,
                                                int64_t ld_src, int32_t F, uint16_t *agg_bf16, int64_t batch_stride_rows,
                                                int64_t ld_bf16, void *stream)
{
    return gather_group<true>(blocks, H_src, dtype, ld_src, F, agg_bf16, nullptr, batch_stride_rows, ld_bf16, stream, norm);
}

extern "C" cr_status cr_gather_aggregate_bwd(const cr_block_set *blocks, int32_t g, const void *d_agg,
                                             const void *d_self, int32_t in_dtype, int64_t ld_in, int32_t F,
                                             const void *relu_out, int32_t relu_dtype, int64_t ld_relu, float *d_src,
                                             uint16_t *d_src_bf16, int64_t ld_bf16, void *stream)
{
    cr_status st = check_block_set(blocks, g, true);
    if (st != CR_OK) return st;
    CR_REQUIRE(d_agg != nullptr && aligned16(d_agg) && aligned16(d_self), CR_ERR_INVALID_ARG, "d_agg / d_self must be 16-byte aligned device pointers");
    CR_REQUIRE(F >= 1 && F <= 1024, CR_ERR_UNSUPPORTED, "F = %d outside 1..1024", F);
    CR_REQUIRE(in_dtype == CR_F32 || in_dtype == CR_BF16, CR_ERR_INVALID_ARG, "in_dtype must be CR_F32 or CR_BF16");
    const int in_vec = in_dtype == CR_BF16 ? 8 : 4;
    CR_REQUIRE(ld_in >= round_up(F, in_vec) && ld_in % in_vec == 0, CR_ERR_INVALID_ARG, "ld_in must be a multiple of %d covering F", in_vec);
    if (relu_out) {
        CR_REQUIRE(relu_dtype == CR_F32 || relu_dtype == CR_BF16, CR_ERR_INVALID_ARG, "relu_dtype must be CR_F32 or CR_BF16");
        CR_REQUIRE(aligned16(relu_out) && ld_relu >= round_up(F, 4) && ld_relu % 4 == 0, CR_ERR_INVALID_ARG, "relu_out must be aligned with ld_relu a multiple of 4 covering F");
        CR_REQUIRE(!(in_dtype == CR_BF16 && relu_dtype == CR_BF16) || ld_relu % 8 == 0, CR_ERR_INVALID_ARG,
                   "with bf16 gradients a bf16 relu_out needs ld_relu to be a multiple of 8");
    }
    CR_REQUIRE(d_src || d_src_bf16, CR_ERR_INVALID_ARG, "no output requested");
    CR_REQUIRE(aligned16(d_src) && aligned16(d_src_bf16), CR_ERR_INVALID_ARG, "outputs must be 16-byte aligned");
    if (d_src_bf16)
        CR_REQUIRE(ld_bf16 % 32 == 0 && ld_bf16 >= F && ld_bf16 <= round_up(F, 64), CR_ERR_INVALID_ARG,
                   "ld_bf16 = %lld must be a multiple of 32 in [F, F rounded up to 64]", (long long)ld_bf16);
    if (dry_run()) return CR_OK;

    run_bwd(blocks, g, d_agg, d_self, in_dtype, ld_in, F, relu_out, relu_dtype, ld_relu, d_src, d_src_bf16, ld_bf16,
            static_cast<hipStream_t>(stream), nullptr);
    CR_LAUNCH_CHECK();
    return CR_OK;
}

extern "C" cr_status cr_sage_layer_bwd(const cr_sage_layer *layer, const cr_block_set *blocks, int32_t g,
                                       const uint16_t *h_self, const uint16_t *agg, int64_t ld_in, const uint16_t *dz_bf16,
                                       float lr, float weight_decay, uint16_t *d_in_bf16, const uint16_t *relu_out_bf16,
                                       int64_t ld_relu, uint16_t *d_src_bf16, int64_t ld_bf16, float *dW_out, float *db_out,
                                       void *ws, size_t ws_bytes, void *stream)
{
    cr_status st = check_block_set(blocks, g, true);
    if (st != CR_OK) return st;
    CR_REQUIRE(layer != nullptr && layer->n_operands == 2, CR_ERR_INVALID_ARG, "a two-operand layer is required");
    CR_REQUIRE(d_in_bf16 != nullptr && d_src_bf16 != nullptr, CR_ERR_INVALID_ARG, "d_in_bf16 and d_src_bf16 must be given");
    CR_REQUIRE(aligned16(d_src_bf16) && aligned16(relu_out_bf16), CR_ERR_INVALID_ARG, "d_src_bf16 / relu_out_bf16 must be 16-byte aligned");
    const int32_t F = layer->F_in;
    CR_REQUIRE(F >= 1 && F <= 1024, CR_ERR_UNSUPPORTED, "F_in = %d outside 1..1024", F);
    if (relu_out_bf16) CR_REQUIRE(ld_relu >= round_up(F, 8) && ld_relu % 8 == 0, CR_ERR_INVALID_ARG, "ld_relu must be a multiple of 8 covering F_in");
    CR_REQUIRE(ld_bf16 % 32 == 0 && ld_bf16 >= F && ld_bf16 <= round_up(F, 64), CR_ERR_INVALID_ARG,
               "ld_bf16 = %lld must be a multiple of 32 in [F_in, F_in rounded up to 64]", (long long)ld_bf16);
    const int32_t *hdr = blocks->hdr + (int64_t)g * CR_HDR_WORDS;
    SgdArgs sgd;
    st = linear_bwd_products(layer, hdr, blocks->cap_dst, h_self, agg, ld_in, dz_bf16, lr, weight_decay, nullptr, nullptr, d_in_bf16,
                             dW_out, db_out, ws, ws_bytes, stream, &sgd);
    if (st != CR_OK) return st;
    if (dry_run()) return CR_OK;

    const int F_pad = (int)round_up(F, 32), N_pad = (int)round_up(layer->F_out, 64);
    const unsigned sgd_blocks = sgd_reduce_blocks(F_pad, N_pad, 2);
    const int32_t *indptr = blocks->indptr + (int64_t)g * (blocks->cap_dst + 1);
    const int32_t *t_indptr = blocks->t_indptr + (int64_t)g * (blocks->cap_src + 1);
    const int32_t *t_indices = blocks->t_indices + (int64_t)g * blocks->cap_nnz;
    hipStream_t s = static_cast<hipStream_t>(stream);
#define CR_BWDS(LPR, NC) launch_bwd_sgd<LPR, NC>(sgd, sgd_blocks, blocks->cap_src, hdr, indptr, t_indptr, t_indices, d_in_bf16 + F_pad, d_in_bf16, \
                                                 2 * (int64_t)F_pad, F, relu_out_bf16, 1, ld_relu, d_src_bf16, ld_bf16, s)
    if (F <= 128) CR_BWDS(16, 1);
    else if (F <= 256) CR_BWDS(32, 1);
    else if (F <= 512) CR_BWDS(64, 1);
    else CR_BWDS(64, 2);
#undef CR_BWDS
    CR_LAUNCH_CHECK();
    return CR_OK;
}

// ------------------------------------------------------------------------------------------------
// GCN propagation on the same blocks
// ------------------------------------------------------------------------------------------------
extern "C" cr_status cr_graph_gcn_norm(const cr_graph *graph, float *norm, void *stream)
{
    CR_REQUIRE(graph != nullptr && graph->indptr != nullptr && graph->n_nodes >= 1, CR_ERR_INVALID_ARG, "graph must carry indptr and at least one node");
    CR_REQUIRE(norm != nullptr && aligned16(norm), CR_ERR_INVALID_ARG, "norm must be a 16-byte aligned device pointer");
    if (dry_run()) return CR_OK;
    hipLaunchKernelGGL(gcn_node_norm_kernel, dim3((unsigned)ceil_div(graph->n_nodes, 256)), dim3(256), 0, static_cast<hipStream_t>(stream),
                       graph->indptr, graph->n_nodes, norm);
    CR_LAUNCH_CHECK();
    return CR_OK;
}

static GcnFwd block_norm_views(const cr_block_set *b, float *blk_norm)
{
    GcnFwd v;
    v.edge_w = blk_norm;
    v.node_norm = nullptr;
    v.dst_scale = blk_norm + b->cap_src;
    v.dst_self = blk_norm + b->cap_src + b->cap_dst;
    return v;
}

extern "C" cr_status cr_gcn_block_norm(const cr_block_set *blocks, int32_t g, const float *norm, float *blk_norm, void *stream)
{
    cr_status st = check_block_set(blocks, g, false);
    if (st != CR_OK) return st;
    CR_REQUIRE(norm && blk_norm, CR_ERR_INVALID_ARG, "norm / blk_norm must not be NULL");
    if (dry_run()) return CR_OK;
    const GcnFwd v = block_norm_views(blocks, blk_norm);
    hipLaunchKernelGGL(gcn_block_norm_kernel, dim3((unsigned)ceil_div(blocks->cap_src, 256)), dim3(256), 0, static_cast<hipStream_t>(stream),
                       blocks->hdr + (int64_t)g * CR_HDR_WORDS, blocks->indptr + (int64_t)g * (blocks->cap_dst + 1),
                       blocks->src_ids + (int64_t)g * blocks->cap_src, norm, const_cast<float *>(v.edge_w),
                       const_cast<float *>(v.dst_scale), const_cast<float *>(v.dst_self));
    CR_LAUNCH_CHECK();
    return CR_OK;
}

extern "C" cr_status cr_gcn_aggregate_fwd(const cr_block_set *blocks, int32_t g, const float *norm, const float *blk_norm,
                                          const void *H_src, int32_t dtype, int64_t ld_src, int32_t F, int32_t indirect,
                                          float *agg, uint16_t *agg_bf16, int64_t ld_bf16, void *stream)
{
    cr_status st = check_block_set(blocks, g, false);
    if (st != CR_OK) return st;
    CR_REQUIRE(norm && blk_norm, CR_ERR_INVALID_ARG, "norm / blk_norm must not be NULL");
    CR_REQUIRE(!indirect || blocks->gather_ids, CR_ERR_UNSUPPORTED, "table addressing by global id needs the block's gather_ids");
    CR_REQUIRE(H_src != nullptr && aligned16(H_src), CR_ERR_INVALID_ARG, "H_src must be a 16-byte aligned device pointer");
    CR_REQUIRE(dtype == CR_F32 || dtype == CR_BF16, CR_ERR_INVALID_ARG, "dtype must be CR_F32 or CR_BF16");
    const int vec = dtype == CR_F32 ? 4 : 8;
    CR_REQUIRE(F >= 1 && F <= 1024, CR_ERR_UNSUPPORTED, "F = %d outside 1..1024", F);
    CR_REQUIRE(ld_src >= round_up(F, vec) && ld_src % vec == 0, CR_ERR_INVALID_ARG,
               "ld_src = %lld must be a multiple of %d and cover F rounded up to it", (long long)ld_src, vec);
    CR_REQUIRE(agg || agg_bf16, CR_ERR_INVALID_ARG, "no output requested");
    CR_REQUIRE(aligned16(agg) && aligned16(agg_bf16), CR_ERR_INVALID_ARG, "outputs must be 16-byte aligned");
    if (agg_bf16)
        CR_REQUIRE(ld_bf16 % 32 == 0 && ld_bf16 >= F && ld_bf16 <= round_up(F, 64), CR_ERR_INVALID_ARG,
                   "ld_bf16 = %lld must be a multiple of 32 in [F, F rounded up to 64]", (long long)ld_bf16);
    if (dry_run()) return CR_OK;
    GcnFwd v = block_norm_views(blocks, const_cast<float *>(blk_norm));
    if (indirect) { v.edge_w = nullptr; v.node_norm = norm; }       // per-edge ids are global: weights by node
    run_fwd(blocks, g, H_src, dtype, ld_src, F, indirect, agg, agg_bf16, nullptr, ld_bf16, static_cast<hipStream_t>(stream), &v);
    CR_LAUNCH_CHECK();
    return CR_OK;
}

extern "C" cr_status cr_gcn_aggregate_bwd(const cr_block_set *blocks, int32_t g, const float *blk_norm, const void *d_out,
                                          int32_t in_dtype, int64_t ld_in, int32_t F, const void *relu_out, int32_t relu_dtype,
                                          int64_t ld_relu, float *d_src, uint16_t *d_src_bf16, int64_t ld_bf16, void *stream)
{
    cr_status st = check_block_set(blocks, g, true);
    if (st != CR_OK) return st;
    CR_REQUIRE(blk_norm != nullptr, CR_ERR_INVALID_ARG, "blk_norm must not be NULL");
    CR_REQUIRE(d_out != nullptr && aligned16(d_out), CR_ERR_INVALID_ARG, "d_out must be a 16-byte aligned device pointer");
    CR_REQUIRE(F >= 1 && F <= 1024, CR_ERR_UNSUPPORTED, "F = %d outside 1..1024", F);
    CR_REQUIRE(in_dtype == CR_F32 || in_dtype == CR_BF16, CR_ERR_INVALID_ARG, "in_dtype must be CR_F32 or CR_BF16");
    const int in_vec = in_dtype == CR_BF16 ? 8 : 4;
    CR_REQUIRE(ld_in >= round_up(F, in_vec) && ld_in % in_vec == 0, CR_ERR_INVALID_ARG, "ld_in must be a multiple of %d covering F", in_vec);
    if (relu_out) {
        CR_REQUIRE(relu_dtype == CR_F32 || relu_dtype == CR_BF16, CR_ERR_INVALID_ARG, "relu_dtype must be CR_F32 or CR_BF16");
        CR_REQUIRE(aligned16(relu_out) && ld_relu >= round_up(F, 4) && ld_relu % 4 == 0, CR_ERR_INVALID_ARG, "relu_out must be aligned with ld_relu a multiple of 4 covering F");
        CR_REQUIRE(!(in_dtype == CR_BF16 && relu_dtype == CR_BF16) || ld_relu % 8 == 0, CR_ERR_INVALID_ARG,
                   "with bf16 gradients a bf16 relu_out needs ld_relu to be a multiple of 8");
    }
    CR_REQUIRE(d_src || d_src_bf16, CR_ERR_INVALID_ARG, "no output requested");
    CR_REQUIRE(aligned16(d_src) && aligned16(d_src_bf16), CR_ERR_INVALID_ARG, "outputs must be 16-byte aligned");
    if (d_src_bf16)
        CR_REQUIRE(ld_bf16 % 32 == 0 && ld_bf16 >= F && ld_bf16 <= round_up(F, 64), CR_ERR_INVALID_ARG,
                   "ld_bf16 = %lld must be a multiple of 32 in [F, F rounded up to 64]", (long long)ld_bf16);
    if (dry_run()) return CR_OK;
    const GcnFwd v = block_norm_views(blocks, const_cast<float *>(blk_norm));
    run_bwd(blocks, g, d_out, d_out, in_dtype, ld_in, F, relu_out, relu_dtype, ld_relu, d_src, d_src_bf16, ld_bf16,
            static_cast<hipStream_t>(stream), &v);
    CR_LAUNCH_CHECK();
    return CR_OK;
}
