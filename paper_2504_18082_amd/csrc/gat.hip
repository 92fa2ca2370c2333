// Graph-attention layer on a sampled block (Section 6.4 applies the method to GAT; the layer is the one of
// Velickovic et al.: shared projection z = xW, scores LeakyReLU(a_l.z_u + a_r.z_v), softmax over the sampled
// in-neighbours, out_v = sum_u alpha_vu z_u + bias, heads concatenated).
//
// Layout: a projected row is `ld` bf16 values (the layer's padded output width, heads*D real columns); a lane owns
// 8 consecutive columns (one 16-byte load), a group of LPR lanes owns one row, the lanes of one head are LH
// consecutive lanes of the group, so a per-head dot product is an xor-shuffle reduction over LH lanes.
// Every sum is taken in a fixed order (rows are dealt to groups by index, partial sums meet in LDS in a fixed
// association), so results are bit-reproducible.
#include "cr_common.h"

#include <math.h>

namespace cr {

__device__ __forceinline__ void load_bf16x8(const uint16_t *p, float (&v)[8])
{
    const uint4 x = *reinterpret_cast<const uint4 *>(p);
    v[0] = __uint_as_float(x.x << 16); v[1] = __uint_as_float(x.x & 0xFFFF0000u);
    v[2] = __uint_as_float(x.y << 16); v[3] = __uint_as_float(x.y & 0xFFFF0000u);
    v[4] = __uint_as_float(x.z << 16); v[5] = __uint_as_float(x.z & 0xFFFF0000u);
    v[6] = __uint_as_float(x.w << 16); v[7] = __uint_as_float(x.w & 0xFFFF0000u);
}

// The same load for a lane whose columns may not exist: such a lane reads the row's last chunk instead and gets
// zeros (mask = 0).  Keeping every load unconditional lets the independent loads of a loop body be issued back
// to back; a load under a branch makes the compiler wait for it before going on.
__device__ __forceinline__ void load_bf16x8(const uint16_t *p, uint32_t mask, float (&v)[8])
{
    uint4 x = *reinterpret_cast<const uint4 *>(p);
    x.x &= mask; x.y &= mask; x.z &= mask; x.w &= mask;
    v[0] = __uint_as_float(x.x << 16); v[1] = __uint_as_float(x.x & 0xFFFF0000u);
    v[2] = __uint_as_float(x.y << 16); v[3] = __uint_as_float(x.y & 0xFFFF0000u);
    v[4] = __uint_as_float(x.z << 16); v[5] = __uint_as_float(x.z & 0xFFFF0000u);
    v[6] = __uint_as_float(x.w << 16); v[7] = __uint_as_float(x.w & 0xFFFF0000u);
}

__device__ __forceinline__ void unpack_bf16x8(uint4 x, uint32_t mask, float (&v)[8])
{
    x.x &= mask; x.y &= mask; x.z &= mask; x.w &= mask;
    v[0] = __uint_as_float(x.x << 16); v[1] = __uint_as_float(x.x & 0xFFFF0000u);
    v[2] = __uint_as_float(x.y << 16); v[3] = __uint_as_float(x.y & 0xFFFF0000u);
    v[4] = __uint_as_float(x.z << 16); v[5] = __uint_as_float(x.z & 0xFFFF0000u);
    v[6] = __uint_as_float(x.w << 16); v[7] = __uint_as_float(x.w & 0xFFFF0000u);
}

__device__ __forceinline__ void store_bf16x8(uint16_t *p, const float (&v)[8])
{
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) w[i] = pack_bf16x2(v[2 * i], v[2 * i + 1]);
    *reinterpret_cast<uint4 *>(p) = make_uint4(w[0], w[1], w[2], w[3]);
}

// sum over the LH lanes of a head (LH a power of two; every lane of the head ends up with the total)
__device__ __forceinline__ float head_sum(float x, int LH)
{
    for (int off = 1; off < LH; off <<= 1) x += __shfl_xor(x, off);
    return x;
}

// the same for N independent values at once: the N reductions advance together, one exchange latency per step
template <int N>
__device__ __forceinline__ void head_sum_n(float (&x)[N], int LH)
{
    for (int off = 1; off < LH; off <<= 1) {
        float y[N];
#pragma unroll
        for (int k = 0; k < N; ++k) y[k] = __shfl_xor(x[k], off);
#pragma unroll
        for (int k = 0; k < N; ++k) x[k] += y[k];
    }
}

__device__ __forceinline__ float dot8(const float (&a)[8], const float (&b)[8])
{
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) s += a[i] * b[i];
    return s;
}

struct GatShape {
    int32_t heads, D, LH;   // LH: lanes per head
    int32_t ld;             // elements per projected row (multiple of 64)
    int32_t max_deg;        // most neighbours a destination row can have (the block's fanout)
    float slope;
};

// what a lane needs to know about its place in the row
struct LaneInfo {
    int gl, grp, col, colc, h;   // colc: col, or the row's last chunk for a lane past the row's end
    uint32_t mask;               // all ones for a live lane, else 0
    bool live, writer;           // live: the lane's columns exist; writer: the lane that stores its head's scalars
};
template <int LPR>
__device__ __forceinline__ LaneInfo lane_info(const GatShape &s)
{
    LaneInfo li;
    li.gl = (int)(threadIdx.x % LPR);
    li.grp = (int)(threadIdx.x / LPR);
    li.col = li.gl * 8;
    li.live = li.col < s.ld;
    li.colc = min(li.col, s.ld - 8);
    li.mask = li.live ? 0xFFFFFFFFu : 0u;
    const int h = s.heads > 1 ? li.col / s.D : 0;
    li.writer = li.live && h < s.heads && (li.gl % s.LH) == 0;
    li.h = min(h, s.heads - 1);
    return li;
}

// ---------------------------------------------------------------------------------------------------------------
// rows_out[i] = bf16(store[ids[i]]), zero padded to ld_out columns: the operand of the first layer's projection.
// ---------------------------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void gather_rows_bf16_kernel(const T *__restrict__ store, int64_t ld_src, int F,
                                                               const int32_t *__restrict__ ids, const int32_t *__restrict__ hdr,
                                                               int hdr_word, int max_n, uint16_t *__restrict__ out, int64_t ld_out)
{
    const int n = min(hdr[hdr_word], max_n);
    const int cpr = (int)(ld_out / 8);                      // 8-column chunks per row
    const int64_t total = (int64_t)n * cpr;
    for (int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x; t < total; t += (int64_t)gridDim.x * 256) {
        const int i = (int)(t / cpr), col = (int)(t % cpr) * 8;
        float v[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        const T *row = store + (int64_t)ids[i] * ld_src;
        if constexpr (sizeof(T) == 4) {
            if (col < ld_src) {
                const float4 a = *reinterpret_cast<const float4 *>(row + col);
                v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
            }
            if (col + 4 < ld_src) {
                const float4 b = *reinterpret_cast<const float4 *>(row + col + 4);
                v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
            }
        } else {
            if (col < ld_src) load_bf16x8(reinterpret_cast<const uint16_t *>(row) + col, v);
        }
#pragma unroll
        for (int k = 0; k < 8; ++k)
            if (col + k >= F) v[k] = 0.f;
        store_bf16x8(out + (int64_t)i * ld_out + col, v);
    }
}

// ---------------------------------------------------------------------------------------------------------------
// el[u,h] = a_l[h] . z[u,h],  er[u,h] = a_r[h] . z[u,h]  for every source row u
// ---------------------------------------------------------------------------------------------------------------
template <int LPR>
__global__ __launch_bounds__(256) void gat_scores_kernel(const int32_t *__restrict__ hdr, GatShape s, const uint16_t *__restrict__ z,
                                                         const float *__restrict__ attn, float *__restrict__ el, float *__restrict__ er)
{
    constexpr int GPB = 256 / LPR;
    const int n_src = hdr[CR_HDR_N_SRC];
    const LaneInfo li = lane_info<LPR>(s);
    float al[8], ar[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        al[i] = li.live ? attn[li.colc + i] : 0.f;
        ar[i] = li.live ? attn[s.ld + li.colc + i] : 0.f;
    }
    constexpr int R = 4;                                     // rows in flight per group
    for (int u0 = (int)blockIdx.x * GPB * R + li.grp; u0 < n_src; u0 += (int)gridDim.x * GPB * R) {
        float v[R][8];
#pragma unroll
        for (int k = 0; k < R; ++k) {
            load_bf16x8(z + (int64_t)min(u0 + k * GPB, n_src - 1) * s.ld + li.colc, li.mask, v[k]);
        }
        float sc[2 * R];
#pragma unroll
        for (int k = 0; k < R; ++k) {
            sc[2 * k] = dot8(v[k], al);
            sc[2 * k + 1] = dot8(v[k], ar);
        }
        head_sum_n<2 * R>(sc, s.LH);
#pragma unroll
        for (int k = 0; k < R; ++k) {
            const int u = u0 + k * GPB;
            if (li.writer && u < n_src) {
                el[(int64_t)u * s.heads + li.h] = sc[2 * k];
                er[(int64_t)u * s.heads + li.h] = sc[2 * k + 1];
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------------------------
// forward: neighbourhood softmax and weighted sum.  stat[v,h] = (er, max score, 1 / sum of exp, -) is kept for the
// backward pass, which recomputes alpha from it instead of storing one weight per edge and head.
// The scores of a row are computed cooperatively: the LH lanes of a head take every LH-th edge each, so a row of
// degree d costs d / LH dependent look-ups instead of d; the per-edge weights pass through a slice of LDS that the
// row's group owns (fanout x heads floats; a group is part of one wave, LDS operations of a wave stay in order).
// ---------------------------------------------------------------------------------------------------------------
__device__ __forceinline__ float head_max(float x, int LH)
{
    for (int off = 1; off < LH; off <<= 1) x = fmaxf(x, __shfl_xor(x, off));
    return x;
}

template <int LPR>
__global__ __launch_bounds__(256) void gat_aggregate_fwd_kernel(const int32_t *__restrict__ hdr, const int32_t *__restrict__ indptr,
                                                                const int32_t *__restrict__ indices, GatShape s,
                                                                const uint16_t *__restrict__ z, const float *__restrict__ attn,
                                                                const float *__restrict__ el, const float *__restrict__ er, int relu,
                                                                float *__restrict__ out, uint16_t *__restrict__ out_bf16,
                                                                float4 *__restrict__ stat)
{
    constexpr int GPB = 256 / LPR;
    constexpr int U = 8;
    extern __shared__ float edge_w[];                       // [GPB][max_deg][heads]
    const int n_dst = hdr[CR_HDR_N_DST];
    const LaneInfo li = lane_info<LPR>(s);
    float *gw = edge_w + (size_t)li.grp * s.max_deg * s.heads + li.h;
    const int sub = li.gl % s.LH;
    float bias[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) bias[i] = li.live ? attn[2 * s.ld + li.colc + i] : 0.f;
    for (int v = (int)blockIdx.x * GPB + li.grp; v < n_dst; v += (int)gridDim.x * GPB) {
        const int b = indptr[v], e = min(indptr[v + 1], b + s.max_deg);
        const float erv = er[(int64_t)v * s.heads + li.h];
        float mx = -INFINITY;
        for (int j = b + sub; j < e; j += s.LH) {
            float x = el[(int64_t)indices[j] * s.heads + li.h] + erv;
            x = x > 0.f ? x : s.slope * x;
            gw[(j - b) * s.heads] = x;
            mx = fmaxf(mx, x);
        }
        mx = head_max(mx, s.LH);
        float sum = 0.f;
        for (int j = b + sub; j < e; j += s.LH) {
            const float w = expf(gw[(j - b) * s.heads] - mx);
            gw[(j - b) * s.heads] = w;
            sum += w;
        }
        sum = head_sum(sum, s.LH);
        const float inv = e > b ? 1.f / sum : 0.f;
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");      // the head's lanes now read each other's weights
        float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        for (int j = b; j < e; j += U) {
            int u[U];
            float w[U], r[U][8];
#pragma unroll
            for (int k = 0; k < U; ++k) u[k] = indices[min(j + k, e - 1)];
#pragma unroll
            for (int k = 0; k < U; ++k) {
                load_bf16x8(z + (int64_t)u[k] * s.ld + li.colc, li.mask, r[k]);
                const float wk = gw[(min(j + k, e - 1) - b) * s.heads];
                w[k] = j + k < e ? wk : 0.f;
            }
#pragma unroll
            for (int k = 0; k < U; ++k)
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[i] += w[k] * r[k][i];
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");      // the slice is reused by the group's next row
        float o[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            o[i] = acc[i] * inv + bias[i];
            if (relu) o[i] = fmaxf(o[i], 0.f);
        }
        if (li.live) {
            if (out) {
                *reinterpret_cast<float4 *>(out + (int64_t)v * s.ld + li.col) = make_float4(o[0], o[1], o[2], o[3]);
                *reinterpret_cast<float4 *>(out + (int64_t)v * s.ld + li.col + 4) = make_float4(o[4], o[5], o[6], o[7]);
            }
            if (out_bf16) store_bf16x8(out_bf16 + (int64_t)v * s.ld + li.col, o);
        }
        if (li.writer) stat[(int64_t)v * s.heads + li.h] = make_float4(erv, e > b ? mx : 0.f, inv, 0.f);
    }
}

// Sum of per-lane column partials over the groups of a workgroup (fixed order), written as row blockIdx.x of `partial`.
template <int LPR>
__device__ __forceinline__ void block_column_sums(const float (&p)[8], const LaneInfo &li, float *lds /*[256 * 8]*/, float *partial, int ld)
{
    constexpr int GPB = 256 / LPR;
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 8; ++i) lds[(li.grp * LPR + li.gl) * 8 + i] = p[i];
    __syncthreads();
    if (li.grp == 0 && li.live) {
        float t[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) t[i] = 0.f;
        for (int g = 0; g < GPB; ++g)
#pragma unroll
            for (int i = 0; i < 8; ++i) t[i] += lds[(g * LPR + li.gl) * 8 + i];
        float *dst = partial + (int64_t)blockIdx.x * ld + li.col;
        *reinterpret_cast<float4 *>(dst) = make_float4(t[0], t[1], t[2], t[3]);
        *reinterpret_cast<float4 *>(dst + 4) = make_float4(t[4], t[5], t[6], t[7]);
    }
}

// ---------------------------------------------------------------------------------------------------------------
// backward, destination side.  With g = dL/d out (ReLU mask applied), per edge d_alpha = g[v,h] . z[u,h]; then
//   t[v,h]    = sum_e alpha_e d_alpha_e                       (softmax backward: d_e = alpha (d_alpha - t))
//   d_er[v,h] = sum_e alpha_e (d_alpha_e - t) lrelu'(x_e)     (every edge's score contains er[v,h])
// One pass over the row's edges collects sum(alpha d_alpha), sum(alpha d_alpha l') and sum(alpha l').  Also writes
// the masked gradient rows (bf16) for the source-side pass and this workgroup's column sums of g (bias gradient).
// ---------------------------------------------------------------------------------------------------------------
template <int LPR>
__global__ __launch_bounds__(256) void gat_bwd_dst_kernel(const int32_t *__restrict__ hdr, const int32_t *__restrict__ indptr,
                                                          const int32_t *__restrict__ indices, GatShape s,
                                                          const uint16_t *__restrict__ z, const float *__restrict__ el,
                                                          const uint16_t *__restrict__ d_out, int64_t ld_dout,
                                                          const uint16_t *__restrict__ relu_out, float4 *__restrict__ stat,
                                                          uint16_t *__restrict__ g_b, float *__restrict__ d_er,
                                                          float *__restrict__ partial_db)
{
    constexpr int GPB = 256 / LPR;
    constexpr int U = 8;
    extern __shared__ float edge_w[];                       // [GPB][max_deg][heads][2]: alpha, alpha * lrelu'
    float *lds = edge_w + (size_t)GPB * s.max_deg * s.heads * 2;     // [256 * 8] for the column sums
    const int n_dst = hdr[CR_HDR_N_DST];
    const LaneInfo li = lane_info<LPR>(s);
    float2 *gw = reinterpret_cast<float2 *>(edge_w) + (size_t)li.grp * s.max_deg * s.heads + li.h;
    const int sub = li.gl % s.LH;
    float dbp[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int v = (int)blockIdx.x * GPB + li.grp; v < n_dst; v += (int)gridDim.x * GPB) {
        float g[8], o[8];
        load_bf16x8(d_out + (int64_t)v * ld_dout + li.colc, li.mask, g);
        // without a ReLU the mask is taken on the gradient row itself (loaded again, from cache) and always passes
        load_bf16x8(relu_out ? relu_out + (int64_t)v * s.ld + li.colc : d_out + (int64_t)v * ld_dout + li.colc, li.mask, o);
#pragma unroll
        for (int i = 0; i < 8; ++i) g[i] = (relu_out == nullptr || o[i] > 0.f) ? g[i] : 0.f;
        if (li.live) store_bf16x8(g_b + (int64_t)v * s.ld + li.col, g);
#pragma unroll
        for (int i = 0; i < 8; ++i) dbp[i] += g[i];
        const int b = indptr[v], e = min(indptr[v + 1], b + s.max_deg);
        const float4 st = stat[(int64_t)v * s.heads + li.h];
        // alpha and alpha * lrelu' of the row's edges, every LH-th edge per lane of the head
        float Cq = 0.f;
        for (int j = b + sub; j < e; j += s.LH) {
            const float x = el[(int64_t)indices[j] * s.heads + li.h] + st.x;
            const bool pos = x > 0.f;
            const float a = expf((pos ? x : s.slope * x) - st.y) * st.z;
            const float alp = pos ? a : s.slope * a;
            gw[(j - b) * s.heads] = make_float2(a, alp);
            Cq += alp;
        }
        Cq = head_sum(Cq, s.LH);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        float A = 0.f, Bq = 0.f;
        for (int j = b; j < e; j += U) {
            int u[U];
            float2 w[U];
            float r[U][8];
#pragma unroll
            for (int k = 0; k < U; ++k) u[k] = indices[min(j + k, e - 1)];
#pragma unroll
            for (int k = 0; k < U; ++k) {
                load_bf16x8(z + (int64_t)u[k] * s.ld + li.colc, li.mask, r[k]);
                const float2 wk = gw[(min(j + k, e - 1) - b) * s.heads];
                w[k] = j + k < e ? wk : make_float2(0.f, 0.f);
            }
            float da[U];
#pragma unroll
            for (int k = 0; k < U; ++k) da[k] = dot8(g, r[k]);
            head_sum_n<U>(da, s.LH);
#pragma unroll
            for (int k = 0; k < U; ++k) {
                A += w[k].x * da[k];
                Bq += w[k].y * da[k];
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        if (li.writer) {
            stat[(int64_t)v * s.heads + li.h] = make_float4(st.x, st.y, st.z, A);
            d_er[(int64_t)v * s.heads + li.h] = Bq - A * Cq;
        }
    }
    block_column_sums<LPR>(dbp, li, lds, partial_db, s.ld);
}

// ---------------------------------------------------------------------------------------------------------------
// backward, source side (pull over the transposed block, no atomics): for source row u with destinations v
//   d_z[u,h] = sum_v alpha_vu g[v,h] + d_el[u,h] a_l[h] + (u < n_dst) d_er[u,h] a_r[h]
//   d_el[u,h] = sum_v alpha_vu (d_alpha_vu - t[v,h]) lrelu'(x_vu)
// and this workgroup's contributions to d_a_l = sum_u d_el[u,h] z[u,h] and d_a_r = sum_v d_er[v,h] z[v,h].
// ---------------------------------------------------------------------------------------------------------------
template <int LPR>
__global__ __launch_bounds__(256) void gat_bwd_src_kernel(const int32_t *__restrict__ hdr, const int32_t *__restrict__ t_indptr,
                                                          const int32_t *__restrict__ t_indices, GatShape s,
                                                          const uint16_t *__restrict__ z, const float *__restrict__ attn,
                                                          const float *__restrict__ el, const float4 *__restrict__ stat,
                                                          const uint16_t *__restrict__ g_b, const float *__restrict__ d_er,
                                                          uint16_t *__restrict__ dz_bf16, float *__restrict__ partial_al,
                                                          float *__restrict__ partial_ar)
{
    constexpr int GPB = 256 / LPR;
    constexpr int U = 2;
    __shared__ float lds[256 * 8];
    const int n_dst = hdr[CR_HDR_N_DST], n_src = hdr[CR_HDR_N_SRC];
    const LaneInfo li = lane_info<LPR>(s);
    float al[8], ar[8], pal[8], par[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        al[i] = li.live ? attn[li.colc + i] : 0.f;
        ar[i] = li.live ? attn[s.ld + li.colc + i] : 0.f;
        pal[i] = 0.f;
        par[i] = 0.f;
    }
    // Most source rows are used by one or two destinations, so a row is a chain of look-ups (row range -> destination
    // ids -> their gradient rows), not a stream.  The chain of the group's next row is started while the current
    // row is worked on: its range and its first U destination ids are fetched one row ahead (clamped, unconditional).
    const int stride = (int)gridDim.x * GPB;
    int u = (int)blockIdx.x * GPB + li.grp;
    if (u < n_src) {
        int b = t_indptr[u], e = t_indptr[u + 1];
        int v0[U];
#pragma unroll
        for (int k = 0; k < U; ++k) v0[k] = t_indices[max(min(b + k, e - 1), 0)];
        uint4 z_raw = *reinterpret_cast<const uint4 *>(z + (int64_t)u * s.ld + li.colc);
        float elu = el[(int64_t)u * s.heads + li.h];
        float der_any = d_er[(int64_t)max(min(u, n_dst - 1), 0) * s.heads + li.h];
        for (; u < n_src; u += stride) {
            // everything the next row starts from: its range, its first destinations, its own row and scalars
            const int un = min(u + stride, n_src - 1);
            const int nb = t_indptr[un], ne = t_indptr[un + 1];
            const uint4 nz_raw = *reinterpret_cast<const uint4 *>(z + (int64_t)un * s.ld + li.colc);
            const float nelu = el[(int64_t)un * s.heads + li.h];
            const float nder = d_er[(int64_t)max(min(un, n_dst - 1), 0) * s.heads + li.h];
            int nv[U];
#pragma unroll
            for (int k = 0; k < U; ++k) nv[k] = t_indices[max(min(nb + k, ne - 1), 0)];
            float zr[8];
            unpack_bf16x8(z_raw, li.mask, zr);
            const float der = u < n_dst ? der_any : 0.f;
            int v[U];
#pragma unroll
            for (int k = 0; k < U; ++k) v[k] = v0[k];
            float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f}, del = 0.f;
            for (int j = b; j < e; j += U) {
                float4 st[U];
                float g[U][8];
#pragma unroll
                for (int k = 0; k < U; ++k) {
                    st[k] = stat[(int64_t)v[k] * s.heads + li.h];
                    load_bf16x8(g_b + (int64_t)v[k] * s.ld + li.colc, li.mask, g[k]);
                }
#pragma unroll
                for (int k = 0; k < U; ++k) v[k] = t_indices[min(j + U + k, e - 1)];      // the next chunk, if any
                float da[U];
#pragma unroll
                for (int k = 0; k < U; ++k) da[k] = dot8(g[k], zr);
                head_sum_n<U>(da, s.LH);
#pragma unroll
                for (int k = 0; k < U; ++k) {
                    const float x = elu + st[k].x;
                    const bool pos = x > 0.f;
                    const float a = j + k < e ? expf((pos ? x : s.slope * x) - st[k].y) * st[k].z : 0.f;
                    del += a * (da[k] - st[k].w) * (pos ? 1.f : s.slope);
#pragma unroll
                    for (int i = 0; i < 8; ++i) acc[i] += a * g[k][i];
                }
            }
            float dz[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                dz[i] = acc[i] + del * al[i] + der * ar[i];
                pal[i] += del * zr[i];
                par[i] += der * zr[i];
            }
            if (li.live) store_bf16x8(dz_bf16 + (int64_t)u * s.ld + li.col, dz);
            b = nb;
            e = ne;
            z_raw = nz_raw;
            elu = nelu;
            der_any = nder;
#pragma unroll
            for (int k = 0; k < U; ++k) v0[k] = nv[k];
        }
    }
    block_column_sums<LPR>(pal, li, lds, partial_al, s.ld);
    block_column_sums<LPR>(par, li, lds, partial_ar, s.ld);
}

// ---------------------------------------------------------------------------------------------------------------
// Sums the workgroups' partial column sums (fixed order) and takes the SGD step on a_l, a_r (with weight decay) and
// the bias (without, as for the dense layers' bias).  blockIdx.y = 0: a_l, 1: a_r, 2: bias; 64 columns per workgroup.
// ---------------------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void gat_param_step_kernel(const float *__restrict__ partial_al, const float *__restrict__ partial_ar,
                                                              const float *__restrict__ partial_db, int nb_src, int nb_dst, int ld, int HD,
                                                              float lr, float wd, float *__restrict__ attn, float *__restrict__ d_attn_out)
{
    __shared__ float red[16][64];
    const int which = (int)blockIdx.y;
    const float *p = which == 0 ? partial_al : (which == 1 ? partial_ar : partial_db);
    const int nb = which == 2 ? nb_dst : nb_src;
    const int lane = (int)(threadIdx.x & 63), wave = (int)(threadIdx.x >> 6);
    const int c = (int)blockIdx.x * 64 + lane;
    float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;          // wave w takes rows w, w + 16, ...; four loads in flight
    if (c < ld) {
        const float *q = p + c;
        int r = wave;
        for (; r + 48 < nb; r += 64) {
            s0 += q[(int64_t)r * ld];
            s1 += q[(int64_t)(r + 16) * ld];
            s2 += q[(int64_t)(r + 32) * ld];
            s3 += q[(int64_t)(r + 48) * ld];
        }
        for (; r < nb; r += 16) s0 += q[(int64_t)r * ld];
    }
    red[wave][lane] = (s0 + s1) + (s2 + s3);
    __syncthreads();
    if (wave != 0 || c >= HD) return;
    float g = 0.f;
#pragma unroll
    for (int w = 0; w < 16; ++w) g += red[w][lane];
    if (d_attn_out) d_attn_out[(int64_t)which * ld + c] = g;
    float w = attn[(int64_t)which * ld + c];
    w -= lr * (g + (which == 2 ? 0.f : wd * w));
    attn[(int64_t)which * ld + c] = w;
}

}  // namespace cr

using namespace cr;

namespace {

constexpr int GAT_MAX_BLOCKS = 1024;    // workgroups of the two backward kernels = rows of their partial sums

int lanes_per_row(int ld) { return ld <= 64 ? 8 : (ld <= 128 ? 16 : (ld <= 256 ? 32 : 64)); }

// LDS of the per-edge weights: one slice of fanout x heads x `words` floats per row group of a workgroup
size_t edge_lds_bytes(int lpr, int heads, int fanout, int words) { return (size_t)(256 / lpr) * fanout * heads * words * sizeof(float); }

cr_status gat_shape(const cr_gat_params *p, int64_t ld, int fanout, GatShape &s)
{
    CR_REQUIRE(p != nullptr && p->attn != nullptr && aligned16(p->attn), CR_ERR_INVALID_ARG, "params / params->attn must be a 16-byte aligned device pointer");
    CR_REQUIRE(p->heads >= 1 && p->D >= 1, CR_ERR_INVALID_ARG, "heads = %d, D = %d must be positive", p->heads, p->D);
    CR_REQUIRE(ld >= 64 && ld % 64 == 0 && ld <= 512, CR_ERR_UNSUPPORTED, "row width ld = %lld must be a multiple of 64 in 64..512", (long long)ld);
    CR_REQUIRE((int64_t)p->heads * p->D <= ld, CR_ERR_INVALID_ARG, "heads * D = %lld exceeds ld = %lld", (long long)p->heads * p->D, (long long)ld);
    CR_REQUIRE(p->slope == p->slope && p->slope >= 0.f && p->slope <= 1.f, CR_ERR_INVALID_ARG, "slope must be in [0, 1]");
    const int lpr = lanes_per_row((int)ld);
    int LH = lpr;
    if (p->heads > 1) {
        CR_REQUIRE(p->D % 8 == 0 && ((p->D / 8) & (p->D / 8 - 1)) == 0, CR_ERR_UNSUPPORTED,
                   "with several heads D = %d must be 8 times a power of two", p->D);
        LH = p->D / 8;
    }
    CR_REQUIRE(fanout >= 1 && fanout <= CR_MAX_FANOUT, CR_ERR_INVALID_ARG, "blocks->fanout = %d outside 1..%d", fanout, CR_MAX_FANOUT);
    CR_REQUIRE(edge_lds_bytes(lpr, p->heads, fanout, 2) + 256 * 8 * sizeof(float) <= 65536, CR_ERR_UNSUPPORTED,
               "%d heads, fanout %d on rows of %lld columns need more LDS than a workgroup has", p->heads, fanout, (long long)ld);
    s.heads = p->heads; s.D = p->D; s.LH = LH; s.ld = (int32_t)ld; s.slope = p->slope; s.max_deg = fanout;
    return CR_OK;
}

cr_status check_blocks(const cr_block_set *b, int32_t g, bool transposed)
{
    CR_REQUIRE(b != nullptr, CR_ERR_INVALID_ARG, "blocks is NULL");
    CR_REQUIRE(g >= 0 && g < b->n_batches, CR_ERR_INVALID_ARG, "batch %d outside 0..%d", g, b->n_batches - 1);
    CR_REQUIRE(b->hdr && b->indptr && b->indices, CR_ERR_INVALID_ARG, "blocks has a NULL array");
    CR_REQUIRE(b->cap_dst >= 1 && b->cap_src >= b->cap_dst, CR_ERR_INVALID_ARG, "blocks capacities are not positive");
    CR_REQUIRE(!transposed || (b->t_indptr && b->t_indices), CR_ERR_INVALID_ARG, "the backward pass needs the transposed block");
    return CR_OK;
}

// Workgroups for `rows` rows, one row group each, at most `cap`: the kernels loop over their rows, and on this part a
// few resident workgroups per compute unit that loop beat many short-lived ones (measured: the same kernel takes
// 16 us with 768 workgroups and 59 us with 8192).
int grid_for(int64_t rows, int lpr, int cap)
{
    const int64_t nb = ceil_div(rows, 256 / lpr);
    return (int)(nb < 1 ? 1 : (nb > cap ? cap : nb));
}

struct GatBwdWs {
    uint16_t *g_b;
    float *d_er, *partial_al, *partial_ar, *partial_db;
    size_t bytes;
};

GatBwdWs carve_bwd(void *ws, int cap_dst, int ld, int heads)
{
    Carver c(ws);
    GatBwdWs w;
    w.g_b = c.take<uint16_t>((size_t)cap_dst * ld);
    w.d_er = c.take<float>((size_t)cap_dst * heads);
    w.partial_al = c.take<float>((size_t)GAT_MAX_BLOCKS * ld);
    w.partial_ar = c.take<float>((size_t)GAT_MAX_BLOCKS * ld);
    w.partial_db = c.take<float>((size_t)GAT_MAX_BLOCKS * ld);
    w.bytes = c.bytes();
    return w;
}

}  // namespace

#define GAT_DISPATCH(lpr, KERNEL, grid, lds_bytes, stream, ...)                                                     \
    do {                                                                                                            \
        switch (lpr) {                                                                                              \
        case 8: hipLaunchKernelGGL(KERNEL<8>, dim3(grid), dim3(256), lds_bytes, stream, __VA_ARGS__); break;        \
        case 16: hipLaunchKernelGGL(KERNEL<16>, dim3(grid), dim3(256), lds_bytes, stream, __VA_ARGS__); break;      \
        case 32: hipLaunchKernelGGL(KERNEL<32>, dim3(grid), dim3(256), lds_bytes, stream, __VA_ARGS__); break;      \
        default: hipLaunchKernelGGL(KERNEL<64>, dim3(grid), dim3(256), lds_bytes, stream, __VA_ARGS__); break;      \
        }                                                                                                           \
    } while (0)

extern "C" cr_status cr_gather_rows_bf16(const void *store, int32_t dtype, int64_t ld_src, int32_t F, const int32_t *ids,
                                         const int32_t *hdr, int32_t hdr_word, int32_t max_n, uint16_t *rows_out,
                                         int64_t ld_out, void *stream)
{
    CR_REQUIRE(store && ids && hdr && rows_out, CR_ERR_INVALID_ARG, "store / ids / hdr / rows_out must not be NULL");
    CR_REQUIRE(dtype == CR_F32 || dtype == CR_BF16, CR_ERR_INVALID_ARG, "dtype must be CR_F32 or CR_BF16");
    const int vec = dtype == CR_F32 ? 4 : 8;
    CR_REQUIRE(F >= 1 && ld_src >= round_up(F, vec) && ld_src % vec == 0, CR_ERR_INVALID_ARG,
               "ld_src = %lld must be a multiple of %d and >= F = %d", (long long)ld_src, vec, F);
    CR_REQUIRE(ld_out >= F && ld_out % 8 == 0, CR_ERR_INVALID_ARG, "ld_out = %lld must be a multiple of 8 and >= F", (long long)ld_out);
    CR_REQUIRE(aligned16(store) && aligned16(rows_out), CR_ERR_INVALID_ARG, "store / rows_out must be 16-byte aligned");
    CR_REQUIRE(hdr_word >= 0 && hdr_word < CR_HDR_WORDS && max_n >= 1, CR_ERR_INVALID_ARG, "hdr_word / max_n out of range");
    if (dry_run()) return CR_OK;
    const int64_t chunks = (int64_t)max_n * (ld_out / 8);
    const unsigned grid = (unsigned)(ceil_div(chunks, 256) > 8192 ? 8192 : ceil_div(chunks, 256));
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (dtype == CR_F32)
        hipLaunchKernelGGL(gather_rows_bf16_kernel<float>, dim3(grid), dim3(256), 0, s, static_cast<const float *>(store), ld_src, F, ids,
                           hdr, hdr_word, max_n, rows_out, ld_out);
    else
        hipLaunchKernelGGL(gather_rows_bf16_kernel<uint16_t>, dim3(grid), dim3(256), 0, s, static_cast<const uint16_t *>(store), ld_src, F,
                           ids, hdr, hdr_word, max_n, rows_out, ld_out);
    CR_LAUNCH_CHECK();
    return CR_OK;
}

extern "C" cr_status cr_gat_attention_fwd(const cr_block_set *blocks, int32_t g, const cr_gat_params *params,
                                          const uint16_t *z_bf16, int64_t ld, int32_t relu, float *el, float *er,
                                          float *stat, float *out, uint16_t *out_bf16, void *stream)
{
    cr_status st = check_blocks(blocks, g, false);
    if (st != CR_OK) return st;
    GatShape s;
    st = gat_shape(params, ld, blocks->fanout, s);
    if (st != CR_OK) return st;
    CR_REQUIRE(z_bf16 && el && er && stat, CR_ERR_INVALID_ARG, "z_bf16 / el / er / stat must not be NULL");
    CR_REQUIRE(aligned16(z_bf16) && aligned16(stat) && aligned16(out) && aligned16(out_bf16), CR_ERR_INVALID_ARG,
               "z_bf16 / stat / out / out_bf16 must be 16-byte aligned");
    CR_REQUIRE(out || out_bf16, CR_ERR_INVALID_ARG, "no output requested");
    if (dry_run()) return CR_OK;
    const int lpr = lanes_per_row(s.ld);
    hipStream_t hs = static_cast<hipStream_t>(stream);
    const int32_t *hdr = blocks->hdr + (int64_t)g * CR_HDR_WORDS;
    const int32_t *indptr = blocks->indptr + (int64_t)g * (blocks->cap_dst + 1);
    const int32_t *indices = blocks->indices + (int64_t)g * blocks->cap_nnz;
    GAT_DISPATCH(lpr, gat_scores_kernel, grid_for(ceil_div(blocks->cap_src, 4), lpr, 768), 0, hs, hdr, s, z_bf16, params->attn, el, er);
    GAT_DISPATCH(lpr, gat_aggregate_fwd_kernel, grid_for(blocks->cap_dst, lpr, GAT_MAX_BLOCKS), edge_lds_bytes(lpr, s.heads, s.max_deg, 1), hs, hdr, indptr, indices, s, z_bf16, params->attn, el, er,
                 relu ? 1 : 0, out, out_bf16, reinterpret_cast<float4 *>(stat));
    CR_LAUNCH_CHECK();
    return CR_OK;
}

extern "C" cr_status cr_gat_attention_bwd_workspace_bytes(int32_t cap_dst, int64_t ld, int32_t heads, size_t *bytes)
{
    CR_REQUIRE(cap_dst >= 1 && ld >= 64 && ld <= 512 && heads >= 1 && bytes != nullptr, CR_ERR_INVALID_ARG,
               "cap_dst / ld / heads out of range or bytes NULL");
    *bytes = carve_bwd(nullptr, cap_dst, (int)ld, heads).bytes;
    return CR_OK;
}

extern "C" cr_status cr_gat_attention_bwd(const cr_block_set *blocks, int32_t g, const cr_gat_params *params,
                                          const uint16_t *z_bf16, int64_t ld, const float *el, float *stat,
                                          const uint16_t *d_out_bf16, int64_t ld_dout, const uint16_t *relu_out_bf16,
                                          float lr, float weight_decay, uint16_t *dz_bf16, float *d_attn_out, void *ws,
                                          size_t ws_bytes, void *stream)
{
    cr_status st = check_blocks(blocks, g, true);
    if (st != CR_OK) return st;
    GatShape s;
    st = gat_shape(params, ld, blocks->fanout, s);
    if (st != CR_OK) return st;
    CR_REQUIRE(z_bf16 && el && stat && d_out_bf16 && dz_bf16, CR_ERR_INVALID_ARG, "z_bf16 / el / stat / d_out_bf16 / dz_bf16 must not be NULL");
    CR_REQUIRE(aligned16(z_bf16) && aligned16(stat) && aligned16(d_out_bf16) && aligned16(relu_out_bf16) && aligned16(dz_bf16),
               CR_ERR_INVALID_ARG, "z_bf16 / stat / d_out_bf16 / relu_out_bf16 / dz_bf16 must be 16-byte aligned");
    CR_REQUIRE(ld_dout >= ld && ld_dout % 8 == 0, CR_ERR_INVALID_ARG, "ld_dout = %lld must be a multiple of 8 and >= ld", (long long)ld_dout);
    CR_REQUIRE(lr == lr && weight_decay == weight_decay, CR_ERR_INVALID_ARG, "lr / weight_decay is NaN");
    const GatBwdWs w = carve_bwd(ws, blocks->cap_dst, s.ld, s.heads);
    CR_REQUIRE(ws != nullptr && aligned16(ws), CR_ERR_INVALID_ARG, "workspace must be a 16-byte aligned device pointer");
    CR_REQUIRE(ws_bytes >= w.bytes, CR_ERR_CAPACITY, "workspace of %zu bytes, %zu needed", ws_bytes, w.bytes);
    if (dry_run()) return CR_OK;
    const int lpr = lanes_per_row(s.ld);
    hipStream_t hs = static_cast<hipStream_t>(stream);
    const int32_t *hdr = blocks->hdr + (int64_t)g * CR_HDR_WORDS;
    const int32_t *indptr = blocks->indptr + (int64_t)g * (blocks->cap_dst + 1);
    const int32_t *indices = blocks->indices + (int64_t)g * blocks->cap_nnz;
    const int32_t *t_indptr = blocks->t_indptr + (int64_t)g * (blocks->cap_src + 1);
    const int32_t *t_indices = blocks->t_indices + (int64_t)g * blocks->cap_nnz;
    const int nb_dst = grid_for(blocks->cap_dst, lpr, GAT_MAX_BLOCKS), nb_src = grid_for(blocks->cap_src, lpr, GAT_MAX_BLOCKS);
    GAT_DISPATCH(lpr, gat_bwd_dst_kernel, nb_dst, edge_lds_bytes(lpr, s.heads, s.max_deg, 2) + 256 * 8 * sizeof(float), hs, hdr, indptr, indices, s, z_bf16, el, d_out_bf16, ld_dout, relu_out_bf16,
                 reinterpret_cast<float4 *>(stat), w.g_b, w.d_er, w.partial_db);
    GAT_DISPATCH(lpr, gat_bwd_src_kernel, nb_src, 0, hs, hdr, t_indptr, t_indices, s, z_bf16, params->attn, el,
                 reinterpret_cast<const float4 *>(stat), w.g_b, w.d_er, dz_bf16, w.partial_al, w.partial_ar);
    hipLaunchKernelGGL(gat_param_step_kernel, dim3((unsigned)(s.ld / 64), 3), dim3(1024), 0, hs, w.partial_al, w.partial_ar, w.partial_db,
                       nb_src, nb_dst, s.ld, s.heads * s.D, lr, weight_decay, params->attn, d_attn_out);
    CR_LAUNCH_CHECK();
    return CR_OK;
}
