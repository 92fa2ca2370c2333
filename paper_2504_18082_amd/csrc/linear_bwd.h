// Shared between the dense kernels (linear.hip) and the fused backward launch of a whole layer (gather.hip):
// the reduction + SGD step of a layer's weight gradient as a device function, and the host routine that launches a
// layer's two backward products.
#pragma once

#include "cr_common.h"

namespace cr {

// Rows of one split of the weight-gradient product, from the block's actual row count (read on the
// device) and the number of partial slots the workspace holds: at most `slots` splits, at least 96 rows each.
__host__ __device__ __forceinline__ int rows_per_split_for(int M, int slots)
{
    int rows = ((M + slots - 1) / slots + 95) / 96 * 96;
    return rows < 96 ? 96 : rows;
}

// sums the partial products of the active splits in a fixed order, applies the SGD step to the float
// master and refreshes both bf16 shadows
struct SgdArgs {
    const int32_t *hdr;
    int32_t max_rows, n_splits;
    const float *partial;
    int32_t F_in, F_out, F_pad, N_pad, n_op;
    float *W, *bias;
    uint16_t *W_bf16, *Wt_bf16;
    float lr, wd;
    float *dW_out, *db_out;
};

// A workgroup owns 64 quadruples of consecutive n (256 outputs).  Its four waves each sum every fourth
// split, eight loads in flight per lane; the four sums meet in LDS and wave 0 finishes in a fixed order.
__device__ __forceinline__ void sgd_reduce_body(const SgdArgs &a, uint32_t bid, float4 (&red)[4][64])
{
    const int M = min(a.hdr[CR_HDR_N_DST], a.max_rows);
    const int rows_per_split = rows_per_split_for(M, a.n_splits);
    const int active = min(a.n_splits, (M + rows_per_split - 1) / rows_per_split);
    const int K2 = a.n_op * a.F_pad;
    const int nq = a.N_pad / 4;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t q = (int64_t)bid * 64 + lane;                   // quadruple index over (K2 + 1) rows of nq quadruples
    const bool in_range = q < (int64_t)(K2 + 1) * nq;
    const int k2 = in_range ? (int)(q / nq) : 0, n = in_range ? (int)(q % nq) * 4 : 0;
    const bool is_bias = k2 == K2;
    const int kin = k2 % a.F_pad, part = k2 / a.F_pad;
    const bool live = in_range && n < a.F_out && (is_bias || kin < a.F_in);

    // the master weights this lane will update are requested now (one 16-byte load when the rows allow it), so that
    // they arrive while the partial sums are added up
    const int64_t wi = (int64_t)(part * a.F_in + kin) * a.F_out + n;
    const bool w_vec = (a.F_out & 3) == 0;
    float4 wq = make_float4(0.f, 0.f, 0.f, 0.f);
    if (w_vec) wq = *reinterpret_cast<const float4 *>(a.W + ((live && !is_bias) ? wi : 0));      // (uniform condition)

    float4 g = make_float4(0.f, 0.f, 0.f, 0.f);
    if (live) {
        const float *pp = a.partial + (int64_t)k2 * a.N_pad + n;
        const int64_t ps = (int64_t)(K2 + 1) * a.N_pad;
        const int last = active > 0 ? active - 1 : 0;
        for (int s = wave; s < active; s += 32) {                 // this wave's splits: wave, wave+4, wave+8, ...
            float4 x[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) x[i] = *reinterpret_cast<const float4 *>(pp + (int64_t)min(s + 4 * i, last) * ps);
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const float keep = s + 4 * i < active ? 1.f : 0.f;
                g.x += keep * x[i].x; g.y += keep * x[i].y; g.z += keep * x[i].z; g.w += keep * x[i].w;
            }
        }
    }
    red[wave][lane] = g;
    __syncthreads();
    if (wave != 0 || !live) return;
    const float4 r0 = red[0][lane], r1 = red[1][lane], r2 = red[2][lane], r3 = red[3][lane];
    const float gs[4] = {(r0.x + r1.x) + (r2.x + r3.x), (r0.y + r1.y) + (r2.y + r3.y),
                         (r0.z + r1.z) + (r2.z + r3.z), (r0.w + r1.w) + (r2.w + r3.w)};
    if (is_bias) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (n + i < a.F_out) {
                if (a.db_out) a.db_out[n + i] = gs[i];
                if (a.bias) a.bias[n + i] -= a.lr * gs[i];
            }
        }
        return;
    }
    const float wv[4] = {wq.x, wq.y, wq.z, wq.w};
    uint16_t wb[4] = {0, 0, 0, 0};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (n + i < a.F_out) {
            float w = w_vec ? wv[i] : a.W[wi + i];
            if (a.dW_out) a.dW_out[wi + i] = gs[i];
            w -= a.lr * (gs[i] + a.wd * w);
            a.W[wi + i] = w;
            wb[i] = f32_to_bf16(w);
            a.Wt_bf16[(int64_t)(n + i) * K2 + k2] = wb[i];
        }
    }
    *reinterpret_cast<uint2 *>(a.W_bf16 + (int64_t)k2 * a.N_pad + n) =
        make_uint2((uint32_t)wb[0] | ((uint32_t)wb[1] << 16), (uint32_t)wb[2] | ((uint32_t)wb[3] << 16));
}

// number of workgroups sgd_reduce_body needs
inline unsigned sgd_reduce_blocks(int F_pad, int N_pad, int n_op)
{
    return (unsigned)ceil_div(((int64_t)n_op * F_pad + 1) * (N_pad / 4), 64);
}

// Validates the arguments of cr_sage_linear_bwd and launches the layer's weight-gradient and input-gradient products.
// With `deferred` == NULL the reduction + SGD step is launched too; otherwise its arguments are returned in
// *deferred for the caller to launch (alone or inside a fused kernel) on the same stream.
cr_status linear_bwd_products(const cr_sage_layer *layer, const int32_t *hdr, int32_t max_rows, const uint16_t *h_self,
                              const uint16_t *agg, int64_t ld_in, const uint16_t *dz_bf16, float lr, float weight_decay,
                              float *d_self, float *d_agg, uint16_t *d_in_bf16, float *dW_out, float *db_out, void *ws,
                              size_t ws_bytes, void *stream, SgdArgs *deferred);

}  // namespace cr
