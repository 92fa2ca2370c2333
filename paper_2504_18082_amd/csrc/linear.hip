// Dense part of a GraphSAGE-mean layer (Eq. 1 of the paper in its GraphSAGE form):
//   Z = H_self W_self + Agg W_neigh + b  (ReLU on hidden layers), its backward, a fused SGD step,
// and the softmax cross-entropy on the root rows.  The contractions run on the bf16 matrix cores
// (v_mfma_f32_32x32x16_bf16) with float accumulation; operands are staged through LDS.
#include "cr_common.h"

namespace cr {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int LDS_ROW = 40;   // 32 bf16 of payload + 8 of padding per staged row (80 bytes)

__device__ __forceinline__ bf16x8 lds_read8(const uint16_t *p)
{
    return *reinterpret_cast<const bf16x8 *>(p);
}

// ------------------------------------------------------------------------------------------------
// C[m][n] = sum_k A[m][k] * B[n][k]     (both operands contiguous along k)
//   A = [A0 | A1]: columns < K0 come from A0, the rest from A1 (same row stride)
//   C = [C0 | C1]: columns < N0 go to C0, the rest to C1 (same row stride)
// Workgroup tile 128 (m) x 64 (n), four waves of 32 x 64; the weights are the first MFMA operand so
// that a lane ends up with four consecutive n of one row m (vector stores along the row).
// ------------------------------------------------------------------------------------------------
struct NtArgs {
    const int32_t *hdr;
    int32_t max_rows;
    const uint16_t *A0, *A1;
    int64_t lda;
    int32_t K0, K;
    const uint16_t *B;       // [N][K]
    int32_t N;
    const float *bias;       // [N] or NULL
    int32_t relu;
    float *C0, *C1;
    int64_t ldc;
    int32_t N0;
    uint16_t *Cb;            // bf16 copy of C (single destination) or NULL
    int64_t ldcb;
};

__global__ __launch_bounds__(256) void gemm_nt_kernel(NtArgs a)
{
    __shared__ __attribute__((aligned(16))) uint16_t As[2][128][LDS_ROW];
    __shared__ __attribute__((aligned(16))) uint16_t Bs[2][64][LDS_ROW];
    const int M = min(a.hdr[CR_HDR_N_DST], a.max_rows);
    const int m0 = blockIdx.y * 128, n0 = blockIdx.x * 64;
    if (m0 >= M) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    // staging assignment: A 128 rows x 4 chunks of 8, two per thread; B 64 rows x 4 chunks, one per thread
    const int a_row0 = tid >> 2, a_row1 = (tid + 256) >> 2, kc = tid & 3;
    const int64_t ga0 = (int64_t)min(m0 + a_row0, M - 1) * a.lda;
    const int64_t ga1 = (int64_t)min(m0 + a_row1, M - 1) * a.lda;
    const uint16_t *gb = a.B + (int64_t)(n0 + (tid >> 2)) * a.K + kc * 8;

    uint4 ra0, ra1, rb;
    auto load_step = [&](int k0) {
        const uint16_t *src = k0 < a.K0 ? a.A0 + k0 : a.A1 + (k0 - a.K0);
        ra0 = *reinterpret_cast<const uint4 *>(src + ga0 + kc * 8);
        ra1 = *reinterpret_cast<const uint4 *>(src + ga1 + kc * 8);
        rb = *reinterpret_cast<const uint4 *>(gb + k0);
    };
    auto store_step = [&](int buf) {
        *reinterpret_cast<uint4 *>(&As[buf][a_row0][kc * 8]) = ra0;
        *reinterpret_cast<uint4 *>(&As[buf][a_row1][kc * 8]) = ra1;
        *reinterpret_cast<uint4 *>(&Bs[buf][tid >> 2][kc * 8]) = rb;
    };

    f32x16 acc[2];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;

    const int nsteps = a.K / 32;
    load_step(0);
    store_step(0);
    __syncthreads();
    for (int step = 0; step < nsteps; ++step) {
        const int buf = step & 1;
        if (step + 1 < nsteps) load_step((step + 1) * 32);
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            const int ko = kk * 16 + 8 * (lane >> 5);
            const bf16x8 act = lds_read8(&As[buf][wave * 32 + (lane & 31)][ko]);
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const bf16x8 wgt = lds_read8(&Bs[buf][t * 32 + (lane & 31)][ko]);
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wgt, act, acc[t], 0, 0, 0);
            }
        }
        if (step + 1 < nsteps) store_step(buf ^ 1);
        __syncthreads();
    }

    const int m = m0 + wave * 32 + (lane & 31);
    if (m >= M) return;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int grp = 0; grp < 4; ++grp) {
            const int n = n0 + t * 32 + 8 * grp + 4 * (lane >> 5);
            float v[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                v[i] = acc[t][grp * 4 + i] + (a.bias ? a.bias[n + i] : 0.f);
                if (a.relu && v[i] < 0.f) v[i] = 0.f;
            }
            if (a.C0) {
                float *dst = n < a.N0 ? a.C0 + (int64_t)m * a.ldc + n : a.C1 + (int64_t)m * a.ldc + (n - a.N0);
                *reinterpret_cast<float4 *>(dst) = make_float4(v[0], v[1], v[2], v[3]);
            }
            if (a.Cb) {
                const uint32_t lo = (uint32_t)f32_to_bf16(v[0]) | ((uint32_t)f32_to_bf16(v[1]) << 16);
                const uint32_t hi = (uint32_t)f32_to_bf16(v[2]) | ((uint32_t)f32_to_bf16(v[3]) << 16);
                *reinterpret_cast<uint2 *>(a.Cb + (int64_t)m * a.ldcb + n) = make_uint2(lo, hi);
            }
        }
}

// ------------------------------------------------------------------------------------------------
// P[s][k][n] = sum_{m in split s} A[m][k] * Z[m][n]      (both operands strided along m: the tiles are
// transposed on their way into LDS).  Also the column sums of Z per split (bias gradient).
// Workgroup tile 64 (k) x 64 (n), four waves of 32 x 32; 32 rows of m per step.
// ------------------------------------------------------------------------------------------------
struct TnArgs {
    const int32_t *hdr;
    int32_t max_rows;
    const uint16_t *A0, *A1;
    int64_t lda;
    int32_t K0, K2;
    const uint16_t *Z;       // [M][N]
    int32_t N;
    int32_t rows_per_split;
    float *partial;          // [S][K2][N]
    float *db_partial;       // [S][N]
};

__global__ __launch_bounds__(256) void gemm_tn_kernel(TnArgs a)
{
    __shared__ __attribute__((aligned(16))) uint16_t At[64][LDS_ROW];
    __shared__ __attribute__((aligned(16))) uint16_t Zt[64][LDS_ROW];
    const int M = min(a.hdr[CR_HDR_N_DST], a.max_rows);
    const int split = blockIdx.y;
    const int m_begin = split * a.rows_per_split;
    if (m_begin >= M) return;                      // inactive split: the reduction skips it too
    const int m_end = min(M, m_begin + a.rows_per_split);
    const int n_tiles = a.N / 64;
    const int k0 = (blockIdx.x / n_tiles) * 64, n0 = (blockIdx.x % n_tiles) * 64;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wk = wave >> 1, wn = wave & 1;

    // staging: 32 rows of m x 8 chunks of 8 columns, one chunk of each operand per thread
    const int sm = tid >> 3, sc = (tid & 7) * 8;
    const int kcol = k0 + sc;
    const uint16_t *srcA = kcol < a.K0 ? a.A0 + kcol : a.A1 + (kcol - a.K0);
    const uint16_t *srcZ = a.Z + n0 + sc;

    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    float colsum = 0.f;

    for (int mb = m_begin; mb < m_end; mb += 32) {
        const int gm = mb + sm;
        uint4 ra = make_uint4(0, 0, 0, 0), rz = make_uint4(0, 0, 0, 0);
        if (gm < m_end) {
            ra = *reinterpret_cast<const uint4 *>(srcA + (int64_t)gm * a.lda);
            rz = *reinterpret_cast<const uint4 *>(srcZ + (int64_t)gm * a.N);
        }
        __syncthreads();                           // previous step's reads are done
        const uint32_t wa[4] = {ra.x, ra.y, ra.z, ra.w}, wz[4] = {rz.x, rz.y, rz.z, rz.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            At[sc + 2 * i][sm] = (uint16_t)(wa[i] & 0xFFFFu);
            At[sc + 2 * i + 1][sm] = (uint16_t)(wa[i] >> 16);
            Zt[sc + 2 * i][sm] = (uint16_t)(wz[i] & 0xFFFFu);
            Zt[sc + 2 * i + 1][sm] = (uint16_t)(wz[i] >> 16);
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            const int mo = kk * 16 + 8 * (lane >> 5);
            const bf16x8 x = lds_read8(&At[wk * 32 + (lane & 31)][mo]);
            const bf16x8 z = lds_read8(&Zt[wn * 32 + (lane & 31)][mo]);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, z, acc, 0, 0, 0);
        }
        if (k0 == 0 && tid < 64) {
#pragma unroll 8
            for (int i = 0; i < 32; ++i) colsum += bf16_to_f32(Zt[tid][i]);
        }
    }

    float *P = a.partial + (int64_t)split * a.K2 * a.N;
    const int n = n0 + wn * 32 + (lane & 31);
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int k = k0 + wk * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        P[(int64_t)k * a.N + n] = acc[r];
    }
    if (k0 == 0 && tid < 64) a.db_partial[(int64_t)split * a.N + n0 + tid] = colsum;
}

// sums the partial products of the active splits in a fixed order, applies the SGD step to the float
// master and refreshes both bf16 shadows
struct SgdArgs {
    const int32_t *hdr;
    int32_t max_rows, rows_per_split, n_splits;
    const float *partial, *db_partial;
    int32_t F_in, F_out, F_pad, N_pad;
    float *W, *bias;
    uint16_t *W_bf16, *Wt_bf16;
    float lr, wd;
    float *dW_out, *db_out;
};

__global__ __launch_bounds__(256) void sgd_reduce_kernel(SgdArgs a)
{
    const int M = min(a.hdr[CR_HDR_N_DST], a.max_rows);
    const int active = min(a.n_splits, (M + a.rows_per_split - 1) / a.rows_per_split);
    const int K2 = 2 * a.F_pad;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)K2 * a.N_pad) return;
    const int k2 = (int)(idx / a.N_pad), n = (int)(idx % a.N_pad);
    const int kin = k2 % a.F_pad, part = k2 / a.F_pad;
    if (kin < a.F_in && n < a.F_out) {
        float g4[4] = {0.f, 0.f, 0.f, 0.f};     // fixed association: split s goes to accumulator s % 4
        const float *pp = a.partial + (int64_t)k2 * a.N_pad + n;
        const int64_t ps = (int64_t)K2 * a.N_pad;
        for (int s = 0; s < active; s += 4) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (s + i < active) g4[i] += pp[(int64_t)(s + i) * ps];
        }
        const float g = (g4[0] + g4[1]) + (g4[2] + g4[3]);
        const int64_t wi = (int64_t)(part * a.F_in + kin) * a.F_out + n;
        float w = a.W[wi];
        if (a.dW_out) a.dW_out[wi] = g;
        w -= a.lr * (g + a.wd * w);
        a.W[wi] = w;
        const uint16_t wb = f32_to_bf16(w);
        a.W_bf16[(int64_t)k2 * a.N_pad + n] = wb;
        a.Wt_bf16[(int64_t)n * K2 + k2] = wb;
    }
    if (k2 == 0 && n < a.F_out) {
        float g = 0.f;
        for (int s = 0; s < active; ++s) g += a.db_partial[(int64_t)s * a.N_pad + n];
        if (a.db_out) a.db_out[n] = g;
        a.bias[n] -= a.lr * g;
    }
}

__global__ __launch_bounds__(256) void refresh_shadows_kernel(const float *W, int F_in, int F_out, int F_pad, int N_pad,
                                                              uint16_t *W_bf16, uint16_t *Wt_bf16)
{
    const int K2 = 2 * F_pad;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)K2 * N_pad) return;
    const int k2 = (int)(idx / N_pad), n = (int)(idx % N_pad);
    const int kin = k2 % F_pad, part = k2 / F_pad;
    uint16_t wb = 0;
    if (kin < F_in && n < F_out) wb = f32_to_bf16(W[(int64_t)(part * F_in + kin) * F_out + n]);
    W_bf16[(int64_t)k2 * N_pad + n] = wb;
    Wt_bf16[(int64_t)n * K2 + k2] = wb;
}

// ------------------------------------------------------------------------------------------------
// softmax cross-entropy on the root rows: one wave per row
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void xent_rows_kernel(const int32_t *hdr, int max_rows, const float *logits, int64_t ld,
                                                        int C, const int32_t *labels, const int32_t *root_ids,
                                                        float *row_loss, float *d_logits, uint16_t *d_logits_bf16)
{
    const int n = min(hdr[CR_HDR_N_DST], max_rows);
    const int row = blockIdx.x * 4 + threadIdx.x / WAVE;
    if (row >= n) return;
    const int lane = lane_id();
    const float *z = logits + (int64_t)row * ld;
    float mx = -INFINITY;
    for (int c = lane; c < C; c += WAVE) mx = fmaxf(mx, z[c]);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
    float den = 0.f;
    for (int c = lane; c < C; c += WAVE) den += expf(z[c] - mx);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) den += __shfl_xor(den, off);
    const int label = labels[root_ids[row]];
    if (lane == 0) row_loss[row] = -(z[label] - mx - logf(den));
    const float inv_n = 1.0f / (float)n;
    for (int c = lane; c < ld; c += WAVE) {
        float d = 0.f;
        if (c < C) d = (expf(z[c] - mx) / den - (c == label ? 1.f : 0.f)) * inv_n;
        if (d_logits) d_logits[(int64_t)row * ld + c] = d;
        if (d_logits_bf16) d_logits_bf16[(int64_t)row * ld + c] = f32_to_bf16(d);
    }
}

__global__ __launch_bounds__(1024) void xent_mean_kernel(const int32_t *hdr, int max_rows, const float *row_loss, float *loss)
{
    __shared__ float part[16];
    const int n = min(hdr[CR_HDR_N_DST], max_rows);
    float s = 0.f;
    for (int i = threadIdx.x; i < n; i += 1024) s += row_loss[i];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off);
    if (lane_id() == 0) part[threadIdx.x / WAVE] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        float t = 0.f;
        for (int w = 0; w < 16; ++w) t += part[w];
        loss[0] = n > 0 ? t / (float)n : 0.f;
    }
}

static void split_plan(int F_pad, int N_pad, int max_rows, int &rows_per_split, int &n_splits)
{
    const int tiles = (2 * F_pad / 64) * (N_pad / 64);
    int target = 1024 / tiles;
    if (target < 1) target = 1;
    if (target > 128) target = 128;
    int rows = (int)round_up(ceil_div(max_rows, target), 32);
    if (rows < 64) rows = 64;
    rows_per_split = rows;
    n_splits = (int)ceil_div(max_rows, rows);
}

}  // namespace cr

using namespace cr;

static cr_status check_layer(const cr_sage_layer *L, int &F_pad, int &N_pad)
{
    CR_REQUIRE(L != nullptr, CR_ERR_INVALID_ARG, "layer is NULL");
    CR_REQUIRE(L->F_in >= 1 && L->F_in <= 8192 && L->F_out >= 1 && L->F_out <= 8192, CR_ERR_INVALID_ARG,
               "layer dims (%d, %d) outside 1..8192", L->F_in, L->F_out);
    CR_REQUIRE(L->W && L->bias && L->W_bf16 && L->Wt_bf16, CR_ERR_INVALID_ARG, "layer has a NULL array");
    CR_REQUIRE(aligned16(L->W) && aligned16(L->bias) && aligned16(L->W_bf16) && aligned16(L->Wt_bf16), CR_ERR_INVALID_ARG,
               "layer arrays must be 16-byte aligned");
    F_pad = (int)round_up(L->F_in, 32);
    N_pad = (int)round_up(L->F_out, 64);
    return CR_OK;
}

extern "C" cr_status cr_sage_padded_dims(int32_t F_in, int32_t F_out, int32_t *F_pad, int32_t *N_pad)
{
    CR_REQUIRE(F_in >= 1 && F_in <= 8192 && F_out >= 1 && F_out <= 8192, CR_ERR_INVALID_ARG, "layer dims (%d, %d) outside 1..8192", F_in, F_out);
    CR_REQUIRE(F_pad && N_pad, CR_ERR_INVALID_ARG, "outputs must not be NULL");
    *F_pad = (int32_t)round_up(F_in, 32);
    *N_pad = (int32_t)round_up(F_out, 64);
    return CR_OK;
}

extern "C" cr_status cr_sage_refresh_shadows(const cr_sage_layer *layer, void *stream)
{
    int F_pad, N_pad;
    cr_status st = check_layer(layer, F_pad, N_pad);
    if (st != CR_OK) return st;
    if (dry_run()) return CR_OK;
    const int64_t n = 2ll * F_pad * N_pad;
    hipLaunchKernelGGL(refresh_shadows_kernel, dim3((unsigned)ceil_div(n, 256)), dim3(256), 0, static_cast<hipStream_t>(stream),
                       layer->W, layer->F_in, layer->F_out, F_pad, N_pad, layer->W_bf16, layer->Wt_bf16);
    CR_LAUNCH_CHECK();
    return CR_OK;
}

extern "C" cr_status cr_sage_linear_fwd(const cr_sage_layer *layer, const int32_t *hdr, int32_t max_rows,
                                        const uint16_t *h_self, const uint16_t *agg, int64_t ld_in, int relu,
                                        float *out, uint16_t *out_bf16, void *stream)
{
    int F_pad, N_pad;
    cr_status st = check_layer(layer, F_pad, N_pad);
    if (st != CR_OK) return st;
    CR_REQUIRE(hdr != nullptr && max_rows >= 1, CR_ERR_INVALID_ARG, "hdr must not be NULL and max_rows must be positive");
    CR_REQUIRE(h_self && agg && aligned16(h_self) && aligned16(agg), CR_ERR_INVALID_ARG, "h_self / agg must be 16-byte aligned device pointers");
    CR_REQUIRE(ld_in >= F_pad && ld_in % 8 == 0, CR_ERR_INVALID_ARG, "ld_in = %lld must be a multiple of 8 and >= %d", (long long)ld_in, F_pad);
    CR_REQUIRE(out || out_bf16, CR_ERR_INVALID_ARG, "no output requested");
    CR_REQUIRE(aligned16(out) && aligned16(out_bf16), CR_ERR_INVALID_ARG, "outputs must be 16-byte aligned");
    if (dry_run()) return CR_OK;
    NtArgs a;
    a.hdr = hdr; a.max_rows = max_rows; a.A0 = h_self; a.A1 = agg; a.lda = ld_in; a.K0 = F_pad; a.K = 2 * F_pad;
    a.B = layer->Wt_bf16; a.N = N_pad; a.bias = layer->bias; a.relu = relu ? 1 : 0;
    a.C0 = out; a.C1 = nullptr; a.ldc = N_pad; a.N0 = N_pad; a.Cb = out_bf16; a.ldcb = N_pad;
    hipLaunchKernelGGL(gemm_nt_kernel, dim3(N_pad / 64, (unsigned)ceil_div(max_rows, 128)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), a);
    CR_LAUNCH_CHECK();
    return CR_OK;
}

extern "C" cr_status cr_sage_linear_bwd_workspace_bytes(int32_t F_in, int32_t F_out, int32_t max_rows, size_t *bytes)
{
    CR_REQUIRE(F_in >= 1 && F_in <= 8192 && F_out >= 1 && F_out <= 8192, CR_ERR_INVALID_ARG, "layer dims (%d, %d) outside 1..8192", F_in, F_out);
    CR_REQUIRE(max_rows >= 1 && bytes != nullptr, CR_ERR_INVALID_ARG, "max_rows must be positive and bytes not NULL");
    const int F_pad = (int)round_up(F_in, 32), N_pad = (int)round_up(F_out, 64);
    int rows, splits;
    split_plan(F_pad, N_pad, max_rows, rows, splits);
    Carver c(nullptr);
    c.take<float>((size_t)splits * 2 * F_pad * N_pad);
    c.take<float>((size_t)splits * N_pad);
    *bytes = c.bytes();
    return CR_OK;
}

extern "C" cr_status cr_sage_linear_bwd(const cr_sage_layer *layer, const int32_t *hdr, int32_t max_rows,
                                        const uint16_t *h_self, const uint16_t *agg, int64_t ld_in,
                                        const uint16_t *dz_bf16, float lr, float weight_decay, float *d_self,
                                        float *d_agg, float *dW_out, float *db_out, void *ws, size_t ws_bytes,
                                        void *stream)
{
    int F_pad, N_pad;
    cr_status st = check_layer(layer, F_pad, N_pad);
    if (st != CR_OK) return st;
    CR_REQUIRE(hdr != nullptr && max_rows >= 1, CR_ERR_INVALID_ARG, "hdr must not be NULL and max_rows must be positive");
    CR_REQUIRE(h_self && agg && dz_bf16 && aligned16(h_self) && aligned16(agg) && aligned16(dz_bf16), CR_ERR_INVALID_ARG,
               "h_self / agg / dz_bf16 must be 16-byte aligned device pointers");
    CR_REQUIRE(ld_in >= F_pad && ld_in % 8 == 0, CR_ERR_INVALID_ARG, "ld_in = %lld must be a multiple of 8 and >= %d", (long long)ld_in, F_pad);
    CR_REQUIRE((d_self == nullptr) == (d_agg == nullptr), CR_ERR_INVALID_ARG, "d_self and d_agg must be given together");
    CR_REQUIRE(aligned16(d_self) && aligned16(d_agg), CR_ERR_INVALID_ARG, "d_self / d_agg must be 16-byte aligned");
    CR_REQUIRE(lr == lr && weight_decay == weight_decay, CR_ERR_INVALID_ARG, "lr / weight_decay is NaN");
    int rows, splits;
    split_plan(F_pad, N_pad, max_rows, rows, splits);
    Carver c(ws);
    float *partial = c.take<float>((size_t)splits * 2 * F_pad * N_pad);
    float *db_partial = c.take<float>((size_t)splits * N_pad);
    CR_REQUIRE(ws != nullptr && aligned16(ws), CR_ERR_INVALID_ARG, "workspace must be a 16-byte aligned device pointer");
    CR_REQUIRE(ws_bytes >= c.bytes(), CR_ERR_CAPACITY, "workspace of %zu bytes, %zu needed", ws_bytes, c.bytes());
    if (dry_run()) return CR_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);

    if (d_self) {   // gradient w.r.t. the layer's inputs, with the weights from before the step
        NtArgs a;
        a.hdr = hdr; a.max_rows = max_rows; a.A0 = dz_bf16; a.A1 = nullptr; a.lda = N_pad; a.K0 = N_pad; a.K = N_pad;
        a.B = layer->W_bf16; a.N = 2 * F_pad; a.bias = nullptr; a.relu = 0;
        a.C0 = d_self; a.C1 = d_agg; a.ldc = F_pad; a.N0 = F_pad; a.Cb = nullptr; a.ldcb = 0;
        hipLaunchKernelGGL(gemm_nt_kernel, dim3(2 * F_pad / 64, (unsigned)ceil_div(max_rows, 128)), dim3(256), 0, s, a);
    }
    TnArgs t;
    t.hdr = hdr; t.max_rows = max_rows; t.A0 = h_self; t.A1 = agg; t.lda = ld_in; t.K0 = F_pad; t.K2 = 2 * F_pad;
    t.Z = dz_bf16; t.N = N_pad; t.rows_per_split = rows; t.partial = partial; t.db_partial = db_partial;
    hipLaunchKernelGGL(gemm_tn_kernel, dim3((2 * F_pad / 64) * (N_pad / 64), splits), dim3(256), 0, s, t);
    SgdArgs g;
    g.hdr = hdr; g.max_rows = max_rows; g.rows_per_split = rows; g.n_splits = splits; g.partial = partial; g.db_partial = db_partial;
    g.F_in = layer->F_in; g.F_out = layer->F_out; g.F_pad = F_pad; g.N_pad = N_pad; g.W = layer->W; g.bias = layer->bias;
    g.W_bf16 = layer->W_bf16; g.Wt_bf16 = layer->Wt_bf16; g.lr = lr; g.wd = weight_decay; g.dW_out = dW_out; g.db_out = db_out;
    hipLaunchKernelGGL(sgd_reduce_kernel, dim3((unsigned)ceil_div(2ll * F_pad * N_pad, 256)), dim3(256), 0, s, g);
    CR_LAUNCH_CHECK();
    return CR_OK;
}

extern "C" cr_status cr_softmax_xent(const int32_t *hdr, int32_t max_rows, const float *logits, int64_t ld,
                                     int32_t n_classes, const int32_t *labels, const int32_t *root_ids, float *loss,
                                     float *row_loss, float *d_logits, uint16_t *d_logits_bf16, void *stream)
{
    CR_REQUIRE(hdr != nullptr && max_rows >= 1, CR_ERR_INVALID_ARG, "hdr must not be NULL and max_rows must be positive");
    CR_REQUIRE(logits && labels && root_ids && loss && row_loss, CR_ERR_INVALID_ARG, "logits / labels / root_ids / loss / row_loss must not be NULL");
    CR_REQUIRE(n_classes >= 1 && ld >= n_classes, CR_ERR_INVALID_ARG, "need 1 <= n_classes <= ld");
    if (dry_run()) return CR_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(xent_rows_kernel, dim3((unsigned)ceil_div(max_rows, 4)), dim3(256), 0, s, hdr, max_rows, logits, ld, n_classes,
                       labels, root_ids, row_loss, d_logits, d_logits_bf16);
    hipLaunchKernelGGL(xent_mean_kernel, dim3(1), dim3(1024), 0, s, hdr, max_rows, row_loss, loss);
    CR_LAUNCH_CHECK();
    return CR_OK;
}
