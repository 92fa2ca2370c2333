// Dense part of a GraphSAGE-mean layer (Eq. 1 of the paper in its GraphSAGE form):
//   Z = H_self W_self + Agg W_neigh + b  (ReLU on hidden layers), its backward, a fused SGD step,
// and the softmax cross-entropy on the root rows.  The contractions run on the bf16 matrix cores
// (v_mfma_f32_32x32x16_bf16) with float accumulation; operands are staged through LDS.
#include <type_traits>

#include "cr_common.h"
#include "linear_bwd.h"

namespace cr {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4v __attribute__((ext_vector_type(4)));
typedef short v4s16 __attribute__((ext_vector_type(4)));

constexpr int TN_BM = 32;     // rows of the operands staged per step of the TN product (a multiple of 16; 96-row splits hold two)
constexpr int TN_ROW = 144;   // staged row of the TN product: 128 columns + 16 of padding (288 bytes)

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

struct NtState {
    const uint16_t *A0, *A1;
    int K0, K;
    int64_t ga0, ga1;
    const uint16_t *gb;       // B row (n0 + tid/4), chunk column kc*8
    int kc, a_row0, a_row1, b_row, act_row, lr, half;
};

// the pieces one thread fetches for one 32-wide K step: two of A, NB of B (rows b_row + 64*i)
template <int NB>
struct NtFetch {
    u32x4v a0, a1, b0, b1, b2, b3;
};

template <int NB>
__device__ __forceinline__ NtFetch<NB> nt_fetch(const NtState &st, int step)
{
    NtFetch<NB> f;
    const int k0 = step * 32;
    const uint16_t *src = k0 < st.K0 ? st.A0 + k0 : st.A1 + (k0 - st.K0);
    f.a0 = *reinterpret_cast<const u32x4v *>(src + st.ga0 + st.kc * 8);
    f.a1 = *reinterpret_cast<const u32x4v *>(src + st.ga1 + st.kc * 8);
    const uint16_t *b = st.gb + k0;
    f.b0 = *reinterpret_cast<const u32x4v *>(b);
    f.b1 = f.b2 = f.b3 = f.b0;
    if constexpr (NB > 1) f.b1 = *reinterpret_cast<const u32x4v *>(b + (int64_t)64 * st.K);
    if constexpr (NB > 2) {
        f.b2 = *reinterpret_cast<const u32x4v *>(b + (int64_t)128 * st.K);
        f.b3 = *reinterpret_cast<const u32x4v *>(b + (int64_t)192 * st.K);
    }
    return f;
}

// one K step: stage the fetched pieces, barrier, MFMA (wave tile 32 m x NTILES*32 n)
template <int NTILES>
__device__ __forceinline__ void nt_step(const NtState &st, const NtFetch<NTILES / 2> &f, int &buf,
                                        uint16_t (&As)[2][128][LDS_ROW], uint16_t (&Bs)[2][NTILES * 32][LDS_ROW],
                                        f32x16 (&acc)[NTILES])
{
    constexpr int NB = NTILES / 2;
    *reinterpret_cast<u32x4v *>(&As[buf][st.a_row0][st.kc * 8]) = f.a0;
    *reinterpret_cast<u32x4v *>(&As[buf][st.a_row1][st.kc * 8]) = f.a1;
    *reinterpret_cast<u32x4v *>(&Bs[buf][st.b_row][st.kc * 8]) = f.b0;
    if constexpr (NB > 1) *reinterpret_cast<u32x4v *>(&Bs[buf][st.b_row + 64][st.kc * 8]) = f.b1;
    if constexpr (NB > 2) {
        *reinterpret_cast<u32x4v *>(&Bs[buf][st.b_row + 128][st.kc * 8]) = f.b2;
        *reinterpret_cast<u32x4v *>(&Bs[buf][st.b_row + 192][st.kc * 8]) = f.b3;
    }
    __syncthreads();               // tile `buf` is complete; everyone is also done reading tile `buf ^ 1`
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
        const int ko = kk * 16 + 8 * st.half;
        const bf16x8 act = lds_read8(&As[buf][st.act_row][ko]);
#pragma unroll
        for (int t = 0; t < NTILES; ++t) {
            const bf16x8 wgt = lds_read8(&Bs[buf][t * 32 + st.lr][ko]);
            acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wgt, act, acc[t], 0, 0, 0);
        }
    }
    buf ^= 1;
}

// ------------------------------------------------------------------------------------------------
// Workgroup tile 128 (m) x NTILES*32 (n), four waves of 32 x NTILES*32; the weights are the first MFMA
// operand so that a lane ends up with four consecutive n of one row m (vector stores along the row).
// K is consumed in chunks of CH 32-wide steps (single steps for the remainder): every global load of a
// chunk is issued before the first one is used, so a chunk costs one memory round trip; its steps then
// go through double-buffered LDS tiles with one barrier each.  NTILES = 8 covers a whole 256-wide
// layer, so the activations are read once (see launch_nt for why it is not the default).
// ------------------------------------------------------------------------------------------------
template <int NTILES, int CH>
__device__ __forceinline__ void gemm_nt_body(const NtArgs &a, uint32_t bid, uint32_t ncol, uint16_t (&As)[2][128][LDS_ROW],
                                             uint16_t (&Bs)[2][NTILES * 32][LDS_ROW])
{
    constexpr int BN = NTILES * 32, NB = NTILES / 2;
    const int M = min(a.hdr[CR_HDR_N_DST], a.max_rows);
    // the column tiles of one row tile run next to each other on one XCD: the activations come from HBM once
    uint32_t tile;
    if (!xcd_compact(bid, (uint32_t)((M + 127) / 128) * ncol, tile)) return;
    const int m0 = (int)(tile / ncol) * 128, n0 = (int)(tile % ncol) * BN;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, lr = lane & 31;

    // staging assignment: A 128 rows x 4 chunks of 8, two per thread; B BN rows x 4 chunks, NB per thread
    const int a_row0 = tid >> 2, a_row1 = (tid + 256) >> 2, kc = tid & 3;
    const int64_t ga0 = (int64_t)min(m0 + a_row0, M - 1) * a.lda;
    const int64_t ga1 = (int64_t)min(m0 + a_row1, M - 1) * a.lda;
    const uint16_t *gb = a.B + (int64_t)(n0 + (tid >> 2)) * a.K + kc * 8;

    f32x16 acc[NTILES];
#pragma unroll
    for (int t = 0; t < NTILES; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;

    const int nsteps = a.K / 32;
    int buf = 0;
    NtState st{a.A0, a.A1, a.K0, a.K, ga0, ga1, gb, kc, a_row0, a_row1, tid >> 2, wave * 32 + lr, lr, half};
    int s0 = 0;
    for (; s0 + CH <= nsteps; s0 += CH) {
        NtFetch<NB> f[CH];
#pragma unroll
        for (int i = 0; i < CH; ++i) f[i] = nt_fetch<NB>(st, s0 + i);
#pragma unroll
        for (int i = 0; i < CH; ++i) nt_step<NTILES>(st, f[i], buf, As, Bs, acc);
    }
    while (s0 < nsteps) {         // the remaining steps (K not a multiple of 32 * CH), again fetched together: up to three at a time
        const int rem = nsteps - s0;
        const NtFetch<NB> f0 = nt_fetch<NB>(st, s0), f1 = nt_fetch<NB>(st, min(s0 + 1, nsteps - 1)),
                          f2 = nt_fetch<NB>(st, min(s0 + 2, nsteps - 1));
        nt_step<NTILES>(st, f0, buf, As, Bs, acc);
        if (rem > 1) nt_step<NTILES>(st, f1, buf, As, Bs, acc);
        if (rem > 2) nt_step<NTILES>(st, f2, buf, As, Bs, acc);
        s0 += 3;
    }

    // Epilogue through LDS (the staging tiles are free after one more barrier): a lane holds 4-column pieces of one
    // row, which would go out as 8/16-byte stores scattered over 32 rows; staged, a wave writes whole 128-byte row
    // segments.  Each wave uses its own quarter of As.
    static_assert(NTILES == 2, "the staged epilogue is laid out for a 32 x 64 wave tile");
    __syncthreads();
    char *region = reinterpret_cast<char *>(&As[0][0][0]) + wave * (2 * 128 * LDS_ROW * 2 / 4);     // 5120 bytes
    const int mw = m0 + wave * 32;
    float v[2][4][4];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int grp = 0; grp < 4; ++grp) {
            const int n = n0 + t * 32 + 8 * grp + 4 * half;
            const float4 bq = a.bias ? *reinterpret_cast<const float4 *>(a.bias + n) : make_float4(0.f, 0.f, 0.f, 0.f);
            v[t][grp][0] = acc[t][grp * 4 + 0] + bq.x; v[t][grp][1] = acc[t][grp * 4 + 1] + bq.y;
            v[t][grp][2] = acc[t][grp * 4 + 2] + bq.z; v[t][grp][3] = acc[t][grp * 4 + 3] + bq.w;
            if (a.relu) {
#pragma unroll
                for (int i = 0; i < 4; ++i) v[t][grp][i] = v[t][grp][i] < 0.f ? 0.f : v[t][grp][i];
            }
        }
    if (a.Cb) {      // both 32-column halves at once: rows of 64 bf16 (+8 of padding)
        uint16_t (*ob)[72] = reinterpret_cast<uint16_t (*)[72]>(region);
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int grp = 0; grp < 4; ++grp) {
                const uint32_t lo = pack_bf16x2(v[t][grp][0], v[t][grp][1]);
                const uint32_t hi = pack_bf16x2(v[t][grp][2], v[t][grp][3]);
                *reinterpret_cast<uint2 *>(&ob[lr][t * 32 + 8 * grp + 4 * half]) = make_uint2(lo, hi);
            }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int c = it * 64 + lane, row = c >> 3, c8 = (c & 7) * 8;
            const u32x4v x = *reinterpret_cast<const u32x4v *>(&ob[row][c8]);
            if (mw + row < M) *reinterpret_cast<u32x4v *>(a.Cb + (int64_t)(mw + row) * a.ldcb + n0 + c8) = x;
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    }
    if (a.C0) {      // one 32-column half at a time: rows of 32 floats (+4 of padding)
        float (*of)[36] = reinterpret_cast<float (*)[36]>(region);
#pragma unroll
        for (int t = 0; t < 2; ++t) {
#pragma unroll
            for (int grp = 0; grp < 4; ++grp)
                *reinterpret_cast<float4 *>(&of[lr][8 * grp + 4 * half]) = make_float4(v[t][grp][0], v[t][grp][1], v[t][grp][2], v[t][grp][3]);
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                const int c = it * 64 + lane, row = c >> 3, c4 = (c & 7) * 4;
                const float4 x = *reinterpret_cast<const float4 *>(&of[row][c4]);
                const int n = n0 + t * 32 + c4;
                if (mw + row < M) {
                    float *dst = n < a.N0 ? a.C0 + (int64_t)(mw + row) * a.ldc + n : a.C1 + (int64_t)(mw + row) * a.ldc + (n - a.N0);
                    *reinterpret_cast<float4 *>(dst) = x;
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        }
    }
}

// Register budget: up to four waves per SIMD.  Four K steps of prefetch at this occupancy measured faster
// than eight steps at two waves per SIMD on the products that fill the chip; a product with few workgroups and a
// long K loop (the reddit-like input layer: 88 row tiles, K = 1216) gains nothing from occupancy and takes the
// eight-step instantiation, which halves the round trips of its K loop.
template <int NTILES, int CH>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(CH == 4 ? 3 : 1, CH == 4 ? 4 : 2))) void gemm_nt_kernel(NtArgs a)
{
    __shared__ __attribute__((aligned(16))) uint16_t As[2][128][LDS_ROW];
    __shared__ __attribute__((aligned(16))) uint16_t Bs[2][NTILES * 32][LDS_ROW];
    gemm_nt_body<NTILES, CH>(a, blockIdx.y * gridDim.x + blockIdx.x, gridDim.x, As, Bs);
}

// ------------------------------------------------------------------------------------------------
// The same product for blocks of few rows (the layers next to the roots: about a thousand rows), where the tiled
// kernel above leaves most of the chip idle and spends its time in K steps taken one after another.  Workgroup tile
// 32 (m) x 64 (n); the four waves split K between them (wave w takes the 16-wide steps w, w + 4, ...) and fetch
// their MFMA operands straight from memory in the layout the matrix cores want (both operands are contiguous along
// k: a lane's fragment is one 16-byte load), up to eight steps in flight, no staging and no barrier inside the
// loop.  The four partial tiles meet in LDS and are added in a fixed order.
// ------------------------------------------------------------------------------------------------
constexpr int SMALL_DEPTH = 8;
constexpr int SMALL_ROW = 68;     // floats per staged row: 64 + 4 of padding (272 bytes, keeps 16-byte alignment)

// loss part of the fused top-layer launch (XENT == true): the product's rows are the roots, its columns the classes
struct XentArgs {
    int32_t n_classes;
    const int32_t *labels, *root_ids;
    float *loss, *row_loss;
    uint16_t *d_logits_bf16;      // [max_rows][64]
    unsigned long long *acc;      // tickets and the fixed-point sum of the workgroups' loss shares; zero between calls
};

// XENT == true (one column tile: at most 64 classes; no ReLU, no bf16 copy): a workgroup holds whole rows of
// logits after the reduction, so the softmax cross-entropy of its rows, their gradient and its share of the mean
// loss are taken right there; the shares meet in one device-side accumulator.
template <bool XENT>
__global__ __launch_bounds__(256) void gemm_nt_small_kernel(NtArgs a, XentArgs x)
{
    __shared__ __attribute__((aligned(16))) float red[4][32][SMALL_ROW];
    __shared__ float wg_loss[32];
    const int M = min(a.hdr[CR_HDR_N_DST], a.max_rows);
    const int m0 = (int)blockIdx.y * 32, n0 = (int)blockIdx.x * 64;
    if (XENT && M <= 0) {
        if (blockIdx.y == 0 && threadIdx.x == 0) x.loss[0] = 0.f;
        return;
    }
    if (m0 >= M) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, lr = lane & 31;
    const int nk = a.K / 16;
    // the label of the row this thread will finish: requested now (two dependent loads), used after the product
    int label = 0;
    if constexpr (XENT) label = x.labels[x.root_ids[min(m0 + (tid >> 3), M - 1)]];
    const int64_t arow = (int64_t)min(m0 + lr, M - 1) * a.lda + 8 * half;
    const uint16_t *b0 = a.B + (int64_t)(n0 + lr) * a.K + 8 * half;
    const uint16_t *b1 = b0 + (int64_t)32 * a.K;

    f32x16 acc[2];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;

    for (int s0 = wave; s0 < nk; s0 += 4 * SMALL_DEPTH) {
        u32x4v xa[SMALL_DEPTH], xb0[SMALL_DEPTH], xb1[SMALL_DEPTH];
#pragma unroll
        for (int i = 0; i < SMALL_DEPTH; ++i) {
            const int k0 = min(s0 + 4 * i, nk - 1) * 16;       // a step past the end re-reads the last one and is not used
            const uint16_t *src = k0 < a.K0 ? a.A0 + k0 : a.A1 + (k0 - a.K0);
            xa[i] = *reinterpret_cast<const u32x4v *>(src + arow);
            xb0[i] = *reinterpret_cast<const u32x4v *>(b0 + k0);
            xb1[i] = *reinterpret_cast<const u32x4v *>(b1 + k0);
        }
#pragma unroll
        for (int i = 0; i < SMALL_DEPTH; ++i) {
            if (s0 + 4 * i < nk) {                              // (uniform over the wave)
                const bf16x8 act = __builtin_bit_cast(bf16x8, xa[i]);
                acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, xb0[i]), act, acc[0], 0, 0, 0);
                acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, xb1[i]), act, acc[1], 0, 0, 0);
            }
        }
    }
    // a lane holds, for row lr, the columns t*32 + 8*grp + 4*half .. + 4
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int grp = 0; grp < 4; ++grp)
            *reinterpret_cast<float4 *>(&red[wave][lr][t * 32 + 8 * grp + 4 * half]) =
                make_float4(acc[t][grp * 4 + 0], acc[t][grp * 4 + 1], acc[t][grp * 4 + 2], acc[t][grp * 4 + 3]);
    __syncthreads();
    const int row = tid >> 3, c8 = (tid & 7) * 8;
    if (!XENT && m0 + row >= M) return;
    const bool row_ok = m0 + row < M;
    float v[8];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const float4 p0 = *reinterpret_cast<const float4 *>(&red[0][row][c8 + 4 * h]), p1 = *reinterpret_cast<const float4 *>(&red[1][row][c8 + 4 * h]);
        const float4 p2 = *reinterpret_cast<const float4 *>(&red[2][row][c8 + 4 * h]), p3 = *reinterpret_cast<const float4 *>(&red[3][row][c8 + 4 * h]);
        v[4 * h + 0] = (p0.x + p1.x) + (p2.x + p3.x); v[4 * h + 1] = (p0.y + p1.y) + (p2.y + p3.y);
        v[4 * h + 2] = (p0.z + p1.z) + (p2.z + p3.z); v[4 * h + 3] = (p0.w + p1.w) + (p2.w + p3.w);
    }
    const int n = n0 + c8;
    if (a.bias) {
        const float4 q0 = *reinterpret_cast<const float4 *>(a.bias + n), q1 = *reinterpret_cast<const float4 *>(a.bias + n + 4);
        v[0] += q0.x; v[1] += q0.y; v[2] += q0.z; v[3] += q0.w; v[4] += q1.x; v[5] += q1.y; v[6] += q1.z; v[7] += q1.w;
    }
    if (a.relu) {
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = v[i] < 0.f ? 0.f : v[i];
    }
    const int64_t m = min(m0 + row, M - 1);
    if (a.C0 && row_ok) {
        float *dst = n < a.N0 ? a.C0 + m * a.ldc + n : a.C1 + m * a.ldc + (n - a.N0);    // (N0 is a multiple of 32: no piece straddles)
        *reinterpret_cast<float4 *>(dst) = make_float4(v[0], v[1], v[2], v[3]);
        *reinterpret_cast<float4 *>(dst + 4) = make_float4(v[4], v[5], v[6], v[7]);
    }
    if (a.Cb && row_ok) {
        u32x4v xb;
#pragma unroll
        for (int i = 0; i < 4; ++i) xb[i] = pack_bf16x2(v[2 * i], v[2 * i + 1]);
        *reinterpret_cast<u32x4v *>(a.Cb + m * a.ldcb + n) = xb;
    }
    if constexpr (XENT) {
        // the eight threads of a row sit in eight neighbouring lanes; rows past the last one compute on row M - 1 and store nothing
        const int C = x.n_classes;
        float mx = -INFINITY;
#pragma unroll
        for (int i = 0; i < 8; ++i) mx = fmaxf(mx, n + i < C ? v[i] : -INFINITY);
#pragma unroll
        for (int off = 1; off < 8; off <<= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
        float e[8], den = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            e[i] = n + i < C ? expf(v[i] - mx) : 0.f;
            den += e[i];
        }
#pragma unroll
        for (int off = 1; off < 8; off <<= 1) den += __shfl_xor(den, off);
        const float inv_n = 1.0f / (float)M;
        u32x4v dq;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float d0 = 0.f, d1 = 0.f;
            if (n + 2 * i < C) d0 = (e[2 * i] / den - (n + 2 * i == label ? 1.f : 0.f)) * inv_n;
            if (n + 2 * i + 1 < C) d1 = (e[2 * i + 1] / den - (n + 2 * i + 1 == label ? 1.f : 0.f)) * inv_n;
            dq[i] = pack_bf16x2(d0, d1);
        }
        if (row_ok) *reinterpret_cast<u32x4v *>(x.d_logits_bf16 + m * 64 + n) = dq;
        if ((tid & 7) == 0) wg_loss[row] = 0.f;
        __syncthreads();
        if (label >= n && label < n + 8) {          // the thread that holds the label's logit
            float zl = v[0];
#pragma unroll
            for (int i = 1; i < 8; ++i) zl = label == n + i ? v[i] : zl;
            const float rl = -(zl - mx - logf(den));
            if (row_ok) { x.row_loss[m] = rl; wg_loss[row] = rl; }
        }
        __syncthreads();
        if (tid < 64) {
            float t = tid < 32 ? wg_loss[tid] : 0.f;
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) t += __shfl_xor(t, off);
            if (tid == 0) {
                // One 64-bit atomic per workgroup carries its share of the loss (fixed point, 2^-20, bits 0..39: integer
                // sums do not depend on the order of arrival, so the mean is reproducible), a ticket (bits 40..55) and a
                // mark for a share that is not finite (bits 56..62).  The workgroup whose ticket is the last one has the
                // whole sum in hand.  No fence, no access to another workgroup's data: the atomic is performed at the
                // memory side.
                const bool finite = t == t && fabsf(t) <= 8192.0f;       // 32 rows of at most ~100 each
                const unsigned long long share = finite ? (unsigned long long)(fmaxf(t, 0.f) * 1048576.0f + 0.5f) : 0ull;
                const unsigned long long add = share | (1ull << 40) | (finite ? 0ull : 1ull << 56);
                const unsigned long long after = __hip_atomic_fetch_add(x.acc, add, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + add;
                if ((int)((after >> 40) & 0xFFFFull) == (M + 31) / 32) {
                    const float mean = (float)((double)(after & ((1ull << 40) - 1ull)) * (1.0 / 1048576.0) / (double)M);
                    x.loss[0] = (after >> 56) ? __builtin_nanf("") : mean;
                    __hip_atomic_store(x.acc, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------
// The same product for the input layer of the large workloads: tens of thousands of rows, N = 256, any K (K <= 256 takes
// the streaming kernel further down; this one serves wider inputs, e.g. 602 features.  GraphSAGE: self | aggregate;
// one-operand layers: all of K from one array).  The tiled kernel
// above reads every activation row four times (once per 64-column tile) and spends most of its time moving operands;
// here one workgroup per compute unit takes 256 rows and ALL columns, so activations pass through a compute unit once:
//   - K is taken in chunks of 128 columns, each operand array's columns in chunks of their own.  A chunk is 256 rows x
//     256 bytes of activations and 256 x 256 bytes of weights: both are fetched with coalesced 16-byte loads (16 per
//     thread each) and laid out in LDS with rows padded by 16 bytes, so that the MFMA fragments are conflict-free
//     16-byte LDS reads; an array's last chunk that reaches past its columns is staged with zeros there;
//   - the next chunk's loads are issued inside the current chunk's K loop, four per step, and travel under its MFMAs
//     (issued in one go they hold the wave, the only one on its SIMD, for as long as the memory pipeline takes them);
//   - a wave owns 64 rows x 256 columns (256 accumulator registers, one wave per SIMD): per 16-wide K step 10 fragment
//     reads feed 16 MFMAs; the fragments of step s + 1 are requested before the MFMAs of step s are issued, because no
//     other wave is there to hide the LDS latency;
//   - the accumulators start from the bias; ReLU and the bf16 conversion happen on the way through LDS again, from
//     where whole 512-byte rows leave.
// ------------------------------------------------------------------------------------------------
constexpr int WIDE_ROWS = 256;          // rows per workgroup
constexpr int WIDE_KH = 128;            // K of one chunk
constexpr int WIDE_N = 256;
constexpr int WIDE_LROW = WIDE_KH + 8;  // staged row: 128 bf16 + 8 of padding (272 bytes)
constexpr int WIDE_OROW = WIDE_N + 8;   // staged output row
constexpr size_t WIDE_LDS_BYTES = (size_t)2 * 256 * WIDE_LROW * sizeof(uint16_t) + WIDE_N * sizeof(float);

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void gemm_nt_wide_kernel(NtArgs a)
{
    constexpr int KSTEPS = WIDE_KH / 16, NTILES = WIDE_N / 32;
    extern __shared__ __attribute__((aligned(16))) uint16_t wide_lds[];
    uint16_t *Ws = wide_lds;                                   // [256 n][WIDE_LROW]
    uint16_t *As = wide_lds + 256 * WIDE_LROW;                 // [256 m][WIDE_LROW]
    float *bias_s = reinterpret_cast<float *>(wide_lds + 2 * 256 * WIDE_LROW);
    static_assert((size_t)4 * 64 * WIDE_OROW * sizeof(uint16_t) <= (size_t)2 * 256 * WIDE_LROW * sizeof(uint16_t), "output staging must fit");
    const int M = min(a.hdr[CR_HDR_N_DST], a.max_rows);
    if ((int)blockIdx.x * WIDE_ROWS >= M) return;
    // the last tile is moved back so that it ends at the last row: it recomputes a few rows of its neighbour (same
    // values, written twice) and no load has to be clamped to the row count.  With fewer than 256 rows the one tile
    // reads rows past the last one: they exist (the arrays hold max_rows >= 16384 rows), rows are independent, and
    // results past the last row are not stored.
    const int m0 = max(0, min((int)blockIdx.x * WIDE_ROWS, M - WIDE_ROWS));
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, lr = lane & 31;
    const int K = a.K, K0 = a.K0;
    // Column k of the product sits in the first operand array for k < K0 and in the second from there on.  Each array's
    // columns are taken in chunks of 128 of their own (the first array's chunks, then the second's), so a chunk lies in
    // one array whatever K0 is; the last chunk of an array whose width is no multiple of 128 is a partial one.
    const int nchunk0 = (K0 + WIDE_KH - 1) / WIDE_KH;
    const int nchunk = nchunk0 + (K - K0 + WIDE_KH - 1) / WIDE_KH;
    // chunk c: its first column within its array, and the columns it has there (128, fewer in a partial chunk)
    auto chunk_off = [&](int c) { return (c < nchunk0 ? c : c - nchunk0) * WIDE_KH; };
    auto chunk_cols = [&](int c) { return min(WIDE_KH, (c < nchunk0 ? K0 : K - K0) - chunk_off(c)); };

    // staging assignment: piece p = i * 256 + tid of a chunk = (row p / 16, 16-byte piece p % 16).  An address is a base
    // that is the same for the whole workgroup (chunk, 16-row group i) plus one per-thread offset that serves all 16
    // pieces: no address registers are held across the K loop.  Pieces past a partial chunk's columns are loaded from the
    // chunk's first piece and staged as zeros.
    const int srow = tid >> 4, spiece = tid & 15;
    u32x4v wreg[16], areg[16];
    auto fetch = [&](int c, int i) {     // pieces i of the chunk's 16 activation and 16 weight pieces of this thread
        const int koff = chunk_off(c);
        const int sp = spiece * 8 < chunk_cols(c) ? spiece * 8 : 0;
        const uint16_t *Ai = (c < nchunk0 ? a.A0 : a.A1) + koff + (int64_t)(m0 + i * 16) * a.lda;
        const uint16_t *Wi = a.B + (c < nchunk0 ? 0 : K0) + koff + (int64_t)(i * 16) * K;
        areg[i] = *reinterpret_cast<const u32x4v *>(Ai + (uint32_t)(srow * (int)a.lda + sp));
        wreg[i] = *reinterpret_cast<const u32x4v *>(Wi + (uint32_t)(srow * K + sp));
    };
    auto stage = [&](int c) {
        const bool full = chunk_cols(c) == WIDE_KH;            // (uniform)
        const bool mine = spiece * 8 < chunk_cols(c);
        const u32x4v zero = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int row = i * 16 + srow;
            *reinterpret_cast<u32x4v *>(&As[row * WIDE_LROW + spiece * 8]) = (full || mine) ? areg[i] : zero;
            *reinterpret_cast<u32x4v *>(&Ws[row * WIDE_LROW + spiece * 8]) = (full || mine) ? wreg[i] : zero;
        }
    };
#pragma unroll
    for (int i = 0; i < 16; ++i) fetch(0, i);
    if (tid < WIDE_N / 4)
        *reinterpret_cast<float4 *>(&bias_s[tid * 4]) = a.bias ? *reinterpret_cast<const float4 *>(a.bias + tid * 4) : make_float4(0.f, 0.f, 0.f, 0.f);
    stage(0);
    __syncthreads();

    // the accumulators start from the bias (a lane's 4-column pieces: columns t*32 + 8*grp + 4*half .. + 4)
    f32x16 acc[2][NTILES];
#pragma unroll
    for (int t = 0; t < NTILES; ++t)
#pragma unroll
        for (int grp = 0; grp < 4; ++grp) {
            const float4 bq = *reinterpret_cast<const float4 *>(&bias_s[t * 32 + 8 * grp + 4 * half]);
#pragma unroll
            for (int rb = 0; rb < 2; ++rb) {
                acc[rb][t][grp * 4 + 0] = bq.x; acc[rb][t][grp * 4 + 1] = bq.y; acc[rb][t][grp * 4 + 2] = bq.z; acc[rb][t][grp * 4 + 3] = bq.w;
            }
        }
    const uint16_t *arow0 = As + (wave * 64 + lr) * WIDE_LROW + 8 * half, *arow1 = arow0 + 32 * WIDE_LROW;
    const uint16_t *wrow = Ws + lr * WIDE_LROW + 8 * half;
    // one chunk's K loop; PREFETCH: the next chunk's loads, two of each per step, travel under the MFMAs
    auto chunk_loop = [&](auto prefetch, int c) {
        constexpr bool PREFETCH = decltype(prefetch)::value;
        bf16x8 wnext[NTILES], anext[2];
        anext[0] = lds_read8(arow0);
        anext[1] = lds_read8(arow1);
#pragma unroll
        for (int t = 0; t < NTILES; ++t) wnext[t] = lds_read8(wrow + t * 32 * WIDE_LROW);
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
            bf16x8 wcur[NTILES];
            const bf16x8 a0 = anext[0], a1 = anext[1];
#pragma unroll
            for (int t = 0; t < NTILES; ++t) wcur[t] = wnext[t];
            if (ks + 1 < KSTEPS) {
                anext[0] = lds_read8(arow0 + (ks + 1) * 16);
                anext[1] = lds_read8(arow1 + (ks + 1) * 16);
#pragma unroll
                for (int t = 0; t < NTILES; ++t) wnext[t] = lds_read8(wrow + t * 32 * WIDE_LROW + (ks + 1) * 16);
            }
            if constexpr (PREFETCH) {
                fetch(c + 1, 2 * ks);
                fetch(c + 1, 2 * ks + 1);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int t = 0; t < NTILES; ++t) {
                acc[0][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wcur[t], a0, acc[0][t], 0, 0, 0);
                acc[1][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wcur[t], a1, acc[1][t], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    // (the last chunk is peeled off: with the prefetch and the staging under a condition inside one loop the compiler
    // keeps the 128 staging registers alive across the whole loop and spills)
    for (int c = 0; c + 1 < nchunk; ++c) {
        chunk_loop(std::true_type{}, c);
        __syncthreads();                  // every wave is done reading this chunk
        stage(c + 1);
        __syncthreads();
    }
    chunk_loop(std::false_type{}, nchunk - 1);
    __syncthreads();

    // epilogue: ReLU, bf16; a lane holds, for row lr of each block, the columns t*32 + 8*grp + 4*half .. + 4
    const float floor_v = a.relu ? 0.f : -INFINITY;
    uint16_t *ob = wide_lds + wave * 64 * WIDE_OROW;
#pragma unroll
    for (int t = 0; t < NTILES; ++t)
#pragma unroll
        for (int grp = 0; grp < 4; ++grp) {
            const int n = t * 32 + 8 * grp + 4 * half;
#pragma unroll
            for (int rb = 0; rb < 2; ++rb) {
                const float v0 = fmaxf(acc[rb][t][grp * 4 + 0], floor_v), v1 = fmaxf(acc[rb][t][grp * 4 + 1], floor_v);
                const float v2 = fmaxf(acc[rb][t][grp * 4 + 2], floor_v), v3 = fmaxf(acc[rb][t][grp * 4 + 3], floor_v);
                *reinterpret_cast<uint2 *>(&ob[(rb * 32 + lr) * WIDE_OROW + n]) = make_uint2(pack_bf16x2(v0, v1), pack_bf16x2(v2, v3));
            }
        }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    constexpr int CPR = WIDE_N / 8;       // 16-byte chunks per output row
    const int mw = m0 + wave * 64;
#pragma unroll 8
    for (int it = 0; it < CPR; ++it) {
        const int c = it * 64 + lane, row = c / CPR, c8 = (c % CPR) * 8;
        const u32x4v x = *reinterpret_cast<const u32x4v *>(&ob[row * WIDE_OROW + c8]);
        if (mw + row < M) *reinterpret_cast<u32x4v *>(a.Cb + (int64_t)(mw + row) * a.ldcb + c8) = x;
    }
}

// ------------------------------------------------------------------------------------------------
// The same product again for K <= 256 (the input layer of the papers-like workload: 2 x 128 features): the weights
// of a wave's 64 output columns fit its registers (64 x 256 bf16 = 128 registers per lane), so they are fetched once
// per workgroup and only activations pass through LDS.  One persistent workgroup per compute unit walks over tiles
// of 64 rows (tile t, t + gridDim.x, ..):
//   - a tile's activations (64 rows x K) travel global -> registers -> LDS; the loads of tiles t+1 and t+2 are in
//     flight while tile t is multiplied (two register sets, two LDS buffers, one barrier per tile), so a compute unit
//     keeps two tiles (64 KB) on the way and the chip about 16 MB: enough to cover the memory latency at full rate;
//   - a wave multiplies all 64 rows by its own 64 columns: per 16-wide K step two fragment reads feed four MFMAs
//     (the activation fragments are the only LDS reads of the K loop);
//   - bias, ReLU and the bf16 conversion happen in the wave's own LDS patch, from where 128-byte row pieces leave;
//     the stores of tile t overlap the loads of the tiles behind it.
// With K = N = 256 the product moves 1 KB per row against 131 K multiply-adds: even at the full memory rate the matrix
// cores can be busy for about 30 % of the time at most.
// ------------------------------------------------------------------------------------------------
constexpr int STREAM_ROWS = 64;
constexpr int STREAM_KMAX = 256;
constexpr int STREAM_LROW = STREAM_KMAX + 8;    // staged activation row: 256 bf16 + 8 of padding (528 bytes)
constexpr int STREAM_OROW = 64 + 8;             // staged output row of one wave
constexpr size_t STREAM_LDS_BYTES = ((size_t)2 * STREAM_ROWS * STREAM_LROW + (size_t)4 * STREAM_ROWS * STREAM_OROW) * sizeof(uint16_t) +
                                    WIDE_N * sizeof(float);

// KS: 16-wide K steps held in registers (8: K <= 128, 16: K <= 256; columns from K on count as zeros).  FULL: at least
// 64 rows, so that every tile is a whole one and nothing in the tile loop is conditional: every wait on the counter of
// outstanding memory operations then leaves exactly the newer loads and stores in flight.
// UNIFORM: each wave's sixteen pieces of a row lie in one operand array (K0 = K or a multiple of 128): a load address is
// then a base that is the same for the whole wave (array, tile, row group) plus one 32-bit offset per thread that never
// changes, so no address registers are computed per tile (the compiler puts such temporaries into the registers the
// previous tile's loads went to, and then waits for loads that have long been consumed).
template <int KS, bool FULL, bool UNIFORM>
__device__ __forceinline__ void nt_stream_body(const NtArgs &a, const int M, uint16_t *stream_lds, const bf16x8 (&wf)[2][KS])
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, lr = lane & 31;
    uint16_t *As0 = stream_lds, *As1 = stream_lds + STREAM_ROWS * STREAM_LROW;
    uint16_t *ob = stream_lds + 2 * STREAM_ROWS * STREAM_LROW + wave * STREAM_ROWS * STREAM_OROW;
    float *bias_s = reinterpret_cast<float *>(stream_lds + 2 * STREAM_ROWS * STREAM_LROW + 4 * STREAM_ROWS * STREAM_OROW);
    const int ntiles = (M + STREAM_ROWS - 1) / STREAM_ROWS;
    const int K = a.K, K0 = a.K0;

    // staging: a thread moves the same 16-byte piece (columns 8 kp ..) of eight rows (srow, srow + 8, ..) of every tile;
    // a wave covers 16 pieces (256 bytes) of four rows per load.
    // The last tile is moved back so that it ends at the last row (it recomputes rows of its neighbour: same values,
    // written twice); with fewer than 64 rows the one tile reads rows past the last one: they exist (the arrays hold
    // max_rows >= 16384 rows), rows are independent, and results past the last row are not stored.  A fetch for a tile
    // past the last one, or of a piece past K, still issues its eight loads (all of the first operand's first bytes).
    const int uwave = __builtin_amdgcn_readfirstlane(wave);
    const int kp = (lane & 15) + 16 * (uwave & 1), srow = (lane >> 4) + 4 * (uwave >> 1);
    const bool mine = kp * 8 < K;
    const uint16_t *col_src = !mine ? a.A0 : (kp * 8 < K0 ? a.A0 + kp * 8 : a.A1 + (kp * 8 - K0));
    // (UNIFORM: the wave's array, the second one addressed from K0 columns in front of it; the host has checked that
    // the arrays are shorter than 2^31 bytes)
    const bool second = 128 * (uwave & 1) >= K0;
    const uint64_t base_v = reinterpret_cast<uint64_t>(second ? a.A1 - K0 : a.A0);
    const uint16_t *wave_src = reinterpret_cast<const uint16_t *>(
        ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(base_v >> 32)) << 32) | (uint32_t)__builtin_amdgcn_readfirstlane((int)base_v));
    const uint32_t ld_bytes = (uint32_t)__builtin_amdgcn_readfirstlane((int)(a.lda * 2));
    const uint32_t records = (uint32_t)__builtin_amdgcn_readfirstlane((int)((uint32_t)a.max_rows * ld_bytes + (second ? 2u * (uint32_t)K0 : 0u)));
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(wave_src), 0, (int)records, 0x00020000);
    // (a thread without a piece of its own -- columns from K on -- reads its array's first bytes: with the second array
    // that is K0 columns past the shifted base, not the base itself, which lies in front of the array)
    const uint32_t lane_off = mine ? (uint32_t)srow * ld_bytes + 16u * (uint32_t)kp : (second ? 2u * (uint32_t)K0 : 0u);
    auto tile_m0 = [&](int t) { return max(0, min(t * STREAM_ROWS, M - STREAM_ROWS)); };
    auto fetch = [&](u32x4v (&r)[8], int t) {
        if constexpr (UNIFORM) {
            // buffer loads: descriptor and row offset in scalar registers, the thread's offset in one register that
            // never changes (a tile past the last one: the first tile's rows again, they exist)
            const uint32_t row0 = t < ntiles ? (uint32_t)tile_m0(t) : 0u;
#pragma unroll
            for (int i = 0; i < 8; ++i)
                r[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)lane_off, (int)((row0 + 8u * i) * ld_bytes), 0);
        } else {
            const bool real = mine && t < ntiles;
            const int64_t ld = real ? a.lda : 0;
            const uint16_t *src = real ? col_src + (int64_t)(tile_m0(t) + srow) * ld : a.A0;
#pragma unroll
            for (int i = 0; i < 8; ++i) r[i] = *reinterpret_cast<const u32x4v *>(src + (int64_t)(8 * i) * ld);
        }
    };
    auto stage = [&](uint16_t *As, const u32x4v (&r)[8]) {
        if (!mine) return;
#pragma unroll
        for (int i = 0; i < 8; ++i) *reinterpret_cast<u32x4v *>(&As[(8 * i + srow) * STREAM_LROW + kp * 8]) = r[i];
    };
    const float floor_v = a.relu ? 0.f : -INFINITY;
    // Two sets of accumulators: while the MFMAs of a tile fill one, the other -- the tile before -- is converted and
    // written to the wave's LDS patch, a sixteenth (K <= 128: an eighth) per K step, in the shadow of that step's MFMAs;
    // this wave is alone on its SIMD, so nothing else would fill the vector pipe while the matrix pipe runs, nor the
    // matrix pipe during a separate epilogue.
    // piece 0..15 of a tile's results: a lane holds, for row lr of each 32-row block rb, the columns
    // 32 cb + 8 grp + 4 half .. + 4 of the wave's 64
    auto convert_piece = [&](const f32x16 (&acc)[2][2], int piece) {
        const int cb = piece >> 3, grp = (piece >> 1) & 3, rb = piece & 1;
        const int n = 32 * cb + 8 * grp + 4 * half;
        const float v0 = fmaxf(acc[rb][cb][grp * 4 + 0], floor_v), v1 = fmaxf(acc[rb][cb][grp * 4 + 1], floor_v);
        const float v2 = fmaxf(acc[rb][cb][grp * 4 + 2], floor_v), v3 = fmaxf(acc[rb][cb][grp * 4 + 3], floor_v);
        *reinterpret_cast<uint2 *>(&ob[(rb * 32 + lr) * STREAM_OROW + n]) = make_uint2(pack_bf16x2(v0, v1), pack_bf16x2(v2, v3));
    };
    // the patch leaves as 128-byte row pieces
    auto flush = [&](int t) {
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        const int m0 = tile_m0(t);
#pragma unroll
        for (int it = 0; it < 8; ++it) {
            const int c = it * 64 + lane, row = c >> 3, c8 = (c & 7) * 8;
            const u32x4v x = *reinterpret_cast<const u32x4v *>(&ob[row * STREAM_OROW + c8]);
            if (FULL || m0 + row < M) *reinterpret_cast<u32x4v *>(a.Cb + (int64_t)(m0 + row) * a.ldcb + 64 * wave + c8) = x;
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");      // the patch is rewritten for the next tile
    };
    auto multiply = [&](const uint16_t *As, f32x16 (&acc)[2][2], const f32x16 (&prev)[2][2], auto with_prev) {
        constexpr bool PREV = decltype(with_prev)::value;
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
            for (int grp = 0; grp < 4; ++grp) {
                const float4 bq = *reinterpret_cast<const float4 *>(&bias_s[64 * wave + 32 * cb + 8 * grp + 4 * half]);
#pragma unroll
                for (int rb = 0; rb < 2; ++rb) {
                    acc[rb][cb][grp * 4 + 0] = bq.x; acc[rb][cb][grp * 4 + 1] = bq.y; acc[rb][cb][grp * 4 + 2] = bq.z; acc[rb][cb][grp * 4 + 3] = bq.w;
                }
            }
        const uint16_t *ar0 = As + lr * STREAM_LROW + 8 * half, *ar1 = ar0 + 32 * STREAM_LROW;
        // (fragments are requested two K steps ahead: four MFMAs do not cover an LDS round trip)
        bf16x8 f0[3], f1[3];
        f0[0] = lds_read8(ar0); f1[0] = lds_read8(ar1);
        f0[1] = lds_read8(ar0 + 16); f1[1] = lds_read8(ar1 + 16);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            if (ks + 2 < KS) {
                f0[(ks + 2) % 3] = lds_read8(ar0 + (ks + 2) * 16);
                f1[(ks + 2) % 3] = lds_read8(ar1 + (ks + 2) * 16);
            }
            const bf16x8 a0 = f0[ks % 3], a1 = f1[ks % 3];
            acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[0][ks], a0, acc[0][0], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[0][ks], a1, acc[1][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[1][ks], a0, acc[0][1], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[1][ks], a1, acc[1][1], 0, 0, 0);
            if constexpr (PREV) {
#pragma unroll
                for (int q = 0; q < 16 / KS; ++q) convert_piece(prev, ks * (16 / KS) + q);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    auto convert_all = [&](const f32x16 (&acc)[2][2]) {
#pragma unroll
        for (int piece = 0; piece < 16; ++piece) convert_piece(acc, piece);
    };

    const int step = (int)gridDim.x;
    int t = (int)blockIdx.x;
    u32x4v ra[8], rb[8];
    fetch(ra, t);
    fetch(rb, t + step);
    if (tid < WIDE_N / 4)
        *reinterpret_cast<float4 *>(&bias_s[tid * 4]) = a.bias ? *reinterpret_cast<const float4 *>(a.bias + tid * 4) : make_float4(0.f, 0.f, 0.f, 0.f);
    if (!mine) {                 // columns from K on stay zero in both buffers
        const u32x4v zero = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            *reinterpret_cast<u32x4v *>(&As0[(8 * i + srow) * STREAM_LROW + kp * 8]) = zero;
            *reinterpret_cast<u32x4v *>(&As1[(8 * i + srow) * STREAM_LROW + kp * 8]) = zero;
        }
    }
    stage(As0, ra);
    __syncthreads();
    f32x16 acc_a[2][2], acc_b[2][2];
    // tile t sits in the first buffer, tile t + step is on its way into rb
    fetch(ra, t + 2 * step);
    multiply(As0, acc_a, acc_b, std::false_type{});
    for (;;) {
        // acc_a holds tile t; tile t + step (if there is one) is on its way into rb
        if (t + step >= ntiles) {
            convert_all(acc_a);
            flush(t);
            break;
        }
        stage(As1, rb);
        __syncthreads();
        fetch(rb, t + 3 * step);
        multiply(As1, acc_b, acc_a, std::true_type{});
        flush(t);
        t += step;
        // acc_b holds tile t; tile t + step is on its way into ra
        if (t + step >= ntiles) {
            convert_all(acc_b);
            flush(t);
            break;
        }
        stage(As0, ra);
        __syncthreads();
        fetch(ra, t + 3 * step);
        multiply(As0, acc_a, acc_b, std::true_type{});
        flush(t);
        t += step;
    }
}

// The wave's weights are requested before the row count is read (they do not depend on it): the two round trips to
// memory overlap.  Columns 64 wave + 32 cb + lr, eight k from 16 ks + 8 half on (K is a multiple of 8).
template <int KS>
__device__ __forceinline__ void nt_stream_run(const NtArgs &a, uint16_t *stream_lds)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int half = lane >> 5, lr = lane & 31;
    const int K = a.K;
    bf16x8 wf[2][KS];
#pragma unroll
    for (int cb = 0; cb < 2; ++cb)
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int k = ks * 16 + 8 * half;
            const uint16_t *src = a.B + (int64_t)(64 * wave + 32 * cb + lr) * K + (k < K ? k : 0);
            const u32x4v x = *reinterpret_cast<const u32x4v *>(src);
            const u32x4v zero = {0u, 0u, 0u, 0u};
            wf[cb][ks] = __builtin_bit_cast(bf16x8, k < K ? x : zero);
        }
    asm volatile("" ::: "memory");      // (keeps the loads above from being moved below the branch on the row count)
    const int M = min(a.hdr[CR_HDR_N_DST], a.max_rows);
    if ((int)blockIdx.x * STREAM_ROWS >= M) return;
    const bool uniform = a.K0 == a.K || a.K0 % 128 == 0;
    if (M < STREAM_ROWS) nt_stream_body<KS, false, false>(a, M, stream_lds, wf);
    else if (uniform) nt_stream_body<KS, true, true>(a, M, stream_lds, wf);
    else nt_stream_body<KS, true, false>(a, M, stream_lds, wf);
}

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void gemm_nt_stream_kernel(NtArgs a)
{
    extern __shared__ __attribute__((aligned(16))) uint16_t stream_lds[];
    if (a.K <= 128) nt_stream_run<8>(a, stream_lds);
    else nt_stream_run<16>(a, stream_lds);
}

constexpr int NT_WIDE_MIN_ROWS = 16384;   // below this the 256-row workgroups leave most compute units idle

constexpr int NT_SMALL_ROWS = 2048;    // blocks of at most this many rows (by capacity) take the kernel above

// Wider tiles (NTILES = 4, 8) read the activations fewer times but measured slower on MI355X for the
// layer widths of this path (K = 256..512, N = 256): these products are bound by memory round trips
// and occupancy, not by the matrix cores, so the smallest tile at the highest occupancy wins.
constexpr int64_t NT_DEEP_MAX_BLOCKS = 512;   // at most two workgroups per compute unit and ...
constexpr int NT_DEEP_MIN_K = 768;            // ... a K loop of at least 24 steps: eight steps of prefetch

static void launch_nt(const NtArgs &a, hipStream_t s)
{
    // many rows, bf16 output only, K small enough for the weights to stay in registers: the streaming kernel
    if (a.max_rows >= NT_WIDE_MIN_ROWS && a.N == WIDE_N && a.K <= STREAM_KMAX && a.K % 8 == 0 && a.K0 % 8 == 0 && a.A1 != nullptr &&
        a.Cb != nullptr && a.C0 == nullptr && a.ldcb == a.N && (int64_t)a.max_rows * a.lda < (1ll << 29)) {
        static const bool ready = [] {
            return hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_nt_stream_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)STREAM_LDS_BYTES) == hipSuccess;
        }();
        if (ready) {
            const int64_t tiles = ceil_div(a.max_rows, STREAM_ROWS);
            hipLaunchKernelGGL(gemm_nt_stream_kernel, dim3((unsigned)(tiles < 256 ? tiles : 256)), dim3(256), STREAM_LDS_BYTES, s, a);
            return;
        }
    }
    // many rows against weights that fit one compute unit's LDS, bf16 output only: the weight-stationary kernel
    if (a.max_rows >= NT_WIDE_MIN_ROWS && a.N == WIDE_N && a.K0 % 8 == 0 && a.K % 8 == 0 && a.A1 != nullptr && a.Cb != nullptr &&
        a.C0 == nullptr && a.ldcb == a.N && a.lda < (1 << 20)) {
        static const bool ready = [] {
            return hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_nt_wide_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)WIDE_LDS_BYTES) == hipSuccess;
        }();
        if (ready) {
            hipLaunchKernelGGL(gemm_nt_wide_kernel, dim3((unsigned)ceil_div(a.max_rows, WIDE_ROWS)), dim3(256), WIDE_LDS_BYTES, s, a);
            return;
        }
    }
    // xcd_compact needs the grid rounded up to a multiple of eight blocks
    const unsigned ncol = (unsigned)(a.N / 64);
    if (a.max_rows <= NT_SMALL_ROWS) {
        hipLaunchKernelGGL(gemm_nt_small_kernel<false>, dim3(ncol, (unsigned)ceil_div(a.max_rows, 32)), dim3(256), 0, s, a, XentArgs{});
        return;
    }
    const dim3 grid(ncol, (unsigned)ceil_div(a.max_rows, 128) + (7 + ncol - 1) / ncol);
    if ((int64_t)grid.x * grid.y <= NT_DEEP_MAX_BLOCKS && a.K >= NT_DEEP_MIN_K) hipLaunchKernelGGL((gemm_nt_kernel<2, 8>), grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL((gemm_nt_kernel<2, 4>), grid, dim3(256), 0, s, a);
}

// ------------------------------------------------------------------------------------------------
// P[s][k][n] = sum_{m in split s} A[m][k] * Z[m][n]      (both operands strided along m).  Also the
// column sums of Z per split (bias gradient).
// Workgroup tile 128 (k) x 128 (n), four waves of 64 x 64; TN_BM rows of m per step (one barrier per step: taller
// steps spread its cost and the LDS round trip over more MFMAs).  Half of the
// threads stage A, half stage Z: a thread fetches one 8-column chunk of TN_BM / 8 consecutive rows and
// writes it transposed as eight 64-bit LDS stores (four m of one column each), so the MFMA operands
// are again 16-byte reads along m.  Global loads run three steps ahead in a register ring.
// ------------------------------------------------------------------------------------------------
struct TnArgs {
    const int32_t *hdr;
    int32_t max_rows;
    const uint16_t *A0, *A1;
    int64_t lda;
    int32_t K0, K2;
    const uint16_t *Z;       // [M][N]
    int32_t N;
    int32_t slots;           // partial slots available
    float *partial;          // [S][K2 + 1][N]: row K2 holds the column sums of Z (bias gradient)
};

// T = [buffer][operand: 0 = A, 1 = Z][m][column]: the tiles are staged as they come from memory (row-major);
// the transposition the MFMA operands need (eight consecutive m of one column per lane) is done by the LDS
// transpose read of gfx950.  Row stride 288 bytes: the four 32-byte row pieces a 16-lane group reads
// fall into disjoint banks.  `bid` is the workgroup's number among the `ntile` x (splits) workgroups of the product.
__device__ __forceinline__ void gemm_tn_body(const TnArgs &a, uint32_t bid, uint32_t ntile, uint16_t (&T)[2][2][TN_BM][TN_ROW])
{
    const int M = min(a.hdr[CR_HDR_N_DST], a.max_rows);
    // the tiles of one split run next to each other on one XCD (they share the split's rows of A and Z);
    // splits past the last row stay inactive, and the reduction skips them too
    uint32_t work;
    const int rows_per_split = rows_per_split_for(M, a.slots);
    if (!xcd_compact(bid, (uint32_t)((M + rows_per_split - 1) / rows_per_split) * ntile, work)) return;
    const int split = (int)(work / ntile), tile_id = (int)(work % ntile);
    const int m_begin = split * rows_per_split;
    const int m_end = min(M, m_begin + rows_per_split);
    const int n_tiles = (a.N + 127) / 128;
    const int k_tiles_part = (a.K0 + 127) / 128;   // k-tiles per operand part (self | agg): a tile never straddles the two
    const int kt = tile_id / n_tiles;
    const int part = kt / k_tiles_part;
    const int kp0 = (kt % k_tiles_part) * 128;     // first column of the tile inside its part
    const int k0 = part * a.K0 + kp0;              // first row of the output tile
    const int k_valid = min(128, a.K0 - kp0);
    const int n0 = (tile_id % n_tiles) * 128;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, lr = lane & 31;
    const int wk = wave >> 1, wn = wave & 1;

    // staging role: waves 0,1 stage A, waves 2,3 stage Z.  Buffer loads return zero past the end of the
    // split's rows (and for columns outside the tile), so no load sits under a branch and the loads of
    // three steps stay in flight together.
    const int op = tid >> 7;                       // 0: A, 1: Z (uniform per wave)
    const int st = tid & 127, mg = st >> 4, sc = (st & 15) * 8;
    // (op is the same for a whole wave; the descriptor is built from values the compiler can see are wave-uniform --
    // with a descriptor it takes for lane-dependent it wraps every load in a loop over the distinct descriptors and then
    // waits for nearly all earlier loads before each new one, which undoes the ring)
    const uint64_t base_v = reinterpret_cast<uint64_t>(op == 0 ? (part == 0 ? a.A0 : a.A1) : a.Z);
    const uint16_t *base = reinterpret_cast<const uint16_t *>(
        ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(base_v >> 32)) << 32) | (uint32_t)__builtin_amdgcn_readfirstlane((int)base_v));
    const uint32_t ld_bytes = (uint32_t)__builtin_amdgcn_readfirstlane((int)((op == 0 ? a.lda : (int64_t)a.N) * 2));
    const bool col_ok = op == 0 ? sc < k_valid : n0 + sc < a.N;
    const uint32_t col_bytes = (uint32_t)((op == 0 ? kp0 + sc : n0 + sc) * 2);
    const __amdgpu_buffer_rsrc_t rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(base), 0, (int)((uint32_t)m_end * ld_bytes), 0x00020000);

    constexpr int RPT = TN_BM / 8;                 // rows per thread and step: row group mg takes rows mg * RPT .. + RPT
    uint4 ring[3][RPT];
    auto fetch = [&](uint4 (&r)[RPT], int step) {
        const uint32_t mrow = (uint32_t)(m_begin + step * TN_BM + mg * RPT);
#pragma unroll
        for (int i = 0; i < RPT; ++i) {
            const uint32_t off = col_ok ? (mrow + i) * ld_bytes + col_bytes : 0xFFFFFFF0u;
            const u32x4v v = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)off, 0, 0);
            r[i] = make_uint4(v[0], v[1], v[2], v[3]);
        }
    };
    // a thread holds an 8-column chunk of RPT consecutive rows: plain 16-byte stores
    float cacc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};      // column sums of Z over this thread's rows (kt == 0 only)
    const bool do_colsum = kt == 0 && op == 1;
    auto stage = [&](const uint4 (&r)[RPT], int buf) {
#pragma unroll
        for (int i = 0; i < RPT; ++i) *reinterpret_cast<uint4 *>(&T[buf][op][mg * RPT + i][sc]) = r[i];
        if (do_colsum) {
#pragma unroll
            for (int i = 0; i < RPT; ++i) {
                cacc[0] += __uint_as_float(r[i].x << 16); cacc[1] += __uint_as_float(r[i].x & 0xFFFF0000u);
                cacc[2] += __uint_as_float(r[i].y << 16); cacc[3] += __uint_as_float(r[i].y & 0xFFFF0000u);
                cacc[4] += __uint_as_float(r[i].z << 16); cacc[5] += __uint_as_float(r[i].z & 0xFFFF0000u);
                cacc[6] += __uint_as_float(r[i].w << 16); cacc[7] += __uint_as_float(r[i].w & 0xFFFF0000u);
            }
        }
    };
    // MFMA operand of lane (lr, half) for the 32-column sub-tile at col0: rows m0 + 8 half .. + 8 of column
    // col0 + lr.  A 16-lane group reads a 4 (m) x 16 (columns) piece: lane i of the group supplies the address of
    // row i / 4, columns 4 (i % 4) .. + 4 and receives column i's four rows.
    const int tl = lane & 15, tcol = ((lane >> 4) & 1) * 16;
    auto operand = [&](int buf, int which, int col0, int m0) -> bf16x8 {
        const uint16_t *p = &T[buf][which][m0 + 8 * half + (tl >> 2)][col0 + tcol + 4 * (tl & 3)];
        const v4s16 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((v4s16 __attribute__((address_space(3))) *)p);
        const v4s16 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((v4s16 __attribute__((address_space(3))) *)(p + 4 * TN_ROW));
        typedef short v8s16 __attribute__((ext_vector_type(8)));
        const v8s16 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        return __builtin_bit_cast(bf16x8, both);
    };

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int nsteps = (m_end - m_begin + TN_BM - 1) / TN_BM;
    fetch(ring[0], 0);
    fetch(ring[1], 1);
    fetch(ring[2], 2);
    stage(ring[0], 0);
    __syncthreads();

    auto body = [&](int t, uint4 (&slot_next_fetch)[RPT], const uint4 (&slot_next_stage)[RPT]) {
        const int buf = t & 1;
        fetch(slot_next_fetch, t + 3);             // the slot that held step t (already staged)
#pragma unroll
        for (int kk = 0; kk < TN_BM / 16; ++kk) {
            bf16x8 x[2], z[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                x[i] = operand(buf, 0, wk * 64 + i * 32, kk * 16);
                z[i] = operand(buf, 1, wn * 64 + i * 32, kk * 16);
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x[i], z[j], acc[i][j], 0, 0, 0);
        }
        // (unconditional, also after the last step, where it stores the zeros that loads past the end return: with a
        // branch here the compiler sees a path on which a ring slot's loads are never waited for, and drains every
        // outstanding load at the head of the loop)
        stage(slot_next_stage, buf ^ 1);
        __syncthreads();
    };
    int t = 0;
    for (; t + 3 <= nsteps; t += 3) {
        body(t, ring[0], ring[1]);
        body(t + 1, ring[1], ring[2]);
        body(t + 2, ring[2], ring[0]);
    }
    if (t < nsteps) body(t, ring[0], ring[1]);
    if (t + 1 < nsteps) body(t + 1, ring[1], ring[2]);

    float *P = a.partial + (int64_t)split * (a.K2 + 1) * a.N;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int n = n0 + wn * 64 + j * 32 + lr;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int kl = wk * 64 + i * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
                if (kl < k_valid && n < a.N) P[(int64_t)(k0 + kl) * a.N + n] = acc[i][j][r];
            }
        }
    // bias gradient: the eight row groups' column sums meet in LDS and are added in a fixed order
    if (kt == 0) {
        float (*csum)[128] = reinterpret_cast<float (*)[128]>(&T[0][0][0][0]);     // the staging tiles are free now
        if (op == 1) {
#pragma unroll
            for (int c = 0; c < 8; ++c) csum[mg][sc + c] = cacc[c];
        }
        __syncthreads();
        if (tid < 128 && n0 + tid < a.N) {
            float tot = 0.f;
#pragma unroll
            for (int g8 = 0; g8 < 8; ++g8) tot += csum[g8][tid];
            P[(int64_t)a.K2 * a.N + n0 + tid] = tot;
        }
    }
}

__global__ __launch_bounds__(256) void gemm_tn_kernel(TnArgs a)
{
    __shared__ __attribute__((aligned(16))) uint16_t T[2][2][TN_BM][TN_ROW];
    gemm_tn_body(a, blockIdx.y * gridDim.x + blockIdx.x, gridDim.x, T);
}

// The two products of a layer's backward pass that need nothing from each other (weight gradient, input
// gradient) in one launch: both are short and bound by memory round trips, so side by side they take about as
// long as the longer one.  The first `tn_blocks` workgroups (a multiple of eight, so that both parts keep their
// XCD mapping) run the weight-gradient product, the rest the input-gradient product.
__global__ __launch_bounds__(256) void gemm_tn_nt_kernel(TnArgs t, NtArgs n, uint32_t tn_blocks, uint32_t tn_tiles, uint32_t nt_cols)
{
    __shared__ __attribute__((aligned(16))) uint16_t lds[2 * 2 * TN_BM * TN_ROW];
    static_assert(sizeof(lds) >= sizeof(uint16_t) * (2 * 128 * LDS_ROW + 2 * 64 * LDS_ROW), "the staging tiles of either product fit");
    if (blockIdx.x < tn_blocks) {
        gemm_tn_body(t, blockIdx.x, tn_tiles, *reinterpret_cast<uint16_t (*)[2][2][TN_BM][TN_ROW]>(lds));
    } else {
        gemm_nt_body<2, 4>(n, blockIdx.x - tn_blocks, nt_cols, *reinterpret_cast<uint16_t (*)[2][128][LDS_ROW]>(lds),
                           *reinterpret_cast<uint16_t (*)[2][64][LDS_ROW]>(lds + 2 * 128 * LDS_ROW));
    }
}

__global__ __launch_bounds__(256) void sgd_reduce_kernel(SgdArgs a)
{
    __shared__ float4 red[4][64];
    sgd_reduce_body(a, blockIdx.x, red);
}

__global__ __launch_bounds__(256) void refresh_shadows_kernel(const float *W, int F_in, int F_out, int F_pad, int N_pad, int n_op,
                                                              uint16_t *W_bf16, uint16_t *Wt_bf16)
{
    const int K2 = n_op * F_pad;
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

// arg-max of every root row against its label; the workgroup's count is added to a device counter
__global__ __launch_bounds__(256) void count_correct_kernel(const int32_t *hdr, int max_rows, const float *logits, int64_t ld,
                                                            int C, const int32_t *labels, const int32_t *root_ids, int32_t *count)
{
    __shared__ int hits[4];
    const int n = min(hdr[CR_HDR_N_DST], max_rows);
    const int row = blockIdx.x * 4 + threadIdx.x / WAVE;
    const int lane = lane_id();
    int hit = 0;
    if (row < n) {
        const float *z = logits + (int64_t)row * ld;
        float best = -INFINITY;
        int arg = 0x7FFFFFFF;
        for (int c = lane; c < C; c += WAVE) {
            const float x = z[c];
            if (x > best) { best = x; arg = c; }          // ascending c per lane: the first maximum stays
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const float ob = __shfl_xor(best, off);
            const int oa = __shfl_xor(arg, off);
            if (ob > best || (ob == best && oa < arg)) { best = ob; arg = oa; }
        }
        hit = arg == labels[root_ids[row]] ? 1 : 0;
    }
    if (lane == 0) hits[threadIdx.x / WAVE] = hit;
    __syncthreads();
    if (threadIdx.x == 0) {
        const int s = hits[0] + hits[1] + hits[2] + hits[3];
        if (s) atomicAdd(count, s);
    }
}

static void split_plan(int F_pad, int N_pad, int n_op, int max_rows, int &rows_per_split, int &n_splits)
{
    const int tiles = (int)(n_op * ceil_div(F_pad, 128) * ceil_div(N_pad, 128));
    // one workgroup per compute unit: with two (the kernel's residency) the product itself is no faster, and the partial
    // sums -- written once and read once by the reduction -- double
    int target = 256 / tiles;
    if (target < 1) target = 1;
    if (target > 128) target = 128;
    int rows = (int)round_up(ceil_div(max_rows, target), 96);
    if (rows < 96) rows = 96;
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
    CR_REQUIRE(L->n_operands == 1 || L->n_operands == 2, CR_ERR_INVALID_ARG, "layer n_operands = %d must be 1 or 2", L->n_operands);
    CR_REQUIRE(L->W && L->W_bf16 && L->Wt_bf16, CR_ERR_INVALID_ARG, "layer has a NULL array");
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
    const int64_t n = (int64_t)layer->n_operands * F_pad * N_pad;
    hipLaunchKernelGGL(refresh_shadows_kernel, dim3((unsigned)ceil_div(n, 256)), dim3(256), 0, static_cast<hipStream_t>(stream),
                       layer->W, layer->F_in, layer->F_out, F_pad, N_pad, layer->n_operands, layer->W_bf16, layer->Wt_bf16);
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
    const int n_op = layer->n_operands;
    CR_REQUIRE(agg && aligned16(h_self) && aligned16(agg), CR_ERR_INVALID_ARG, "h_self / agg must be 16-byte aligned device pointers");
    CR_REQUIRE((h_self != nullptr) == (n_op == 2), CR_ERR_INVALID_ARG, "h_self must be given for a two-operand layer and NULL for a one-operand layer");
    CR_REQUIRE(ld_in >= F_pad && ld_in % 8 == 0, CR_ERR_INVALID_ARG, "ld_in = %lld must be a multiple of 8 and >= %d", (long long)ld_in, F_pad);
    CR_REQUIRE(out || out_bf16, CR_ERR_INVALID_ARG, "no output requested");
    CR_REQUIRE(aligned16(out) && aligned16(out_bf16), CR_ERR_INVALID_ARG, "outputs must be 16-byte aligned");
    if (dry_run()) return CR_OK;
    NtArgs a;
    a.hdr = hdr; a.max_rows = max_rows; a.A0 = n_op == 2 ? h_self : agg; a.A1 = agg; a.lda = ld_in; a.K0 = F_pad; a.K = n_op * F_pad;
    a.B = layer->Wt_bf16; a.N = N_pad; a.bias = layer->bias; a.relu = relu ? 1 : 0;
    a.C0 = out; a.C1 = nullptr; a.ldc = N_pad; a.N0 = N_pad; a.Cb = out_bf16; a.ldcb = N_pad;
    launch_nt(a, static_cast<hipStream_t>(stream));
    CR_LAUNCH_CHECK();
    return CR_OK;
}

extern "C" cr_status cr_sage_linear_fwd_xent(const cr_sage_layer *layer, const int32_t *hdr, int32_t max_rows,
                                             const uint16_t *h_self, const uint16_t *agg, int64_t ld_in, float *logits,
                                             int32_t n_classes, const int32_t *labels, const int32_t *root_ids, float *loss,
                                             float *row_loss, uint16_t *d_logits_bf16, void *scratch, void *stream)
{
    int F_pad, N_pad;
    cr_status st = check_layer(layer, F_pad, N_pad);
    if (st != CR_OK) return st;
    CR_REQUIRE(hdr != nullptr && max_rows >= 1, CR_ERR_INVALID_ARG, "hdr must not be NULL and max_rows must be positive");
    const int n_op = layer->n_operands;
    CR_REQUIRE(agg && aligned16(h_self) && aligned16(agg), CR_ERR_INVALID_ARG, "h_self / agg must be 16-byte aligned device pointers");
    CR_REQUIRE((h_self != nullptr) == (n_op == 2), CR_ERR_INVALID_ARG, "h_self must be given for a two-operand layer and NULL for a one-operand layer");
    CR_REQUIRE(ld_in >= F_pad && ld_in % 8 == 0, CR_ERR_INVALID_ARG, "ld_in = %lld must be a multiple of 8 and >= %d", (long long)ld_in, F_pad);
    CR_REQUIRE(logits && d_logits_bf16 && aligned16(logits) && aligned16(d_logits_bf16), CR_ERR_INVALID_ARG,
               "logits / d_logits_bf16 must be 16-byte aligned device pointers");
    CR_REQUIRE(labels && root_ids && loss && row_loss, CR_ERR_INVALID_ARG, "labels / root_ids / loss / row_loss must not be NULL");
    CR_REQUIRE(n_classes >= 1 && n_classes <= layer->F_out, CR_ERR_INVALID_ARG, "need 1 <= n_classes <= F_out");
    CR_REQUIRE(scratch != nullptr && aligned16(scratch), CR_ERR_INVALID_ARG, "scratch must be a 16-byte aligned device pointer");
    if (dry_run()) return CR_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    NtArgs a;
    a.hdr = hdr; a.max_rows = max_rows; a.A0 = n_op == 2 ? h_self : agg; a.A1 = agg; a.lda = ld_in; a.K0 = F_pad; a.K = n_op * F_pad;
    a.B = layer->Wt_bf16; a.N = N_pad; a.bias = layer->bias; a.relu = 0;
    a.C0 = logits; a.C1 = nullptr; a.ldc = N_pad; a.N0 = N_pad; a.Cb = nullptr; a.ldcb = N_pad;
    if (N_pad == 64 && max_rows <= NT_SMALL_ROWS) {
        XentArgs x;
        x.n_classes = n_classes; x.labels = labels; x.root_ids = root_ids; x.loss = loss; x.row_loss = row_loss;
        x.d_logits_bf16 = d_logits_bf16; x.acc = static_cast<unsigned long long *>(scratch);
        hipLaunchKernelGGL(gemm_nt_small_kernel<true>, dim3(1, (unsigned)ceil_div(max_rows, 32)), dim3(256), 0, s, a, x);
    } else {
        launch_nt(a, s);
        hipLaunchKernelGGL(xent_rows_kernel, dim3((unsigned)ceil_div(max_rows, 4)), dim3(256), 0, s, hdr, max_rows, logits, (int64_t)N_pad,
                           n_classes, labels, root_ids, row_loss, (float *)nullptr, d_logits_bf16);
        hipLaunchKernelGGL(xent_mean_kernel, dim3(1), dim3(1024), 0, s, hdr, max_rows, row_loss, loss);
    }
    CR_LAUNCH_CHECK();
    return CR_OK;
}

extern "C" cr_status cr_sage_linear_bwd_workspace_bytes(int32_t F_in, int32_t F_out, int32_t max_rows, size_t *bytes)
{
    CR_REQUIRE(F_in >= 1 && F_in <= 8192 && F_out >= 1 && F_out <= 8192, CR_ERR_INVALID_ARG, "layer dims (%d, %d) outside 1..8192", F_in, F_out);
    CR_REQUIRE(max_rows >= 1 && bytes != nullptr, CR_ERR_INVALID_ARG, "max_rows must be positive and bytes not NULL");
    const int F_pad = (int)round_up(F_in, 32), N_pad = (int)round_up(F_out, 64);
    int rows, splits, splits1;
    split_plan(F_pad, N_pad, 2, max_rows, rows, splits);
    split_plan(F_pad, N_pad, 1, max_rows, rows, splits1);       // enough for either kind of layer
    const size_t need2 = (size_t)splits * (2 * F_pad + 1) * N_pad, need1 = (size_t)splits1 * (F_pad + 1) * N_pad;
    Carver c(nullptr);
    c.take<float>(need2 > need1 ? need2 : need1);
    *bytes = c.bytes();
    return CR_OK;
}

cr_status cr::linear_bwd_products(const cr_sage_layer *layer, const int32_t *hdr, int32_t max_rows, const uint16_t *h_self,
                                  const uint16_t *agg, int64_t ld_in, const uint16_t *dz_bf16, float lr, float weight_decay,
                                  float *d_self, float *d_agg, uint16_t *d_in_bf16, float *dW_out, float *db_out, void *ws,
                                  size_t ws_bytes, void *stream, SgdArgs *deferred)
{
    int F_pad, N_pad;
    cr_status st = check_layer(layer, F_pad, N_pad);
    if (st != CR_OK) return st;
    CR_REQUIRE(hdr != nullptr && max_rows >= 1, CR_ERR_INVALID_ARG, "hdr must not be NULL and max_rows must be positive");
    const int n_op = layer->n_operands;
    CR_REQUIRE(agg && dz_bf16 && aligned16(h_self) && aligned16(agg) && aligned16(dz_bf16), CR_ERR_INVALID_ARG,
               "h_self / agg / dz_bf16 must be 16-byte aligned device pointers");
    CR_REQUIRE((h_self != nullptr) == (n_op == 2), CR_ERR_INVALID_ARG, "h_self must be given for a two-operand layer and NULL for a one-operand layer");
    CR_REQUIRE(n_op == 2 || d_self == nullptr, CR_ERR_INVALID_ARG, "a one-operand layer has no d_self");
    CR_REQUIRE(ld_in >= F_pad && ld_in % 8 == 0, CR_ERR_INVALID_ARG, "ld_in = %lld must be a multiple of 8 and >= %d", (long long)ld_in, F_pad);
    CR_REQUIRE(n_op == 1 || (d_self == nullptr) == (d_agg == nullptr), CR_ERR_INVALID_ARG, "d_self and d_agg must be given together");
    CR_REQUIRE(aligned16(d_self) && aligned16(d_agg) && aligned16(d_in_bf16), CR_ERR_INVALID_ARG, "d_self / d_agg / d_in_bf16 must be 16-byte aligned");
    CR_REQUIRE(lr == lr && weight_decay == weight_decay, CR_ERR_INVALID_ARG, "lr / weight_decay is NaN");
    CR_REQUIRE(!(d_agg || d_in_bf16) || (n_op * F_pad) % 64 == 0, CR_ERR_UNSUPPORTED,
               "input gradients of a one-operand layer need F_in rounded up to 32 to be a multiple of 64");
    CR_REQUIRE((int64_t)max_rows * ld_in * 2 < 0x7FFFFFFFll && (int64_t)max_rows * N_pad * 2 < 0x7FFFFFFFll, CR_ERR_UNSUPPORTED,
               "operand of %d rows exceeds the 2 GiB reach of 32-bit buffer offsets", max_rows);
    int rows, splits;
    split_plan(F_pad, N_pad, n_op, max_rows, rows, splits);
    Carver c(ws);
    float *partial = c.take<float>((size_t)splits * (n_op * F_pad + 1) * N_pad);
    CR_REQUIRE(ws != nullptr && aligned16(ws), CR_ERR_INVALID_ARG, "workspace must be a 16-byte aligned device pointer");
    CR_REQUIRE(ws_bytes >= c.bytes(), CR_ERR_CAPACITY, "workspace of %zu bytes, %zu needed", ws_bytes, c.bytes());
    if (dry_run()) return CR_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);

    const unsigned tn_tiles = (unsigned)(n_op * ceil_div(F_pad, 128) * ceil_div(N_pad, 128));
    if (d_agg || d_in_bf16) {
        // the input-gradient product shares the launch and the 512 resident workgroup slots: fewer, longer splits so
        // that both parts fit one round (its tiles counted at ~0.7 of the capacity, the usual fill of a sampled block)
        const int64_t nt_share = (int64_t)(n_op * F_pad / 64) * ceil_div(max_rows, 128) * 7 / 10;
        const int64_t room = (512 - nt_share) / tn_tiles;
        if (room >= 8 && room < splits) splits = (int)room;
    }
    TnArgs t;
    t.hdr = hdr; t.max_rows = max_rows; t.A0 = n_op == 2 ? h_self : agg; t.A1 = agg; t.lda = ld_in; t.K0 = F_pad; t.K2 = n_op * F_pad;
    t.Z = dz_bf16; t.N = N_pad; t.slots = splits; t.partial = partial;
    if (d_agg || d_in_bf16) {   // also the gradient w.r.t. the layer's inputs (weights from before the step), in the same launch
        NtArgs a;
        a.hdr = hdr; a.max_rows = max_rows; a.A0 = dz_bf16; a.A1 = nullptr; a.lda = N_pad; a.K0 = N_pad; a.K = N_pad;
        a.B = layer->W_bf16; a.N = n_op * F_pad; a.bias = nullptr; a.relu = 0;
        a.C0 = n_op == 2 ? d_self : d_agg; a.C1 = d_agg; a.ldc = F_pad; a.N0 = F_pad; a.Cb = d_in_bf16; a.ldcb = n_op * F_pad;
        const unsigned nt_cols = (unsigned)(a.N / 64);
        const unsigned tn_blocks = (unsigned)round_up((int64_t)tn_tiles * splits + 7, 8);
        const unsigned nt_blocks = (unsigned)round_up((int64_t)nt_cols * ceil_div(max_rows, 128) + 7, 8);
        hipLaunchKernelGGL(gemm_tn_nt_kernel, dim3(tn_blocks + nt_blocks), dim3(256), 0, s, t, a, tn_blocks, tn_tiles, nt_cols);
    } else {
        hipLaunchKernelGGL(gemm_tn_kernel, dim3(tn_tiles, (unsigned)splits + (7 + tn_tiles - 1) / tn_tiles), dim3(256), 0, s, t);
    }
    SgdArgs g;
    g.hdr = hdr; g.max_rows = max_rows; g.n_splits = splits; g.partial = partial;
    g.F_in = layer->F_in; g.F_out = layer->F_out; g.F_pad = F_pad; g.N_pad = N_pad; g.n_op = n_op; g.W = layer->W; g.bias = layer->bias;
    g.W_bf16 = layer->W_bf16; g.Wt_bf16 = layer->Wt_bf16; g.lr = lr; g.wd = weight_decay; g.dW_out = dW_out; g.db_out = db_out;
    if (deferred) *deferred = g;
    else hipLaunchKernelGGL(sgd_reduce_kernel, dim3(sgd_reduce_blocks(F_pad, N_pad, n_op)), dim3(256), 0, s, g);
    CR_LAUNCH_CHECK();
    return CR_OK;
}

extern "C" cr_status cr_sage_linear_bwd(const cr_sage_layer *layer, const int32_t *hdr, int32_t max_rows,
                                        const uint16_t *h_self, const uint16_t *agg, int64_t ld_in,
                                        const uint16_t *dz_bf16, float lr, float weight_decay, float *d_self,
                                        float *d_agg, uint16_t *d_in_bf16, float *dW_out, float *db_out, void *ws,
                                        size_t ws_bytes, void *stream)
{
    return linear_bwd_products(layer, hdr, max_rows, h_self, agg, ld_in, dz_bf16, lr, weight_decay, d_self, d_agg, d_in_bf16,
                               dW_out, db_out, ws, ws_bytes, stream, nullptr);
}

extern "C" cr_status cr_sage_linear_bwd_input(const cr_sage_layer *layer, const int32_t *hdr, int32_t max_rows,
                                              const uint16_t *dz_bf16, float *d_self, float *d_agg, uint16_t *d_in_bf16,
                                              void *stream)
{
    int F_pad, N_pad;
    cr_status st = check_layer(layer, F_pad, N_pad);
    if (st != CR_OK) return st;
    CR_REQUIRE(hdr != nullptr && max_rows >= 1, CR_ERR_INVALID_ARG, "hdr must not be NULL and max_rows must be positive");
    CR_REQUIRE(dz_bf16 && aligned16(dz_bf16), CR_ERR_INVALID_ARG, "dz_bf16 must be a 16-byte aligned device pointer");
    const int n_op = layer->n_operands;
    CR_REQUIRE(n_op == 2 || d_self == nullptr, CR_ERR_INVALID_ARG, "a one-operand layer has no d_self");
    CR_REQUIRE(n_op == 1 || (d_self == nullptr) == (d_agg == nullptr), CR_ERR_INVALID_ARG, "d_self and d_agg must be given together");
    CR_REQUIRE(d_agg || d_in_bf16, CR_ERR_INVALID_ARG, "no output requested");
    CR_REQUIRE(aligned16(d_self) && aligned16(d_agg) && aligned16(d_in_bf16), CR_ERR_INVALID_ARG, "d_self / d_agg / d_in_bf16 must be 16-byte aligned");
    CR_REQUIRE((n_op * F_pad) % 64 == 0, CR_ERR_UNSUPPORTED, "input gradients of a one-operand layer need F_in rounded up to 32 to be a multiple of 64");
    if (dry_run()) return CR_OK;
    NtArgs a;
    a.hdr = hdr; a.max_rows = max_rows; a.A0 = dz_bf16; a.A1 = nullptr; a.lda = N_pad; a.K0 = N_pad; a.K = N_pad;
    a.B = layer->W_bf16; a.N = n_op * F_pad; a.bias = nullptr; a.relu = 0;
    a.C0 = n_op == 2 ? d_self : d_agg; a.C1 = d_agg; a.ldc = F_pad; a.N0 = F_pad; a.Cb = d_in_bf16; a.ldcb = n_op * F_pad;
    launch_nt(a, static_cast<hipStream_t>(stream));
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

namespace cr {
// acc[0] += value * rows, acc[1] += rows, acc[2] = their ratio (one thread: the calls of a pass are ordered on their stream)
__global__ void mean_accumulate_kernel(const int32_t *hdr, int max_rows, const float *value, double *acc)
{
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    const int n = min(hdr[CR_HDR_N_DST], max_rows);
    if (n <= 0) return;
    const double sum = acc[0] + (double)value[0] * (double)n, rows = acc[1] + (double)n;
    acc[0] = sum;
    acc[1] = rows;
    acc[2] = sum / rows;
}
}  // namespace cr

extern "C" cr_status cr_mean_accumulate(const int32_t *hdr, int32_t max_rows, const float *value, double *acc, void *stream)
{
    CR_REQUIRE(hdr != nullptr && max_rows >= 1, CR_ERR_INVALID_ARG, "hdr must not be NULL and max_rows must be positive");
    CR_REQUIRE(value != nullptr && acc != nullptr, CR_ERR_INVALID_ARG, "value / acc must not be NULL");
    CR_REQUIRE((reinterpret_cast<uintptr_t>(acc) & 7u) == 0, CR_ERR_INVALID_ARG, "acc must be 8-byte aligned");
    if (dry_run()) return CR_OK;
    hipLaunchKernelGGL(mean_accumulate_kernel, dim3(1), dim3(64), 0, static_cast<hipStream_t>(stream), hdr, max_rows, value, acc);
    CR_LAUNCH_CHECK();
    return CR_OK;
}

extern "C" cr_status cr_count_correct(const int32_t *hdr, int32_t max_rows, const float *logits, int64_t ld,
                                      int32_t n_classes, const int32_t *labels, const int32_t *root_ids,
                                      int32_t *count, void *stream)
{
    CR_REQUIRE(hdr != nullptr && max_rows >= 1, CR_ERR_INVALID_ARG, "hdr must not be NULL and max_rows must be positive");
    CR_REQUIRE(logits && labels && root_ids && count, CR_ERR_INVALID_ARG, "logits / labels / root_ids / count must not be NULL");
    CR_REQUIRE(n_classes >= 1 && ld >= n_classes, CR_ERR_INVALID_ARG, "need 1 <= n_classes <= ld");
    if (dry_run()) return CR_OK;
    hipLaunchKernelGGL(count_correct_kernel, dim3((unsigned)ceil_div(max_rows, 4)), dim3(256), 0, static_cast<hipStream_t>(stream), hdr,
                       max_rows, logits, ld, n_classes, labels, root_ids, count);
    CR_LAUNCH_CHECK();
    return CR_OK;
}
