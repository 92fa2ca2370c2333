/*
 * oracle.c -- plain, single-threaded CPU statement of the COMM-RAND hot path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct model
 * that the GPU library is checked against.  It shares no code, header, table
 * or helper with the HIP sources and must never be called from the product
 * path; only the test-suite, the smoke check and the benchmark's cpu_baseline
 * leg load it.
 *
 * What it states (paper = "Efficient GNN Training Through Structure-Aware
 * Randomized Mini-batching", COMM-RAND):
 *   - Step-1 of Algorithm 1 (root node partitioning) under the policies of
 *     Table 1 and the mix knob of Section 4.1      -> orc_build_batches
 *   - Step-2 of Algorithm 1 (sub-graph construction) with the intra-community
 *     probability knob p of Section 4.2            -> orc_sample_hop
 *   - the message-passing layer of Eq. 1 in its GraphSAGE-mean form, the
 *     loss on root labels (Section 2) and the exact backward of both
 *                                                   -> orc_gather_mean*, orc_sage_linear_*,
 *                                                      orc_softmax_xent
 * The paper fixes the policy level only; the random stream, the
 * without-replacement rule and the block layout are this build's readings and
 * are written out next to each function.
 *
 * Floating point: every sum is accumulated in double.  Where the GPU path
 * feeds bf16 operands to its matrix cores the caller asks for the same operand
 * rounding here (round-to-nearest-even on the fp32 bit pattern); accumulation
 * stays in double.
 *
 * Threads: the library the tests load is built without OpenMP and runs on one
 * thread.  The "#pragma omp parallel for" lines sit on loops over destination /
 * output rows whose iterations are independent (every output element is still
 * one thread's sum, in the same order); they take effect only in the second
 * build (-fopenmp) that the benchmark times as its all-cores CPU baseline.
 *
 * Parity pins: every function below is pinned by tests/test_oracle_*.py
 * (known-answer vectors, closed forms, brute force, dense-matrix identities,
 * finite differences).  Nothing here is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ */
/* Random stream: Philox4x32-10 (Salmon et al., "Parallel random      */
/* numbers: as easy as 1, 2, 3", SC'11).                               */
/* ------------------------------------------------------------------ */

void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Domains of the stream (4 bits of counter word 3). */
enum { DOM_COMMUNITY = 0, DOM_NODE = 1, DOM_NEIGHBOUR = 2 };

/* One block of four words for (seed, epoch, batch, layer, node, slot/4). */
static void stream_block(uint64_t seed, uint32_t epoch, uint32_t domain, uint32_t layer,
                         uint32_t batch, uint32_t node, uint32_t slot_block, uint32_t out[4])
{
    uint32_t ctr[4], key[2];
    ctr[0] = slot_block;
    ctr[1] = node;
    ctr[2] = batch;
    ctr[3] = (epoch << 8) | (domain << 4) | layer;
    key[0] = (uint32_t)(seed & 0xFFFFFFFFu);
    key[1] = (uint32_t)(seed >> 32);
    orc_philox4x32_10(ctr, key, out);
}

/* 64-bit shuffle key of a community (domain 0) or a node (domain 1). */
uint64_t orc_shuffle_key(uint64_t seed, uint32_t epoch, uint32_t domain, uint32_t id)
{
    uint32_t w[4];
    stream_block(seed, epoch, domain, 0, 0, id, 0, w);
    return ((uint64_t)w[0] << 32) | w[1];
}

/* 32-bit word of adjacency slot `slot` of node `node`. */
uint32_t orc_slot_word(uint64_t seed, uint32_t epoch, uint32_t batch, uint32_t layer,
                       uint32_t node, uint32_t slot)
{
    uint32_t w[4];
    stream_block(seed, epoch, DOM_NEIGHBOUR, layer, batch, node, slot >> 2, w);
    return w[slot & 3];
}

/* ------------------------------------------------------------------ */
/* Step-1: root node partitioning (Algorithm 1 Step-1; Section 4.1;    */
/* Table 1).                                                           */
/*                                                                     */
/* policy 0 = NORAND-ROOTS : the training set as given, every epoch.   */
/* policy 1 = COMM-RAND    : shuffle the communities present in the    */
/*            training set as whole blocks, merge every `mix`          */
/*            consecutive ones of that shuffled order into a           */
/*            super-block (the last may be short), shuffle inside each */
/*            super-block.  mix = 1 is COMM-RAND-MIX-0%.               */
/* policy 2 = RAND-ROOTS   : one uniform shuffle of the whole set.     */
/*                                                                     */
/* A shuffle is "sort by an independent random key"; equal keys fall   */
/* back to the smaller id, so the result is a function of the keys     */
/* alone.  Mini-batches are consecutive slices of the result.          */
/* ------------------------------------------------------------------ */

typedef struct { uint64_t key; int32_t id; } keyed_id;

static int cmp_keyed_id(const void *a, const void *b)
{
    const keyed_id *x = (const keyed_id *)a, *y = (const keyed_id *)b;
    if (x->key != y->key) return x->key < y->key ? -1 : 1;
    if (x->id != y->id) return x->id < y->id ? -1 : 1;
    return 0;
}

typedef struct { int32_t block; uint64_t key; int32_t id; } blocked_id;

static int cmp_blocked_id(const void *a, const void *b)
{
    const blocked_id *x = (const blocked_id *)a, *y = (const blocked_id *)b;
    if (x->block != y->block) return x->block < y->block ? -1 : 1;
    if (x->key != y->key) return x->key < y->key ? -1 : 1;
    if (x->id != y->id) return x->id < y->id ? -1 : 1;
    return 0;
}

/* returns 0, or -1 on bad arguments / out of memory */
int orc_build_batches(int policy, int32_t mix, uint64_t seed, uint32_t epoch,
                      const int32_t *train_ids, int64_t n_train,
                      const int32_t *comm, int32_t n_comm, int32_t *perm)
{
    if (policy < 0 || policy > 2 || n_train < 0 || n_comm < 1) return -1;
    if (policy == 0) {
        for (int64_t i = 0; i < n_train; ++i) perm[i] = train_ids[i];
        return 0;
    }
    if (policy == 1 && mix < 1) return -1;

    /* super-block number of every community */
    int32_t *block_of = (int32_t *)calloc((size_t)n_comm, sizeof(int32_t));
    if (!block_of) return -1;
    if (policy == 1) {
        char *present = (char *)calloc((size_t)n_comm, 1);
        keyed_id *order = (keyed_id *)malloc(sizeof(keyed_id) * (size_t)n_comm);
        if (!present || !order) { free(present); free(order); free(block_of); return -1; }
        for (int64_t i = 0; i < n_train; ++i) present[comm[train_ids[i]]] = 1;
        int32_t n_present = 0;
        for (int32_t c = 0; c < n_comm; ++c)
            if (present[c]) {
                order[n_present].key = orc_shuffle_key(seed, epoch, DOM_COMMUNITY, (uint32_t)c);
                order[n_present].id = c;
                ++n_present;
            }
        qsort(order, (size_t)n_present, sizeof(keyed_id), cmp_keyed_id);
        for (int32_t r = 0; r < n_present; ++r) block_of[order[r].id] = r / mix;
        free(present);
        free(order);
    }
    /* policy 2: every community in super-block 0 */

    blocked_id *items = (blocked_id *)malloc(sizeof(blocked_id) * (size_t)(n_train ? n_train : 1));
    if (!items) { free(block_of); return -1; }
    for (int64_t i = 0; i < n_train; ++i) {
        int32_t v = train_ids[i];
        items[i].block = block_of[comm[v]];
        items[i].key = orc_shuffle_key(seed, epoch, DOM_NODE, (uint32_t)v);
        items[i].id = v;
    }
    qsort(items, (size_t)n_train, sizeof(blocked_id), cmp_blocked_id);
    for (int64_t i = 0; i < n_train; ++i) perm[i] = items[i].id;
    free(items);
    free(block_of);
    return 0;
}

/* ------------------------------------------------------------------ */
/* Step-2: biased neighbourhood sampling (Algorithm 1 Step-2;          */
/* Section 4.2; Section 5 "Software and implementation": unnormalised  */
/* edge weight p for intra-community, 1-p for inter-community edges).  */
/*                                                                     */
/* Without-replacement rule: successive sampling proportional to       */
/* weight, realised with exponential clocks (Efraimidis & Spirakis):   */
/* slot j gets clock E_j / w_j with E_j = -log2(U_j); the `fanout`     */
/* smallest clocks win.  With two weight classes E_j/w_j is ordered    */
/* like E_j * w_other, so no division is needed.  All of it is integer */
/* arithmetic so that any machine computes the same set.               */
/* ------------------------------------------------------------------ */

/* E(r) = -log2((2r+1) / 2^33) in Q24 fixed point, bit by bit. */
uint32_t orc_exp_clock_q24(uint32_t r)
{
    uint64_t x = 2 * (uint64_t)r + 1;           /* odd, in [1, 2^33) */
    int t = 63;
    while (!((x >> t) & 1)) --t;                /* floor(log2 x), 0..32 */
    uint64_t y = (x << (63 - t)) >> 32;         /* mantissa in [2^31, 2^32): Q1.31 in [1,2) */
    uint32_t frac = 0;
    for (int i = 0; i < 24; ++i) {
        uint64_t y2 = y * y;                    /* Q2.62 in [1,4) */
        if (y2 >> 63) { frac = (frac << 1) | 1; y = y2 >> 32; }
        else          { frac = (frac << 1);     y = y2 >> 31; }
    }
    return ((uint32_t)(33 - t) << 24) - frac;
}

/* Sampling key of one adjacency slot.  q_in = round(p * 65536). */
uint64_t orc_slot_key(uint32_t r, int intra, uint32_t q_in)
{
    uint32_t q_out = 65536u - q_in;
    if (q_in == q_out) return (uint64_t)r;                                   /* p = 0.5 : uniform */
    if (q_out == 0) return (intra ? 0 : ((uint64_t)1 << 62)) + (uint64_t)r;  /* p = 1 : intra first */
    return (uint64_t)orc_exp_clock_q24(r) * (uint64_t)(intra ? q_out : q_in);
}

typedef struct { uint64_t key; int32_t slot; } keyed_slot;

static int cmp_keyed_slot(const void *a, const void *b)
{
    const keyed_slot *x = (const keyed_slot *)a, *y = (const keyed_slot *)b;
    if (x->key != y->key) return x->key < y->key ? -1 : 1;
    if (x->slot != y->slot) return x->slot < y->slot ? -1 : 1;
    return 0;
}

static int cmp_int32(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/*
 * One hop: expand the destination rows dst_ids[0..n_dst) of GNN layer `layer`.
 *
 *   graph     : CSR (indptr int64[N+1], indices int32), comm int32[N]
 *   strict    : 1 = never take an inter-community neighbour when p = 1
 *               (rows may come out short or empty), 0 = fill up to
 *               min(fanout, degree) with inter-community ones after every
 *               intra-community neighbour has been taken
 *   pos_map   : caller scratch int32[N], all -1 on entry and on return
 *   out_indptr[n_dst+1], out_indices[<= n_dst*fanout] (positions in out_src),
 *   out_src[<= n_dst*(1+fanout)] (global ids; first n_dst are dst_ids, then
 *   every new neighbour in order of first appearance: rows ascending, slots
 *   ascending), *out_n_src.
 *   out_slots (may be NULL): the chosen adjacency slot of every edge.
 * returns nnz, or -1 on error.
 */
int64_t orc_sample_hop(const int64_t *indptr, const int32_t *indices, const int32_t *comm,
                       const int32_t *dst_ids, int32_t n_dst, int32_t fanout,
                       uint32_t q_in, int strict, uint64_t seed, uint32_t epoch,
                       uint32_t batch, uint32_t layer, int32_t *pos_map,
                       int32_t *out_indptr, int32_t *out_indices, int32_t *out_src,
                       int32_t *out_n_src, int32_t *out_slots)
{
    if (fanout < 1 || q_in < 32768u || q_in > 65536u) return -1;
    int64_t max_deg = 0;
    for (int32_t i = 0; i < n_dst; ++i) {
        int64_t d = indptr[dst_ids[i] + 1] - indptr[dst_ids[i]];
        if (d > max_deg) max_deg = d;
    }
    keyed_slot *cand = (keyed_slot *)malloc(sizeof(keyed_slot) * (size_t)(max_deg ? max_deg : 1));
    int32_t *chosen = (int32_t *)malloc(sizeof(int32_t) * (size_t)fanout);
    if (!cand || !chosen) { free(cand); free(chosen); return -1; }

    int32_t n_src = 0;
    for (int32_t i = 0; i < n_dst; ++i) { out_src[n_src] = dst_ids[i]; pos_map[dst_ids[i]] = n_src; ++n_src; }

    int64_t nnz = 0;
    out_indptr[0] = 0;
    for (int32_t i = 0; i < n_dst; ++i) {
        int32_t v = dst_ids[i];
        int64_t base = indptr[v];
        int32_t deg = (int32_t)(indptr[v + 1] - base);
        for (int32_t j = 0; j < deg; ++j) {
            int32_t u = indices[base + j];
            uint32_t r = orc_slot_word(seed, epoch, batch, layer, (uint32_t)v, (uint32_t)j);
            cand[j].key = orc_slot_key(r, comm[u] == comm[v], q_in);
            cand[j].slot = j;
        }
        qsort(cand, (size_t)deg, sizeof(keyed_slot), cmp_keyed_slot);
        int32_t k = deg < fanout ? deg : fanout;
        int32_t taken = 0;
        for (int32_t t = 0; t < k; ++t) {
            if (strict && q_in == 65536u && cand[t].key >= ((uint64_t)1 << 62)) break;
            chosen[taken++] = cand[t].slot;
        }
        qsort(chosen, (size_t)taken, sizeof(int32_t), cmp_int32);
        for (int32_t t = 0; t < taken; ++t) {
            int32_t u = indices[base + chosen[t]];
            if (pos_map[u] < 0) { pos_map[u] = n_src; out_src[n_src++] = u; }
            out_indices[nnz] = pos_map[u];
            if (out_slots) out_slots[nnz] = chosen[t];
            ++nnz;
        }
        out_indptr[i + 1] = (int32_t)nnz;
    }
    for (int32_t s = 0; s < n_src; ++s) pos_map[out_src[s]] = -1;
    *out_n_src = n_src;
    free(cand);
    free(chosen);
    return nnz;
}

/* Transposed block: for every source position the destination rows that
 * contain it, ascending (the gradient of the mean flows along these). */
void orc_transpose_block(int32_t n_dst, int32_t n_src, const int32_t *indptr,
                         const int32_t *indices, int32_t *t_indptr, int32_t *t_indices)
{
    for (int32_t s = 0; s <= n_src; ++s) t_indptr[s] = 0;
    for (int32_t e = 0; e < indptr[n_dst]; ++e) t_indptr[indices[e] + 1]++;
    for (int32_t s = 0; s < n_src; ++s) t_indptr[s + 1] += t_indptr[s];
    if (n_src < 0 || n_dst < 0) return;
    int32_t *fill = (int32_t *)malloc(sizeof(int32_t) * ((size_t)n_src + 1));
    for (int32_t s = 0; s < n_src; ++s) fill[s] = t_indptr[s];
    for (int32_t v = 0; v < n_dst; ++v)
        for (int32_t e = indptr[v]; e < indptr[v + 1]; ++e) t_indices[fill[indices[e]]++] = v;
    free(fill);
}

/* ------------------------------------------------------------------ */
/* Message passing, GraphSAGE-mean form of Eq. 1:                      */
/*   Agg[v] = (1/|N_s(v)|) * sum_{u in N_s(v)} H[u]   (0 if N_s empty) */
/*   Z[v]   = H[v] W_self + Agg[v] W_neigh + b,  ReLU on hidden layers */
/* ------------------------------------------------------------------ */

static float bf16_round(float x)
{
    uint32_t u;
    memcpy(&u, &x, 4);
    if ((u & 0x7F800000u) == 0x7F800000u) return x;      /* inf / nan unchanged */
    u += 0x7FFFu + ((u >> 16) & 1u);                     /* round to nearest even */
    u &= 0xFFFF0000u;
    memcpy(&x, &u, 4);
    return x;
}

static double bf16_to_double(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

void orc_round_bf16(const double *in, int64_t n, double *out)
{
    for (int64_t i = 0; i < n; ++i) out[i] = (double)bf16_round((float)in[i]);
}

/* table_dtype: 0 = float32, 1 = bfloat16 (raw uint16), 2 = float64.  row_map (may be NULL)
 * sends a block-local source position to a table row (layer 0: the frontier's
 * global node ids). */
static double table_at(const void *table, int table_dtype, int64_t ld, int64_t row, int32_t col)
{
    if (table_dtype == 0) return (double)((const float *)table)[row * ld + col];
    if (table_dtype == 2) return ((const double *)table)[row * ld + col];
    return bf16_to_double(((const uint16_t *)table)[row * ld + col]);
}

void orc_gather_mean(int32_t n_dst, const int32_t *indptr, const int32_t *indices,
                     const int32_t *row_map, const void *table, int table_dtype, int64_t ld,
                     int32_t F, double *agg /*[n_dst*F]*/, double *self_rows /*[n_dst*F] or NULL*/)
{
#pragma omp parallel for schedule(static)
    for (int32_t v = 0; v < n_dst; ++v) {
        int32_t deg = indptr[v + 1] - indptr[v];
        for (int32_t c = 0; c < F; ++c) {
            double s = 0.0;
            for (int32_t e = indptr[v]; e < indptr[v + 1]; ++e) {
                int64_t row = row_map ? row_map[indices[e]] : indices[e];
                s += table_at(table, table_dtype, ld, row, c);
            }
            agg[(int64_t)v * F + c] = deg ? s / (double)deg : 0.0;
            if (self_rows) {
                int64_t row = row_map ? row_map[v] : v;
                self_rows[(int64_t)v * F + c] = table_at(table, table_dtype, ld, row, c);
            }
        }
    }
}

/* Gradient of the mean w.r.t. the source rows, plus the self path:
 * d_src[u] = sum_{v : u in N_s(v)} d_agg[v] / |N_s(v)|  (+ d_self[u] for u < n_dst). */
void orc_gather_mean_bwd(int32_t n_dst, int32_t n_src, const int32_t *indptr,
                         const int32_t *indices, const double *d_agg, const double *d_self,
                         int32_t F, double *d_src /*[n_src*F]*/)
{
    for (int64_t i = 0; i < (int64_t)n_src * F; ++i) d_src[i] = 0.0;
    for (int32_t v = 0; v < n_dst; ++v) {
        int32_t deg = indptr[v + 1] - indptr[v];
        for (int32_t e = indptr[v]; e < indptr[v + 1]; ++e)
            for (int32_t c = 0; c < F; ++c)
                d_src[(int64_t)indices[e] * F + c] += d_agg[(int64_t)v * F + c] / (double)deg;
    }
    if (d_self)
        for (int64_t i = 0; i < (int64_t)n_dst * F; ++i) d_src[i] += d_self[i];
}

static double opnd(double x, int round_operands)
{
    return round_operands ? (double)bf16_round((float)x) : x;
}

/* W is [2*F_in, F_out] row-major: rows 0..F_in-1 = W_self, F_in..2F_in-1 = W_neigh. */
void orc_sage_linear_fwd(int32_t M, int32_t F_in, int32_t F_out, const double *h_self,
                         const double *agg, const double *W, const double *bias, int relu,
                         int round_operands, double *out /*[M*F_out]*/)
{
#pragma omp parallel for schedule(static)
    for (int32_t m = 0; m < M; ++m)
        for (int32_t n = 0; n < F_out; ++n) {
            double s = 0.0;
            for (int32_t k = 0; k < F_in; ++k)
                s += opnd(h_self[(int64_t)m * F_in + k], round_operands) *
                     opnd(W[(int64_t)k * F_out + n], round_operands);
            for (int32_t k = 0; k < F_in; ++k)
                s += opnd(agg[(int64_t)m * F_in + k], round_operands) *
                     opnd(W[(int64_t)(F_in + k) * F_out + n], round_operands);
            s += bias[n];
            out[(int64_t)m * F_out + n] = (relu && s < 0.0) ? 0.0 : s;
        }
}

/* Backward of the layer above.  d_out is dL/d(out); with relu the mask is
 * out > 0.  Writes dW [2F_in*F_out], db [F_out], and (if non-NULL) d_self,
 * d_agg [M*F_in]. */
void orc_sage_linear_bwd(int32_t M, int32_t F_in, int32_t F_out, const double *h_self,
                         const double *agg, const double *W, const double *out,
                         const double *d_out, int relu, int round_operands,
                         double *dW, double *db, double *d_self, double *d_agg)
{
    double *dz = (double *)malloc(sizeof(double) * (size_t)M * (size_t)F_out + 8);
    for (int64_t i = 0; i < (int64_t)M * F_out; ++i)
        dz[i] = (relu && !(out[i] > 0.0)) ? 0.0 : d_out[i];
    for (int32_t n = 0; n < F_out; ++n) {
        double s = 0.0;
        for (int32_t m = 0; m < M; ++m) s += dz[(int64_t)m * F_out + n];
        db[n] = s;
    }
#pragma omp parallel for schedule(static)
    for (int32_t k = 0; k < 2 * F_in; ++k)
        for (int32_t n = 0; n < F_out; ++n) {
            double s = 0.0;
            for (int32_t m = 0; m < M; ++m) {
                double a = k < F_in ? h_self[(int64_t)m * F_in + k] : agg[(int64_t)m * F_in + (k - F_in)];
                s += opnd(a, round_operands) * opnd(dz[(int64_t)m * F_out + n], round_operands);
            }
            dW[(int64_t)k * F_out + n] = s;
        }
    for (int part = 0; part < 2; ++part) {
        double *dx = part == 0 ? d_self : d_agg;
        if (!dx) continue;
#pragma omp parallel for schedule(static)
        for (int32_t m = 0; m < M; ++m)
            for (int32_t k = 0; k < F_in; ++k) {
                double s = 0.0;
                for (int32_t n = 0; n < F_out; ++n)
                    s += opnd(dz[(int64_t)m * F_out + n], round_operands) *
                         opnd(W[(int64_t)(part * F_in + k) * F_out + n], round_operands);
                dx[(int64_t)m * F_in + k] = s;
            }
    }
    free(dz);
}

/* Plain SGD with L2 weight decay on the weights (not on the bias). */
void orc_sgd_step(int64_t n_w, double *W, const double *dW, int64_t n_b, double *b,
                  const double *db, double lr, double weight_decay)
{
    for (int64_t i = 0; i < n_w; ++i) W[i] -= lr * (dW[i] + weight_decay * W[i]);
    for (int64_t i = 0; i < n_b; ++i) b[i] -= lr * db[i];
}

/* Mean softmax cross-entropy over the n root rows and its gradient. */
double orc_softmax_xent(int32_t n, int32_t C, const double *logits, int64_t ld,
                        const int32_t *labels, double *d_logits /*[n*ld] or NULL*/)
{
    double loss = 0.0;
    for (int32_t i = 0; i < n; ++i) {
        const double *z = logits + (int64_t)i * ld;
        double mx = z[0];
        for (int32_t c = 1; c < C; ++c) if (z[c] > mx) mx = z[c];
        double den = 0.0;
        for (int32_t c = 0; c < C; ++c) den += exp(z[c] - mx);
        loss += -(z[labels[i]] - mx - log(den));
        if (d_logits)
            for (int32_t c = 0; c < C; ++c)
                d_logits[(int64_t)i * ld + c] =
                    (exp(z[c] - mx) / den - (c == labels[i] ? 1.0 : 0.0)) / (double)n;
    }
    return n ? loss / (double)n : 0.0;
}

/* Number of rows whose largest logit (lowest index on ties) is the label: the accuracy numerator of the
 * validation pass of the training protocol (Section 5 "Training methodology"). */
int32_t orc_count_correct(int32_t n, int32_t C, const double *logits, int64_t ld, const int32_t *labels)
{
    int32_t ok = 0;
    for (int32_t i = 0; i < n; ++i) {
        const double *z = logits + (int64_t)i * ld;
        int32_t best = 0;
        for (int32_t c = 1; c < C; ++c) if (z[c] > z[best]) best = c;
        ok += best == labels[i];
    }
    return ok;
}

/* Software-managed feature cache in front of a slower feature store (Section 6.5, impact of software-managed
 * caches: an LRU cache of node-feature rows in GPU memory).  The paper names the policy (LRU) and the capacity, not
 * the organisation; the reading here is a set-associative cache (set = node id mod n_sets, `ways` rows per set)
 * that is updated once per mini-batch:
 *   1. every distinct input node of the batch is looked up; a hit refreshes its row's stamp to this batch's stamp;
 *   2. the misses of a set, in the order the nodes appear in the batch, replace that set's rows in order of
 *      (stamp ascending, way ascending), never a row hit or filled in this same batch (empty rows carry stamp -1,
 *      so they go first);
 *   3. misses that find no such row in their set are served from the store without being cached (slot -1 here).
 * With one set, and batches of a single node, this is textbook LRU.
 * keys / stamps: [n_sets*ways], -1 = empty.  ids: n distinct node ids.  slot_out[i] = n_sets-major slot of ids[i]
 * after the update, or -1.  Returns the number of misses. */
int32_t orc_cache_fetch(int32_t n_sets, int32_t ways, int32_t *keys, int32_t *stamps, const int32_t *ids, int32_t n,
                        int32_t stamp, int32_t *slot_out)
{
    int32_t n_miss = 0;
    /* 1. look-ups */
    for (int32_t i = 0; i < n; ++i) {
        const int32_t set = ids[i] % n_sets;
        slot_out[i] = -2;                                   /* miss, not yet placed */
        for (int32_t w = 0; w < ways; ++w) {
            const int64_t s = (int64_t)set * ways + w;
            if (keys[s] == ids[i]) { slot_out[i] = (int32_t)s; stamps[s] = stamp; break; }
        }
        if (slot_out[i] == -2) ++n_miss;
    }
    /* 2. + 3. replacements, set by set; the misses of a set are visited in batch order */
    for (int32_t i = 0; i < n; ++i) {
        if (slot_out[i] != -2) continue;
        const int32_t set = ids[i] % n_sets;
        int32_t best = -1;
        for (int32_t w = 0; w < ways; ++w) {
            const int64_t s = (int64_t)set * ways + w;
            if (stamps[s] == stamp) continue;               /* hit or filled in this batch */
            if (best < 0 || stamps[s] < stamps[(int64_t)set * ways + best]) best = w;
        }
        if (best < 0) { slot_out[i] = -1; continue; }
        const int64_t s = (int64_t)set * ways + best;
        keys[s] = ids[i];
        stamps[s] = stamp;
        slot_out[i] = (int32_t)s;
    }
    return n_miss;
}
