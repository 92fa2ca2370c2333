/* Test infrastructure: drives every oracle routine once over a small synthetic graph with heap buffers of exactly the
 * documented sizes, so that a build with -fsanitize=address,undefined reports any access outside them, any signed
 * overflow, misaligned access or invalid shift inside the oracle.  No result is checked here (the pins and the parity
 * tests do that); the program prints "ok" and returns 0 when every call returned normally.
 *
 *   gcc -O1 -g -fsanitize=address,undefined -fno-sanitize-recover=all oracle/oracle.c oracle/sanitize_driver.c -lm
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

uint64_t orc_shuffle_key(uint64_t, uint32_t, uint32_t, uint32_t);
uint32_t orc_slot_word(uint64_t, uint32_t, uint32_t, uint32_t, uint32_t, uint32_t);
int orc_build_batches(int, int32_t, uint64_t, uint32_t, const int32_t *, int64_t, const int32_t *, int32_t, int32_t *);
uint64_t orc_slot_key(uint32_t, int, uint32_t);
int64_t orc_sample_hop(const int64_t *, const int32_t *, const int32_t *, const int32_t *, int32_t, int32_t, uint32_t, int,
                       uint64_t, uint32_t, uint32_t, uint32_t, int32_t *, int32_t *, int32_t *, int32_t *, int32_t *, int32_t *);
void orc_transpose_block(int32_t, int32_t, const int32_t *, const int32_t *, int32_t *, int32_t *);
void orc_gather_mean(int32_t, const int32_t *, const int32_t *, const int32_t *, const void *, int, int64_t, int32_t, double *,
                     double *);
void orc_gather_mean_bwd(int32_t, int32_t, const int32_t *, const int32_t *, const double *, const double *, int32_t, double *);
void orc_sage_linear_fwd(int32_t, int32_t, int32_t, const double *, const double *, const double *, const double *, int, int,
                         double *);
void orc_sage_linear_bwd(int32_t, int32_t, int32_t, const double *, const double *, const double *, const double *,
                         const double *, int, int, double *, double *, double *, double *);
void orc_sgd_step(int64_t, double *, const double *, int64_t, double *, const double *, double, double);
double orc_softmax_xent(int32_t, int32_t, const double *, int64_t, const int32_t *, double *);
int32_t orc_count_correct(int32_t, int32_t, const double *, int64_t, const int32_t *);
int32_t orc_cache_fetch(int32_t, int32_t, int32_t *, int32_t *, const int32_t *, int32_t, int32_t, int32_t *);
void orc_round_bf16(const double *, int64_t, double *);

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd(void)
{
    rng_state = rng_state * 6364136223846793005ull + 1442695040888963407ull;
    return (uint32_t)(rng_state >> 33);
}
static double rndf(void) { return (double)rnd() / 2147483648.0 - 0.5; }
static void *xmalloc(size_t n)
{
    void *p = malloc(n ? n : 1);
    if (!p) { fprintf(stderr, "out of memory\n"); exit(2); }
    return p;
}

#define N_NODES 300
#define N_COMM 7

int main(void)
{
    /* a small directed graph: node v has (v * 7) % 23 neighbours, node 5 a hub with 200, nodes 10..14 isolated */
    int64_t *indptr = xmalloc(sizeof(int64_t) * (N_NODES + 1));
    int32_t *comm = xmalloc(sizeof(int32_t) * N_NODES);
    indptr[0] = 0;
    for (int v = 0; v < N_NODES; ++v) {
        int deg = (v * 7) % 23;
        if (v == 5) deg = 200;
        if (v >= 10 && v < 15) deg = 0;
        indptr[v + 1] = indptr[v] + deg;
        comm[v] = (int32_t)((int64_t)v * N_COMM / N_NODES);          /* ids contiguous by community */
    }
    const int64_t nnz_g = indptr[N_NODES];
    int32_t *indices = xmalloc(sizeof(int32_t) * (size_t)nnz_g);
    for (int v = 0; v < N_NODES; ++v) {
        const int deg = (int)(indptr[v + 1] - indptr[v]);
        for (int j = 0; j < deg; ++j) indices[indptr[v] + j] = (int32_t)((v + 1 + (int64_t)j * 3) % N_NODES);   /* distinct for deg <= 100 */
        if (v == 5) for (int j = 0; j < deg; ++j) indices[indptr[v] + j] = (int32_t)((6 + j) % N_NODES);
    }

    /* Step 1: the three root policies over the training set (every third node), and an empty set */
    const int64_t n_train = N_NODES / 3;
    int32_t *train = xmalloc(sizeof(int32_t) * (size_t)n_train), *perm = xmalloc(sizeof(int32_t) * (size_t)n_train);
    for (int64_t i = 0; i < n_train; ++i) train[i] = (int32_t)(3 * i);
    for (int policy = 0; policy < 3; ++policy)
        for (int32_t mix = 1; mix <= 3; ++mix)
            if (orc_build_batches(policy, mix, 11u, 2u, train, n_train, comm, N_COMM, perm) != 0) return 3;
    if (orc_build_batches(2, 1, 11u, 2u, train, 0, comm, N_COMM, perm) != 0) return 3;
    (void)orc_shuffle_key(1u, 2u, 1u, 3u);
    (void)orc_slot_word(1u, 2u, 3u, 1u, 4u, 5u);
    (void)orc_slot_key(0u, 1, 32768u);
    (void)orc_slot_key(0xFFFFFFFFu, 0, 58982u);
    (void)orc_slot_key(123u, 0, 65536u);

    /* Step 2: two hops for p = 0.5, 0.9, 1 (also strict), roots include the hub and an isolated node */
    const int32_t fanouts[2] = {4, 3};
    const uint32_t q[3] = {32768u, 58982u, 65536u};
    int32_t *pos_map = xmalloc(sizeof(int32_t) * N_NODES);
    for (int i = 0; i < N_NODES; ++i) pos_map[i] = -1;
    int32_t roots[9] = {0, 5, 12, 33, 36, 99, 150, 299, 3};
    for (int qi = 0; qi < 3; ++qi)
        for (int strict = 0; strict < 2; ++strict) {
            int32_t n_dst = 9;
            int32_t *dst = xmalloc(sizeof(int32_t) * 9);
            memcpy(dst, roots, sizeof(roots));
            for (int l = 1; l >= 0; --l) {
                const int32_t f = fanouts[l];
                int32_t *o_indptr = xmalloc(sizeof(int32_t) * (size_t)(n_dst + 1));
                int32_t *o_indices = xmalloc(sizeof(int32_t) * (size_t)(n_dst * f));
                int32_t *o_slots = xmalloc(sizeof(int32_t) * (size_t)(n_dst * f));
                int32_t *o_src = xmalloc(sizeof(int32_t) * (size_t)(n_dst * (1 + f)));
                int32_t n_src = 0;
                const int64_t nnz = orc_sample_hop(indptr, indices, comm, dst, n_dst, f, q[qi], strict, 7u, 1u, 2u, (uint32_t)l, pos_map,
                                                   o_indptr, o_indices, o_src, &n_src, l ? o_slots : NULL);
                if (nnz < 0) return 4;
                int32_t *t_indptr = xmalloc(sizeof(int32_t) * (size_t)(n_src + 1));
                int32_t *t_indices = xmalloc(sizeof(int32_t) * (size_t)(nnz > 0 ? nnz : 1));
                orc_transpose_block(n_dst, n_src, o_indptr, o_indices, t_indptr, t_indices);

                /* Step 3 on this block: float32, bf16 and float64 tables; through the frontier (indirect) and direct */
                const int32_t F = 5;
                const int64_t ld = 6;
                float *tab32 = xmalloc(sizeof(float) * N_NODES * (size_t)ld);
                uint16_t *tab16 = xmalloc(sizeof(uint16_t) * N_NODES * (size_t)ld);
                double *tab64 = xmalloc(sizeof(double) * (size_t)n_src * (size_t)F);
                for (int64_t i = 0; i < N_NODES * ld; ++i) { tab32[i] = (float)rndf(); tab16[i] = (uint16_t)(0x3F00u + (rnd() & 0xFFu)); }
                for (int64_t i = 0; i < (int64_t)n_src * F; ++i) tab64[i] = rndf();
                double *agg = xmalloc(sizeof(double) * (size_t)n_dst * F), *self_rows = xmalloc(sizeof(double) * (size_t)n_dst * F);
                orc_gather_mean(n_dst, o_indptr, o_indices, o_src, tab32, 0, ld, F, agg, self_rows);
                orc_gather_mean(n_dst, o_indptr, o_indices, o_src, tab16, 1, ld, F, agg, NULL);
                orc_gather_mean(n_dst, o_indptr, o_indices, NULL, tab64, 2, F, F, agg, self_rows);
                double *d_agg = xmalloc(sizeof(double) * (size_t)n_dst * F), *d_self = xmalloc(sizeof(double) * (size_t)n_dst * F);
                double *d_src = xmalloc(sizeof(double) * (size_t)n_src * F);
                for (int64_t i = 0; i < (int64_t)n_dst * F; ++i) { d_agg[i] = rndf(); d_self[i] = rndf(); }
                orc_gather_mean_bwd(n_dst, n_src, o_indptr, o_indices, d_agg, d_self, F, d_src);
                orc_gather_mean_bwd(n_dst, n_src, o_indptr, o_indices, d_agg, NULL, F, d_src);

                /* dense layer, forward and backward, with and without ReLU / operand rounding / input gradient */
                const int32_t Fo = 4;
                double *W = xmalloc(sizeof(double) * 2 * F * Fo), *b = xmalloc(sizeof(double) * Fo);
                double *out = xmalloc(sizeof(double) * (size_t)n_dst * Fo), *d_out = xmalloc(sizeof(double) * (size_t)n_dst * Fo);
                double *dW = xmalloc(sizeof(double) * 2 * F * Fo), *db = xmalloc(sizeof(double) * Fo);
                for (int i = 0; i < 2 * F * Fo; ++i) W[i] = rndf();
                for (int i = 0; i < Fo; ++i) b[i] = rndf();
                for (int64_t i = 0; i < (int64_t)n_dst * Fo; ++i) d_out[i] = rndf();
                for (int relu = 0; relu < 2; ++relu)
                    for (int ro = 0; ro < 2; ++ro) {
                        orc_sage_linear_fwd(n_dst, F, Fo, self_rows, agg, W, b, relu, ro, out);
                        orc_sage_linear_bwd(n_dst, F, Fo, self_rows, agg, W, out, d_out, relu, ro, dW, db, d_self, d_agg);
                        orc_sage_linear_bwd(n_dst, F, Fo, self_rows, agg, W, out, d_out, relu, ro, dW, db, NULL, NULL);
                    }
                orc_sgd_step(2 * F * Fo, W, dW, Fo, b, db, 0.1, 5e-4);
                orc_round_bf16(out, (int64_t)n_dst * Fo, out);

                /* loss on the rows of this block (labels in range), padded leading dimension */
                {
                    const int32_t C = 3;
                    const int64_t ldl = 4;
                    double *logits = xmalloc(sizeof(double) * (size_t)n_dst * (size_t)ldl), *dl = xmalloc(sizeof(double) * (size_t)n_dst * (size_t)ldl);
                    int32_t *labels = xmalloc(sizeof(int32_t) * (size_t)n_dst);
                    for (int64_t i = 0; i < (int64_t)n_dst * ldl; ++i) logits[i] = 8.0 * rndf();
                    for (int32_t i = 0; i < n_dst; ++i) labels[i] = (int32_t)(rnd() % (uint32_t)C);
                    (void)orc_softmax_xent(n_dst, C, logits, ldl, labels, dl);
                    (void)orc_softmax_xent(n_dst, C, logits, ldl, labels, NULL);
                    (void)orc_count_correct(n_dst, C, logits, ldl, labels);
                    free(logits); free(dl); free(labels);
                }
                free(W); free(b); free(out); free(d_out); free(dW); free(db);
                free(tab32); free(tab16); free(tab64); free(agg); free(self_rows); free(d_agg); free(d_self); free(d_src);
                free(t_indptr); free(t_indices); free(o_indptr); free(o_indices); free(o_slots);
                free(dst);
                dst = o_src;            /* the frontier is the next hop's destination list (first n_src entries) */
                n_dst = n_src;
            }
            free(dst);
        }
    for (int i = 0; i < N_NODES; ++i)
        if (pos_map[i] != -1) return 5;

    /* empty batch */
    {
        int32_t o_indptr[1], n_src = -1, dummy[1];
        if (orc_sample_hop(indptr, indices, comm, dummy, 0, 3, 32768u, 0, 1u, 0u, 0u, 0u, pos_map, o_indptr, dummy, dummy, &n_src, NULL) != 0) return 6;
        (void)orc_softmax_xent(0, 3, NULL, 4, NULL, NULL);
    }

    /* software cache: more distinct ids per set than ways, several batches (the ids of a batch are distinct) */
    {
        const int32_t n_sets = 4, ways = 3, n = 40;
        int32_t *keys = xmalloc(sizeof(int32_t) * n_sets * ways), *stamps = xmalloc(sizeof(int32_t) * n_sets * ways);
        int32_t *ids = xmalloc(sizeof(int32_t) * n), *slot = xmalloc(sizeof(int32_t) * n);
        for (int i = 0; i < n_sets * ways; ++i) { keys[i] = -1; stamps[i] = 0; }
        for (int32_t step = 1; step <= 5; ++step) {
            for (int i = 0; i < n; ++i) ids[i] = (int32_t)((step * 7 + i * 3) % 200);
            (void)orc_cache_fetch(n_sets, ways, keys, stamps, ids, n, step, slot);
        }
        (void)orc_cache_fetch(n_sets, ways, keys, stamps, ids, 0, 6, slot);
        free(keys); free(stamps); free(ids); free(slot);
    }
    free(indptr); free(indices); free(comm); free(train); free(perm); free(pos_map);
    printf("ok\n");
    return 0;
}
