// Test infrastructure: the library's host side (argument validation, capacity and workspace arithmetic, context handling)
// under AddressSanitizer + UndefinedBehaviorSanitizer.  Every call is made under a dry-run context, so it stops after the
// host-side checks and no GPU is needed; device pointers are dummy addresses that are never dereferenced.  The structures
// the library reads on the host (configurations, the per-layer block-set array, layer descriptors) live in heap blocks of
// exactly their size, so a read past them is reported.  Prints "ok" and returns 0 when every call returned the status it
// should.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>

#include "../include/commrand.h"

static int failures = 0;
#define EXPECT(call, want)                                                                                       \
    do {                                                                                                         \
        const cr_status got_ = (call);                                                                           \
        if (got_ != (want)) { std::fprintf(stderr, "line %d: status %d, expected %d (%s)\n", __LINE__, (int)got_, (int)(want), cr_last_error()); ++failures; } \
    } while (0)

template <typename T> static T *heap(const T &v) { T *p = static_cast<T *>(std::malloc(sizeof(T))); *p = v; return p; }
static void *dev(uintptr_t n) { return reinterpret_cast<void *>(0x10000u * n); }      // aligned dummy device address

int main()
{
    cr_ctx *ctx = nullptr;
    EXPECT(cr_ctx_create(nullptr, 0, CR_CTX_DRY_RUN, nullptr), CR_ERR_INVALID_ARG);
    EXPECT(cr_ctx_create(&ctx, -1, CR_CTX_DRY_RUN, nullptr), CR_ERR_INVALID_ARG);
    EXPECT(cr_ctx_create(&ctx, 0, 0x80u, nullptr), CR_ERR_INVALID_ARG);
    EXPECT(cr_ctx_create(&ctx, 0, CR_CTX_DRY_RUN, nullptr), CR_OK);
    EXPECT(cr_ctx_make_current(ctx), CR_OK);
    (void)cr_version();

    // ---- root partitioning
    size_t bytes = 0;
    EXPECT(cr_build_batches_workspace_bytes(100000, 500, &bytes), CR_OK);
    EXPECT(cr_build_batches_workspace_bytes(-1, 500, &bytes), CR_ERR_INVALID_ARG);
    cr_batch_cfg *bc = heap(cr_batch_cfg{CR_ROOTS_COMM_RAND, 3, 1024, 7u, 1ull});
    int64_t nb = 0;
    EXPECT(cr_build_batches(bc, (const int32_t *)dev(1), 100000, (const int32_t *)dev(2), 500, dev(3), bytes, (int32_t *)dev(4), &nb, nullptr), CR_OK);
    EXPECT(cr_build_batches(bc, (const int32_t *)dev(1), 100000, (const int32_t *)dev(2), 500, dev(3), bytes / 2, (int32_t *)dev(4), &nb, nullptr), CR_ERR_CAPACITY);
    EXPECT(cr_build_batches_static(bc, (const int32_t *)dev(1), 100000, (const int32_t *)dev(2), 500, (int32_t *)dev(4), &nb, nullptr), CR_OK);
    EXPECT(cr_build_batches_static(bc, (const int32_t *)dev(1), CR_STATIC_MAX_TRAIN + 1, (const int32_t *)dev(2), 500, (int32_t *)dev(4), &nb, nullptr), CR_ERR_CAPACITY);
    bc->mix_count = 0;
    EXPECT(cr_build_batches(bc, (const int32_t *)dev(1), 100000, (const int32_t *)dev(2), 500, dev(3), bytes, (int32_t *)dev(4), &nb, nullptr), CR_ERR_INVALID_ARG);
    (void)cr_mix_count_from_percent(12.5, 500);
    (void)cr_mix_count_from_percent(0.0, 0);
    std::free(bc);

    // ---- sampling: capacities, workspace, block sets of exactly n_layers entries
    for (int L = 1; L <= 3; ++L) {
        cr_sample_cfg *sc = heap(cr_sample_cfg{});
        sc->n_layers = L;
        const int32_t fan[3] = {15, 10, 5};
        for (int l = 0; l < L; ++l) sc->fanout[l] = fan[l];
        sc->p_intra = 0.9; sc->seed = 3; sc->epoch = 2; sc->first_batch = 4; sc->flags = CR_SAMPLE_ROW_ORDER;
        int32_t *cap_dst = static_cast<int32_t *>(std::malloc(sizeof(int32_t) * L)), *cap_src = static_cast<int32_t *>(std::malloc(sizeof(int32_t) * L)),
                *cap_nnz = static_cast<int32_t *>(std::malloc(sizeof(int32_t) * L));
        const int64_t n_nodes = 170000;
        EXPECT(cr_block_capacities(sc, n_nodes, 1024, cap_dst, cap_src, cap_nnz), CR_OK);
        size_t ws = 0;
        EXPECT(cr_sample_blocks_workspace_bytes(sc, n_nodes, 1024, 8, &ws), CR_OK);
        int32_t kind = -1;
        EXPECT(cr_sample_blocks_dedup_table(sc, n_nodes, 1024, &kind), CR_OK);
        cr_graph *gr = heap(cr_graph{n_nodes, 2400000, (const int64_t *)dev(1), (const int32_t *)dev(2), (const int32_t *)dev(3), 500, 0, (const uint32_t *)dev(4)});
        cr_block_set *layers = static_cast<cr_block_set *>(std::malloc(sizeof(cr_block_set) * L));
        for (int l = 0; l < L; ++l) {
            cr_block_set b{};
            b.n_batches = 8; b.fanout = sc->fanout[l]; b.cap_dst = cap_dst[l]; b.cap_src = cap_src[l]; b.cap_nnz = cap_nnz[l];
            b.hdr = (int32_t *)dev(10 + l); b.src_ids = (int32_t *)dev(20 + l); b.indptr = (int32_t *)dev(30 + l); b.indices = (int32_t *)dev(40 + l);
            if (l >= 1) { b.t_indptr = (int32_t *)dev(50 + l); b.t_indices = (int32_t *)dev(60 + l); }
            b.gather_ids = (int32_t *)dev(70 + l);
            layers[l] = b;
        }
        EXPECT(cr_sample_blocks(gr, sc, (const int32_t *)dev(5), 8 * 1024 - 100, 1024, 8, dev(6), ws, layers, nullptr), CR_OK);
        EXPECT(cr_sample_blocks(gr, sc, (const int32_t *)dev(5), 8 * 1024 - 100, 1024, 8, dev(6), ws / 4, layers, nullptr), CR_ERR_CAPACITY);
        layers[L - 1].cap_dst -= 1;
        EXPECT(cr_sample_blocks(gr, sc, (const int32_t *)dev(5), 8 * 1024 - 100, 1024, 8, dev(6), ws, layers, nullptr), CR_ERR_CAPACITY);
        layers[L - 1].cap_dst += 1;
        sc->flags |= CR_SAMPLE_INPUT_GLOBAL_IDS | CR_SAMPLE_EXACT_RANKING;
        EXPECT(cr_sample_blocks(gr, sc, (const int32_t *)dev(5), 8 * 1024 - 100, 1024, 8, dev(6), ws, layers, nullptr), CR_OK);
        sc->p_intra = 0.3;
        EXPECT(cr_sample_blocks(gr, sc, (const int32_t *)dev(5), 8 * 1024 - 100, 1024, 8, dev(6), ws, layers, nullptr), CR_ERR_INVALID_ARG);
        sc->p_intra = 1.0;
        // the calls that read one block set
        EXPECT(cr_gather_aggregate_fwd(&layers[0], 7, dev(7), 0, 128, 128, 1, nullptr, (uint16_t *)dev(8), (uint16_t *)dev(9), 128, nullptr), CR_OK);
        EXPECT(cr_gather_aggregate_fwd(&layers[0], 8, dev(7), 0, 128, 128, 1, nullptr, (uint16_t *)dev(8), (uint16_t *)dev(9), 128, nullptr), CR_ERR_INVALID_ARG);
        std::free(layers); std::free(gr); std::free(cap_dst); std::free(cap_src); std::free(cap_nnz); std::free(sc);
    }
    EXPECT(cr_selftest_clock_approximation(nullptr, nullptr), CR_ERR_INVALID_ARG);
    EXPECT(cr_selftest_clock_approximation((float *)dev(1), nullptr), CR_OK);

    // ---- dense layers
    int32_t F_pad = 0, N_pad = 0;
    EXPECT(cr_sage_padded_dims(100, 47, &F_pad, &N_pad), CR_OK);
    EXPECT(cr_sage_padded_dims(0, 47, &F_pad, &N_pad), CR_ERR_INVALID_ARG);
    cr_sage_layer *lay = heap(cr_sage_layer{100, 47, 2, 0, (float *)dev(1), (float *)dev(2), (uint16_t *)dev(3), (uint16_t *)dev(4)});
    EXPECT(cr_sage_refresh_shadows(lay, nullptr), CR_OK);
    EXPECT(cr_sage_linear_fwd(lay, (const int32_t *)dev(5), 4096, (const uint16_t *)dev(6), (const uint16_t *)dev(7), 128, 1, (float *)dev(8), (uint16_t *)dev(9), nullptr), CR_OK);
    EXPECT(cr_sage_linear_fwd(lay, (const int32_t *)dev(5), 4096, nullptr, (const uint16_t *)dev(7), 128, 1, (float *)dev(8), nullptr, nullptr), CR_ERR_INVALID_ARG);
    EXPECT(cr_sage_linear_fwd(lay, (const int32_t *)dev(5), 4096, (const uint16_t *)dev(6), (const uint16_t *)dev(7), 100, 1, (float *)dev(8), nullptr, nullptr), CR_ERR_INVALID_ARG);
    size_t wsb = 0;
    EXPECT(cr_sage_linear_bwd_workspace_bytes(100, 47, 4096, &wsb), CR_OK);
    EXPECT(cr_sage_linear_bwd(lay, (const int32_t *)dev(5), 4096, (const uint16_t *)dev(6), (const uint16_t *)dev(7), 128, (const uint16_t *)dev(8), 0.1f, 5e-4f,
                              nullptr, nullptr, (uint16_t *)dev(9), nullptr, nullptr, dev(10), wsb, nullptr), CR_OK);
    EXPECT(cr_sage_linear_bwd(lay, (const int32_t *)dev(5), 4096, (const uint16_t *)dev(6), (const uint16_t *)dev(7), 128, (const uint16_t *)dev(8), 0.1f, 5e-4f,
                              nullptr, nullptr, (uint16_t *)dev(9), nullptr, nullptr, dev(10), wsb / 2, nullptr), CR_ERR_CAPACITY);
    lay->n_operands = 3;
    EXPECT(cr_sage_refresh_shadows(lay, nullptr), CR_ERR_INVALID_ARG);
    std::free(lay);
    EXPECT(cr_softmax_xent((const int32_t *)dev(1), 1024, (const float *)dev(2), 64, 47, (const int32_t *)dev(3), (const int32_t *)dev(4), (float *)dev(5), (float *)dev(6),
                           (float *)dev(7), (uint16_t *)dev(8), nullptr), CR_OK);
    EXPECT(cr_mean_accumulate((const int32_t *)dev(1), 1024, (const float *)dev(2), (double *)dev(3), nullptr), CR_OK);

    // ---- contexts: polling a context without status words, switching and destroying the current one
    int64_t need = -1;
    (void)cr_ctx_poll_error(ctx, &need, 1, nullptr);
    EXPECT(cr_ctx_poll_error(nullptr, &need, 1, nullptr), CR_ERR_INVALID_ARG);
    EXPECT(cr_ctx_destroy(ctx), CR_OK);
    EXPECT(cr_ctx_destroy(nullptr), CR_OK);
    if (failures) { std::fprintf(stderr, "%d unexpected statuses\n", failures); return 1; }
    std::printf("ok\n");
    return 0;
}
