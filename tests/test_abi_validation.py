"""CPU-only: every entry point validates its arguments on the host before touching the GPU.
With cr_set_dry_run(1) a call stops after validation, so error paths run without a device."""
import ctypes as C

import pytest

from paper_2504_18082_amd import binding as B

FAKE = 0x10000          # a non-null, 16-byte aligned "device" address (never dereferenced in dry-run mode)


@pytest.fixture(autouse=True)
def dry_run():
    B.cr_set_dry_run(True)
    yield
    B.cr_set_dry_run(False)


def status_of(call):
    try:
        call()
        return B.CR_OK
    except B.CrError as e:
        assert str(e)            # carries cr_last_error()
        return e.status


def vp(x=FAKE):
    return C.c_void_p(x)


def block_set(n_batches=1, fanout=5, cap_dst=8, cap_src=48, cap_nnz=40, t=True, null=None):
    ptrs = dict(hdr=FAKE, src_ids=FAKE, indptr=FAKE, indices=FAKE, t_indptr=FAKE if t else None,
                t_indices=FAKE if t else None, gather_ids=None)
    if null:
        ptrs[null] = None
    return B.cr_block_set(n_batches, fanout, cap_dst, cap_src, cap_nnz, 0, ptrs["hdr"], ptrs["src_ids"], ptrs["indptr"],
                          ptrs["indices"], ptrs["t_indptr"], ptrs["t_indices"], ptrs["gather_ids"])


def build_batches(policy=1, mix=1, batch=256, epoch=0, n_train=1000, n_comm=10, ws_bytes=None, train=FAKE, out=FAKE, ws=FAKE):
    lib = B.lib()
    cfg = B.cr_batch_cfg(policy, mix, batch, epoch, 0)
    need = C.c_size_t(0)
    lib.cr_build_batches_workspace_bytes(max(n_train, 0), max(n_comm, 1), C.byref(need))
    nb = C.c_int64(-1)
    st = lib.cr_build_batches(C.byref(cfg), vp(train), n_train, vp(), n_comm, vp(ws), need.value if ws_bytes is None else ws_bytes,
                              vp(out), C.byref(nb), None)
    return st, nb.value


def test_build_batches_validation():
    assert build_batches() == (B.CR_OK, 4)
    assert build_batches(n_train=1025) == (B.CR_OK, 5)                 # the short last batch is kept
    assert build_batches(policy=3)[0] == B.CR_ERR_INVALID_ARG
    assert build_batches(policy=1, mix=0)[0] == B.CR_ERR_INVALID_ARG
    assert build_batches(policy=0, mix=0)[0] == B.CR_OK                # mix_count only matters for COMM-RAND
    assert build_batches(batch=0)[0] == B.CR_ERR_INVALID_ARG
    assert build_batches(epoch=1 << 24)[0] == B.CR_ERR_INVALID_ARG
    assert build_batches(n_comm=0)[0] == B.CR_ERR_INVALID_ARG
    assert build_batches(train=None)[0] == B.CR_ERR_INVALID_ARG
    assert build_batches(ws=FAKE + 4)[0] == B.CR_ERR_INVALID_ARG       # misaligned workspace
    assert build_batches(ws_bytes=16)[0] == B.CR_ERR_CAPACITY
    assert b"workspace" in B.lib().cr_last_error()


def test_build_batches_static_validation():
    lib = B.lib()

    def call(n_train=1000, n_comm=10, policy=1, mix=1, train=FAKE, out=FAKE):
        cfg = B.cr_batch_cfg(policy, mix, 256, 0, 0)
        nb = C.c_int64(-1)
        return lib.cr_build_batches_static(C.byref(cfg), vp(train), n_train, vp(), n_comm, vp(out), C.byref(nb), None), nb.value

    assert call() == (B.CR_OK, 4)
    assert call(n_train=B.CR_STATIC_MAX_TRAIN, n_comm=B.CR_STATIC_MAX_COMM)[0] == B.CR_OK       # the stated maximum fits the array
    assert call(n_train=B.CR_STATIC_MAX_TRAIN + 1)[0] == B.CR_ERR_CAPACITY
    assert b"fixed scratch array" in lib.cr_last_error()
    assert call(n_comm=B.CR_STATIC_MAX_COMM + 1)[0] == B.CR_ERR_CAPACITY
    assert call(policy=3)[0] == B.CR_ERR_INVALID_ARG
    assert call(policy=1, mix=0)[0] == B.CR_ERR_INVALID_ARG
    assert call(train=None)[0] == B.CR_ERR_INVALID_ARG


def sample(fanouts=(10, 5), p=0.9, epoch=0, n_nodes=10000, batch=8, n_batches=1, n_roots=8, flags=0, layers=None,
           ws_bytes=None, graph_null=None):
    lib = B.lib()
    cfg = B.make_sample_cfg(list(fanouts), p, 0, epoch, 0, flags)
    graph = B.cr_graph(n_nodes, 100, FAKE, FAKE, FAKE, 5, 0, None)
    if graph_null:
        setattr(graph, graph_null, None)
    need = C.c_size_t(0)
    lib.cr_sample_blocks_workspace_bytes(C.byref(cfg), n_nodes, batch, n_batches, C.byref(need))
    if layers is None:
        a, b, c = (C.c_int32 * 8)(), (C.c_int32 * 8)(), (C.c_int32 * 8)()
        if lib.cr_block_capacities(C.byref(cfg), n_nodes, batch, a, b, c) != B.CR_OK:
            a[0] = b[0] = c[0] = 1
        layers = [block_set(n_batches, fanouts[l], a[l], b[l], c[l], t=(l >= 1)) for l in range(len(fanouts))]
    arr = (B.cr_block_set * len(layers))(*layers)
    return lib.cr_sample_blocks(C.byref(graph), C.byref(cfg), vp(), n_roots, batch, n_batches, vp(), need.value if ws_bytes is None else ws_bytes,
                                arr, None)


def test_sample_blocks_validation():
    assert sample() == B.CR_OK
    assert sample(n_batches=3, n_roots=17) == B.CR_OK                   # 8 + 8 + 1
    assert sample(n_batches=3, n_roots=16) == B.CR_ERR_INVALID_ARG      # would leave the last batch empty
    assert sample(n_batches=3, n_roots=25) == B.CR_ERR_INVALID_ARG
    assert sample(p=0.4) == B.CR_ERR_INVALID_ARG
    assert sample(p=1.1) == B.CR_ERR_INVALID_ARG
    assert sample(fanouts=(10, 0)) == B.CR_ERR_INVALID_ARG
    assert sample(fanouts=(10, 65)) == B.CR_ERR_INVALID_ARG
    assert sample(fanouts=()) == B.CR_ERR_INVALID_ARG
    assert sample(epoch=1 << 24) == B.CR_ERR_INVALID_ARG
    assert sample(graph_null="comm") == B.CR_ERR_INVALID_ARG
    assert sample(ws_bytes=64) == B.CR_ERR_CAPACITY
    small = [block_set(1, 10, 48, 10, 480, t=False), block_set(1, 5, 8, 48, 40)]
    assert sample(layers=small) == B.CR_ERR_CAPACITY                    # frontier capacity below the bound
    with_t0 = [block_set(1, 10, 48, 528, 480, t=True), block_set(1, 5, 8, 48, 40)]
    assert sample(layers=with_t0) == B.CR_ERR_UNSUPPORTED               # layer 0 takes no transposed block
    wrong_fanout = [block_set(1, 9, 48, 528, 480, t=False), block_set(1, 5, 8, 48, 40)]
    assert sample(layers=wrong_fanout) == B.CR_ERR_INVALID_ARG
    # leaving the input-side block in global ids needs somewhere to put them
    assert sample(flags=B.CR_SAMPLE_INPUT_GLOBAL_IDS) == B.CR_ERR_INVALID_ARG
    with_ids = [block_set(1, 10, 48, 528, 480, t=False), block_set(1, 5, 8, 48, 40)]
    with_ids[0].gather_ids = FAKE
    assert sample(layers=with_ids, flags=B.CR_SAMPLE_INPUT_GLOBAL_IDS) == B.CR_OK
    # a processing order of the rows is filled on request only: the flag sizes the workspace
    with_ids[0].row_order = FAKE
    assert sample(layers=with_ids, flags=B.CR_SAMPLE_INPUT_GLOBAL_IDS) == B.CR_ERR_INVALID_ARG
    assert sample(layers=with_ids, flags=B.CR_SAMPLE_INPUT_GLOBAL_IDS | B.CR_SAMPLE_ROW_ORDER) == B.CR_OK


def test_edge_classes_validation():
    lib = B.lib()
    graph = B.cr_graph(1000, 100, FAKE, FAKE, FAKE, 5, 0, None)
    assert lib.cr_graph_edge_classes(C.byref(graph), vp(), None) == B.CR_OK
    assert lib.cr_graph_edge_classes(C.byref(graph), None, None) == B.CR_ERR_INVALID_ARG
    graph.comm = None
    assert lib.cr_graph_edge_classes(C.byref(graph), vp(), None) == B.CR_ERR_INVALID_ARG


def test_block_capacities_are_the_worst_case_bounds():
    cfg = B.make_sample_cfg([15, 10, 5], 0.5, 0, 0)
    cap_dst, cap_src, cap_nnz = B.cr_block_capacities(cfg, 2_450_000, 1024)
    assert cap_dst == [67584, 6144, 1024] and cap_src == [1081344, 67584, 6144] and cap_nnz == [1013760, 61440, 5120]
    cap_dst, cap_src, cap_nnz = B.cr_block_capacities(cfg, 170_000, 1024)
    assert cap_src == [170000, 67584, 6144]                             # a frontier cannot exceed the graph


def test_gather_validation():
    lib = B.lib()
    bs = block_set()
    ok = lambda **kw: lib.cr_gather_aggregate_fwd(C.byref(kw.get("bs", bs)), kw.get("g", 0), vp(kw.get("H", FAKE)), kw.get("dtype", 0),
                                                  kw.get("ld", 64), kw.get("F", 64), 1, vp(kw.get("agg", FAKE)), None, None, 0, None)
    assert ok() == B.CR_OK
    assert ok(g=1) == B.CR_ERR_INVALID_ARG
    assert ok(H=None) == B.CR_ERR_INVALID_ARG
    assert ok(H=FAKE + 8) == B.CR_ERR_INVALID_ARG
    assert ok(dtype=2) == B.CR_ERR_INVALID_ARG
    assert ok(F=1025, ld=1028) == B.CR_ERR_UNSUPPORTED
    assert ok(F=100, ld=98) == B.CR_ERR_INVALID_ARG
    assert ok(agg=None) == B.CR_ERR_INVALID_ARG                          # no output requested
    assert ok(bs=block_set(null="indptr")) == B.CR_ERR_INVALID_ARG
    # bf16 outputs need a padded stride
    bad_ld = lib.cr_gather_aggregate_fwd(C.byref(bs), 0, vp(), 0, 100, 100, 1, None, vp(), None, 100, None)
    assert bad_ld == B.CR_ERR_INVALID_ARG
    good_ld = lib.cr_gather_aggregate_fwd(C.byref(bs), 0, vp(), 0, 100, 100, 1, None, vp(), None, 128, None)
    assert good_ld == B.CR_OK
    # backward needs the transposed block
    no_t = block_set(t=False)
    st = lib.cr_gather_aggregate_bwd(C.byref(no_t), 0, vp(), None, B.CR_F32, 64, 64, None, 0, 0, vp(), None, 0, None)
    assert st == B.CR_ERR_INVALID_ARG
    st = lib.cr_gather_aggregate_bwd(C.byref(bs), 0, vp(), None, B.CR_F32, 64, 64, vp(), 7, 64, vp(), None, 0, None)
    assert st == B.CR_ERR_INVALID_ARG                                    # unknown relu_dtype
    st = lib.cr_gather_aggregate_bwd(C.byref(bs), 0, vp(), None, 9, 64, 64, None, 0, 0, vp(), None, 0, None)
    assert st == B.CR_ERR_INVALID_ARG                                    # unknown in_dtype
    st = lib.cr_gather_aggregate_bwd(C.byref(bs), 0, vp(), None, B.CR_BF16, 68, 64, None, 0, 0, vp(), None, 0, None)
    assert st == B.CR_ERR_INVALID_ARG                                    # bf16 rows need a stride that is a multiple of 8
    st = lib.cr_gather_aggregate_bwd(C.byref(bs), 0, vp(), None, B.CR_BF16, 128, 64, vp(), B.CR_BF16, 64, vp(), None, 0, None)
    assert st == B.CR_OK
    st = lib.cr_gather_aggregate_bwd(C.byref(bs), 0, vp(), None, B.CR_F32, 64, 64, vp(), B.CR_BF16, 64, vp(), None, 0, None)
    assert st == B.CR_OK


def test_linear_and_loss_validation():
    lib = B.lib()
    layer = B.cr_sage_layer(100, 47, 2, 0, FAKE, FAKE, FAKE, FAKE)
    fp, np_ = B.cr_sage_padded_dims(100, 47)
    assert (fp, np_) == (128, 64)
    fwd = lambda **kw: lib.cr_sage_linear_fwd(C.byref(kw.get("layer", layer)), vp(kw.get("hdr", FAKE)), kw.get("rows", 100), vp(kw.get("h", FAKE)),
                                              vp(), kw.get("ld", 128), 1, vp(kw.get("out", FAKE)), None, None)
    assert fwd() == B.CR_OK
    assert fwd(hdr=None) == B.CR_ERR_INVALID_ARG
    assert fwd(rows=0) == B.CR_ERR_INVALID_ARG
    assert fwd(ld=96) == B.CR_ERR_INVALID_ARG                            # operands narrower than F_pad
    assert fwd(h=FAKE + 2) == B.CR_ERR_INVALID_ARG
    assert fwd(out=None) == B.CR_ERR_INVALID_ARG
    # one-operand (GCN) layers take no h_self; their input gradients need the padded input width to be a multiple of 64
    one = B.cr_sage_layer(256, 47, 1, 0, FAKE, FAKE, FAKE, FAKE)
    assert fwd(layer=one, ld=256) == B.CR_ERR_INVALID_ARG
    assert fwd(layer=one, ld=256, h=None) == B.CR_OK
    assert fwd(h=None) == B.CR_ERR_INVALID_ARG                           # two operands need both
    assert fwd(layer=B.cr_sage_layer(100, 47, 3, 0, FAKE, FAKE, FAKE, FAKE)) == B.CR_ERR_INVALID_ARG
    one_bwd = lambda lay, **kw: lib.cr_sage_linear_bwd(C.byref(lay), vp(), 1000, None, vp(), kw.get("ld", 256), vp(), C.c_float(0.01), C.c_float(0.0),
                                                       vp(kw.get("ds", None)), vp(kw.get("da", None)), vp(kw.get("db", None)), None, None, vp(),
                                                       B.cr_sage_linear_bwd_workspace_bytes(256, 47, 1000), None)
    assert one_bwd(one) == B.CR_OK and one_bwd(one, da=FAKE) == B.CR_OK and one_bwd(one, db=FAKE) == B.CR_OK
    assert one_bwd(one, ds=FAKE, da=FAKE) == B.CR_ERR_INVALID_ARG
    odd = B.cr_sage_layer(96, 47, 1, 0, FAKE, FAKE, FAKE, FAKE)
    assert one_bwd(odd, ld=96) == B.CR_OK and one_bwd(odd, ld=96, db=FAKE) == B.CR_ERR_UNSUPPORTED
    assert fwd(layer=B.cr_sage_layer(0, 47, 2, 0, FAKE, FAKE, FAKE, FAKE)) == B.CR_ERR_INVALID_ARG
    assert fwd(layer=B.cr_sage_layer(100, 47, 2, 0, None, FAKE, FAKE, FAKE)) == B.CR_ERR_INVALID_ARG
    need = B.cr_sage_linear_bwd_workspace_bytes(100, 47, 1000)
    bwd = lambda **kw: lib.cr_sage_linear_bwd(C.byref(layer), vp(), 1000, vp(), vp(), 128, vp(), C.c_float(kw.get("lr", 0.01)), C.c_float(0.0),
                                              vp(kw.get("ds", FAKE)), vp(kw.get("da", FAKE)), vp(kw.get("db", None)), None, None, vp(),
                                              kw.get("ws", need), None)
    assert bwd() == B.CR_OK
    assert bwd(ds=None, da=None) == B.CR_OK                              # layer 0: no input gradient
    assert bwd(ds=None, da=None, db=FAKE) == B.CR_OK                     # input gradient in bf16 only
    assert bwd(db=FAKE + 8) == B.CR_ERR_INVALID_ARG                      # misaligned
    bwd_in = lambda ds, da, db: lib.cr_sage_linear_bwd_input(C.byref(layer), vp(), 1000, vp(), vp(ds), vp(da), vp(db), None)
    assert bwd_in(FAKE, FAKE, None) == B.CR_OK and bwd_in(None, None, FAKE) == B.CR_OK
    assert bwd_in(None, None, None) == B.CR_ERR_INVALID_ARG and bwd_in(FAKE, None, FAKE) == B.CR_ERR_INVALID_ARG
    assert bwd(ds=None) == B.CR_ERR_INVALID_ARG                          # only one of the two
    assert bwd(ws=need - 1) == B.CR_ERR_CAPACITY
    assert bwd(lr=float("nan")) == B.CR_ERR_INVALID_ARG
    xent = lambda **kw: lib.cr_softmax_xent(vp(), 100, vp(kw.get("logits", FAKE)), kw.get("ld", 64), kw.get("C", 47), vp(), vp(), vp(), vp(), None, None, None)
    assert xent() == B.CR_OK
    assert xent(C=65) == B.CR_ERR_INVALID_ARG
    assert xent(C=0) == B.CR_ERR_INVALID_ARG
    assert xent(logits=None) == B.CR_ERR_INVALID_ARG
    cnt = lambda **kw: lib.cr_count_correct(vp(), kw.get("rows", 100), vp(kw.get("logits", FAKE)), kw.get("ld", 64), kw.get("C", 47), vp(), vp(),
                                            vp(kw.get("count", FAKE)), None)
    assert cnt() == B.CR_OK
    assert cnt(C=65) == B.CR_ERR_INVALID_ARG
    assert cnt(rows=0) == B.CR_ERR_INVALID_ARG
    assert cnt(logits=None) == B.CR_ERR_INVALID_ARG
    assert cnt(count=None) == B.CR_ERR_INVALID_ARG


def test_fused_layer_backward_validation():
    lib = B.lib()
    layer = B.cr_sage_layer(100, 47, 2, 0, FAKE, FAKE, FAKE, FAKE)
    need = B.cr_sage_linear_bwd_workspace_bytes(100, 47, 8)

    def call(**kw):
        blocks = kw.get("blocks", block_set())
        return lib.cr_sage_layer_bwd(C.byref(kw.get("layer", layer)), C.byref(blocks), kw.get("g", 0), vp(kw.get("h", FAKE)), vp(),
                                     kw.get("ld", 128), vp(kw.get("dz", FAKE)), C.c_float(0.01), C.c_float(0.0), vp(kw.get("d_in", FAKE)),
                                     vp(kw.get("relu", FAKE)), kw.get("ld_relu", 128), vp(kw.get("d_src", FAKE)), kw.get("ld_bf16", 128),
                                     None, None, vp(), kw.get("ws", need), None)
    assert call() == B.CR_OK
    assert call(relu=None) == B.CR_OK                                     # no ReLU below
    assert call(g=1) == B.CR_ERR_INVALID_ARG
    assert call(blocks=block_set(t=False)) == B.CR_ERR_INVALID_ARG        # needs the transposed block
    assert call(layer=B.cr_sage_layer(128, 47, 1, 0, FAKE, FAKE, FAKE, FAKE), h=None) == B.CR_ERR_INVALID_ARG
    assert call(d_in=None) == B.CR_ERR_INVALID_ARG and call(d_src=None) == B.CR_ERR_INVALID_ARG
    assert call(ld_relu=100) == B.CR_ERR_INVALID_ARG and call(ld_bf16=96) == B.CR_ERR_INVALID_ARG
    assert call(ld=96) == B.CR_ERR_INVALID_ARG and call(dz=None) == B.CR_ERR_INVALID_ARG
    assert call(d_src=FAKE + 4) == B.CR_ERR_INVALID_ARG
    assert call(ws=need - 1) == B.CR_ERR_CAPACITY


def test_forward_with_loss_validation():
    lib = B.lib()
    layer = B.cr_sage_layer(100, 47, 2, 0, FAKE, FAKE, FAKE, FAKE)

    def call(**kw):
        return lib.cr_sage_linear_fwd_xent(C.byref(kw.get("layer", layer)), vp(kw.get("hdr", FAKE)), kw.get("rows", 1024), vp(kw.get("h", FAKE)), vp(),
                                           kw.get("ld", 128), vp(kw.get("logits", FAKE)), kw.get("C", 47), vp(kw.get("labels", FAKE)), vp(),
                                           vp(kw.get("loss", FAKE)), vp(), vp(kw.get("d", FAKE)), vp(kw.get("scratch", FAKE)), None)
    assert call() == B.CR_OK
    assert call(rows=100000) == B.CR_OK                                   # large blocks take the separate kernels
    assert call(hdr=None) == B.CR_ERR_INVALID_ARG and call(rows=0) == B.CR_ERR_INVALID_ARG
    assert call(ld=96) == B.CR_ERR_INVALID_ARG and call(h=None) == B.CR_ERR_INVALID_ARG
    assert call(logits=None) == B.CR_ERR_INVALID_ARG and call(d=None) == B.CR_ERR_INVALID_ARG and call(d=FAKE + 2) == B.CR_ERR_INVALID_ARG
    assert call(C=48) == B.CR_ERR_INVALID_ARG and call(C=0) == B.CR_ERR_INVALID_ARG
    assert call(labels=None) == B.CR_ERR_INVALID_ARG and call(loss=None) == B.CR_ERR_INVALID_ARG
    assert call(scratch=None) == B.CR_ERR_INVALID_ARG


def test_feature_cache_validation():
    lib = B.lib()
    def cache(**kw):
        return B.cr_feature_cache(kw.get("n_sets", 64), kw.get("ways", 16), kw.get("row_bytes", 256), kw.get("n_overflow", 1000),
                                  FAKE, FAKE, kw.get("rows", FAKE), FAKE, FAKE, FAKE)
    fetch = lambda c, **kw: lib.cr_cache_fetch(C.byref(c), vp(kw.get("store", FAKE)), kw.get("ld", 256), vp(), vp(), kw.get("word", 1),
                                               kw.get("max_n", 1000), kw.get("stamp", 0), vp(), None)
    assert lib.cr_cache_reset(C.byref(cache()), None) == B.CR_OK
    assert fetch(cache()) == B.CR_OK
    assert fetch(cache(ways=65)) == B.CR_ERR_INVALID_ARG
    assert fetch(cache(ways=0)) == B.CR_ERR_INVALID_ARG
    assert fetch(cache(n_sets=0)) == B.CR_ERR_INVALID_ARG
    assert fetch(cache(row_bytes=100)) == B.CR_ERR_INVALID_ARG
    assert fetch(cache(rows=None)) == B.CR_ERR_INVALID_ARG
    assert fetch(cache(n_overflow=999)) == B.CR_ERR_CAPACITY            # the overflow area must hold a whole batch
    assert fetch(cache(), ld=128) == B.CR_ERR_INVALID_ARG               # store rows shorter than cache rows
    assert fetch(cache(), word=8) == B.CR_ERR_INVALID_ARG
    assert fetch(cache(), stamp=-1) == B.CR_ERR_INVALID_ARG
    assert fetch(cache(), store=None) == B.CR_ERR_INVALID_ARG
    h, d = C.c_void_p(), C.c_void_p()
    assert lib.cr_host_alloc(0, C.byref(h), C.byref(d)) == B.CR_ERR_INVALID_ARG
    assert lib.cr_host_alloc(1024, C.byref(h), C.byref(d)) == B.CR_OK   # dry run: validated, nothing allocated
    assert h.value is None and d.value is None
    assert lib.cr_host_free(None) == B.CR_OK


def test_graph_attention_validation():
    lib = B.lib()
    # the transposed input block needs its flag, and excludes the global-id input block
    with_t0 = [block_set(1, 10, 48, 528, 480, t=True), block_set(1, 5, 8, 48, 40)]
    assert sample(layers=with_t0, flags=B.CR_SAMPLE_TRANSPOSE_INPUT) == B.CR_OK
    with_t0[0].gather_ids = FAKE
    assert sample(layers=with_t0, flags=B.CR_SAMPLE_TRANSPOSE_INPUT | B.CR_SAMPLE_INPUT_GLOBAL_IDS) == B.CR_ERR_INVALID_ARG

    rows = lambda **kw: lib.cr_gather_rows_bf16(vp(kw.get("store", FAKE)), kw.get("dtype", 0), kw.get("ld_src", 604), kw.get("F", 602), vp(),
                                                vp(), kw.get("word", 1), kw.get("max_n", 100), vp(), kw.get("ld_out", 608), None)
    assert rows() == B.CR_OK
    assert rows(dtype=2) == B.CR_ERR_INVALID_ARG
    assert rows(ld_src=602) == B.CR_ERR_INVALID_ARG            # float rows must keep 16-byte alignment
    assert rows(ld_out=600) == B.CR_ERR_INVALID_ARG            # narrower than F
    assert rows(ld_out=604) == B.CR_ERR_INVALID_ARG            # not a multiple of 8
    assert rows(store=None) == B.CR_ERR_INVALID_ARG
    assert rows(word=8) == B.CR_ERR_INVALID_ARG
    assert rows(max_n=0) == B.CR_ERR_INVALID_ARG

    def params(heads=4, D=64, slope=0.2, attn=FAKE):
        return B.cr_gat_params(heads, D, slope, 0, attn)
    bs = block_set()
    fwd = lambda p, **kw: lib.cr_gat_attention_fwd(C.byref(kw.get("blocks", bs)), kw.get("g", 0), C.byref(p), vp(kw.get("z", FAKE)),
                                                   kw.get("ld", 256), 1, vp(), vp(), vp(kw.get("stat", FAKE)), vp(kw.get("out", FAKE)),
                                                   vp(kw.get("out_b", FAKE)), None)
    assert fwd(params()) == B.CR_OK
    assert fwd(params(heads=1, D=41), ld=64) == B.CR_OK
    assert fwd(params(heads=0)) == B.CR_ERR_INVALID_ARG
    assert fwd(params(heads=4, D=65)) == B.CR_ERR_INVALID_ARG         # heads * D wider than the row
    assert fwd(params(heads=4, D=24), ld=128) == B.CR_ERR_UNSUPPORTED  # several heads: D must be 8 * 2^k
    assert fwd(params(), ld=100) == B.CR_ERR_UNSUPPORTED
    assert fwd(params(heads=16, D=64), ld=1024) == B.CR_ERR_UNSUPPORTED
    assert fwd(params(slope=1.5)) == B.CR_ERR_INVALID_ARG
    assert fwd(params(attn=None)) == B.CR_ERR_INVALID_ARG
    assert fwd(params(), z=None) == B.CR_ERR_INVALID_ARG
    assert fwd(params(), stat=FAKE + 4) == B.CR_ERR_INVALID_ARG
    assert fwd(params(), out=None, out_b=None) == B.CR_ERR_INVALID_ARG
    assert fwd(params(), g=1) == B.CR_ERR_INVALID_ARG
    assert fwd(params(), blocks=block_set(null="indices")) == B.CR_ERR_INVALID_ARG

    need = C.c_size_t(0)
    assert lib.cr_gat_attention_bwd_workspace_bytes(8, 256, 4, C.byref(need)) == B.CR_OK and need.value > 0
    assert lib.cr_gat_attention_bwd_workspace_bytes(0, 256, 4, C.byref(need)) == B.CR_ERR_INVALID_ARG
    bwd = lambda p, **kw: lib.cr_gat_attention_bwd(C.byref(kw.get("blocks", bs)), 0, C.byref(p), vp(), kw.get("ld", 256), vp(), vp(),
                                                   vp(kw.get("d_out", FAKE)), kw.get("ld_dout", 256), vp(), kw.get("lr", 0.1), 0.0,
                                                   vp(kw.get("dz", FAKE)), None, vp(kw.get("ws", FAKE)), kw.get("ws_bytes", need.value), None)
    lib.cr_gat_attention_bwd_workspace_bytes(8, 256, 4, C.byref(need))
    assert bwd(params()) == B.CR_OK
    assert bwd(params(), blocks=block_set(t=False)) == B.CR_ERR_INVALID_ARG     # needs the transposed block
    assert bwd(params(), ld_dout=128) == B.CR_ERR_INVALID_ARG
    assert bwd(params(), d_out=None) == B.CR_ERR_INVALID_ARG
    assert bwd(params(), dz=None) == B.CR_ERR_INVALID_ARG
    assert bwd(params(), lr=float("nan")) == B.CR_ERR_INVALID_ARG
    assert bwd(params(), ws=None) == B.CR_ERR_INVALID_ARG
    assert bwd(params(), ws_bytes=need.value - 1) == B.CR_ERR_CAPACITY

    # a dense layer without a bias term is valid; one without weights is not
    layer = B.cr_sage_layer(64, 64, 1, 0, FAKE, None, FAKE, FAKE)
    assert lib.cr_sage_linear_fwd(C.byref(layer), vp(), 8, None, vp(), 64, 0, vp(), None, None) == B.CR_OK
    layer.W = None
    assert lib.cr_sage_linear_fwd(C.byref(layer), vp(), 8, None, vp(), 64, 0, vp(), None, None) == B.CR_ERR_INVALID_ARG


def test_grouped_gather_validation():
    lib = B.lib()
    def blocks(**kw):
        b = block_set(4, 10, 48, 528, 480, t=False)
        b.gather_ids = kw.get("gather_ids", FAKE)
        b.group_order = kw.get("group_order", FAKE)
        return b
    call = lambda b, **kw: lib.cr_gather_aggregate_fwd_group(C.byref(b), vp(kw.get("H", FAKE)), kw.get("dtype", 0), kw.get("ld_src", 128),
                                                             kw.get("F", 128), vp(kw.get("agg", FAKE)), vp(kw.get("self_", FAKE)),
                                                             kw.get("stride", 48), kw.get("ld", 128), None)
    assert call(blocks()) == B.CR_OK
    assert call(blocks(group_order=None)) == B.CR_ERR_INVALID_ARG       # needs the group's order ...
    assert call(blocks(gather_ids=None)) == B.CR_ERR_INVALID_ARG        # ... and the per-edge global ids
    assert call(blocks(), stride=47) == B.CR_ERR_INVALID_ARG            # batches would overlap
    assert call(blocks(), agg=None) == B.CR_ERR_INVALID_ARG
    assert call(blocks(), ld=100) == B.CR_ERR_INVALID_ARG
    assert call(blocks(), ld_src=126) == B.CR_ERR_INVALID_ARG
    assert call(blocks(), dtype=3) == B.CR_ERR_INVALID_ARG
    assert call(blocks(), H=None) == B.CR_ERR_INVALID_ARG
    assert call(blocks(), self_=None) == B.CR_ERR_INVALID_ARG           # GraphSAGE needs the self rows too
    gcn = lambda b, **kw: lib.cr_gcn_aggregate_fwd_group(C.byref(b), vp(kw.get("norm", FAKE)), vp(kw.get("H", FAKE)), kw.get("dtype", 0),
                                                         kw.get("ld_src", 128), kw.get("F", 128), vp(kw.get("agg", FAKE)), kw.get("stride", 48),
                                                         kw.get("ld", 128), None)
    assert gcn(blocks()) == B.CR_OK
    assert gcn(blocks(), norm=None) == B.CR_ERR_INVALID_ARG
    assert gcn(blocks(group_order=None)) == B.CR_ERR_INVALID_ARG and gcn(blocks(), agg=None) == B.CR_ERR_INVALID_ARG
    assert gcn(blocks(), stride=47) == B.CR_ERR_INVALID_ARG and gcn(blocks(), ld=100) == B.CR_ERR_INVALID_ARG
