"""GPU parity: cr_sage_linear_fwd / _bwd (+SGD) and cr_softmax_xent against the oracle.

The GPU feeds bf16 operands to the matrix cores and accumulates in float; the oracle is asked for the
same operand rounding and accumulates in double.  Tolerance 2e-2 relative (bf16 path)."""
import ctypes as C

import numpy as np
import pytest

import oracle
from paper_2504_18082_amd import synth
from gpu_util import assert_close, bf16_tensor_to_float

pytestmark = pytest.mark.gpu
RTOL_BF16 = 2e-2
RTOL_F32 = 1e-5


@pytest.fixture(scope="module")
def torch_mod():
    import torch
    assert torch.cuda.is_available()
    return torch


def to_bf16_dev(torch, x, ld):
    """float array [M, F] -> device int16 [M, ld] of bf16 bits, zero padded."""
    M, F = x.shape
    buf = np.zeros((M, ld), dtype=np.uint16)
    buf[:, :F] = synth.float_to_bf16_bits(x.astype(np.float32))
    return torch.from_numpy(buf.view(np.int16)).cuda()


def hdr_for(torch, n_rows):
    h = torch.zeros(8, dtype=torch.int32, device="cuda")
    h[0] = n_rows
    return h


@pytest.mark.parametrize("M,F_in,F_out,relu", [(300, 64, 64, True), (1000, 100, 256, True), (517, 256, 40, False),
                                               (130, 602, 256, True), (64, 32, 10, False), (1, 64, 64, True),
                                               (33001, 64, 256, True), (66010, 100, 128, False),     # several workgroup rounds
                                               (5000, 400, 256, True)])                             # few workgroups, long K loop
def test_linear_fwd(torch_mod, M, F_in, F_out, relu):
    torch = torch_mod
    from paper_2504_18082_amd import binding as B
    rng = np.random.default_rng(M + F_in)
    print(f"case fwd M={M} F_in={F_in} F_out={F_out}", flush=True)
    hs = rng.standard_normal((M, F_in)).astype(np.float32)
    ag = rng.standard_normal((M, F_in)).astype(np.float32) * 0.5
    W = (rng.standard_normal((2 * F_in, F_out)) / np.sqrt(2 * F_in)).astype(np.float32)
    b = rng.standard_normal(F_out).astype(np.float32) * 0.1
    want = oracle.sage_linear_fwd(hs, ag, W, b, relu, True)

    layer = B.SageLayer(W, b)
    layer.refresh()
    cap = M + 37                                     # capacity above the live row count
    ld_in = layer.F_pad
    d_hs, d_ag = to_bf16_dev(torch, np.pad(hs, ((0, 37), (0, 0))), ld_in), to_bf16_dev(torch, np.pad(ag, ((0, 37), (0, 0))), ld_in)
    out = torch.full((cap, layer.N_pad), np.nan, dtype=torch.float32, device="cuda")
    out_b = torch.full((cap, layer.N_pad), 0x7FC0, dtype=torch.int16, device="cuda")
    hdr = hdr_for(torch, M)
    B.cr_sage_linear_fwd(layer, C.c_void_p(hdr.data_ptr()), cap, d_hs, d_ag, ld_in, relu, out, out_b)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert_close(got[:M, :F_out], want, RTOL_BF16, "out")
    # far tighter in practice: only the accumulation differs
    assert_close(got[:M, :F_out], want, 1e-4, "out (accumulation only)")
    assert np.all(got[:M, F_out:] == 0) or not relu
    assert np.all(np.isnan(got[M:]))                  # rows past the header's count untouched
    gb = bf16_tensor_to_float(out_b)
    assert_close(gb[:M, :F_out], want, RTOL_BF16, "out_bf16")


@pytest.mark.parametrize("M,F_in,F_out,relu,cap,n_op", [
    (20001, 128, 256, True, None, 2), (61221, 100, 256, True, None, 2), (16384, 128, 200, False, None, 2),
    (17003, 256, 256, True, None, 2),          # K = 512: four chunks of 128
    (100, 128, 256, True, 16500, 2),           # fewer rows than one tile holds, capacity still large
    (16640, 128, 256, False, 16700, 2),        # last tile moved back onto its neighbour
    (18000, 602, 256, False, None, 1),         # one operand, K = 608: five chunks, the last one a partial one
    (16500, 32, 256, True, None, 1),           # one operand, K = 32: a single partial chunk
    (40, 128, 256, True, 16500, 2),            # fewer rows than the streaming kernel's 64-row tile
    (19201, 64, 256, False, None, 2),          # K = 128: the streaming kernel with half the weight registers; a moved-back tile
    (70003, 128, 256, True, None, 2),          # several tiles per workgroup of the persistent streaming kernel
    (16500, 128, 256, True, None, 1),          # one operand, K = 128: half of the streaming kernel's waves have no piece to load
    (17003, 602, 256, True, None, 2),          # two operands of 608 columns: five chunks each, both with a partial last one
    (16400, 96, 256, True, None, 2),           # K = 192 with the operands meeting inside a wave's sixteen pieces (per-thread addresses)
    (16400, 256, 256, False, None, 1),         # one operand, K = 256: every wave loads from the same array
    (5000, 602, 256, True, None, 2),           # a few thousand rows against K = 1216: the tiled kernel with the deep prefetch
    (4200, 800, 256, False, None, 1),          # the same, one operand of 800 columns
    (0, 128, 256, True, 16500, 2)])            # no live row at all: nothing may be written
def test_linear_fwd_many_rows_bf16_output(torch_mod, M, F_in, F_out, relu, cap, n_op):
    """The input layer of the large workloads: tens of thousands of rows, N = 256 after padding, bf16 output only
    (K <= 256: the streaming kernel, weights in registers, 64-row tiles; larger K: the weight-stationary kernel, 256 rows
    x all columns per workgroup, K in chunks of 128)."""
    torch = torch_mod
    from paper_2504_18082_amd import binding as B
    rng = np.random.default_rng(M + F_in)
    print(f"case fwd wide M={M} F_in={F_in} F_out={F_out} cap={cap} operands={n_op}", flush=True)
    hs = rng.standard_normal((M, F_in)).astype(np.float32)
    ag = rng.standard_normal((M, F_in)).astype(np.float32) * 0.5
    W = (rng.standard_normal((n_op * F_in, F_out)) / np.sqrt(n_op * F_in)).astype(np.float32)
    b = rng.standard_normal(F_out).astype(np.float32) * 0.1
    oracle.use_all_cores(True)
    try:
        if n_op == 2:
            want = oracle.sage_linear_fwd(hs, ag, W, b, relu, True)
        else:                                        # (zero self operand against zero weights adds exact zeros)
            want = oracle.sage_linear_fwd(np.zeros_like(ag), ag, np.vstack([np.zeros_like(W), W]), b, relu, True)
    finally:
        oracle.use_all_cores(False)
    layer = B.SageLayer(W, b, n_operands=n_op)
    layer.refresh()
    cap = cap or M + 300                             # capacity above the live row count: whole workgroups without rows
    ld_in = layer.F_pad
    pad = ((0, cap - M), (0, 0))
    # rows past the live ones hold NaNs: they may be read but must not reach any stored result
    d_hs = to_bf16_dev(torch, np.pad(hs, pad, constant_values=np.nan), ld_in)
    d_ag = to_bf16_dev(torch, np.pad(ag, pad, constant_values=np.nan), ld_in)
    out_b = torch.full((cap, layer.N_pad), 0x7FC0, dtype=torch.int16, device="cuda")
    hdr = hdr_for(torch, M)
    B.cr_sage_linear_fwd(layer, C.c_void_p(hdr.data_ptr()), cap, d_hs if n_op == 2 else None, d_ag, ld_in, relu, None, out_b)
    torch.cuda.synchronize()
    gb = bf16_tensor_to_float(out_b)
    # one rounding to bf16 (2^-9 relative) on top of the float accumulation
    assert_close(gb[:M, :F_out], want, 2.0 ** -8, "out_bf16")
    assert np.all(gb[:M, F_out:] == 0)
    assert np.all(out_b[M:].cpu().numpy() == 0x7FC0)          # rows past the header's count untouched


@pytest.mark.parametrize("M,F_in,F_out,need_dx", [(300, 64, 64, True), (2500, 100, 256, False), (777, 256, 40, True),
                                                  (200, 602, 256, False), (33, 32, 10, True)])
def test_linear_bwd_and_sgd(torch_mod, M, F_in, F_out, need_dx):
    torch = torch_mod
    from paper_2504_18082_amd import binding as B
    rng = np.random.default_rng(M * 3 + F_out)
    print(f"case bwd M={M} F_in={F_in} F_out={F_out} need_dx={need_dx}", flush=True)
    hs = rng.standard_normal((M, F_in)).astype(np.float32)
    ag = rng.standard_normal((M, F_in)).astype(np.float32) * 0.5
    W = (rng.standard_normal((2 * F_in, F_out)) / np.sqrt(2 * F_in)).astype(np.float32)
    b = rng.standard_normal(F_out).astype(np.float32) * 0.1
    dz = (rng.standard_normal((M, F_out)) / M).astype(np.float32)
    dz[rng.random((M, F_out)) < 0.4] = 0.0            # as after a ReLU mask
    # oracle: relu flag off, the mask is already in dz; `out` unused then
    dW, db, d_self, d_agg = oracle.sage_linear_bwd(hs, ag, W, np.ones((M, F_out)), dz, False, True, need_dx=need_dx)
    # db sums the bf16-rounded dz on the GPU (it reads the same operand as the matrix cores)
    db = oracle.round_bf16(dz).sum(axis=0)
    lr, wd = 0.05, 5e-4
    W_new, b_new = oracle.sgd_step(W, dW, b, db, lr, wd)

    layer = B.SageLayer(W, b)
    layer.refresh()
    cap = M + 100
    ld_in = layer.F_pad
    pad = lambda x: np.pad(x, ((0, 100), (0, 0)), constant_values=3.0)     # junk rows past the live count
    d_hs, d_ag = to_bf16_dev(torch, pad(hs), ld_in), to_bf16_dev(torch, pad(ag), ld_in)
    d_dz = to_bf16_dev(torch, pad(dz), layer.N_pad)
    ws = torch.empty(B.cr_sage_linear_bwd_workspace_bytes(F_in, F_out, cap), dtype=torch.uint8, device="cuda")
    g_self = torch.full((cap, layer.F_pad), np.nan, dtype=torch.float32, device="cuda") if need_dx else None
    g_agg = torch.full((cap, layer.F_pad), np.nan, dtype=torch.float32, device="cuda") if need_dx else None
    dW_out = torch.zeros((2 * F_in, F_out), dtype=torch.float32, device="cuda")
    db_out = torch.zeros(F_out, dtype=torch.float32, device="cuda")
    hdr = hdr_for(torch, M)
    g_in_b = torch.full((cap, 2 * layer.F_pad), 0x7FC0, dtype=torch.int16, device="cuda") if need_dx else None
    B.cr_sage_linear_bwd(layer, C.c_void_p(hdr.data_ptr()), cap, d_hs, d_ag, ld_in, d_dz, lr, wd, g_self, g_agg, ws, dW_out, db_out,
                         d_in_bf16=g_in_b)
    torch.cuda.synchronize()
    assert_close(dW_out.cpu().numpy(), dW, RTOL_BF16, "dW")
    assert_close(dW_out.cpu().numpy(), dW, 1e-4, "dW (accumulation only)")
    assert_close(db_out.cpu().numpy(), db, 1e-4, "db")
    assert_close(layer.W.cpu().numpy(), W_new, RTOL_F32, "W after SGD")
    assert_close(layer.bias.cpu().numpy()[:F_out], b_new, RTOL_F32, "bias after SGD")
    # shadows follow the master
    wb = bf16_tensor_to_float(layer.W_bf16)
    wt = bf16_tensor_to_float(layer.Wt_bf16)
    Wn = layer.W.cpu().numpy()
    Fp = layer.F_pad
    for part in (0, 1):
        blockW = wb[part * Fp:part * Fp + F_in, :F_out]
        np.testing.assert_array_equal(blockW.astype(np.float64), oracle.round_bf16(Wn[part * F_in:(part + 1) * F_in]))
        assert np.all(wb[part * Fp + F_in:(part + 1) * Fp] == 0)
    assert np.all(wb[:, F_out:] == 0)
    np.testing.assert_array_equal(wt, wb.T)
    if need_dx:
        assert_close(g_self.cpu().numpy()[:M, :F_in], d_self, RTOL_BF16, "d_self")
        assert_close(g_agg.cpu().numpy()[:M, :F_in], d_agg, RTOL_BF16, "d_agg")
        assert_close(g_self.cpu().numpy()[:M, :F_in], d_self, 1e-4, "d_self (accumulation only)")
        assert np.all(g_self.cpu().numpy()[:M, F_in:] == 0)
        # the bf16 copy is the float result rounded to nearest even, [d_self | d_agg] side by side
        both = np.concatenate([g_self.cpu().numpy()[:M], g_agg.cpu().numpy()[:M]], axis=1)
        np.testing.assert_array_equal(g_in_b.cpu().numpy()[:M].view(np.uint16), synth.float_to_bf16_bits(both))


@pytest.mark.parametrize("M,F_in,F_out", [(777, 100, 40), (70000, 64, 64)])
def test_linear_bwd_input_only(torch_mod, M, F_in, F_out):
    """cr_sage_linear_bwd_input against the oracle, float and bf16 outputs."""
    torch = torch_mod
    from paper_2504_18082_amd import binding as B
    rng = np.random.default_rng(M + 5 * F_out)
    print(f"case bwd_input M={M} F_in={F_in} F_out={F_out}", flush=True)
    W = (rng.standard_normal((2 * F_in, F_out)) / np.sqrt(2 * F_in)).astype(np.float32)
    dz = (rng.standard_normal((M, F_out)) / 8).astype(np.float32)
    zeros = np.zeros((M, F_in), dtype=np.float32)
    _, _, d_self, d_agg = oracle.sage_linear_bwd(zeros, zeros, W, np.ones((M, F_out)), dz, False, True, need_dx=True)
    layer = B.SageLayer(W, np.zeros(F_out, np.float32))
    layer.refresh()
    cap = M + 50
    d_dz = to_bf16_dev(torch, np.pad(dz, ((0, 50), (0, 0)), constant_values=2.0), layer.N_pad)
    g_self = torch.full((cap, layer.F_pad), np.nan, dtype=torch.float32, device="cuda")
    g_agg = torch.full((cap, layer.F_pad), np.nan, dtype=torch.float32, device="cuda")
    g_in_b = torch.full((cap, 2 * layer.F_pad), 0x7FC0, dtype=torch.int16, device="cuda")
    hdr = hdr_for(torch, M)
    B.cr_sage_linear_bwd_input(layer, C.c_void_p(hdr.data_ptr()), cap, d_dz, g_self, g_agg, d_in_bf16=g_in_b)
    torch.cuda.synchronize()
    gs, ga = g_self.cpu().numpy(), g_agg.cpu().numpy()
    assert_close(gs[:M, :F_in], d_self, 1e-4, "d_self")
    assert_close(ga[:M, :F_in], d_agg, 1e-4, "d_agg")
    assert np.all(gs[:M, F_in:] == 0) and np.all(ga[:M, F_in:] == 0)
    assert np.all(np.isnan(gs[M:])) and np.all(np.isnan(ga[M:]))
    np.testing.assert_array_equal(g_in_b.cpu().numpy()[:M].view(np.uint16), synth.float_to_bf16_bits(np.concatenate([gs[:M], ga[:M]], axis=1)))
    assert np.all(g_in_b.cpu().numpy()[M:].view(np.uint16) == 0x7FC0)


@pytest.mark.parametrize("n,Cn", [(256, 10), (1024, 40), (1000, 172), (1, 7)])
def test_softmax_xent(torch_mod, n, Cn):
    torch = torch_mod
    from paper_2504_18082_amd import binding as B
    rng = np.random.default_rng(n + Cn)
    ld = (Cn + 63) // 64 * 64
    logits = np.zeros((n + 5, ld), dtype=np.float32)
    logits[:, :Cn] = rng.standard_normal((n + 5, Cn)).astype(np.float32) * 4
    logits[:, Cn:] = 99.0                               # padded columns must be ignored
    n_nodes = 5000
    labels_all = rng.integers(0, Cn, size=n_nodes).astype(np.int32)
    roots = rng.choice(n_nodes, size=n + 5, replace=False).astype(np.int32)
    want_loss, want_d = oracle.softmax_xent(logits[:n].astype(np.float64), labels_all[roots[:n]], n_classes=Cn)
    up = lambda a: torch.from_numpy(a).cuda()
    d_roots = up(roots)
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    row_loss = torch.zeros(n + 5, dtype=torch.float32, device="cuda")
    d = torch.full((n + 5, ld), np.nan, dtype=torch.float32, device="cuda")
    db = torch.full((n + 5, ld), 0x7FC0, dtype=torch.int16, device="cuda")
    hdr = hdr_for(torch, n)
    B.cr_softmax_xent(C.c_void_p(hdr.data_ptr()), n + 5, up(logits), ld, Cn, up(labels_all), C.c_void_p(d_roots.data_ptr()),
                      loss, row_loss, d, db)
    torch.cuda.synchronize()
    assert abs(float(loss.cpu()[0]) - want_loss) <= RTOL_F32 * max(1.0, abs(want_loss))
    got = d.cpu().numpy()
    assert_close(got[:n], want_d, RTOL_F32, "d_logits")
    assert np.all(got[:n, Cn:] == 0) and np.all(np.isnan(got[n:]))
    assert_close(bf16_tensor_to_float(db)[:n], want_d, 2.0 ** -8, "d_logits bf16")


@pytest.mark.parametrize("M,F_in,Cn,cap_extra", [(1000, 256, 40, 24), (1024, 100, 47, 0), (33, 64, 64, 7), (1, 32, 3, 0),
                                                 (300, 64, 172, 5), (2500, 64, 10, 12),      # these and the next: separate kernels inside
                                                 (9000, 32, 172, 100)])
def test_linear_fwd_with_loss(torch_mod, M, F_in, Cn, cap_extra):
    """cr_sage_linear_fwd_xent: logits bit-identical to cr_sage_linear_fwd, loss and gradient against the oracle's
    softmax cross-entropy of those logits; two calls in a row on the same scratch, the second on fewer rows."""
    torch = torch_mod
    from paper_2504_18082_amd import binding as B
    rng = np.random.default_rng(M + 3 * Cn)
    hs = rng.standard_normal((M, F_in)).astype(np.float32)
    ag = rng.standard_normal((M, F_in)).astype(np.float32) * 0.5
    W = (rng.standard_normal((2 * F_in, Cn)) * 3 / np.sqrt(2 * F_in)).astype(np.float32)
    b = rng.standard_normal(Cn).astype(np.float32) * 0.1
    layer = B.SageLayer(W, b)
    layer.refresh()
    cap = M + cap_extra
    ld_in, Np = layer.F_pad, layer.N_pad
    d_hs = to_bf16_dev(torch, np.pad(hs, ((0, cap_extra), (0, 0))), ld_in)
    d_ag = to_bf16_dev(torch, np.pad(ag, ((0, cap_extra), (0, 0))), ld_in)
    n_nodes = 12000
    labels_all = rng.integers(0, Cn, size=n_nodes).astype(np.int32)
    roots = rng.choice(n_nodes, size=cap, replace=False).astype(np.int32)
    up = lambda a: torch.from_numpy(a).cuda()
    d_labels, d_roots = up(labels_all), up(roots)
    scratch = torch.zeros(B.CR_XENT_SCRATCH_BYTES, dtype=torch.uint8, device="cuda")
    for rows in (M, max(1, M // 3)):
        print(f"case fwd+loss M={rows} F_in={F_in} classes={Cn} cap={cap}", flush=True)
        hdr = hdr_for(torch, rows)
        ref = torch.full((cap, Np), np.nan, dtype=torch.float32, device="cuda")
        B.cr_sage_linear_fwd(layer, C.c_void_p(hdr.data_ptr()), cap, d_hs, d_ag, ld_in, False, ref, None)
        logits = torch.full((cap, Np), np.nan, dtype=torch.float32, device="cuda")
        loss = torch.full((1,), np.nan, dtype=torch.float32, device="cuda")
        row_loss = torch.zeros(cap, dtype=torch.float32, device="cuda")
        db = torch.full((cap, Np), 0x7FC0, dtype=torch.int16, device="cuda")
        B.cr_sage_linear_fwd_xent(layer, C.c_void_p(hdr.data_ptr()), cap, d_hs, d_ag, ld_in, logits, Cn, d_labels,
                                  C.c_void_p(d_roots.data_ptr()), loss, row_loss, db, scratch)
        torch.cuda.synchronize()
        got = logits.cpu().numpy()
        np.testing.assert_array_equal(got[:rows], ref.cpu().numpy()[:rows])
        assert np.all(np.isnan(got[rows:]))
        want_loss, want_d = oracle.softmax_xent(got[:rows].astype(np.float64), labels_all[roots[:rows]], n_classes=Cn)
        assert abs(float(loss.cpu()[0]) - want_loss) <= RTOL_F32 * max(1.0, abs(want_loss))
        gd = bf16_tensor_to_float(db)
        assert_close(gd[:rows, :Cn], want_d[:, :Cn], 2.0 ** -8, "d_logits bf16")
        assert np.all(gd[:rows, Cn:] == 0)
        assert np.all(db.cpu().numpy()[rows:].view(np.uint16) == 0x7FC0)
        assert np.all(scratch.cpu().numpy()[:8] == 0)            # the accumulator is back at zero


@pytest.mark.parametrize("n,Cn", [(256, 10), (1024, 40), (1000, 172), (1, 7), (3, 1)])
def test_count_correct(torch_mod, n, Cn):
    """Integer result: the same float32 logits go to both sides, so the counts must agree exactly
    (ties included: the lowest class index wins on both sides)."""
    torch = torch_mod
    from paper_2504_18082_amd import binding as B
    rng = np.random.default_rng(7 * n + Cn)
    ld = (Cn + 63) // 64 * 64
    logits = np.zeros((n + 5, ld), dtype=np.float32)
    logits[:, :Cn] = np.round(rng.standard_normal((n + 5, Cn)) * 2).astype(np.float32)    # coarse values: many exact ties
    logits[:, Cn:] = 99.0                               # padded columns must be ignored
    n_nodes = 5000
    labels_all = rng.integers(0, Cn, size=n_nodes).astype(np.int32)
    roots = rng.choice(n_nodes, size=n + 5, replace=False).astype(np.int32)
    # make about half of the rows correct so that the count is not trivially small
    for i in range(0, n, 2):
        labels_all[roots[i]] = int(np.argmax(logits[i, :Cn]))
    want = oracle.count_correct(logits[:n, :Cn].astype(np.float64), labels_all[roots[:n]])
    up = lambda a: torch.from_numpy(a).cuda()
    d_roots = up(roots)
    count = torch.full((1,), 11, dtype=torch.int32, device="cuda")     # accumulates on top of what is there
    hdr = hdr_for(torch, n)
    B.cr_count_correct(C.c_void_p(hdr.data_ptr()), n + 5, up(logits), ld, Cn, up(labels_all), C.c_void_p(d_roots.data_ptr()), count)
    torch.cuda.synchronize()
    assert int(count.cpu()[0]) == 11 + want


@pytest.mark.parametrize("M,F_in,F_out,relu,need_dx", [(300, 64, 64, True, True), (1000, 100, 256, True, False), (517, 256, 40, False, True),
                                                       (2500, 128, 256, True, True), (1, 64, 64, True, True)])
def test_one_operand_layer(torch_mod, M, F_in, F_out, relu, need_dx):
    """A layer with a single aggregated input (GCN): Z = Agg W + b, its backward and SGD step.  The oracle is the
    two-operand one with a zero self operand and zero W_self rows, which adds exact zeros."""
    torch = torch_mod
    from paper_2504_18082_amd import binding as B
    rng = np.random.default_rng(M * 7 + F_in)
    print(f"case one-operand M={M} F_in={F_in} F_out={F_out}", flush=True)
    ag = rng.standard_normal((M, F_in)).astype(np.float32)
    W = (rng.standard_normal((F_in, F_out)) / np.sqrt(F_in)).astype(np.float32)
    b = rng.standard_normal(F_out).astype(np.float32) * 0.1
    zeros, W2 = np.zeros_like(ag), np.vstack([np.zeros_like(W), W])
    want = oracle.sage_linear_fwd(zeros, ag, W2, b, relu, True)
    dz = (rng.standard_normal((M, F_out)) / M).astype(np.float32)
    dz[rng.random((M, F_out)) < 0.4] = 0.0
    dW2, _, _, d_agg = oracle.sage_linear_bwd(zeros, ag, W2, np.ones((M, F_out)), dz, False, True, need_dx=need_dx)
    dW = dW2[F_in:]
    db = oracle.round_bf16(dz).sum(axis=0)
    lr, wd = 0.05, 5e-4
    W_new2, b_new = oracle.sgd_step(W2, dW2, b, db, lr, wd)

    layer = B.SageLayer(W, b, n_operands=1)
    layer.refresh()
    cap = M + 37
    ld_in = layer.F_pad
    d_ag = to_bf16_dev(torch, np.pad(ag, ((0, 37), (0, 0)), constant_values=2.0), ld_in)
    out = torch.full((cap, layer.N_pad), np.nan, dtype=torch.float32, device="cuda")
    hdr = hdr_for(torch, M)
    B.cr_sage_linear_fwd(layer, C.c_void_p(hdr.data_ptr()), cap, None, d_ag, ld_in, relu, out, None)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert_close(got[:M, :F_out], want, 1e-4, "out")
    assert np.all(np.isnan(got[M:]))

    d_dz = to_bf16_dev(torch, np.pad(dz, ((0, 37), (0, 0)), constant_values=3.0), layer.N_pad)
    ws = torch.empty(B.cr_sage_linear_bwd_workspace_bytes(F_in, F_out, cap), dtype=torch.uint8, device="cuda")
    g_agg = torch.full((cap, layer.F_pad), np.nan, dtype=torch.float32, device="cuda") if need_dx else None
    g_in_b = torch.full((cap, layer.F_pad), 0x7FC0, dtype=torch.int16, device="cuda") if need_dx else None
    dW_out = torch.zeros((F_in, F_out), dtype=torch.float32, device="cuda")
    db_out = torch.zeros(F_out, dtype=torch.float32, device="cuda")
    B.cr_sage_linear_bwd(layer, C.c_void_p(hdr.data_ptr()), cap, None, d_ag, ld_in, d_dz, lr, wd, None, g_agg, ws, dW_out, db_out,
                         d_in_bf16=g_in_b)
    torch.cuda.synchronize()
    assert_close(dW_out.cpu().numpy(), dW, 1e-4, "dW")
    assert_close(db_out.cpu().numpy(), db, 1e-4, "db")
    assert_close(layer.W.cpu().numpy(), W_new2[F_in:], RTOL_F32, "W after SGD")
    assert_close(layer.bias.cpu().numpy()[:F_out], b_new, RTOL_F32, "bias after SGD")
    wb = bf16_tensor_to_float(layer.W_bf16)
    np.testing.assert_array_equal(wb[:F_in, :F_out].astype(np.float64), oracle.round_bf16(layer.W.cpu().numpy()))
    np.testing.assert_array_equal(bf16_tensor_to_float(layer.Wt_bf16), wb.T)
    if need_dx:
        assert_close(g_agg.cpu().numpy()[:M, :F_in], d_agg, 1e-4, "d_agg")
        np.testing.assert_array_equal(g_in_b.cpu().numpy()[:M].view(np.uint16), synth.float_to_bf16_bits(g_agg.cpu().numpy()[:M]))
