"""GPU: cr_build_batches_static (root partitioning with the library's fixed scratch array, for callers that cannot
allocate device memory) against cr_build_batches, bit for bit, on two calls in a row, the second on a smaller input.
Runs last (file name) so that a failure here hides no other test."""
import numpy as np
import pytest

from paper_2504_18082_amd import synth

pytestmark = pytest.mark.gpu


def _both(B, torch, w, policy, mix, epoch, seed):
    cfg = w.cfg
    train = torch.from_numpy(w.train_ids.astype(np.int32)).cuda()
    comm = torch.from_numpy(w.comm.astype(np.int32)).cuda()
    ws = torch.empty(B.cr_build_batches_workspace_bytes(train.numel(), cfg.n_comm), dtype=torch.uint8, device="cuda")
    want = torch.full((train.numel(),), -1, dtype=torch.int32, device="cuda")
    got = torch.full((train.numel(),), -2, dtype=torch.int32, device="cuda")
    nb_want = B.cr_build_batches(policy, mix, cfg.batch_size, seed, epoch, train, comm, cfg.n_comm, ws, want)
    before = torch.cuda.memory_allocated()
    nb_got = B.cr_build_batches_static(policy, mix, cfg.batch_size, seed, epoch, train, comm, cfg.n_comm, got)
    assert torch.cuda.memory_allocated() == before            # (torch's view; the library itself calls no allocator)
    torch.cuda.synchronize()
    assert nb_got == nb_want
    assert np.array_equal(got.cpu().numpy(), want.cpu().numpy())
    return got.cpu().numpy()


def test_static_scratch_entry_point_matches_workspace_entry_point(arxiv_workload, tiny_workload):
    import torch
    from paper_2504_18082_amd import binding as B
    import oracle
    print("case: arxiv-like training set, COMM-RAND mix 62, then tiny, RAND and COMM-RAND mix 6", flush=True)
    big = _both(B, torch, arxiv_workload, B.CR_ROOTS_COMM_RAND, 62, 3, 0)
    # the larger call left its keys, histograms and community tables in the shared array: a smaller input, another
    # policy and another seed must not see them
    small = _both(B, torch, tiny_workload, B.CR_ROOTS_RAND, 1, 1, 7)
    small2 = _both(B, torch, tiny_workload, B.CR_ROOTS_COMM_RAND, 6, 2, 0)
    _both(B, torch, tiny_workload, B.CR_ROOTS_NORAND, 1, 0, 0)
    # and both equal the oracle's partition
    w = tiny_workload
    assert np.array_equal(small, oracle.build_batches(oracle.RAND, 1, 7, 1, w.train_ids, w.comm, w.cfg.n_comm))
    assert np.array_equal(small2, oracle.build_batches(oracle.COMM_RAND, 6, 0, 2, w.train_ids, w.comm, w.cfg.n_comm))
    w = arxiv_workload
    assert np.array_equal(big, oracle.build_batches(oracle.COMM_RAND, 62, 0, 3, w.train_ids, w.comm, w.cfg.n_comm))
