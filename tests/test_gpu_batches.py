"""GPU parity: cr_build_batches against the oracle, bit-exact."""
import numpy as np
import pytest

import oracle

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_mod():
    import torch
    assert torch.cuda.is_available()
    return torch


def run_gpu(torch, policy, mix, seed, epoch, train_ids, comm, n_comm, batch_size=256):
    from paper_2504_18082_amd import binding as B
    d_train = torch.from_numpy(np.ascontiguousarray(train_ids, dtype=np.int32)).cuda()
    d_comm = torch.from_numpy(np.ascontiguousarray(comm, dtype=np.int32)).cuda()
    ws = torch.empty(B.cr_build_batches_workspace_bytes(len(train_ids), n_comm), dtype=torch.uint8, device="cuda")
    out = torch.full((max(1, len(train_ids)),), -1, dtype=torch.int32, device="cuda")
    nb = B.cr_build_batches(policy, mix, batch_size, seed, epoch, d_train, d_comm, n_comm, ws, out)
    torch.cuda.synchronize()
    assert nb == -(-len(train_ids) // batch_size)
    return out.cpu().numpy()[:len(train_ids)]


@pytest.mark.parametrize("policy,mix", [(0, 1), (2, 1), (1, 1), (1, 6), (1, 12), (1, 25), (1, 49), (1, 50), (1, 1000)])
def test_tiny(torch_mod, tiny_workload, policy, mix):
    w = tiny_workload
    for seed, epoch in ((0, 0), (12345678901234567, 7)):
        print(f"case tiny policy={policy} mix={mix} seed={seed} epoch={epoch}", flush=True)
        want = oracle.build_batches(policy, mix, seed, epoch, w.train_ids, w.comm, w.cfg.n_comm)
        got = run_gpu(torch_mod, policy, mix, seed, epoch, w.train_ids, w.comm, w.cfg.n_comm)
        assert np.array_equal(got, want)


@pytest.mark.parametrize("policy,mix", [(2, 1), (1, 1), (1, 62), (1, 125)])
def test_arxiv(torch_mod, arxiv_workload, policy, mix):
    w = arxiv_workload      # 93K training nodes: 46 sort tiles and a ragged tail; power-law community sizes
    print(f"case arxiv policy={policy} mix={mix}", flush=True)
    want = oracle.build_batches(policy, mix, 5, 3, w.train_ids, w.comm, w.cfg.n_comm)
    got = run_gpu(torch_mod, policy, mix, 5, 3, w.train_ids, w.comm, w.cfg.n_comm, 1024)
    assert np.array_equal(got, want)


def test_unordered_membership_absent_communities_and_tiny_sets(torch_mod):
    rng = np.random.default_rng(0)
    comm = rng.integers(0, 37, size=5000).astype(np.int32)
    comm[comm == 11] = 12                                   # community 11 is empty
    train = np.sort(rng.choice(5000, size=1700, replace=False)).astype(np.int32)
    train = train[comm[train] != 20]                        # community 20 has nodes but none in training
    for policy, mix in ((1, 1), (1, 4), (2, 1)):
        want = oracle.build_batches(policy, mix, 9, 1, train, comm, 37)
        got = run_gpu(torch_mod, policy, mix, 9, 1, train, comm, 37)
        assert np.array_equal(got, want), (policy, mix)
    one = np.array([4242], dtype=np.int32)
    for policy in (0, 1, 2):
        assert run_gpu(torch_mod, policy, 1, 1, 1, one, comm, 37).tolist() == [4242]
    two = np.array([7, 4242], dtype=np.int32)
    for epoch in range(4):
        want = oracle.build_batches(1, 1, 1, epoch, two, comm, 37)
        assert np.array_equal(run_gpu(torch_mod, 1, 1, 1, epoch, two, comm, 37), want)
