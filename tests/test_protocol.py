"""Host logic of the training protocol (Section 5, training methodology): the plateau scheduler against
PyTorch's ReduceLROnPlateau, early stopping against its definition, and the validation split of the
synthetic workloads."""
import numpy as np
import pytest

from paper_2504_18082_amd import protocol, synth


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_plateau_scheduler_matches_torch(seed):
    import torch
    rng = np.random.default_rng(seed)
    # a noisy, slowly flattening loss curve with a few long plateaus
    n = 80
    curve = 2.0 * np.exp(-np.arange(n) / 10.0) + 0.5 + 0.02 * rng.standard_normal(n)
    curve[30:45] = curve[29] + 0.01
    param = torch.nn.Parameter(torch.zeros(1))
    opt = torch.optim.SGD([param], lr=0.01)
    ref = torch.optim.lr_scheduler.ReduceLROnPlateau(opt, mode="min", factor=0.1, patience=3)
    mine = protocol.PlateauScheduler(0.01, patience=3, factor=0.1)
    for v in curve:
        ref.step(float(v))
        lr = mine.step(float(v))
        assert lr == pytest.approx(opt.param_groups[0]["lr"], rel=1e-12)
    assert mine.lr < 0.01          # the curve does contain a plateau, so the test exercised a cut


def test_early_stopping_definition():
    es = protocol.EarlyStopping(patience=3)
    seq = [1.0, 0.9, 0.95, 0.91, 0.8, 0.81, 0.82, 0.83, 0.7]
    stops = [es.step(v, i) for i, v in enumerate(seq)]
    # best at index 4 (0.8); three epochs without improvement end at index 7
    assert stops == [False, False, False, False, False, False, False, True, False]
    es = protocol.EarlyStopping(patience=2)
    assert [es.step(v, i) for i, v in enumerate([3.0, 2.0, 1.0, 0.5])] == [False] * 4
    assert es.best == 0.5 and es.best_epoch == 3


def test_history_summary():
    h = protocol.History(epoch_ms=[10.0, 12.0, 11.0], train_loss=[2, 1, 0.9], val_loss=[2.0, 1.2, 1.3], val_acc=[0.2, 0.6, 0.58],
                         lr=[0.01] * 3)
    s = h.summary()
    assert s["epochs"] == 3 and s["best_val_acc"] == 0.6 and s["final_val_acc"] == 0.58
    assert s["total_train_ms"] == pytest.approx(33.0)


def test_validation_split(tiny_workload):
    w = tiny_workload
    assert w.val_ids.dtype == np.int32 and np.all(np.diff(w.val_ids) > 0)
    assert np.intersect1d(w.val_ids, w.train_ids).size == 0
    frac = w.val_ids.size / w.cfg.n_nodes
    assert abs(frac - w.cfg.val_fraction) < 0.02
    # the training set is what it was before the split existed (same seed stream)
    w2 = synth.make_workload("tiny", seed=0, with_features=False)
    assert np.array_equal(w2.train_ids, w.train_ids) and np.array_equal(w2.val_ids, w.val_ids)
