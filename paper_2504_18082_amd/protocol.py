"""Host-side logic of the paper's training protocol (Section 5 "Training methodology"): train for up to a
maximum number of epochs, stop early when the validation loss has not improved for `patience` epochs, and
cut the learning rate when it has plateaued for `lr_patience` epochs (the behaviour of PyTorch's
ReduceLROnPlateau with its default relative threshold of 1e-4 and factor 0.1).  Pure bookkeeping: no
tensor arithmetic happens here."""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List


@dataclass
class PlateauScheduler:
    lr: float
    patience: int = 3
    factor: float = 0.1
    threshold: float = 1e-4
    min_lr: float = 0.0
    eps: float = 1e-8               # cuts smaller than this are not applied
    best: float = float("inf")
    bad_epochs: int = 0

    def step(self, metric: float) -> float:
        """Feed one epoch's validation loss; returns the learning rate for the next epoch."""
        if metric < self.best * (1.0 - self.threshold):
            self.best = metric
            self.bad_epochs = 0
        else:
            self.bad_epochs += 1
        if self.bad_epochs > self.patience:
            new_lr = max(self.min_lr, self.lr * self.factor)
            if self.lr - new_lr > self.eps:
                self.lr = new_lr
            self.bad_epochs = 0
        return self.lr


@dataclass
class EarlyStopping:
    patience: int = 6
    best: float = float("inf")
    best_epoch: int = -1
    bad_epochs: int = 0

    def step(self, metric: float, epoch: int) -> bool:
        """Feed one epoch's validation loss; returns True when training should stop."""
        if metric < self.best:
            self.best = metric
            self.best_epoch = epoch
            self.bad_epochs = 0
        else:
            self.bad_epochs += 1
        return self.bad_epochs >= self.patience


@dataclass
class History:
    epoch_ms: List[float] = field(default_factory=list)
    train_loss: List[float] = field(default_factory=list)
    val_loss: List[float] = field(default_factory=list)
    val_acc: List[float] = field(default_factory=list)
    lr: List[float] = field(default_factory=list)
    stopped_early: bool = False

    @property
    def epochs(self) -> int:
        return len(self.val_loss)

    def summary(self) -> dict:
        best = min(range(self.epochs), key=lambda i: self.val_loss[i]) if self.epochs else -1
        return dict(epochs=self.epochs, stopped_early=self.stopped_early,
                    final_val_acc=self.val_acc[-1] if self.epochs else None,
                    best_val_acc=self.val_acc[best] if self.epochs else None,
                    mean_epoch_ms=sum(self.epoch_ms) / max(1, len(self.epoch_ms)),
                    total_train_ms=sum(self.epoch_ms))
