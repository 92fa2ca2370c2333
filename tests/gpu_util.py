"""Helpers shared by the GPU parity tests."""
import numpy as np


def assert_close(got, want, rtol, what="", scale=None):
    """|a-b| <= rtol * (|b| + scale), element-wise.

    `scale` is the magnitude of the terms that were summed into each element (so that a result made
    small by cancellation is judged against what was added up, the usual backward-error measure);
    it defaults to the root-mean-square of the expected values."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    if want.size == 0:
        return
    if scale is None:
        scale = np.sqrt(np.mean(want * want))
    bound = rtol * (np.abs(want) + scale)
    err = np.abs(got - want)
    bad = err > bound
    if bad.any():
        i = np.unravel_index(np.argmax(err - bound), err.shape)
        raise AssertionError(f"{what}: {int(bad.sum())} of {want.size} outside rtol={rtol}; worst at {i}: "
                             f"got {got[i]!r} want {want[i]!r}")


def bf16_tensor_to_float(t):
    """torch int16 tensor holding raw bf16 -> numpy float32."""
    a = t.cpu().numpy().view(np.uint16).astype(np.uint32) << 16
    return a.view(np.float32)


def worst_rel_err(got, want, scale=None):
    """max over elements of |a-b| / (|b| + scale), scale = rms(b) by default: the quantity assert_close bounds."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    if want.size == 0:
        return 0.0
    if scale is None:
        scale = np.sqrt(np.mean(want * want))
    return float(np.max(np.abs(got - want) / (np.abs(want) + scale + 1e-300)))


def assert_weight_step(W_after, W_before, ref_after, ref_before, rtol, what):
    """Compares the CHANGE of a parameter array over one SGD step with the oracle's change.  (Comparing the weights
    themselves would pass for any gradient: lr * dW is far below a bf16-sized tolerance times |W|.)  The scale is the
    change's own root-mean-square plus what one float32 rounding of the updated master weight is worth."""
    W_before = np.asarray(W_before, dtype=np.float64)
    got = np.asarray(W_after, dtype=np.float64) - W_before
    want = np.asarray(ref_after, dtype=np.float64) - np.asarray(ref_before, dtype=np.float64)
    scale = np.sqrt(np.mean(want * want)) + 2.0 ** -24 * np.max(np.abs(W_before), initial=0.0) / rtol
    assert_close(got, want, rtol, what, scale=scale)


def rms_rel_err(got, want):
    """root-mean-square of (a - b) over the root-mean-square of b."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    return float(np.sqrt(np.mean((got - want) ** 2)) / (np.sqrt(np.mean(want * want)) + 1e-300))


def frac_outside(got, want, rtol):
    """Fraction of elements outside |a-b| <= rtol (|b| + rms b)."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    return float(np.mean(np.abs(got - want) > rtol * (np.abs(want) + np.sqrt(np.mean(want * want)))))
