"""Helpers shared by the GPU parity tests."""
import numpy as np


def assert_close(got, want, rtol, what="", scale=None, extra=None):
    """|a-b| <= rtol * (|b| + scale) (+ extra, an absolute allowance per element), element-wise.

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
    if extra is not None:
        bound = bound + extra
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


def assert_weight_step(W_after, W_before, ref_after, ref_before, rtol, what, extra=None):
    """Compares the CHANGE of a parameter array over one SGD step with the oracle's change.  (Comparing the weights
    themselves would pass for any gradient: lr * dW is far below a bf16-sized tolerance times |W|.)  The scale is the
    change's own root-mean-square plus what one float32 rounding of the updated master weight is worth."""
    W_before = np.asarray(W_before, dtype=np.float64)
    got = np.asarray(W_after, dtype=np.float64) - W_before
    want = np.asarray(ref_after, dtype=np.float64) - np.asarray(ref_before, dtype=np.float64)
    scale = np.sqrt(np.mean(want * want)) + 2.0 ** -24 * np.max(np.abs(W_before), initial=0.0) / rtol
    assert_close(got, want, rtol, what, scale=scale, extra=extra)


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


def relu_flip_allowance(gpu_out, ref_out, gpu_dz, ref_dz, operands):
    """ReLU decisions at the boundary.  The mask of a hidden layer is the sign of an activation; where the activation is
    within rounding of zero the GPU path (float accumulation) and the oracle (double) may decide differently, and the
    gradient element dZ[m, n] is then present on one side and zero on the other.  Both decisions are correct to
    rounding, so the comparison must not fail on them: this returns, for the layer's weight gradient dW[k, n] =
    sum_m A[m, k] dZ[m, n] and bias gradient db[n] = sum_m dZ[m, n], the exact size of what the differing decisions
    contribute, sum over flipped (m, n) of |A[m, k]| |dZ[m, n]| and of |dZ[m, n]|, as an absolute allowance.
    It first checks that every differing decision really is at the boundary: both activations tiny next to the layer's
    typical activation.
      gpu_out, ref_out : activations after the ReLU [M, N] (GPU's stored bf16 values, oracle's);  gpu_dz, ref_dz : dL/dZ
      of the layer [M, N];  operands : the oracle's [H_self | Agg] rows of the layer [M, K]
    Returns (allow_dW [K, N], allow_db [N], number of differing decisions)."""
    gpu_out, ref_out = np.asarray(gpu_out, dtype=np.float64), np.asarray(ref_out, dtype=np.float64)
    flip = (gpu_out > 0) != (ref_out > 0)
    K, N = operands.shape[1], ref_out.shape[1]
    allow_dW, allow_db = np.zeros((K, N)), np.zeros(N)
    if not flip.any():
        return allow_dW, allow_db, 0
    typical = np.sqrt(np.mean(ref_out * ref_out))
    assert np.all(np.maximum(np.abs(gpu_out[flip]), np.abs(ref_out[flip])) <= 2.0 ** -7 * typical), \
        "a ReLU decision differs away from the boundary"
    for m, n in zip(*np.nonzero(flip)):
        dz = max(abs(float(gpu_dz[m, n])), abs(float(ref_dz[m, n])))
        allow_dW[:, n] += np.abs(operands[m]) * dz
        allow_db[n] += dz
    return allow_dW, allow_db, int(flip.sum())
