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
