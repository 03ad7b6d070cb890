"""The two evaluations of the parity bound (numpy on the host, PyTorch float64 where the data is) agree."""
import numpy as np
import pytest


@pytest.mark.parametrize("kind", ["rows", "columns", "whole", "v"])
def test_device_comparison_is_the_host_comparison(kind):
    import torch
    import gpu_harness as H
    rng = np.random.default_rng(7)
    n_blocks, bn = 37, 48
    want = rng.standard_normal(n_blocks * bn) * np.repeat(np.exp(rng.standard_normal(n_blocks) * 3), bn)
    want[5] = np.nan
    got = (want * (1 + 2e-7 * rng.standard_normal(want.size))).astype(np.float32)
    kw = dict(rows=dict(block_numel=bn), columns=dict(block_numel=bn, strided=True), whole={}, v=dict(is_v=True))[kind]
    a = H.assert_state_close("x", got, want, 1e-5, **kw)
    b = H.assert_state_close_on_device("x", torch.from_numpy(got), want, 1e-5, **kw)
    assert a > 0 and abs(a - b) <= 1e-12 * a
    # one element just outside the bound of its own block, and a misplaced NaN: both must refuse
    bad = got.copy()
    bad[100] += np.float32(1e-3 * max(abs(want[100]), 1.0))
    for fn, arg in ((H.assert_state_close, bad), (H.assert_state_close_on_device, torch.from_numpy(bad))):
        with pytest.raises(AssertionError, match="elements off"):
            fn("x", arg, want, 1e-5, **kw)
    bad = got.copy()
    bad[6] = np.nan
    for fn, arg in ((H.assert_state_close, bad), (H.assert_state_close_on_device, torch.from_numpy(bad))):
        with pytest.raises(AssertionError, match="non-finite"):
            fn("x", arg, want, 1e-5, **kw)
