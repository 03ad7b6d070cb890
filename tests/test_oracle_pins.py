"""CPU pins of the oracle (run without a GPU)."""
import pytest

import oracle_pins


@pytest.mark.parametrize("pin", oracle_pins.ALL_PINS, ids=lambda f: f.__name__)
def test_pin(oracle, pin):
    pin(oracle.default_lib())


def test_fp32_storage_mode_only_adds_storage_rounding(oracle):
    """The diagnostic mode that rounds p, m, v to fp32 after every step stays within a few fp32 ulps per step of
    the fp64-state oracle and keeps its state exactly representable in fp32."""
    import numpy as np
    import oracle as orc
    rng = np.random.default_rng(9)
    numel, bnum = [6 * 64, 40, 3 * 1000], [64, 1, 1000]
    p0 = [rng.normal(0, 0.02, n) for n in numel]
    hp = orc.Hyper.from_f32(1e-3, 0.9, 0.95, 1e-8, 0.1)
    a = orc.OracleState(numel, bnum, None, p0)
    b = orc.OracleState(numel, bnum, None, [x.astype(np.float32) for x in p0], storage="f32")
    steps = 10
    for t in range(steps):
        g = [rng.normal(0, 1e-3, n).astype(np.float32) for n in numel]
        a.step(g, hp)
        b.step(g, hp)
    for k in range(len(numel)):
        for x, y in ((a.p[k], b.p[k]), (a.m[k], b.m[k]), (a.v[k], b.v[k])):
            assert np.array_equal(y, y.astype(np.float32).astype(np.float64))
            rms = np.sqrt(np.mean(x * x))
            assert np.max(np.abs(x - y)) <= 4 * steps * 2.0 ** -24 * max(rms, np.max(np.abs(x)))
            assert np.max(np.abs(x - y)) > 0.0        # the rounding is really applied
    with pytest.raises(ValueError):
        orc.OracleState(numel, bnum, None, p0, storage="bf16")
