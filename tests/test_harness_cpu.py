"""Host-side checks of the parity harness itself (no GPU)."""
import numpy as np

import workloads as W
from oracle import lopt_oracle as O
from tests import harness as Hn


def test_pooled_oracle_calls_equal_serial_ones_bit_for_bit():
    # the GPU parity tests step independent tensors through the oracle on a thread pool; the pool must not change a bit
    cfg = O.OracleConfig()
    w = W.small_fc_weights(0, 32)
    specs = [W.TensorSpec(f"t{i}", s) for i, s in enumerate([(700, 768), (768,), (600, 1000), (3072,), (900, 640)] * 4)]

    def one(i):
        p = W.init_param(150, i, specs[i]).astype(np.float64)
        st = O.init_state(*p.shape, cfg)
        return O.tensor_step(p, W.grad(150, i, 0, specs[i], "gauss_logscale"), st, w, cfg, 0, 1.0, 0.01)

    pooled = Hn.pool_map(one, range(len(specs)))
    for i in (0, 2, 4, 7, 19):
        assert np.array_equal(pooled[i], one(i))


def test_delta_err_discounts_only_the_rounding_of_the_stored_parameter():
    p_old = np.array([1.0, -2.0, 0.5])
    p_new = np.array([0.9, -2.1, 0.5])
    assert Hn.delta_err(p_old, p_new, p_old, p_new) == 0.0
    off = p_new + np.array([0.0, 2.0 ** -24 * 2.1, 0.0])          # within the fp32 rounding of p_new: not an error
    assert Hn.delta_err(p_old, off, p_old, p_new) == 0.0
    off = p_new + np.array([1e-3, 0.0, 0.0])                       # an error of the update: d = (0.1, 0.1, 0)
    rms = np.sqrt((0.01 + 0.01) / 3)
    assert abs(Hn.delta_err(p_old, off, p_old, p_new) - (1e-3 - 0.9 * 2.0 ** -23) / (0.1 + rms)) < 1e-9
