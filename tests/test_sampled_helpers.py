"""CPU check of the sampled-output helpers used by the full-size GPU tests: on small tensors the
sampled values must equal the oracle run on the whole tensor."""
import numpy as np
import pytest

from oracle import layers as L
from tests.sampled import sampled_conv_bwd_data_check, sampled_conv_bwd_filter_check, sampled_conv_fwd_check


@pytest.mark.parametrize("shape", [(2, 3, 9, 8, 4, 3, 1, 1), (2, 2, 10, 10, 3, 5, 1, 2), (1, 3, 12, 12, 2, 7, 2, 3),
                                   (2, 4, 6, 6, 3, 1, 1, 0), (1, 2, 23, 23, 3, 11, 4, 0)])
def test_sampled_helpers_agree_with_whole_tensor_oracle(shape):
    n, c, h, w, k, r, st, pd = shape
    rng = np.random.default_rng(5)
    x = rng.standard_normal((n, c, h, w)).astype(np.float32)
    wt = rng.standard_normal((k, c, r, r))
    y = L.conv_fwd(x, wt, st, pd)
    dy = rng.standard_normal(y.shape).astype(np.float32)
    assert sampled_conv_fwd_check(x, wt, y, st, pd, False, rng, 40) < 1e-12
    assert sampled_conv_fwd_check(x, wt, L.relu_fwd(y), st, pd, True, rng, 40) < 1e-12
    assert sampled_conv_bwd_filter_check(x, dy, L.conv_bwd_filter(x, dy, wt.shape, st, pd), st, pd, rng, 4) < 1e-12
    if st == 1:
        assert sampled_conv_bwd_data_check(dy, wt, L.conv_bwd_data(dy, wt, x.shape, st, pd), pd, rng, 40) < 1e-12
    # and they do notice a wrong tensor
    bad = y.copy()
    bad[:, :, 0, 0] += 1.0
    assert sampled_conv_fwd_check(x, wt, bad, st, pd, False, rng, 40) > 1e-3
