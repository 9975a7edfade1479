"""The sampled-column gather used by the large GPU tests reproduces the oracle's lowering."""
import numpy as np
import pytest

import oracle
from paper_2311_14272_amd import synth

from gpu_util import lowering_gather_index


@pytest.mark.parametrize("geo", [(3, 9, 8, 2, 3, 3, 1, 1), (4, 8, 8, 1, 1, 1, 2, 0), (2, 11, 11, 2, 7, 7, 2, 3),
                                 (5, 6, 7, 3, 1, 1, 1, 0), (3, 7, 7, 2, 3, 3, 2, 1)])
def test_gather_index_matches_oracle_lowering(geo):
    C, H, W, batch, kh, kw, stride, pad = geo
    rng = np.random.default_rng(sum(geo))
    act = synth.f32_to_bf16_bits(rng.standard_normal((C, batch, H, W)).astype(np.float32))
    X = oracle.im2col(act, kh, kw, stride, pad)
    cols = np.arange(X.shape[1])[::3]
    idx, inside = lowering_gather_index(C, H, W, batch, kh, kw, stride, pad, cols)
    got = np.where(inside, act.reshape(-1)[idx], np.uint16(0))
    assert (got == X[:, cols]).all()
