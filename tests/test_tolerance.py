"""The store allowance of the bf16 parity bar (gpu_util.bf16_half_spacing) against the format itself: it must
equal the largest error a round-to-nearest bf16 store can make on a given value, no more.  CPU only."""
import numpy as np

import workloads as W
from gpu_util import attn_error, attn_error_raw, bf16_half_spacing


def test_half_spacing_is_the_exact_bound_of_a_bf16_store():
    g = np.random.default_rng(0)
    y = np.concatenate([(g.random(400000) * 16 + 1e-3), -(g.random(1000) * 3), [1.0, 2.0, 4.0, 0.0]]).astype(np.float32)
    stored = W.bf16_bits_to_f32(W.f32_to_bf16_bits(y)).astype(np.float64)
    h = bf16_half_spacing(y)
    assert (np.abs(stored - y) <= h).all()                 # a store never moves a value further
    nz = h > 0
    assert (np.abs(stored - y)[nz] / h[nz]).max() > 0.999  # and the bound is reached: nothing is given away
    assert np.array_equal(bf16_half_spacing(np.array([1.0, 1.99, 2.0, 3.5, 0.75, 0.0, -5.0])),
                          np.array([2.0 ** -8, 2.0 ** -8, 2.0 ** -7, 2.0 ** -7, 2.0 ** -9, 0.0, 2.0 ** -6]))


def test_a_perfectly_rounded_result_has_zero_allowanced_error_and_a_visible_raw_one():
    g = np.random.default_rng(1)
    ref = g.standard_normal((3, 50, 128)) * np.array([1.0, 0.1, 5.0])[:, None, None]
    got = W.bf16_bits_to_f32(W.f32_to_bf16_bits(ref.astype(np.float32)))
    assert attn_error("bf16", got, ref.astype(np.float32).astype(np.float64)) == 0.0
    assert 0.0 < attn_error_raw("bf16", got, ref) < 2e-2
    off = got.copy()
    off[1, 7, 3] += 0.05                                    # an arithmetic error of half a row RMS is charged in full
    assert attn_error("bf16", off, ref) > 0.4
