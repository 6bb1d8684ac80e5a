"""The seeded input generators: determinism, storage rounding, structure of the draws.  CPU only."""
import numpy as np
import torch

import workloads as W


def test_bf16_rounding_matches_library_conversion():
    x = np.random.default_rng(0).standard_normal(100000).astype(np.float32) * 37.0
    x[:4] = [0.0, -0.0, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8]       # exact ties: round to even
    bits = W.f32_to_bf16_bits(x)
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, want)
    assert np.array_equal(W.bf16_bits_to_f32(bits), torch.from_numpy(x).to(torch.bfloat16).float().numpy())


def test_draws_are_reproducible_and_distinct_per_tensor():
    a, b = W.normal(2, 1, (1000,)), W.normal(2, 1, (1000,))
    assert np.array_equal(a, b)
    assert not np.array_equal(a, W.normal(2, 2, (1000,)))
    assert abs(float(a.std()) - 1.0) < 0.1


def test_config1_shapes_and_bias_targets_half_keep():
    wl = W.config1()
    assert wl.x.f32.shape == (1, 128, 256) and wl.q.f32.shape == (1, 4, 128, 64)
    assert wl.k.f32.shape == (1, 4, 128, 64) and wl.bias.shape == (4,) and wl.n_sink == 1
    assert np.allclose(wl.bias, 0.0)      # 50 % keep at tau = 0.5 needs no shift


def test_run_flags_keep_ratio_and_runs():
    f = W.run_flags(4, 6, 4, 32768, 16.0, 0.3)
    assert f.shape == (4, 32768) and set(np.unique(f)) <= {0, 1}
    assert abs(f.mean() - 0.3) < 0.03
    d = np.diff(f[0].astype(np.int8))
    n_runs = (d == 1).sum()
    assert 10 < f[0].sum() / max(n_runs, 1) < 24      # mean kept-run length near 16


def test_decode_batch_structure():
    wl = W.config3(B=2, steps=4, max_len=256)
    U = 64
    assert wl.len0.shape == (U,) and wl.row_off[-1] == (wl.len0.astype(np.int64) + 4).sum()
    assert wl.k_cache.bits.shape == (int(wl.row_off[-1]), 128)
    for u in range(U):
        ix = wl.idx[wl.row_off[u]:wl.row_off[u] + wl.len0[u]]
        assert (np.diff(ix) > 0).all() and (ix >= 0).all() and (ix < 256).all()
    q, kn, vn, nf = wl.step_inputs(0)
    assert q.bits.shape == (2, 32, 128) and nf.shape == (2, 32)


def test_config5_decode_lens_follow_the_layer_keep_ratios():
    for layer in (0, 16, 31):
        lens = W.config5_decode_lens(layer).reshape(16, 32)
        rho = 0.9 - 0.8 * layer / 31
        live = lens[:, lens[0] > 0]
        assert abs(live.mean() / 2048 - rho) < 0.04
        assert lens.min() >= 0 and lens.max() <= 2048
        assert np.array_equal(W.config5_decode_lens(layer), lens.reshape(-1))   # seeded
    dead = (W.config5_decode_lens(31).reshape(16, 32) == 0).all(0)
    assert dead.sum() >= 1   # fully evicted heads in the deepest layer, the same heads for every sequence


def test_config5_gate_params_are_the_layers_own():
    """The light-weight accessor gives the same gate (weights, bias, dead heads) as the full layer workload."""
    import numpy as np
    import workloads as W
    for layer in (3, 27):
        wl = W.config5_layer(layer, B=1, L=8)
        w, bias, keep, dead = W.config5_gate_params(layer)
        assert np.array_equal(w.bits, wl.w_gate.bits) and np.array_equal(bias, wl.bias)
        assert np.array_equal(dead, wl.extra["dead_heads"]) and np.allclose(keep, wl.keep)
