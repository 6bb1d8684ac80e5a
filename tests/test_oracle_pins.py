"""Pins for the CPU oracle: every oracle function is checked against something other than
itself -- hand-worked fixtures from the paper's equations, brute-force dense-mask attention
through a library matmul, closed forms, library routines and invariants.  CPU only."""
import itertools
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------ helpers
def eq5_mask(flags, n_recent=1):
    """Eq. 5 written independently of the oracle as a dense 0/1 matrix (numpy indexing)."""
    L = len(flags)
    j = np.arange(L)[:, None]
    t = np.arange(L)[None, :]
    m = np.where(j < t, 0, np.where(j - t < n_recent, 1, np.asarray(flags)[None, :]))
    return m.astype(np.float64)


def dense_masked_attention(q, k, v, mask, scale):
    """Eq. 2 literally: Softmax(Q K^T * scale - INF (1 - M)) V with a large finite INF, fp64."""
    s = (q.astype(np.float64) @ k.astype(np.float64).T) * scale - 1e30 * (1.0 - mask)
    s = s - s.max(axis=1, keepdims=True)
    p = np.exp(s)
    p /= p.sum(axis=1, keepdims=True)
    return p @ v.astype(np.float64)


def rnd(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape).astype(np.float32)


def read_rows(name, conv):
    rows = []
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            rows.append([conv(x) for x in line.split()])
    return rows


# ------------------------------------------------------------------ fixtures from the equations
def test_eq5_mask_fixture_matches_oracle_visibility():
    """The hand-written Eq. 5 mask equals what the oracle attends to: with Q = 0 and one-hot V the
    output row j is (visible set indicator) / |visible set|."""
    flags = np.array([1, 0, 1, 0, 0], dtype=np.uint8)
    M = np.array(read_rows("eq5_mask_n5.txt", int), dtype=np.float64)
    assert np.array_equal(M, eq5_mask(flags))          # the helper agrees with the hand-written mask
    L = 5
    q = np.zeros((1, 1, L, L), dtype=np.float32)
    k = rnd(1, 1, 1, L, L)
    v = np.eye(L, dtype=np.float32).reshape(1, 1, L, L)
    out = oracle.prefill_attn(q, k, v, flags.reshape(1, 1, L), 1.0)[0, 0]
    assert np.array_equal(out > 0, M > 0)
    np.testing.assert_allclose(out, M / M.sum(axis=1, keepdims=True), rtol=0, atol=1e-15)


def test_recent_window_mask_fixture_fixes_the_width_convention():
    """Table 6 (appendix "More Ablation"): "n recent tokens" counts the current token (setting (1), the diagonal
    alone, is one recent token).  The hand-written mask for 3 recent tokens pins the oracle's n_recent argument,
    and the helper eq5_mask used by the dense comparisons below, to that reading: off by one in either direction
    changes rows 3 to 5 of the fixture."""
    flags = np.array([1, 0, 0, 1, 0, 0], dtype=np.uint8)
    M = np.array(read_rows("eq5_mask_recent3_n6.txt", int), dtype=np.float64)
    assert M.shape == (6, 6)
    assert np.array_equal(M, eq5_mask(flags, 3))
    assert not np.array_equal(M, eq5_mask(flags, 2)) and not np.array_equal(M, eq5_mask(flags, 4))
    L = 6
    q = np.zeros((1, 1, L, L), dtype=np.float32)
    v = np.eye(L, dtype=np.float32).reshape(1, 1, L, L)
    out = oracle.prefill_attn(q, rnd(14, 1, 1, L, L), v, flags.reshape(1, 1, L), 1.0, n_recent=3)[0, 0]
    assert np.array_equal(out > 0, M > 0)
    np.testing.assert_allclose(out, M / M.sum(axis=1, keepdims=True), rtol=0, atol=1e-15)
    rows = oracle.prefill_rows(q, rnd(14, 1, 1, L, L), v, flags.reshape(1, 1, L), 1.0, np.arange(L), n_recent=3)[0, 0]
    np.testing.assert_allclose(rows, out, rtol=0, atol=0)
    # one recent token is Eq. 5 itself
    one = oracle.prefill_attn(q, rnd(14, 1, 1, L, L), v, flags.reshape(1, 1, L), 1.0, n_recent=1)[0, 0]
    assert np.array_equal(one > 0, eq5_mask(flags) > 0)


def test_uniform_attention_fixture():
    want = np.array(read_rows("uniform_attention_n5.txt", lambda s: float(Fraction(s))))
    flags = np.array([1, 0, 1, 0, 0], dtype=np.uint8).reshape(1, 1, 5)
    q = np.zeros((1, 1, 5, 5), dtype=np.float32)
    v = np.eye(5, dtype=np.float32).reshape(1, 1, 5, 5)
    out = oracle.prefill_attn(q, rnd(2, 1, 1, 5, 5), v, flags, 0.37)[0, 0]
    np.testing.assert_allclose(out, want, rtol=0, atol=1e-15)


# ------------------------------------------------------------------ brute force
def test_all_flag_patterns_small_L_vs_dense_mask():
    L, D = 8, 4
    q, k, v = rnd(3, L, D), rnd(4, L, D), rnd(5, L, D)
    scale = 1.0 / math.sqrt(D)
    pats = np.array(list(itertools.product([0, 1], repeat=L)), dtype=np.uint8)     # 256 patterns
    P = len(pats)
    out = oracle.prefill_attn(np.broadcast_to(q, (P, 1, L, D)), np.broadcast_to(k, (P, 1, L, D)),
                              np.broadcast_to(v, (P, 1, L, D)), pats.reshape(P, 1, L), scale)
    for p in range(P):
        want = dense_masked_attention(q, k, v, eq5_mask(pats[p]), scale)
        np.testing.assert_allclose(out[p, 0], want, rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("Hq,Hkv", [(4, 4), (8, 2), (4, 1)])
def test_random_flags_vs_dense_mask_with_gqa(Hq, Hkv):
    B, L, D = 2, 61, 16
    q, k, v = rnd(6, B, Hq, L, D), rnd(7, B, Hkv, L, D), rnd(8, B, Hkv, L, D)
    flags = (np.random.default_rng(9).random((B, Hkv, L)) < 0.4).astype(np.uint8)
    scale = 0.3
    out = oracle.prefill_attn(q, k, v, flags, scale)
    # GQA: expand KV heads explicitly (query head i reads KV head i // (Hq/Hkv))
    kk = np.repeat(k, Hq // Hkv, axis=1)
    vv = np.repeat(v, Hq // Hkv, axis=1)
    ff = np.repeat(flags, Hq // Hkv, axis=1)
    for b in range(B):
        for i in range(Hq):
            want = dense_masked_attention(q[b, i], kk[b, i], vv[b, i], eq5_mask(ff[b, i]), scale)
            np.testing.assert_allclose(out[b, i], want, rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("n_recent", [1, 5, 10])
def test_recent_window_vs_dense_mask(n_recent):
    """Table 6 (appendix "More Ablation"), settings (6-1)/(6-2): the last n_recent keys stay visible whatever their flag."""
    L, D = 40, 8
    q, k, v = rnd(10, 1, 1, L, D), rnd(11, 1, 1, L, D), rnd(12, 1, 1, L, D)
    flags = (np.random.default_rng(13).random((1, 1, L)) < 0.3).astype(np.uint8)
    out = oracle.prefill_attn(q, k, v, flags, 0.5, n_recent=n_recent)[0, 0]
    want = dense_masked_attention(q[0, 0], k[0, 0], v[0, 0], eq5_mask(flags[0, 0], n_recent), 0.5)
    np.testing.assert_allclose(out, want, rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("n_recent", [1, 4])
def test_sampled_rows_vs_dense_mask_with_gqa(n_recent):
    """prefill_rows (used for sampled checks of large problems) against Eq. 2/5 written densely: GQA head
    mapping, an unsorted row list with a repeat, first and last row."""
    B, Hq, Hkv, L, D = 2, 6, 2, 53, 16
    q, k, v = rnd(40, B, Hq, L, D), rnd(41, B, Hkv, L, D), rnd(42, B, Hkv, L, D)
    flags = (np.random.default_rng(43).random((B, Hkv, L)) < 0.4).astype(np.uint8)
    rows = np.array([52, 0, 17, 17, 31, 1])
    out = oracle.prefill_rows(q, k, v, flags, 0.25, rows, n_recent=n_recent)
    assert out.shape == (B, Hq, len(rows), D)
    for b in range(B):
        for i in range(Hq):
            g = i // (Hq // Hkv)
            want = dense_masked_attention(q[b, i], k[b, g], v[b, g], eq5_mask(flags[b, g], n_recent), 0.25)
            np.testing.assert_allclose(out[b, i], want[rows], rtol=1e-12, atol=1e-13)
    assert oracle.prefill_rows(q, k, v, flags, 0.25, np.zeros(0, dtype=np.int32)).shape == (B, Hq, 0, D)


# ------------------------------------------------------------------ main gate module (MHA' + projection)
def test_gate_mha_vs_dense_write_up():
    """Eq. 3 written out densely per head (explicit causal mask, numpy softmax) against oracle.gate_mha."""
    B, L, d, hp, dp, H = 2, 19, 24, 3, 8, 5
    x, wqkv, wo = rnd(50, B, L, d), rnd(51, d, 3 * hp * dp) * 0.3, rnd(52, hp * dp, H) * 0.4
    bias = rnd(53, H) * 0.1
    logits, flags = oracle.gate_mha(x, wqkv, hp, dp, wo, bias, 0.4, n_sink=1)
    causal = np.tril(np.ones((L, L)))
    for b in range(B):
        proj = x[b].astype(np.float64) @ wqkv.astype(np.float64)            # [L, 3*hp*dp]
        heads = []
        for h in range(hp):
            q, k, v = (proj[:, i * hp * dp + h * dp: i * hp * dp + (h + 1) * dp] for i in range(3))
            heads.append(dense_masked_attention(q, k, v, causal, 1.0 / np.sqrt(dp)))
        want = np.concatenate(heads, axis=1) @ wo.astype(np.float64) + bias
        np.testing.assert_allclose(logits[b], want, rtol=1e-5, atol=1e-6)    # features pass through fp32 in gate()
        f = (want > np.log(0.4 / 0.6)).T.astype(np.uint8)
        f[:, 0] = 1
        far = np.abs(want - np.log(0.4 / 0.6)).T > 1e-5
        assert np.array_equal(flags[b][far], f[far])


def test_gate_mha_closed_forms():
    """W_q = 0 makes every causal softmax uniform, so A_j is the running mean of V'; L = 1 gives A = V'."""
    B, L, d, hp, dp, H = 1, 11, 12, 2, 4, 3
    x, wqkv, wo = rnd(54, B, L, d), rnd(55, d, 3 * hp * dp), rnd(56, hp * dp, H)
    wqkv[:, :hp * dp] = 0.0
    bias = np.zeros(H, np.float32)
    logits, _ = oracle.gate_mha(x, wqkv, hp, dp, wo, bias, 0.5)
    vprime = x[0].astype(np.float64) @ wqkv[:, 2 * hp * dp:].astype(np.float64)   # heads side by side = concat
    run_mean = np.cumsum(vprime, axis=0) / np.arange(1, L + 1)[:, None]
    np.testing.assert_allclose(logits[0], run_mean @ wo.astype(np.float64), rtol=1e-5, atol=1e-6)
    one, _ = oracle.gate_mha(x[:, :1], rnd(57, d, 3 * hp * dp), hp, dp, wo, bias, 0.5)
    v1 = x[0, :1].astype(np.float64) @ rnd(57, d, 3 * hp * dp)[:, 2 * hp * dp:].astype(np.float64)
    np.testing.assert_allclose(one[0], v1 @ wo.astype(np.float64), rtol=1e-5, atol=1e-6)


def test_gate_mha_storage_rounding_is_round_to_nearest_even_bf16():
    vals = np.array([1.0, 1.00390625, 1.005859375, 1.01171875, -3.140625, 0.0], dtype=np.float64)
    # 1 + 2^-8 is a tie between 1 and 1 + 2^-7 -> even (1.0); 1 + 3*2^-9 rounds up; 1 + 3*2^-8 is a tie -> 1 + 2^-6
    got = oracle._round_to(vals, "bf16")
    assert got.tolist() == [1.0, 1.0, 1.0078125, 1.015625, -3.140625, 0.0]
    assert oracle._round_to(vals, None) is not None and np.array_equal(oracle._round_to(vals, None), vals)


# ------------------------------------------------------------------ special cases -> library routines
def test_all_kept_is_causal_sdpa():
    B, H, L, D = 2, 3, 50, 32
    q, k, v = rnd(14, B, H, L, D), rnd(15, B, H, L, D), rnd(16, B, H, L, D)
    out = oracle.prefill_attn(q, k, v, np.ones((B, H, L), np.uint8), 1.0 / math.sqrt(D))
    want = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q).double(), torch.from_numpy(k).double(), torch.from_numpy(v).double(),
        is_causal=True).numpy()
    np.testing.assert_allclose(out, want, rtol=1e-11, atol=1e-12)


def test_all_evicted_outputs_own_value_exactly():
    B, H, L, D = 1, 2, 33, 8
    q, k, v = rnd(17, B, H, L, D), rnd(18, B, H, L, D), rnd(19, B, H, L, D)
    out = oracle.prefill_attn(q, k, v, np.zeros((B, H, L), np.uint8), 0.7)
    assert np.array_equal(out, v.astype(np.float64))


def test_q_zero_reads_out_prefix_counts():
    """Q = 0 => o_j = (v_j + sum_{t<j} f_t v_t) / (cnt_j + 1); with V = ones in column 0 of kept-or-self
    rows the denominator is the exclusive prefix count of the flags plus one."""
    L, D = 70, 3
    flags = (np.random.default_rng(20).random(L) < 0.5).astype(np.uint8)
    v = rnd(21, L, D)
    out = oracle.prefill_attn(np.zeros((1, 1, L, D), np.float32), rnd(22, 1, 1, L, D), v.reshape(1, 1, L, D),
                              flags.reshape(1, 1, L), 1.0)[0, 0]
    cnt = np.concatenate([[0], np.cumsum(flags)[:-1]])
    pref = np.concatenate([np.zeros((1, D)), np.cumsum(v.astype(np.float64) * flags[:, None], axis=0)[:-1]])
    want = (v.astype(np.float64) + pref) / (cnt + 1)[:, None]
    np.testing.assert_allclose(out, want, rtol=1e-12, atol=1e-13)


def test_sharp_softmax_selects_best_visible_key_and_evicted_keys_vanish():
    """Orthonormal keys, huge scale: row j returns the value of the visible key with the largest
    score; evicting that key must switch the output to the runner-up."""
    L = D = 12
    k = np.eye(L, dtype=np.float32)
    v = rnd(23, L, D)
    # query j scores key 2 highest, key 5 second, itself third
    q = np.zeros((L, D), np.float32)
    q[:, 2], q[:, 5] = 3.5, 2.0
    q[np.arange(L), np.arange(L)] += 1.0
    for f2, f5 in [(1, 1), (0, 1), (0, 0)]:
        flags = np.ones(L, np.uint8)
        flags[2], flags[5] = f2, f5
        out = oracle.prefill_attn(q.reshape(1, 1, L, D), k.reshape(1, 1, L, D), v.reshape(1, 1, L, D),
                                  flags.reshape(1, 1, L), 200.0)[0, 0]
        for j in range(L):
            cand = [t for t in range(j + 1) if t == j or flags[t]]
            best = max(cand, key=lambda t: float(q[j] @ k[t]))
            np.testing.assert_allclose(out[j], v[best].astype(np.float64), rtol=0, atol=1e-12)


def test_nan_in_evicted_rows_never_leaks():
    B, H, L, D = 1, 2, 45, 8
    q, k, v = rnd(24, B, H, L, D), rnd(25, B, H, L, D), rnd(26, B, H, L, D)
    flags = (np.random.default_rng(27).random((B, H, L)) < 0.5).astype(np.uint8)
    clean = oracle.prefill_attn(q, k, v, flags, 0.35)
    kp, vp = k.copy(), v.copy()
    ev = flags == 0
    kp[ev] = np.nan
    vp[ev] = np.nan
    out = oracle.prefill_attn(q, kp, vp, flags, 0.35)
    keep_rows = flags == 1        # evicted rows see their own (poisoned) k/v on the diagonal
    assert np.array_equal(out[keep_rows], clean[keep_rows])
    assert np.isfinite(out[keep_rows]).all()


def test_units_are_independent_under_permutation():
    B, H, L, D = 2, 4, 30, 8
    q, k, v = rnd(28, B, H, L, D), rnd(29, B, H, L, D), rnd(30, B, H, L, D)
    flags = (np.random.default_rng(31).random((B, H, L)) < 0.5).astype(np.uint8)
    out = oracle.prefill_attn(q, k, v, flags, 0.4)
    perm = np.array([2, 0, 3, 1])
    outp = oracle.prefill_attn(q[:, perm], k[:, perm], v[:, perm], flags[:, perm], 0.4)
    assert np.array_equal(outp, out[:, perm])
    outb = oracle.prefill_attn(q[::-1], k[::-1], v[::-1], flags[::-1], 0.4)
    assert np.array_equal(outb, out[::-1])


# ------------------------------------------------------------------ gate
def test_gate_logits_vs_library_matmul_and_threshold_rule():
    B, L, d, H = 2, 37, 96, 5
    x, w, bias = rnd(32, B, L, d), rnd(33, d, H) / 8, rnd(34, H)
    for tau in (0.5, 0.3, 0.9):
        logits, flags = oracle.gate(x, w, bias, tau)
        want = x.astype(np.float64) @ w.astype(np.float64) + bias.astype(np.float64)
        np.testing.assert_allclose(logits, want, rtol=1e-12, atol=1e-13)
        sig = 1.0 / (1.0 + np.exp(-want))
        far = np.abs(want - math.log(tau / (1 - tau))) > 1e-6
        got = flags.transpose(0, 2, 1).astype(bool)      # [B,L,H]
        assert np.array_equal(got[far], (sig > tau)[far])   # Eq. 4 in probability space


def test_gate_threshold_is_strict_and_tau_half_means_positive_logit():
    assert oracle.logit_threshold(0.5) == 0.0
    assert abs(oracle.logit_threshold(0.3) - math.log(0.3 / 0.7)) < 1e-15
    # one feature, weight 1: the logit is the feature itself (+ bias)
    x = np.array([-1.0, -0.0, 0.0, 1e-30, 1.0], np.float32).reshape(1, 5, 1)
    _, flags = oracle.gate(x, np.ones((1, 1), np.float32), np.zeros(1, np.float32), 0.5)
    assert flags[0, 0].tolist() == [0, 0, 0, 1, 1]        # tie (s = 0 at tau = 0.5) evicts
    # gamma inside the sigmoid (Sec. 3.5): Sigmoid(s + gamma) > tau
    _, flags = oracle.gate(x, np.ones((1, 1), np.float32), np.full(1, 0.5, np.float32), 0.5)
    assert flags[0, 0].tolist() == [0, 1, 1, 1, 1]
    # forced sink tokens
    _, flags = oracle.gate(x, np.ones((1, 1), np.float32), np.zeros(1, np.float32), 0.5, n_sink=2)
    assert flags[0, 0].tolist() == [1, 1, 0, 1, 1]


@pytest.mark.parametrize("tau,gamma", [(0.5, 2.0), (0.3, 0.0)])
def test_gate_with_the_papers_settings_in_probability_space(tau, gamma):
    """Sec. 4.1 / Sec. 4.2 settings: flag = Sigmoid(s + gamma) > tau (Eq. 4 with the constant of Sec. 3.5), gamma
    passed as a bias of gamma in every head."""
    B, L, d, H = 1, 200, 16, 4
    x, w = rnd(61, B, L, d), rnd(62, d, H)
    _, flags = oracle.gate(x, w, np.full(H, gamma, np.float32), tau)
    s = x.astype(np.float64) @ w.astype(np.float64)
    sig = 1.0 / (1.0 + np.exp(-(s + gamma)))
    far = np.abs(sig - tau) > 1e-9
    assert np.array_equal(flags.transpose(0, 2, 1).astype(bool)[far], (sig > tau)[far])
    if gamma > 0:  # the constant pushes the retention up
        assert flags.mean() > oracle.gate(x, w, np.zeros(H, np.float32), tau)[1].mean()


def test_gate_flag_layout_is_head_major():
    B, L, d, H = 2, 6, 3, 4
    x = rnd(35, B, L, d)
    w = rnd(36, d, H)
    logits, flags = oracle.gate(x, w, np.zeros(H, np.float32), 0.5)
    assert flags.shape == (B, H, L)
    assert np.array_equal(flags, (logits.astype(np.float32) > 0).transpose(0, 2, 1).astype(np.uint8))


# ------------------------------------------------------------------ compaction
@pytest.mark.parametrize("dtype", [np.float32, np.uint16])
def test_compaction_invariants(dtype):
    B, H, L, D = 2, 3, 257, 16
    rng = np.random.default_rng(37)
    k = rng.integers(0, 60000, (B, H, L, D)).astype(dtype)
    v = rng.integers(0, 60000, (B, H, L, D)).astype(dtype)
    flags = (rng.random((B, H, L)) < 0.45).astype(np.uint8)
    flags[0, 1] = 0              # fully evicted unit
    flags[1, 2] = 1              # fully kept unit
    ro = oracle.slab_row_off(B * H, L + 3)
    cache, over = oracle.compact_kv(k, v, flags, ro, pos0=1000, fill=7)
    assert over == 0
    fl = flags.reshape(B * H, L)
    kk, vv = k.reshape(B * H, L, D), v.reshape(B * H, L, D)
    assert np.array_equal(cache.len, fl.sum(axis=1))
    for u in range(B * H):
        n, r0 = cache.len[u], ro[u]
        idx = cache.idx[r0:r0 + n] - 1000
        assert np.array_equal(idx, np.flatnonzero(fl[u]))               # stable, each kept token once
        assert np.array_equal(cache.k[r0:r0 + n], kk[u][idx])
        assert np.array_equal(cache.v[r0:r0 + n], vv[u][idx])
        assert (cache.k[r0 + n:ro[u + 1]] == 7).all() and (cache.idx[r0 + n:ro[u + 1]] == -1).all()


def test_compaction_capacity_overflow_is_reported_and_bounded():
    k = np.arange(2 * 10 * 2, dtype=np.float32).reshape(1, 2, 10, 2)
    flags = np.ones((1, 2, 10), np.uint8)
    ro = np.array([0, 4, 14], dtype=np.int64)
    cache, over = oracle.compact_kv(k, k, flags, ro)
    assert over == 1 and cache.len.tolist() == [4, 10]
    assert np.array_equal(cache.k[:4], k[0, 0, :4]) and np.array_equal(cache.k[4:], k[0, 1])


# ------------------------------------------------------------------ decode
def dense_decode(q, K, V, scale):
    s = (K.astype(np.float64) @ q.astype(np.float64)) * scale
    p = np.exp(s - s.max())
    return (p / p.sum()) @ V.astype(np.float64)


def test_decode_step_vs_dense_and_append_rules():
    B, Hq, Hkv, D = 2, 4, 2, 8
    lens = np.array([5, 0, 1, 9], np.int32)
    ro = oracle.slab_row_off(B * Hkv, lens + 2)
    total = int(ro[-1])
    cache = oracle.Cache(rnd(38, total, D), rnd(39, total, D), np.full(total, -1, np.int32), ro, lens.copy())
    ref = cache.copy()
    q, kn, vn = rnd(40, B, Hq, D), rnd(41, B, Hkv, D), rnd(42, B, Hkv, D)
    nf = np.array([1, 0, 1, 0], np.uint8)
    out, dropped = oracle.decode_step(q, kn, vn, nf, 77, cache, 0.5)
    assert dropped == 0
    for b in range(B):
        for i in range(Hq):
            u = b * Hkv + i // 2
            K = np.concatenate([ref.k[ro[u]:ro[u] + lens[u]], kn.reshape(-1, D)[u:u + 1]])
            V = np.concatenate([ref.v[ro[u]:ro[u] + lens[u]], vn.reshape(-1, D)[u:u + 1]])
            np.testing.assert_allclose(out[b, i], dense_decode(q[b, i], K, V, 0.5), rtol=1e-12, atol=1e-13)
    assert cache.len.tolist() == (lens + nf).tolist()
    for u in range(4):
        r = ro[u] + lens[u]
        if nf[u]:
            assert np.array_equal(cache.k[r], kn.reshape(-1, D)[u]) and cache.idx[r] == 77
        else:
            assert np.array_equal(cache.k[r], ref.k[r]) and cache.idx[r] == -1
    # empty cache (fully evicted head): the output is the new token's own value, exactly
    assert np.array_equal(out[0, 2], vn[0, 1].astype(np.float64))
    assert np.array_equal(out[0, 3], vn[0, 1].astype(np.float64))
    # NULL flags keep every generated token; capacity overflow drops the row and reports it
    for step in range(3):
        out, dropped = oracle.decode_step(q, kn, vn, None, 78 + step, cache, 0.5)
    assert dropped > 0 and (cache.len <= lens + 2).all()


def test_prefill_then_decode_equals_longer_prefill():
    """Row L of a prefill over L+1 tokens == prefill over L tokens, compaction, one decode step."""
    B, Hq, Hkv, L, D = 2, 4, 2, 29, 8
    q, k, v = rnd(43, B, Hq, L + 1, D), rnd(44, B, Hkv, L + 1, D), rnd(45, B, Hkv, L + 1, D)
    flags = (np.random.default_rng(46).random((B, Hkv, L + 1)) < 0.5).astype(np.uint8)
    full = oracle.prefill_attn(q, k, v, flags, 0.3)
    ro = oracle.slab_row_off(B * Hkv, L + 1)
    cache, _ = oracle.compact_kv(k[:, :, :L], v[:, :, :L], flags[:, :, :L], ro)
    out, _ = oracle.decode_step(q[:, :, L], k[:, :, L], v[:, :, L], flags[:, :, L], L, cache, 0.3)
    np.testing.assert_allclose(out, full[:, :, L], rtol=1e-12, atol=1e-13)
    # and the cache now equals the compaction of all L+1 tokens
    cache2, _ = oracle.compact_kv(k, v, flags, ro)
    assert np.array_equal(cache.len, cache2.len)
    for u in range(B * Hkv):
        n = cache.len[u]
        assert np.array_equal(cache.k[ro[u]:ro[u] + n], cache2.k[ro[u]:ro[u] + n])
        assert np.array_equal(cache.idx[ro[u]:ro[u] + n], cache2.idx[ro[u]:ro[u] + n])


def test_decode_len_after_many_steps_counts_flags():
    B, H, D, T = 1, 3, 4, 20
    lens = np.array([2, 0, 7], np.int32)
    ro = oracle.slab_row_off(3, lens + T)
    total = int(ro[-1])
    cache = oracle.Cache(rnd(47, total, D), rnd(48, total, D), np.zeros(total, np.int32), ro, lens.copy())
    rng = np.random.default_rng(49)
    tot = np.zeros(3, np.int64)
    for s in range(T):
        nf = (rng.random(3) < 0.5).astype(np.uint8)
        tot += nf
        oracle.decode_step(rnd(50 + s, B, H, D), rnd(80 + s, B, H, D), rnd(110 + s, B, H, D), nf, 100 + s, cache, 1.0)
    assert np.array_equal(cache.len, lens + tot)
    for u in range(3):
        new_idx = cache.idx[ro[u] + lens[u]:ro[u] + cache.len[u]]
        assert (np.diff(new_idx) > 0).all()


# ------------------------------------------------------------------ K/V projection (Eq. 2)
def test_project_kv_selector_weights_read_out_the_features():
    """W that copies feature block h into head h: K_h = X[:, hD:(h+1)D] and V_h = -X[:, ...] exactly, which pins the
    column order (K heads first, then V heads), the head-major output layout and the absence of any scaling."""
    B, L, H, D = 2, 5, 3, 4
    d = H * D
    x = rnd(71, B, L, d)
    w = np.zeros((d, 2 * H * D), np.float32)
    for c in range(H * D):
        w[c, c] = 1.0
        w[c, H * D + c] = -1.0
    k, v = oracle.project_kv(x, w, H, D)
    for h in range(H):
        assert np.array_equal(k[:, h], x[:, :, h * D:(h + 1) * D].astype(np.float64))
        assert np.array_equal(v[:, h], -x[:, :, h * D:(h + 1) * D].astype(np.float64))


def test_project_kv_matches_per_element_sums_and_rounds_to_bf16_on_request():
    B, L, d, H, D = 1, 3, 6, 2, 2
    x, w = rnd(72, B, L, d), rnd(73, d, 2 * H * D)
    k, v = oracle.project_kv(x, w, H, D)
    for t in range(L):
        for h in range(H):
            for e in range(D):
                want_k = sum(float(x[0, t, c]) * float(w[c, h * D + e]) for c in range(d))
                want_v = sum(float(x[0, t, c]) * float(w[c, H * D + h * D + e]) for c in range(d))
                assert abs(k[0, h, t, e] - want_k) < 1e-12 and abs(v[0, h, t, e] - want_v) < 1e-12
    kb, _ = oracle.project_kv(x, w, H, D, store="bf16")
    bits = kb.astype(np.float32).view(np.uint32)
    assert np.all(bits & 0xffff == 0)                       # representable in bf16
    assert np.all(np.abs(kb - k) <= np.abs(k) * 2.0 ** -8)  # and the nearest such value (half a spacing at most)


# ------------------------------------------------------------------ normalisation ahead of the gate
def test_rmsnorm_closed_forms():
    """Rows with a known answer: a constant row c gives sign(c) g / sqrt(1 + eps / c^2); a one-hot row a e_k gives
    sign(a) sqrt(d) g_k at k and 0 elsewhere as eps -> 0 (the mean is over all d features, not a sum and not over the
    non-zero ones); with g = 1 the mean square of an output row is ms / (ms + eps)."""
    d = 12
    g = rnd(81, d) + 2.0
    eps = 1e-3
    h = np.zeros((1, 3, d), np.float32)
    h[0, 0] = -3.0
    h[0, 1, 5] = 2.5
    h[0, 2] = rnd(82, d)
    x = oracle.rmsnorm(h, g, eps)
    assert np.allclose(x[0, 0], -g.astype(np.float64) / np.sqrt(1.0 + eps / 9.0), rtol=1e-12)
    want = np.zeros(d)
    want[5] = float(g[5]) * 2.5 / np.sqrt(2.5 ** 2 / d + eps)
    assert np.allclose(x[0, 1], want, rtol=1e-12) and abs(want[5] / (np.sqrt(d) * g[5]) - 1.0) < 1e-3
    x1 = oracle.rmsnorm(h, np.ones(d, np.float32), eps)
    ms = float(np.mean(h[0, 2].astype(np.float64) ** 2))
    assert abs(np.mean(x1[0, 2] ** 2) - ms / (ms + eps)) < 1e-12


def test_rmsnorm_is_scale_invariant_and_matches_the_library_routine():
    B, L, d = 2, 7, 64
    h, g = rnd(83, B, L, d), rnd(84, d)
    x = oracle.rmsnorm(h, g, 1e-5)
    assert np.allclose(oracle.rmsnorm(4.0 * h, g, 16.0 * 1e-5), x, rtol=1e-12, atol=0)   # h -> a h, eps -> a^2 eps
    lib = torch.nn.functional.rms_norm(torch.from_numpy(h.astype(np.float64)), (d,),
                                       torch.from_numpy(g.astype(np.float64)), eps=1e-5).numpy()
    assert np.allclose(x, lib, rtol=1e-12, atol=1e-15)
    xb = oracle.rmsnorm(h, g, 1e-5, store="bf16")
    assert np.all(xb.astype(np.float32).view(np.uint32) & 0xffff == 0)
    assert np.all(np.abs(xb - x) <= np.abs(x) * 2.0 ** -8)


def test_rmsnorm_gate_is_the_gate_of_the_stored_x():
    """A gate weight that reads out feature c (bias 0, tau 1/2) keeps a token iff x_c > 0, i.e. iff h_c g_c > 0: the
    normalisation never changes a sign; the logits are those of the gate applied to the x that is returned."""
    B, L, d = 1, 40, 16
    h, g = rnd(85, B, L, d), rnd(86, d)
    w = np.zeros((d, 4), np.float32)
    for j, c in enumerate((0, 3, 7, 15)):
        w[c, j] = 1.0
    x, logits, flags = oracle.rmsnorm_gate(h, g, 1e-6, w, np.zeros(4, np.float32), 0.5, 0, store="bf16")
    for j, c in enumerate((0, 3, 7, 15)):
        assert np.array_equal(flags[0, j], (h[0, :, c] * g[c] > 0).astype(np.uint8))
        assert np.array_equal(logits[0, :, j], x[0, :, c])
    l2, f2 = oracle.gate(x, w, np.zeros(4, np.float32), 0.5, 0)
    assert np.array_equal(l2, logits) and np.array_equal(f2, flags)


# ------------------------------------------------------------------ memory safety of the checker itself
def test_oracle_runs_clean_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    """oracle/ag_oracle.c compiled together with tests/oracle_sanitized.c by gcc with
    -fsanitize=address,undefined (host code; statically linked runtime) and run on edge shapes: L = 1, a prompt
    shorter than the recent window, GQA, empty and full units, caches with no room and with exactly enough.  Any
    out-of-bounds access, overflow or leak in the oracle aborts the run."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    exe = str(tmp_path / "oracle_sanitized")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-Wall", "-Wextra", "-Werror", "-o", exe, os.path.join(root, "tests", "oracle_sanitized.c"),
           os.path.join(root, "oracle", "ag_oracle.c"), "-lm"]
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=180)
    if r.returncode != 0 and ("cannot find" in r.stderr or "libasan" in r.stderr):
        pytest.skip("sanitizer runtime not installed: " + r.stderr[-200:])
    assert r.returncode == 0, r.stderr
    r = subprocess.run([exe], capture_output=True, text=True, timeout=180,
                       env=dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", OMP_NUM_THREADS="4"))
    assert r.returncode == 0 and r.stdout.strip().endswith("ok"), r.stdout + r.stderr[-3000:]


def test_packed_row_off_hand_example_and_closed_form():
    """Packed cache layout (Sec. 3.3: only retained rows take memory): worked by hand for three units, then the
    prefix-sum closed form on random flags, with and without the cut at total_rows."""
    flags = np.array([[1, 0, 1], [0, 0, 0], [1, 1, 1]], dtype=np.uint8)      # kept 2, 0, 3
    ro, need = oracle.packed_row_off(flags, 2, 100)
    assert ro.tolist() == [0, 4, 6, 11] and need == 11
    ro, need = oracle.packed_row_off(flags, 2, 8)                              # the allocation ends inside unit 2
    assert ro.tolist() == [0, 4, 6, 8] and need == 11
    ro, need = oracle.packed_row_off(flags.reshape(1, 3, 3), 0, 100)           # [B, Hkv, L] input, no spare rows
    assert ro.tolist() == [0, 2, 2, 5] and need == 5
    g = np.random.default_rng(5)
    f = (g.random((7, 50)) < 0.4).astype(np.uint8)
    ro, need = oracle.packed_row_off(f, 3, 10 ** 9)
    assert np.array_equal(ro[1:], np.cumsum(f.sum(axis=1) + 3)) and need == int(f.sum()) + 21
    assert np.array_equal(np.diff(ro), f.sum(axis=1) + 3)
