"""Parity of the HIP path (through the C ABI) against the CPU oracle, element by element, on seeded inputs.

Bars: flags, idx, len and cached rows bit-exact (gate logits within 1e-3 of the threshold are excluded from
the flag comparison and counted); attention outputs within 1e-5 max-abs (fp32) or, for bf16, max-abs within
2e-2 of the RMS of the output row the element belongs to (see gpu_util.attn_error for why per row)."""
import math

import numpy as np
import pytest
import torch

import oracle
import paper_2410_12876_amd as ag
import workloads as W
from gpu_util import (DEV, attn_error, attn_error_raw, attn_rms_error, attn_tolerance, cache_from_host, dev, ensure_built, host_bits, host_f32, make_ctx,
                      new_cache, torch_dtype)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _lib():
    ensure_built()


def code(name):
    return ag.AG_BF16 if name == "bf16" else ag.AG_F32


def rand_t(seed, shape, dtype, std=1.0):
    return W.store(np.random.default_rng(seed).standard_normal(shape).astype(np.float32) * std, dtype)


def rand_flags(seed, shape, keep):
    return (np.random.default_rng(seed).random(shape) < keep).astype(np.uint8)


# ----------------------------------------------------------------------------------------------- gate
def run_gate(x, w, bias, tau, n_sink):
    B, L, d_in = x.f32.shape
    H = w.f32.shape[1]
    ctx = make_ctx(B, L, H, H, 64, code("bf16" if x.is_bf16 else "f32"), d_in=d_in)
    logits = torch.empty(B, L, H, dtype=torch.float32, device=DEV)
    flags = torch.empty(B, H, L, dtype=torch.uint8, device=DEV)
    ag.ag_gate(ctx, dev(x), dev(w), dev(bias), tau, n_sink, logits, flags)
    torch.cuda.synchronize()
    ctx.close()
    return logits.cpu().numpy(), flags.cpu().numpy()


def check_gate(x, w, bias, tau, n_sink, logit_tol):
    logits, flags = run_gate(x, w, bias, tau, n_sink)
    ref_logits, ref_flags = oracle.gate(x.f32, w.f32, bias, tau, n_sink)
    assert np.abs(logits - ref_logits).max() <= logit_tol
    thr = oracle.logit_threshold(tau)
    near = (np.abs(ref_logits - thr) < 1e-3).transpose(0, 2, 1)        # [B,H,L], excluded and counted
    assert np.array_equal(flags[~near], ref_flags[~near])
    assert set(np.unique(flags)) <= {0, 1}
    return int(near.sum()), int((flags != ref_flags).sum())


def test_gate_config1_fp32():
    wl = W.config1()
    near, diff = check_gate(wl.x, wl.w_gate, wl.bias, wl.tau, wl.n_sink, 2e-5)
    print("cfg1 gate: %d logits within 1e-3 of the threshold, %d flags differ there" % (near, diff))


@pytest.mark.parametrize("B,L,d_in,H,tau,n_sink", [(1, 100, 256, 4, 0.5, 0), (2, 77, 512, 8, 0.3, 2),
                                                   (1, 1, 64, 32, 0.5, 0), (3, 333, 1024, 32, 0.7, 1)])
def test_gate_bf16_shapes(B, L, d_in, H, tau, n_sink):
    x = rand_t(1, (B, L, d_in), "bf16", 0.5)
    w = rand_t(2, (d_in, H), "bf16", 1.0 / math.sqrt(d_in))
    bias = np.random.default_rng(3).standard_normal(H).astype(np.float32) * 0.2
    check_gate(x, w, bias, tau, n_sink, 1e-4)


@pytest.mark.parametrize("B,L,d_in,H,misalign", [(1, 2048, 256, 4, False), (2, 1500, 512, 8, False), (1, 4100, 1024, 12, False),
                                                  (1, 9000, 128, 20, False), (1, 2100, 2048, 32, False), (1, 2048, 256, 6, False),
                                                  (1, 3000, 512, 8, True), (3, 3000, 4096, 32, False)])
def test_gate_bf16_many_tokens(B, L, d_in, H, misalign):
    """Enough tokens for the fused gate kernel: head counts that are and are not a multiple of 4 (the latter take the
    pre-packed weights), a weight tensor that is not 16-byte aligned (also pre-packed), launches with and without
    K splits across workgroups and with one and two workgroups per CU, twice in a row (the arrival counters must be
    back at zero)."""
    x = rand_t(11, (B, L, d_in), "bf16", 0.5)
    w = rand_t(12, (d_in, H), "bf16", 1.0 / math.sqrt(d_in))
    bias = np.random.default_rng(13).standard_normal(H).astype(np.float32) * 0.2
    ref_logits, ref_flags = oracle.gate(x.f32, w.f32, bias, 0.5, 1)
    near = (np.abs(ref_logits - oracle.logit_threshold(0.5)) < 1e-3).transpose(0, 2, 1)
    ctx = make_ctx(B, L, H, H, 64, code("bf16"), d_in=d_in)
    dw = dev(w)
    if misalign:
        buf = torch.zeros(d_in * H + 4, dtype=torch.bfloat16, device=DEV)
        buf[4:].copy_(dw.reshape(-1))
        dw = buf[4:].view(d_in, H)
        assert dw.data_ptr() % 16 == 8
    dx, db = dev(x), dev(bias)
    for rep in range(2):
        logits = torch.zeros(B, L, H, dtype=torch.float32, device=DEV)
        flags = torch.full((B, H, L), 7, dtype=torch.uint8, device=DEV)
        ag.ag_gate(ctx, dx, dw, db, 0.5, 1, logits, flags)
        torch.cuda.synchronize()
        assert np.abs(logits.cpu().numpy() - ref_logits).max() <= 1e-4
        got = flags.cpu().numpy()
        assert np.array_equal(got[~near], ref_flags[~near]) and set(np.unique(got)) <= {0, 1}
    ctx.close()


def test_gate_fp32_ragged():
    x = rand_t(4, (2, 50, 96), "f32")
    w = rand_t(5, (96, 5), "f32", 0.1)
    check_gate(x, w, np.zeros(5, np.float32), 0.5, 0, 2e-5)


def test_gate_config2_full_size():
    wl = W.config2(with_qkv=False)
    near, diff = check_gate(wl.x, wl.w_gate, wl.bias, wl.tau, wl.n_sink, 1e-4)
    _, flags = oracle.gate(wl.x.f32, wl.w_gate.f32, wl.bias, wl.tau, wl.n_sink)
    keep = flags[0].mean(axis=1)
    assert np.abs(keep - wl.keep).max() < 0.05          # the bias recipe lands near the target keep ratios
    print("cfg2 gate: %d of %d logits within 1e-3 of the threshold (%d flags differ there)" %
          (near, flags.size, diff))


# ------------------------------------------------------------------------------- normalisation + gate
def check_rmsnorm_gate(h, g, eps, w, bias, tau, n_sink, misalign=False, what=""):
    """x against the fp64 definition (nearest bf16 up to the fp32 arithmetic: within 2^-8 (1 + 2^-10) of the exact
    value, and at most one bf16 spacing from the oracle's stored x), logits and flags against the oracle's gate of
    the x the kernel stored, in place == out of place, and the unfused ag_gate on that x agrees."""
    B, L, d = h.f32.shape
    H = w.f32.shape[1]
    ctx = make_ctx(B, L, H, H, 64, ag.AG_BF16, d_in=d)
    dh, dg, db = dev(h), dev(g), dev(bias)
    dw = dev(w)
    if misalign:
        buf = torch.zeros(d * H + 4, dtype=torch.bfloat16, device=DEV)
        buf[4:].copy_(dw.reshape(-1))
        dw = buf[4:].view(d, H)
    x = torch.full_like(dh, 7.0)
    logits = torch.zeros(B, L, H, dtype=torch.float32, device=DEV)
    flags = torch.full((B, H, L), 7, dtype=torch.uint8, device=DEV)
    ag.ag_rmsnorm_gate(ctx, dh, dg, eps, dw, db, tau, n_sink, x, logits, flags)
    torch.cuda.synchronize()
    got_x = host_f32(x).astype(np.float64)
    exact = oracle.rmsnorm(h.f32, g.f32, eps)
    stored = oracle.rmsnorm(h.f32, g.f32, eps, store="bf16")
    assert np.all(np.abs(got_x - exact) <= np.abs(exact) * (2.0 ** -8) * (1 + 2.0 ** -10) + 1e-30), what
    assert np.all(np.abs(got_x - stored) <= np.abs(stored) * 2.0 ** -7), what
    n_off = int((got_x != stored).sum())
    assert n_off <= 1e-3 * got_x.size + 2, (what, n_off)
    ref_logits, ref_flags = oracle.gate(got_x.astype(np.float32), w.f32, bias, tau, n_sink)
    got_l, got_f = logits.cpu().numpy(), flags.cpu().numpy()
    assert np.abs(got_l - ref_logits).max() <= 1e-4, what
    near = (np.abs(ref_logits - oracle.logit_threshold(tau)) < 1e-3).transpose(0, 2, 1)
    assert np.array_equal(got_f[~near], ref_flags[~near]) and set(np.unique(got_f)) <= {0, 1}, what
    # in place
    x2 = dh.clone()
    l2, f2 = torch.zeros_like(logits), torch.zeros_like(flags)
    ag.ag_rmsnorm_gate(ctx, x2, dg, eps, dw, db, tau, n_sink, x2, l2, f2)
    torch.cuda.synchronize()
    assert torch.equal(x2, x) and torch.equal(l2, logits) and torch.equal(f2, flags), what
    # the unfused gate on the stored x
    l3, f3 = torch.zeros_like(logits), torch.zeros_like(flags)
    ag.ag_gate(ctx, x, dw, db, tau, n_sink, l3, f3)
    torch.cuda.synchronize()
    assert (l3 - logits).abs().max().item() <= 1e-4, what
    assert np.array_equal(f3.cpu().numpy()[~near], got_f[~near]), what
    ctx.poll_error()
    ctx.close()
    return n_off, bool(torch.equal(l3, logits))


@pytest.mark.parametrize("B,L,d,H,tau,n_sink,misalign", [
    (1, 100, 256, 4, 0.5, 0, False), (2, 77, 512, 8, 0.3, 2, False), (1, 1, 64, 32, 0.5, 0, False),
    (1, 33, 4096, 32, 0.5, 1, False), (3, 333, 1024, 6, 0.7, 1, False), (1, 2100, 2048, 32, 0.5, 0, False),
    (1, 64, 3072, 12, 0.5, 0, True), (2, 50, 4032, 20, 0.4, 0, False), (1, 40, 8192, 32, 0.5, 0, False),
    (2, 300, 5120, 8, 0.5, 1, False), (1, 70, 6144, 6, 0.5, 0, False)])
def test_rmsnorm_gate_shapes(B, L, d, H, tau, n_sink, misalign):
    """Feature counts that fill all, some and (d = 64, 256) not even one chunk per wave, head counts that take the
    weights as stored and pre-packed, ragged last tiles; rows of very different scale, an all-zero row and a row with
    one huge feature among them."""
    g0 = np.random.default_rng(21)
    hv = g0.standard_normal((B, L, d)).astype(np.float32) * np.exp(g0.uniform(-3, 3, size=(B, L, 1))).astype(np.float32)
    hv[0, L // 2] = 0.0
    hv[0, L - 1, d // 3] = 3.0e4
    h = W.store(hv, "bf16")
    g = W.store(1.0 + 0.2 * g0.standard_normal(d).astype(np.float32), "bf16")
    w = rand_t(22, (d, H), "bf16", 1.0 / math.sqrt(d))
    bias = g0.standard_normal(H).astype(np.float32) * 0.2
    check_rmsnorm_gate(h, g, 1e-5, w, bias, tau, n_sink, misalign, "B%d L%d d%d H%d" % (B, L, d, H))


def test_rmsnorm_gate_many_tokens_equals_the_unfused_gate_bit_for_bit():
    """With 8192 tokens or more ag_gate runs its fused kernel without K splits, whose order of additions the fused
    normalisation + gate kernel repeats: the logits of the two are the same bits."""
    B, L, d, H = 2, 4500, 1024, 32
    g0 = np.random.default_rng(23)
    h = W.store(g0.standard_normal((B, L, d)).astype(np.float32) * 2.5, "bf16")
    g = W.store(1.0 + 0.2 * g0.standard_normal(d).astype(np.float32), "bf16")
    w = rand_t(24, (d, H), "bf16", 1.0 / math.sqrt(d))
    _, same_bits = check_rmsnorm_gate(h, g, 1e-6, w, np.zeros(H, np.float32), 0.5, 0, False, "many tokens")
    assert same_bits


# ----------------------------------------------------------------------------------------------- compaction
def run_compact(k, v, flags, row_off, pos0, fill=None):
    B, Hkv, L, D = k.f32.shape
    dt = "bf16" if k.is_bf16 else "f32"
    ctx = make_ctx(B, L, Hkv, Hkv, D, code(dt))
    cache = new_cache(B, Hkv, D, torch_dtype(dt), row_off, fill)
    ag.ag_compact_kv(ctx, dev(k), dev(v), dev(flags), pos0, cache)
    torch.cuda.synchronize()
    return ctx, cache


def check_compact(k, v, flags, cap, pos0=0):
    B, Hkv, L, D = k.f32.shape
    ro = oracle.slab_row_off(B * Hkv, cap)
    ctx, cache = run_compact(k, v, flags, ro, pos0)
    ref, over = oracle.compact_kv(k.storage, v.storage, flags, ro, pos0)
    got_len = cache.len.cpu().numpy()
    assert np.array_equal(got_len, ref.len)
    gk, gv, gi = host_bits(cache.k), host_bits(cache.v), cache.idx.cpu().numpy()
    for u in range(B * Hkv):
        a, n = int(ro[u]), int(ref.len[u])
        assert np.array_equal(gi[a:a + n], ref.idx[a:a + n])
        assert np.array_equal(gk[a:a + n], ref.k[a:a + n]) and np.array_equal(gv[a:a + n], ref.v[a:a + n])
        # rows past len stay untouched (zeros / -1)
        assert not gk[a + n:int(ro[u + 1])].any() and (gi[a + n:int(ro[u + 1])] == -1).all()
    if over:
        with pytest.raises(ag.AgError) as e:
            ctx.poll_error()
        assert e.value.status == ag.AG_ECAPACITY
    ctx.poll_error()          # clean (or cleared)
    ctx.close()


@pytest.mark.parametrize("dtype,B,H,L,D,keep", [("f32", 1, 4, 128, 64, 0.5), ("bf16", 2, 3, 1000, 128, 0.4),
                                                ("bf16", 1, 2, 63, 64, 0.7), ("bf16", 1, 1, 1, 128, 1.0),
                                                ("bf16", 1, 5, 65, 128, 0.1), ("f32", 1, 2, 200, 128, 0.5),
                                                ("bf16", 1, 2, 4096, 128, 0.55)])
def test_compact_bit_exact(dtype, B, H, L, D, keep):
    k, v = rand_t(6, (B, H, L, D), dtype), rand_t(7, (B, H, L, D), dtype)
    flags = rand_flags(8, (B, H, L), keep)
    check_compact(k, v, flags, L, pos0=17)


@pytest.mark.parametrize("seed", range(12))
def test_compact_shape_sweep(seed):
    """Seeded sweep over the scan + compaction launch: ragged lengths (word, 256-token-group and 4-byte alignment of a
    unit's flags all vary), both dtypes and head sizes, keep ratios from nothing to everything per head, and slabs
    that are sometimes too small (surplus rows dropped and reported)."""
    g = np.random.default_rng(500 + seed)
    dtype = "f32" if seed % 3 == 2 else "bf16"
    D = int(g.choice([64, 128]))
    B, H = int(g.integers(1, 4)), int(g.integers(1, 6))
    L = int(g.choice([1, 3, 63, 64, 65, 255, 256, 257, 511, 1000, 1023, 1025, 2050, 3001]))
    keep = g.choice([0.0, 0.05, 0.3, 0.5, 0.8, 1.0], size=(B, H, 1))
    flags = (g.random((B, H, L)) < keep).astype(np.uint8) * np.uint8(g.choice([1, 255]))
    k, v = rand_t(600 + seed, (B, H, L, D), dtype), rand_t(700 + seed, (B, H, L, D), dtype)
    most = int((flags != 0).reshape(B * H, L).sum(1).max())
    cap = L if seed % 4 else max(1, most - int(g.integers(0, max(2, most // 3))))
    check_compact(k, v, flags, cap, pos0=int(g.integers(0, 100)))


def test_compact_all_evicted_all_kept_and_overflow():
    B, H, L, D = 1, 3, 300, 128
    k, v = rand_t(9, (B, H, L, D), "bf16"), rand_t(10, (B, H, L, D), "bf16")
    flags = rand_flags(11, (B, H, L), 0.5)
    flags[0, 0] = 0
    flags[0, 1] = 1
    check_compact(k, v, flags, L)
    check_compact(k, v, flags, np.array([10, 100, 300]))       # unit 1 overflows: rows dropped, error word set


# ----------------------------------------------------------------------------------------------- prefill
def run_prefill(q, k, v, flags, scale, with_cache):
    B, Hq, L, D = q.f32.shape
    Hkv = k.f32.shape[1]
    dt = "bf16" if q.is_bf16 else "f32"
    ctx = make_ctx(B, L, Hq, Hkv, D, code(dt))
    dq, dk, dv, df = dev(q), dev(k), dev(v), dev(flags)
    out = torch.empty_like(dq)
    cache = None
    if with_cache:
        cache = new_cache(B, Hkv, D, torch_dtype(dt), oracle.slab_row_off(B * Hkv, L))
        ag.ag_compact_kv(ctx, dk, dv, df, 0, cache)
    ag.ag_prefill_attn(ctx, dq, dk, dv, df, scale, cache, out)
    torch.cuda.synchronize()
    ctx.poll_error()
    ctx.close()
    return host_f32(out)


def check_prefill(q, k, v, flags, scale, with_cache=True):
    dt = "bf16" if q.is_bf16 else "f32"
    got = run_prefill(q, k, v, flags, scale, with_cache)
    ref = oracle.prefill_attn(q.f32, k.f32, v.f32, flags, scale)
    tol = attn_tolerance(dt, ref)
    err = attn_error(dt, got, ref)
    assert np.isfinite(got).all()
    assert err <= tol, "error %.3g exceeds %.3g (raw max-abs %.3g)" % (err, tol, np.abs(got - ref).max())
    if dt == "bf16":
        assert attn_rms_error(got, ref) <= 5e-3
    return err, tol


def test_prefill_config1_fp32():
    wl = W.config1()
    _, flags = oracle.gate(wl.x.f32, wl.w_gate.f32, wl.bias, wl.tau, wl.n_sink)
    err, tol = check_prefill(wl.q, wl.k, wl.v, flags, wl.scale)
    print("cfg1 prefill max-abs err %.3g (tol %.3g)" % (err, tol))


@pytest.mark.parametrize("Hq,Hkv,L,D,keep,with_cache", [(2, 2, 300, 128, 0.5, True), (4, 4, 129, 128, 0.3, False),
                                                        (8, 2, 200, 128, 0.6, True), (4, 2, 257, 128, 0.5, True),
                                                        (16, 2, 70, 128, 0.5, True), (2, 2, 333, 64, 0.5, True),
                                                        (8, 2, 100, 64, 0.4, False), (1, 1, 1, 128, 1.0, True),
                                                        (2, 1, 31, 128, 0.9, True)])
def test_prefill_bf16_shapes(Hq, Hkv, L, D, keep, with_cache):
    B = 2
    q, k, v = rand_t(12, (B, Hq, L, D), "bf16"), rand_t(13, (B, Hkv, L, D), "bf16"), rand_t(14, (B, Hkv, L, D), "bf16")
    flags = rand_flags(15, (B, Hkv, L), keep)
    check_prefill(q, k, v, flags, 1.0 / math.sqrt(D), with_cache)


@pytest.mark.parametrize("dtype,D", [("bf16", 128), ("f32", 64)])
def test_prefill_fully_evicted_head_returns_own_value_and_all_kept_is_causal(dtype, D):
    B, H, L = 1, 3, 150
    q, k, v = rand_t(16, (B, H, L, D), dtype), rand_t(17, (B, H, L, D), dtype), rand_t(18, (B, H, L, D), dtype)
    flags = rand_flags(19, (B, H, L), 0.5)
    flags[0, 0] = 0          # fully evicted head: out == v exactly
    flags[0, 1] = 1          # nothing evicted: ordinary causal attention
    got = run_prefill(q, k, v, flags, 0.1, True)
    assert np.array_equal(got[0, 0], v.f32[0, 0])
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q.f32[:, 1:2]).double(), torch.from_numpy(k.f32[:, 1:2]).double(),
        torch.from_numpy(v.f32[:, 1:2]).double(), is_causal=True, scale=0.1).numpy()
    assert attn_error(dtype, got[:, 1:2], ref) <= attn_tolerance(dtype, ref)


@pytest.mark.parametrize("dtype,D,scale_mult,offset", [("bf16", 128, 8.0, 0.0), ("bf16", 128, 1.0, 300.0), ("bf16", 64, 6.0, 0.0),
                                                       ("f32", 64, 3.0, 0.0)])
def test_prefill_sharp_and_shifted_scores(dtype, D, scale_mult, offset):
    """Scores whose row maximum jumps by far more than the kernel's lazy-rescale gap from tile to tile (a scale 6 to 8
    times 1/sqrt(D): nearly one-hot softmax rows), and scores shifted by a large common offset (a constant
    component in q and k: every score near +300, differences of order one) -- the running maximum must absorb both.
    (fp32 only with moderate magnitudes: its 1e-5 bound cannot hold once the scores themselves, computed in fp32,
    are hundreds -- one unit in the last place of a score of 400 is already 3e-5.)"""
    B, H, L = 1, 2, 700
    g = np.random.default_rng(int(D + 10 * scale_mult + offset))
    qf, kf = g.standard_normal((B, H, L, D)), g.standard_normal((B, H, L, D))
    if offset:
        qf[..., 0] = math.sqrt(offset * math.sqrt(D))
        kf[..., 0] = math.sqrt(offset * math.sqrt(D))
    q, k = W.store(qf.astype(np.float32), dtype), W.store(kf.astype(np.float32), dtype)
    v = rand_t(41, (B, H, L, D), dtype)
    flags = rand_flags(42, (B, H, L), 0.5)
    check_prefill(q, k, v, flags, scale_mult / math.sqrt(D))
    check_prefill(q, k, v, flags, scale_mult / math.sqrt(D), with_cache=False)


def test_prefill_poisoned_evicted_rows_do_not_leak():
    """NaN in the K/V rows of evicted tokens must not reach any kept token's output row."""
    B, H, L, D = 1, 2, 200, 128
    q, k, v = rand_t(20, (B, H, L, D), "bf16"), rand_t(21, (B, H, L, D), "bf16"), rand_t(22, (B, H, L, D), "bf16")
    flags = rand_flags(23, (B, H, L), 0.5)
    clean = run_prefill(q, k, v, flags, 0.09, True)
    kp, vp = k.f32.copy(), v.f32.copy()
    kp[flags == 0] = np.nan
    vp[flags == 0] = np.nan
    got = run_prefill(q, W.store(kp, "bf16"), W.store(vp, "bf16"), flags, 0.09, True)
    kept = flags == 1
    assert np.array_equal(got[kept], clean[kept]) and np.isfinite(got[kept]).all()


def test_prefill_config2_full_size_every_row_of_every_head():
    """Full Llama2-7B layer shape in the launch configuration the benchmark times; every output row of all 32
    heads against the oracle."""
    wl = W.config2()
    _, flags = oracle.gate(wl.x.f32, wl.w_gate.f32, wl.bias, wl.tau, wl.n_sink)
    got = run_prefill(wl.q, wl.k, wl.v, flags, wl.scale, True)
    ref = oracle.prefill_attn(wl.q.f32, wl.k.f32, wl.v.f32, flags, wl.scale)
    worst = 0.0
    for h in range(wl.Hq):
        err = attn_error("bf16", got[:, h:h + 1], ref[:, h:h + 1])
        worst = max(worst, err)
        assert err <= attn_tolerance("bf16") and attn_rms_error(got[:, h:h + 1], ref[:, h:h + 1]) <= 5e-3, \
            "head %d (keep %.2f): %.3g" % (h, flags[0, h].mean(), err)
    print("cfg2 all %d heads x %d rows: worst max-abs err / row RMS beyond the store %.3g (raw %.3g), RMS err / RMS %.3g"
          % (wl.Hq, wl.L, worst, attn_error_raw("bf16", got, ref), attn_rms_error(got, ref)))
    assert np.isfinite(got).all()


# ----------------------------------------------------------------------------------------------- decode
def check_decode(wl: W.DecodeWorkload, steps, keep_prob, tol_name, always_keep=(), overflow_step=False):
    """`steps` decode steps against the oracle, every unit, every step; then the appended rows bit for bit.
    Units listed in always_keep get flag 1 at every step (they reach their capacity len0 + steps exactly);
    overflow_step adds one more step in which exactly those units overflow: rows dropped, error reported."""
    B, Hq, Hkv, D = wl.B, wl.Hq, wl.Hkv, wl.D
    ctx = make_ctx(B, 1, Hq, Hkv, D, code(wl.dtype), cache_rows=int(wl.row_off[-1]))
    cache = cache_from_host(B, Hkv, D, wl.k_cache, wl.v_cache, wl.idx, wl.row_off, wl.len0)
    ref = oracle.Cache(wl.k_cache.f32.copy(), wl.v_cache.f32.copy(), wl.idx.copy(), wl.row_off.copy(), wl.len0.copy())
    out = torch.empty(B, Hq, D, dtype=torch_dtype(wl.dtype), device=DEV)
    worst = 0.0
    always_keep = np.asarray(always_keep, dtype=np.int64)

    def one_step(s):
        q, kn, vn, nf = wl.step_inputs(s, keep_prob)
        if nf is not None and len(always_keep):
            nf.reshape(-1)[always_keep] = 1
        ag.ag_decode_attn(ctx, dev(q), dev(kn), dev(vn), None if nf is None else dev(nf), wl.pos0 + s, wl.scale,
                          cache, out)
        want, dropped = oracle.decode_step(q.f32, kn.f32, vn.f32, nf, wl.pos0 + s, ref, wl.scale)
        got = host_f32(out)
        tol = attn_tolerance(tol_name, want)
        err = attn_error(tol_name, got, want)
        assert np.isfinite(got).all() and err <= tol, "step %d: err %.3g > tol %.3g" % (s, err, tol)
        assert np.array_equal(cache.len.cpu().numpy(), ref.len)
        return err / tol, dropped

    for s in range(steps):
        r, dropped = one_step(s)
        assert dropped == 0
        worst = max(worst, r)
    ctx.poll_error()
    if len(always_keep):
        cap = (wl.row_off[1:] - wl.row_off[:-1])[always_keep]
        assert np.array_equal(ref.len[always_keep], cap) and steps == wl.steps    # the capacity edge is reached
    if overflow_step:
        _, dropped = one_step(steps)
        assert dropped == len(always_keep) > 0
        with pytest.raises(ag.AgError) as e:
            ctx.poll_error()
        assert e.value.status == ag.AG_ECAPACITY
    # final cache state: appended rows and positions bit-exact
    gk, gv, gi = host_f32(cache.k), host_f32(cache.v), cache.idx.cpu().numpy()
    for u in range(B * Hkv):
        a, n = int(wl.row_off[u]), int(ref.len[u])
        assert np.array_equal(gk[a:a + n], ref.k[a:a + n]) and np.array_equal(gi[a:a + n], ref.idx[a:a + n])
        assert np.array_equal(gv[a:a + n], ref.v[a:a + n])
    ctx.close()
    return worst


def test_decode_config1_fp32_16_steps():
    """Config 1: gate -> compaction -> 16 decode steps (all new tokens kept), fp32."""
    wl = W.config1()
    _, flags = oracle.gate(wl.x.f32, wl.w_gate.f32, wl.bias, wl.tau, wl.n_sink)
    ro = oracle.slab_row_off(4, wl.L + 16)
    c, _ = oracle.compact_kv(wl.k.f32, wl.v.f32, flags, ro)
    dw = W.DecodeWorkload("cfg1_decode", 1, "f32", 1, 4, 4, 64, wl.scale, 16, c.len, ro, W.Tensor(c.k), W.Tensor(c.v),
                          c.idx, wl.L)
    check_decode(dw, 16, None, "f32")


@pytest.mark.parametrize("dtype,B,Hq,Hkv,D,max_len", [("bf16", 2, 4, 4, 128, 700), ("bf16", 1, 8, 2, 128, 1500),
                                                      ("bf16", 2, 4, 2, 64, 300), ("f32", 1, 4, 1, 128, 520),
                                                      ("bf16", 1, 16, 2, 128, 260)])
def test_decode_ragged_shapes(dtype, B, Hq, Hkv, D, max_len):
    g = np.random.default_rng(24)
    len0 = np.rint(max_len * (0.05 + 0.95 * g.random(B * Hkv))).astype(np.int32)
    len0[0] = 0           # an empty (fully evicted) unit: output = the new token's own value
    len0[-1] = 1
    wl = W.decode_batch(30, "t", dtype, B, Hq, Hkv, D, len0, 6, pos0=max_len)
    check_decode(wl, 6, 0.5, dtype)


@pytest.mark.parametrize("G,scale_mult", [(1, 8.0), (4, 6.0), (2, 1.0)])
def test_decode_sharp_and_shifted_scores(G, scale_mult):
    """Decode rows that are nearly one-hot (a scale several times 1/sqrt(D)) and, for the last case, scores with a
    large common offset (cache keys and queries share a constant component): the per-lane-group running maxima and
    the merges of their states must absorb both."""
    B, Hkv, D, steps = 2, 2, 128, 3
    g = np.random.default_rng(int(10 * scale_mult) + G)
    len0 = np.array([900, 130, 257, 1], np.int32)
    wl = W.decode_batch(33, "t", "bf16", B, Hkv * G, Hkv, D, len0, steps, pos0=1000)
    shift = scale_mult == 1.0
    if shift:  # every key of the cache gets the same large first component
        kf = wl.k_cache.f32.copy()
        kf[:, 0] = 60.0
        wl.k_cache = W.store(kf, "bf16")
    wl.scale = scale_mult / math.sqrt(D)
    ctx = make_ctx(B, 1, wl.Hq, Hkv, D, ag.AG_BF16, cache_rows=int(wl.row_off[-1]))
    cache = cache_from_host(B, Hkv, D, wl.k_cache, wl.v_cache, wl.idx, wl.row_off, wl.len0)
    ref = oracle.Cache(wl.k_cache.f32.copy(), wl.v_cache.f32.copy(), wl.idx.copy(), wl.row_off.copy(), wl.len0.copy())
    out = torch.empty(B, wl.Hq, D, dtype=torch.bfloat16, device=DEV)
    for s in range(steps):
        q, kn, vn, nf = wl.step_inputs(s, 0.5)
        if shift:
            qf, knf = q.f32.copy(), kn.f32.copy()
            qf[..., 0] = 60.0
            knf[..., 0] = 60.0
            q, kn = W.store(qf, "bf16"), W.store(knf, "bf16")
        ag.ag_decode_attn(ctx, dev(q), dev(kn), dev(vn), dev(nf), wl.pos0 + s, wl.scale, cache, out)
        want, dropped = oracle.decode_step(q.f32, kn.f32, vn.f32, nf, wl.pos0 + s, ref, wl.scale)
        got = host_f32(out)
        assert dropped == 0 and np.isfinite(got).all()
        assert attn_error("bf16", got, want) <= attn_tolerance("bf16", want), "step %d" % s
    ctx.close()


def test_decode_empty_cache_returns_new_value_exactly_and_overflow_is_dropped():
    B, H, D = 1, 2, 128
    wl = W.decode_batch(31, "t", "bf16", B, H, H, D, np.array([0, 3], np.int32), 1, pos0=10)
    ctx = make_ctx(B, 1, H, H, D, ag.AG_BF16, cache_rows=int(wl.row_off[-1]))
    cache = cache_from_host(B, H, D, wl.k_cache, wl.v_cache, wl.idx, wl.row_off, wl.len0)
    out = torch.empty(B, H, D, dtype=torch.bfloat16, device=DEV)
    q, kn, vn, _ = wl.step_inputs(0, None)
    ag.ag_decode_attn(ctx, dev(q), dev(kn), dev(vn), None, 10, wl.scale, cache, out)
    torch.cuda.synchronize()
    assert np.array_equal(host_f32(out)[0, 0], vn.f32[0, 0])
    ctx.poll_error()
    assert cache.len.cpu().numpy().tolist() == [1, 4]
    ag.ag_decode_attn(ctx, dev(q), dev(kn), dev(vn), None, 11, wl.scale, cache, out)     # capacity is len0 + 1
    with pytest.raises(ag.AgError) as e:
        ctx.poll_error()
    assert e.value.status == ag.AG_ECAPACITY
    assert cache.len.cpu().numpy().tolist() == [1, 4]
    ctx.close()


def test_decode_config3_reduced_batch():
    """Config 3's recipe (len ~ round(4096 U[0.1,1]), 5 % of units at length 1, Bernoulli(0.5) appends) at B=4."""
    wl = W.config3(B=4, steps=8)
    worst = check_decode(wl, 8, 0.5, "bf16")
    print("cfg3 (B=4) worst err/tol %.3f" % worst)


# ----------------------------------------------------------------------------------------------- whole path
def test_whole_path_config1():
    """gate -> compaction -> masked prefill -> decode, each stage fed by the HIP path's own previous stage."""
    wl = W.config1()
    ctx = make_ctx(1, wl.L, 4, 4, 64, ag.AG_F32, d_in=wl.d_model, cache_rows=4 * (wl.L + 16))
    flags = torch.empty(1, 4, wl.L, dtype=torch.uint8, device=DEV)
    dq, dk, dv = dev(wl.q), dev(wl.k), dev(wl.v)
    ag.ag_gate(ctx, dev(wl.x), dev(wl.w_gate), dev(wl.bias), wl.tau, wl.n_sink, None, flags)
    ro = oracle.slab_row_off(4, wl.L + 16)
    cache = new_cache(1, 4, 64, torch.float32, ro)
    ag.ag_compact_kv(ctx, dk, dv, flags, 0, cache)
    out = torch.empty_like(dq)
    ag.ag_prefill_attn(ctx, dq, dk, dv, flags, wl.scale, cache, out)
    torch.cuda.synchronize()
    rl, rf = oracle.gate(wl.x.f32, wl.w_gate.f32, wl.bias, wl.tau, wl.n_sink)
    far = (np.abs(rl - oracle.logit_threshold(wl.tau)) >= 1e-3).transpose(0, 2, 1)
    assert np.array_equal(flags.cpu().numpy()[far], rf[far])
    rf = flags.cpu().numpy()          # later stages are checked on the flags the HIP gate produced
    assert (rf[:, :, 0] == 1).all()                                  # token 0 always kept
    ref = oracle.prefill_attn(wl.q.f32, wl.k.f32, wl.v.f32, rf, wl.scale)
    assert np.abs(host_f32(out) - ref).max() <= 1e-5
    rc, _ = oracle.compact_kv(wl.k.f32, wl.v.f32, rf, ro)
    assert np.array_equal(cache.len.cpu().numpy(), rc.len)
    o = torch.empty(1, 4, 64, dtype=torch.float32, device=DEV)
    for s in range(16):
        q, kn, vn = (rand_t(100 + 3 * s + i, (1, 4, 64), "f32") for i in range(3))
        ag.ag_decode_attn(ctx, dev(q), dev(kn), dev(vn), None, wl.L + s, wl.scale, cache, o)
        want, _ = oracle.decode_step(q.f32, kn.f32, vn.f32, None, wl.L + s, rc, wl.scale)
        assert np.abs(host_f32(o) - want).max() <= 1e-5
    assert np.array_equal(cache.len.cpu().numpy(), rc.len)
    ctx.poll_error()
    ctx.close()
