"""Full-size parity runs of configs 3, 4 and 5, the launch shapes of the tuned kernels, reproducibility and
HIP-graph replay.  Problems too large for the oracle to compute whole are checked on sampled query rows of every
head (oracle.prefill_rows computes a chosen row from the definition); integer results are compared whole."""
import math

import numpy as np
import pytest
import torch

import oracle
import paper_2410_12876_amd as ag
import workloads as W
from gpu_util import (DEV, attn_error, attn_rms_error, attn_tolerance, cache_from_host, dev, ensure_built, host_bits,
                      host_f32, make_ctx, new_cache, torch_dtype)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _lib():
    ensure_built()


def sample_rows(L, seed, n_random=8):
    """Query positions that include the first/last rows and both sides of the 64- and 128-row tile edges."""
    fixed = [0, 1, 62, 63, 64, 65, 127, 128, 129, 255, 256, L // 2 - 1, L // 2, L - 130, L - 129, L - 128, L - 65, L - 64,
             L - 2, L - 1]
    rnd = np.random.default_rng(seed).integers(0, L, n_random).tolist()
    return np.array(sorted({r for r in fixed + rnd if 0 <= r < L}), dtype=np.int32)


def check_sampled_rows(got_f32, q, k, v, flags, scale, rows, what):
    ref = oracle.prefill_rows(q.f32, k.f32, v.f32, flags, scale, rows)
    got = got_f32[:, :, rows, :]
    err, tol = attn_error("bf16", got, ref), attn_tolerance("bf16", ref)
    rel = attn_rms_error(got, ref)
    print("%s: %d rows x %d heads: max-abs err / row RMS %.3g (tol %.3g), RMS err / RMS %.3g" %
          (what, len(rows), got.shape[0] * got.shape[1], err, tol, rel))
    assert np.isfinite(got).all() and err <= tol and rel <= 5e-3


def compact_and_check(ctx, wl, dk, dv, dflags, flags_np, cap):
    """ag_compact_kv into per-unit slabs of `cap` rows; rows, idx and len compared bit for bit."""
    U = wl.B * wl.Hkv
    ro = oracle.slab_row_off(U, cap)
    cache = new_cache(wl.B, wl.Hkv, wl.D, torch.bfloat16, ro, fill=float("nan"))    # slack rows poisoned
    ag.ag_compact_kv(ctx, dk, dv, dflags, 0, cache)
    torch.cuda.synchronize()
    ctx.poll_error()
    ref, over = oracle.compact_kv(wl.k.storage, wl.v.storage, flags_np, ro)
    assert over == 0
    assert np.array_equal(cache.len.cpu().numpy(), ref.len)
    gk, gv, gi = host_bits(cache.k), host_bits(cache.v), cache.idx.cpu().numpy()
    for u in range(U):
        a, n = int(ro[u]), int(ref.len[u])
        assert np.array_equal(gk[a:a + n], ref.k[a:a + n]) and np.array_equal(gv[a:a + n], ref.v[a:a + n])
        assert np.array_equal(gi[a:a + n], ref.idx[a:a + n])
    return cache, ref, ro


def decode_and_check(ctx, wl, cache, ref_bits: "oracle.Cache", ro, steps, seed, keep_prob):
    """`steps` decode steps on the cache the compaction left, against the oracle's decode on the same rows."""
    B, Hq, Hkv, D = wl.B, wl.Hq, wl.Hkv, wl.D
    ref = oracle.Cache(W.bf16_bits_to_f32(ref_bits.k), W.bf16_bits_to_f32(ref_bits.v), ref_bits.idx.copy(), ro.copy(),
                       ref_bits.len.copy())
    out = torch.empty(B, Hq, D, dtype=torch.bfloat16, device=DEV)
    g = np.random.default_rng(seed)
    for s in range(steps):
        q, kn, vn = (W.store(g.standard_normal(shape).astype(np.float32), "bf16")
                     for shape in ((B, Hq, D), (B, Hkv, D), (B, Hkv, D)))
        nf = None if keep_prob is None else (g.random((B, Hkv)) < keep_prob).astype(np.uint8)
        ag.ag_decode_attn(ctx, dev(q), dev(kn), dev(vn), None if nf is None else dev(nf), wl.L + s, wl.scale, cache, out)
        want, dropped = oracle.decode_step(q.f32, kn.f32, vn.f32, nf, wl.L + s, ref, wl.scale)
        got = host_f32(out)
        assert dropped == 0 and np.isfinite(got).all()
        assert attn_error("bf16", got, want) <= attn_tolerance("bf16", want)
        assert np.array_equal(cache.len.cpu().numpy(), ref.len)
    ctx.poll_error()


# ------------------------------------------------------------------------------------------------ config 4
def test_config4_full_size_gqa_long_prompt():
    """Llama-3-8B layer shape (32 query / 8 KV heads, L = 32768, run-structured flags, keep 0.3): compaction whole,
    prefill on sampled rows of all 32 query heads, then the 64 decode steps on the 8 long caches (every new
    token kept, so every unit ends exactly at its capacity L + 64; cache slack is NaN)."""
    wl = W.config4()
    B, L, Hq, Hkv, D = wl.B, wl.L, wl.Hq, wl.Hkv, wl.D
    steps = 64
    ctx = make_ctx(B, L, Hq, Hkv, D, ag.AG_BF16, cache_rows=B * Hkv * (L + steps))
    dq, dk, dv, df = dev(wl.q), dev(wl.k), dev(wl.v), dev(wl.flags)
    cache, ref, ro = compact_and_check(ctx, wl, dk, dv, df, wl.flags, L + steps)
    print("cfg4 keep %.3f" % wl.flags.mean())
    out = torch.empty_like(dq)
    ag.ag_prefill_attn(ctx, dq, dk, dv, df, wl.scale, cache, out)
    torch.cuda.synchronize()
    ctx.poll_error()
    check_sampled_rows(host_f32(out), wl.q, wl.k, wl.v, wl.flags, wl.scale, sample_rows(L, 44, 12), "cfg4 prefill")
    decode_and_check(ctx, wl, cache, ref, ro, steps, 45, None)
    assert (cache.len.cpu().numpy() == ref.len + steps).all() and int(ro[1] - ro[0]) == L + steps
    ctx.close()


# ------------------------------------------------------------------------------------------------ config 5
def _config5_layer_check(layer, B, steps=2, n_rows=4):
    """One layer of config 5 through the whole path against the oracle: gate whole, compaction whole, prefill on
    sampled rows of every head (fully evicted heads: whole output equals V bit for bit), decode steps over all
    caches.  With B < 16 the inputs are the first B sequences of the layer's B = 16 draw (the generator fills
    sequence after sequence), i.e. a subset of the configuration's (layer, sequence, head) units."""
    wl = W.config5_layer(layer, B=B)
    B, L, H, D, d = wl.B, wl.L, wl.Hq, wl.D, wl.d_model
    ctx = make_ctx(B, L, H, H, D, ag.AG_BF16, d_in=d, cache_rows=B * H * (L + steps))
    flags = torch.empty(B, H, L, dtype=torch.uint8, device=DEV)
    logits = torch.empty(B, L, H, dtype=torch.float32, device=DEV)
    ag.ag_gate(ctx, dev(wl.x), dev(wl.w_gate), dev(wl.bias), wl.tau, wl.n_sink, logits, flags)
    torch.cuda.synchronize()
    ref_logits, ref_flags = oracle.gate(wl.x.f32, wl.w_gate.f32, wl.bias, wl.tau, wl.n_sink)
    live = ~wl.extra["dead_heads"]
    assert np.abs(logits.cpu().numpy() - ref_logits)[:, :, live].max() <= 2e-4
    near = (np.abs(ref_logits - oracle.logit_threshold(wl.tau)) < 1e-3).transpose(0, 2, 1)
    fl = flags.cpu().numpy()
    assert np.array_equal(fl[~near], ref_flags[~near])
    print("cfg5 layer %d: keep %.3f, %d logits within 1e-3 of the threshold (excluded), %d of them differ, %d dead heads"
          % (layer, fl.mean(), int(near.sum()), int((fl != ref_flags).sum()), int((~live).sum())))
    assert (fl[:, ~live] == 0).all()
    # later stages are checked on the flags the HIP gate produced
    dq, dk, dv = dev(wl.q), dev(wl.k), dev(wl.v)
    cache, ref, ro = compact_and_check(ctx, wl, dk, dv, flags, fl, L + steps)
    if (~live).any():
        assert (ref.len.reshape(B, H)[:, ~live] == 0).all()
    out = torch.empty_like(dq)
    ag.ag_prefill_attn(ctx, dq, dk, dv, flags, wl.scale, cache, out)
    torch.cuda.synchronize()
    ctx.poll_error()
    for h in np.nonzero(~live)[0]:
        assert torch.equal(out[:, h], dv[:, h])            # fully evicted head: every row is its own value
    check_sampled_rows(host_f32(out), wl.q, wl.k, wl.v, fl, wl.scale, sample_rows(L, 50 + layer, n_rows),
                       "cfg5 layer %d prefill" % layer)
    decode_and_check(ctx, wl, cache, ref, ro, steps, 60 + layer, 0.5)
    ctx.close()
    return int((~live).sum())


@pytest.mark.parametrize("layer", [0, 31])
def test_config5_layer_full_size(layer):
    """One layer of the 32-layer stack at full size (B=16, L=2048, 32 heads): first layer (keep 0.9) and last
    layer (keep 0.1, several fully evicted heads)."""
    _config5_layer_check(layer, 16)


@pytest.mark.timeout(600)
def test_config5_every_layer_with_dead_heads_on_two_sequences_each():
    """Config 5's deep layers (24 to 31, where about a tenth of the heads are fully evicted): the first two sequences
    of every such layer through gate, compaction, prefill and decode -- 8 layers x 2 sequences x 32 heads = 512
    (layer, sequence, head) units, every dead head among them -- and every second shallower layer on one sequence."""
    dead = 0
    for layer in range(24, 32):
        dead += _config5_layer_check(layer, 2, n_rows=2)
    assert dead >= 8                      # the recipe gives each deep layer about three dead heads
    for layer in range(2, 24, 2):
        _config5_layer_check(layer, 1, steps=1, n_rows=0)


# ------------------------------------------------------------------------------------------------ config 3
@pytest.mark.timeout(900)
def test_config3_full_batch_all_256_steps_to_the_capacity_edge():
    """Config 3 as specified: B = 32 (1024 ragged caches, 2.3 M rows), all 256 steps, every unit checked at every
    step.  Cache slack (the rows between len and capacity) is NaN on both sides, so a read past len would show.
    Sixteen units are always kept, so they end exactly at their capacity len0 + 256; one further step makes
    exactly those overflow (rows dropped, AG_ECAPACITY, nothing written out of bounds)."""
    from test_parity_gpu import check_decode
    wl = W.config3(B=32, steps=256, fill_slack=float("nan"))
    edge = np.concatenate([np.arange(8), np.nonzero(wl.len0 == 1)[0][:4], np.argsort(wl.len0)[-4:]])
    worst = check_decode(wl, 256, 0.5, "bf16", always_keep=np.unique(edge), overflow_step=True)
    print("cfg3 (B=32, 256 steps) worst err/tol %.3f" % worst)


# ------------------------------------------------------------------------------- launch shapes of the D=128 kernel
def _prefill_case(B, Hq, Hkv, L, flags, seed, with_cache=True, D=128):
    g = np.random.default_rng(seed)
    q, k, v = (W.store(g.standard_normal(s).astype(np.float32), "bf16")
               for s in ((B, Hq, L, D), (B, Hkv, L, D), (B, Hkv, L, D)))
    ctx = make_ctx(B, L, Hq, Hkv, D, ag.AG_BF16)
    dq, dk, dv, df = dev(q), dev(k), dev(v), dev(flags)
    out = torch.empty_like(dq)
    cache = None
    if with_cache:
        cache = new_cache(B, Hkv, D, torch.bfloat16, oracle.slab_row_off(B * Hkv, L))
        ag.ag_compact_kv(ctx, dk, dv, df, 0, cache)
    ag.ag_prefill_attn(ctx, dq, dk, dv, df, 1.0 / math.sqrt(D), cache, out)
    torch.cuda.synchronize()
    ctx.poll_error()
    ctx.close()
    return q, k, v, out


@pytest.mark.parametrize("name,B,Hq,Hkv,L,D", [
    ("split in two key chunks, balanced order", 1, 16, 16, 2048, 128),
    ("few heads: up to 8 key chunks per item, heads not a multiple of 8 (no reordering)", 1, 3, 3, 4096, 128),
    ("few heads, GQA, long prompt: 4 key chunks", 1, 8, 2, 8192, 128),
    ("large launch, no split", 4, 32, 32, 2048, 128),
    ("more than 1024 units (plan off)", 36, 32, 32, 256, 128),
    ("GQA split", 1, 32, 8, 2048, 128),
    ("ragged length", 2, 16, 4, 1987, 128),
    ("head dimension 64: split in two key chunks, balanced order", 1, 16, 16, 2048, 64),
    ("head dimension 64: few heads, GQA, 4 key chunks", 1, 8, 2, 8192, 64),
    ("head dimension 64: many heads, head-major order, ragged length", 5, 32, 32, 700, 64),
])
def test_prefill_bf16_launch_shapes(name, B, Hq, Hkv, L, D):
    """The workgroup-to-item mapping, the head order and the key-chunk split change with the launch size; every
    variant must give the same rows.  Keep ratios differ strongly between heads (0.05 .. 1.0) so that chunking and
    ordering see uneven work; head 0 keeps everything, head 1 nothing."""
    g = np.random.default_rng(70)
    keep = np.linspace(1.0, 0.05, Hkv)[None, :, None]
    flags = (g.random((B, Hkv, L)) < keep).astype(np.uint8)
    flags[:, 0] = 1
    if Hkv > 1:
        flags[:, 1] = 0
    q, k, v, out = _prefill_case(B, Hq, Hkv, L, flags, 71, D=D)
    check_sampled_rows(host_f32(out), q, k, v, flags, 1.0 / math.sqrt(D), sample_rows(L, 72, 6), name)
    if Hkv > 1:
        G = Hq // Hkv
        assert torch.equal(out[:, G:2 * G], dev(v)[:, 1:2].expand(-1, G, -1, -1))


def test_prefill_and_gate_are_reproducible_bit_for_bit():
    """Two runs of the split/merge prefill and of the K-split gate give identical bits (fixed merge orders)."""
    B, H, L = 1, 32, 4096
    g = np.random.default_rng(80)
    flags = (g.random((B, H, L)) < np.linspace(0.2, 0.9, H)[None, :, None]).astype(np.uint8)
    a = _prefill_case(B, H, H, L, flags, 81)[3]
    b = _prefill_case(B, H, H, L, flags, 81)[3]
    assert torch.equal(a, b)
    c = _prefill_case(B, H, H, L, flags, 81, with_cache=False)[3]      # internal compaction: same rows, same result
    assert torch.equal(a, c)
    # few heads: items are cut into up to 8 key chunks, whose states are added in chunk order whoever arrives last
    flags4 = (g.random((1, 4, L)) < np.array([1.0, 0.9, 0.5, 0.2])[None, :, None]).astype(np.uint8)
    runs = [_prefill_case(1, 4, 4, L, flags4, 82)[3] for _ in range(3)]
    assert torch.equal(runs[0], runs[1]) and torch.equal(runs[0], runs[2])
    x = W.store(g.standard_normal((B, L, 4096)).astype(np.float32) * 0.5, "bf16")
    w = W.store(g.standard_normal((4096, H)).astype(np.float32) / 64.0, "bf16")
    bias = np.zeros(H, np.float32)
    res = []
    for _ in range(2):
        ctx = make_ctx(B, L, H, H, 128, ag.AG_BF16, d_in=4096)
        lo = torch.empty(B, L, H, dtype=torch.float32, device=DEV)
        fo = torch.empty(B, H, L, dtype=torch.uint8, device=DEV)
        ag.ag_gate(ctx, dev(x), dev(w), dev(bias), 0.5, 0, lo, fo)
        torch.cuda.synchronize()
        ctx.close()
        res.append((lo, fo))
    assert torch.equal(res[0][0], res[1][0]) and torch.equal(res[0][1], res[1][1])


def test_prefill_split_merge_is_reproducible_whichever_chunk_arrives_last():
    """Items cut into key chunks are merged by the chunk that arrives last, and which one that is changes with the
    load on the chip.  Two problems alternate on one context (so a state left over from the previous launch would be
    another problem's), half of the launches beside a stream of HBM traffic: every result must be the bits of the
    problem's first run.  (A product contracted into a fused multiply-add made the sum depend on the arrival order
    by one fp32 rounding; this is the regression test.)"""
    B, H, L, D = 1, 16, 2048, 128
    g = np.random.default_rng(83)
    sets = []
    for s in range(2):
        q, k, v = (dev(W.store(g.standard_normal((B, H, L, D)).astype(np.float32) * (1.0 + s), "bf16")) for _ in range(3))
        keep = np.linspace(0.95, 0.3, H)[None, :, None]
        sets.append((q, k, v, dev((g.random((B, H, L)) < keep).astype(np.uint8))))
    ro = oracle.slab_row_off(B * H, L)
    ctx = make_ctx(B, L, H, H, D, ag.AG_BF16)
    side = torch.cuda.Stream()
    junk = torch.empty(64 << 20, dtype=torch.uint8, device=DEV)

    def run(s, load):
        q, k, v, flags = sets[s]
        cache = new_cache(B, H, D, torch.bfloat16, ro)
        out = torch.empty_like(q)
        if load:
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                for _ in range(4):
                    junk.add_(1)
        ag.ag_compact_prefill_attn(ctx, q, k, v, flags, 1.0 / math.sqrt(D), 0, cache, out)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        return out

    base = [run(0, False), run(1, False)]
    for it in range(80):
        assert torch.equal(run(it % 2, it % 4 >= 2), base[it % 2]), it
    ctx.poll_error()
    ctx.close()


def test_gate_and_decode_are_reproducible_beside_other_traffic():
    """The gate's K splits across workgroups and the decode step's partial states are combined in a fixed order; two
    problems alternate on one context, half of the calls beside a stream of HBM traffic, and every result must be the
    bits of the problem's first run."""
    side = torch.cuda.Stream()
    junk = torch.empty(64 << 20, dtype=torch.uint8, device=DEV)

    def loaded(fn, load):
        if load:
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                for _ in range(4):
                    junk.add_(1)
        r = fn()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        return r

    def alternate(fns, n):
        base = [loaded(f, False) for f in fns]
        for it in range(n):
            got = loaded(fns[it % 2], it % 4 >= 2)
            assert all(torch.equal(a, b) for a, b in zip(got, base[it % 2])), it

    g = np.random.default_rng(84)
    B, L, d, H = 1, 2100, 2048, 32                         # 16-token tiles and 2 K splits across workgroups
    ctx = make_ctx(B, L, H, H, 128, ag.AG_BF16, d_in=d)
    xs = [dev(W.store(g.standard_normal((B, L, d)).astype(np.float32) * (0.5 + s), "bf16")) for s in range(2)]
    ws = [dev(W.store(g.standard_normal((d, H)).astype(np.float32) / math.sqrt(d), "bf16")) for s in range(2)]
    bias = dev(np.zeros(H, np.float32))

    def gate(s):
        def f():
            lo = torch.empty(B, L, H, dtype=torch.float32, device=DEV)
            fl = torch.empty(B, H, L, dtype=torch.uint8, device=DEV)
            ag.ag_gate(ctx, xs[s], ws[s], bias, 0.5, 0, lo, fl)
            return lo, fl
        return f
    alternate([gate(0), gate(1)], 40)
    ctx.close()

    B, Hq, Hkv, D, cap = 8, 32, 8, 128, 4200
    ctx = make_ctx(B, 4096, Hq, Hkv, D, ag.AG_BF16, cache_rows=B * Hkv * cap)
    ro = oracle.slab_row_off(B * Hkv, cap)
    sets = []
    for s in range(2):
        lens = g.integers(1, 4000, size=B * Hkv).astype(np.int32)
        kc = torch.randn(B * Hkv * cap, D, device=DEV).to(torch.bfloat16) * (1 + s)
        q = torch.randn(B, Hq, D, device=DEV).to(torch.bfloat16)
        kn = torch.randn(B, Hkv, D, device=DEV).to(torch.bfloat16)
        sets.append((lens, kc, torch.randn_like(kc), q, kn, torch.randn_like(kn)))

    def decode(s):
        lens, kc, vc, q, kn, vn = sets[s]

        def f():
            cache = ag.KVCache(kc.clone(), vc.clone(), torch.zeros(B * Hkv * cap, dtype=torch.int32, device=DEV),
                               torch.from_numpy(ro).to(DEV), torch.from_numpy(lens).to(DEV), B, Hkv, D)
            out = torch.empty_like(q)
            ag.ag_decode_attn(ctx, q, kn, vn, None, 4096, 1.0 / math.sqrt(D), cache, out)
            return out, cache.len
        return f
    alternate([decode(0), decode(1)], 40)
    ctx.poll_error()
    ctx.close()


# ------------------------------------------------------------------------------------------------ HIP graph
def test_whole_step_replays_from_a_hip_graph():
    """gate -> compaction -> prefill -> decode captured once in a HIP graph: several replays, with eager work of
    the same library between them, must reproduce the eager step bit for bit (the kernels re-zero their own
    counters, nothing is cleared by a memset node)."""
    B, H, L, D, d = 1, 16, 2048, 128, 1024
    g = np.random.default_rng(90)
    x = dev(W.store(g.standard_normal((B, L, d)).astype(np.float32) * 0.5, "bf16"))
    w = dev(W.store(g.standard_normal((d, H)).astype(np.float32) / 32.0, "bf16"))
    bias = dev(np.linspace(-0.3, 0.3, H).astype(np.float32))
    q, k, v = (dev(W.store(g.standard_normal((B, H, L, D)).astype(np.float32), "bf16")) for _ in range(3))
    dq, dk, dv = (dev(W.store(g.standard_normal((B, H, D)).astype(np.float32), "bf16")) for _ in range(3))
    cap = L + 4
    ctx = make_ctx(B, L, H, H, D, ag.AG_BF16, d_in=d, cache_rows=B * H * cap)
    cache = new_cache(B, H, D, torch.bfloat16, oracle.slab_row_off(B * H, cap))
    flags = torch.empty(B, H, L, dtype=torch.uint8, device=DEV)
    out, dout = torch.empty_like(q), torch.empty_like(dq)

    def step():
        ag.ag_gate(ctx, x, w, bias, 0.5, 0, None, flags)
        ag.ag_compact_kv(ctx, k, v, flags, 0, cache)
        ag.ag_prefill_attn(ctx, q, k, v, flags, 1.0 / math.sqrt(D), cache, out)
        ag.ag_decode_attn(ctx, dq, dk, dv, None, L, 1.0 / math.sqrt(D), cache, dout)

    step()
    torch.cuda.synchronize()
    ref = [t.clone() for t in (flags, out, dout, cache.len, cache.k, cache.idx)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    for r in range(4):
        for t in (flags, out, dout, cache.len):
            t.zero_()
        graph.replay()
        torch.cuda.synchronize()
        for got, want in zip((flags, out, dout, cache.len, cache.k, cache.idx), ref):
            assert torch.equal(got, want), "replay %d differs from the eager step" % r
        step()                                              # eager work between the replays
        torch.cuda.synchronize()
    ctx.poll_error()
    ctx.close()


# ------------------------------------------------------------------------------------- recent-token window
def _prefill_recent(q, k, v, flags, scale, n_recent, with_cache=True):
    B, Hq, L, D = q.f32.shape
    Hkv = k.f32.shape[1]
    dt = ag.AG_BF16 if q.is_bf16 else ag.AG_F32
    ctx = make_ctx(B, L, Hq, Hkv, D, dt)
    dq, dk, dv, df = dev(q), dev(k), dev(v), dev(flags)
    out = torch.empty_like(dq)
    cache = None
    if with_cache:
        cache = new_cache(B, Hkv, D, dq.dtype, oracle.slab_row_off(B * Hkv, L))
        ag.ag_compact_kv(ctx, dk, dv, df, 0, cache)
    ag.ag_prefill_attn_recent(ctx, dq, dk, dv, df, scale, cache, n_recent, out)
    torch.cuda.synchronize()
    ctx.poll_error()
    ctx.close()
    return out


@pytest.mark.parametrize("dtype,B,Hq,Hkv,L,D,keep,n_recent,with_cache", [
    ("f32", 1, 4, 4, 128, 64, 0.5, 5, True),
    ("f32", 2, 4, 2, 77, 128, 0.3, 10, False),
    ("bf16", 2, 4, 4, 300, 64, 0.4, 5, True),        # generic MFMA kernel
    ("bf16", 1, 8, 2, 200, 64, 0.5, 10, True),       # ... with four query heads per workgroup
    ("bf16", 2, 2, 2, 300, 128, 0.5, 5, True),       # tuned D = 128 kernel
    ("bf16", 1, 4, 4, 257, 128, 0.3, 10, False),
    ("bf16", 1, 8, 2, 333, 128, 0.5, 10, True),      # GQA, 32 queries per workgroup
    ("bf16", 1, 4, 2, 500, 128, 0.2, 64, True),      # widest window, 64 queries per workgroup
    ("bf16", 1, 2, 2, 3, 128, 0.5, 10, True),        # prompt shorter than the window
    ("bf16", 1, 2, 2, 130, 128, 0.0, 5, True),       # nothing kept: plain sliding-window attention
])
def test_prefill_recent_window(dtype, B, Hq, Hkv, L, D, keep, n_recent, with_cache):
    """Table 6's recent-token settings (appendix "More Ablation", (6-1) and (6-2)): keys within n_recent - 1 positions before the query stay visible."""
    g = np.random.default_rng(100 + L + n_recent)
    q, k, v = (W.store(g.standard_normal(s).astype(np.float32), dtype)
               for s in ((B, Hq, L, D), (B, Hkv, L, D), (B, Hkv, L, D)))
    flags = (g.random((B, Hkv, L)) < keep).astype(np.uint8)
    scale = 1.0 / math.sqrt(D)
    got = host_f32(_prefill_recent(q, k, v, flags, scale, n_recent, with_cache))
    ref = oracle.prefill_attn(q.f32, k.f32, v.f32, flags, scale, n_recent=n_recent)
    err, tol = attn_error(dtype, got, ref), attn_tolerance(dtype, ref)
    assert np.isfinite(got).all() and err <= tol, "err %.3g > tol %.3g" % (err, tol)
    # the window changes the result (the case would pass vacuously otherwise)
    if keep < 1.0 and L > 2:
        assert np.abs(ref - oracle.prefill_attn(q.f32, k.f32, v.f32, flags, scale)).max() > 1e-3


def test_prefill_recent_window_full_size_and_window_of_one():
    """Config-2-sized launch (key-chunk split, balanced head order) with a window of 10, on sampled rows; and a
    window of 1 is ag_prefill_attn bit for bit."""
    B, H, L, D = 1, 32, 4096, 128
    g = np.random.default_rng(110)
    q, k, v = (W.store(g.standard_normal((B, H, L, D)).astype(np.float32), "bf16") for _ in range(3))
    flags = (g.random((B, H, L)) < np.linspace(0.2, 0.9, H)[None, :, None]).astype(np.uint8)
    scale = 1.0 / math.sqrt(D)
    out = _prefill_recent(q, k, v, flags, scale, 10)
    rows = sample_rows(L, 111, 6)
    ref = oracle.prefill_rows(q.f32, k.f32, v.f32, flags, scale, rows, n_recent=10)
    got = host_f32(out)[:, :, rows, :]
    assert attn_error("bf16", got, ref) <= attn_tolerance("bf16", ref) and attn_rms_error(got, ref) <= 5e-3
    one = _prefill_recent(q, k, v, flags, scale, 1)
    ctx = make_ctx(B, L, H, H, D, ag.AG_BF16)
    dq, dk, dv, df = dev(q), dev(k), dev(v), dev(flags)
    cache = new_cache(B, H, D, torch.bfloat16, oracle.slab_row_off(B * H, L))
    ag.ag_compact_kv(ctx, dk, dv, df, 0, cache)
    plain = torch.empty_like(dq)
    ag.ag_prefill_attn(ctx, dq, dk, dv, df, scale, cache, plain)
    torch.cuda.synchronize()
    ctx.close()
    assert torch.equal(one, plain)


@pytest.mark.parametrize("dtype,B,Hq,Hkv,D,L,n_recent,keep", [("bf16", 2, 4, 2, 128, 50, 5, 0.4),
                                                               ("f32", 1, 4, 4, 64, 37, 10, 0.5),
                                                               ("bf16", 1, 8, 2, 128, 3, 10, 0.5),
                                                               ("bf16", 2, 2, 2, 64, 200, 2, 0.1)])
def test_decode_recent_window_against_the_prefill_definition(dtype, B, Hq, Hkv, D, L, n_recent, keep):
    """Decoding with the ring of recent tokens: step s must equal row L + s of the windowed prefill definition over
    the whole history (prompt + generated tokens with their flags), which the oracle computes from scratch each
    step.  The cache itself evolves as without a window and is compared with the oracle's decode bit for bit."""
    steps = 14
    g = np.random.default_rng(120 + L)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    k_all = W.store(g.standard_normal((B, Hkv, L + steps, D)).astype(np.float32), dtype)
    v_all = W.store(g.standard_normal((B, Hkv, L + steps, D)).astype(np.float32), dtype)
    q_all = W.store(g.standard_normal((B, Hq, L + steps, D)).astype(np.float32), dtype)
    f_all = (g.random((B, Hkv, L + steps)) < keep).astype(np.uint8)
    scale = 1.0 / math.sqrt(D)
    U = B * Hkv
    ro = oracle.slab_row_off(U, L + steps)
    ctx = make_ctx(B, L, Hq, Hkv, D, ag.AG_BF16 if dtype == "bf16" else ag.AG_F32, cache_rows=int(ro[-1]))
    dk, dv, df = dev(k_all), dev(v_all), dev(f_all)
    kp, vp, fp = dk[:, :, :L].contiguous(), dv[:, :, :L].contiguous(), df[:, :, :L].contiguous()
    cache = new_cache(B, Hkv, D, tdt, ro)
    ag.ag_compact_kv(ctx, kp, vp, fp, 0, cache)
    ring = ag.RecentRing(torch.zeros(U, n_recent, D, dtype=tdt, device=DEV), torch.zeros(U, n_recent, D, dtype=tdt, device=DEV),
                         torch.zeros(U, n_recent, dtype=torch.uint8, device=DEV),
                         torch.zeros(U, n_recent, dtype=torch.int32, device=DEV), n_recent)
    ag.ag_recent_fill(ctx, kp, vp, fp, 0, ring)
    ref_cache, _ = oracle.compact_kv(k_all.f32[:, :, :L], v_all.f32[:, :, :L], f_all[:, :, :L], ro)
    out = torch.empty(B, Hq, D, dtype=tdt, device=DEV)
    dq = dev(q_all)
    for s in range(steps):
        p = L + s
        ag.ag_decode_attn_recent(ctx, dq[:, :, p].contiguous(), dk[:, :, p].contiguous(), dv[:, :, p].contiguous(),
                                 df[:, :, p].contiguous(), p, scale, cache, ring, out)
        want = oracle.prefill_rows(q_all.f32[:, :, :p + 1], k_all.f32[:, :, :p + 1], v_all.f32[:, :, :p + 1],
                                   f_all[:, :, :p + 1], scale, np.array([p]), n_recent=n_recent)[:, :, 0]
        got = host_f32(out)
        assert np.isfinite(got).all() and attn_error(dtype, got, want) <= attn_tolerance(dtype, want), "step %d" % s
        oracle.decode_step(q_all.f32[:, :, p], k_all.f32[:, :, p], v_all.f32[:, :, p], f_all[:, :, p], p, ref_cache, scale)
        assert np.array_equal(cache.len.cpu().numpy(), ref_cache.len)
    gk, gi = host_f32(cache.k), cache.idx.cpu().numpy()
    for u in range(U):
        a, n = int(ro[u]), int(ref_cache.len[u])
        assert np.array_equal(gk[a:a + n], ref_cache.k[a:a + n]) and np.array_equal(gi[a:a + n], ref_cache.idx[a:a + n])
    # the ring now holds the last n_recent positions, each in slot position % n_recent, with its flag
    end = L + steps
    rp, rf, rk = ring.pos.cpu().numpy(), ring.flags.cpu().numpy(), host_f32(ring.k)
    for p in range(max(0, end - n_recent), end):
        assert (rp[:, p % n_recent] == p).all()
        assert np.array_equal(rf[:, p % n_recent], f_all[:, :, p].reshape(U))
        assert np.array_equal(rk[:, p % n_recent], k_all.f32[:, :, p].reshape(U, D))
    ctx.poll_error()
    ctx.close()


# --------------------------------------------------------------------------------- main gate module (MHA')
def _gate_mha_case(B, L, d, hp, H, seed, tau=0.5, n_sink=0):
    g = np.random.default_rng(seed)
    x = W.store(g.standard_normal((B, L, d)).astype(np.float32) * 0.5, "bf16")
    wqkv = W.store(g.standard_normal((d, 3 * hp * 128)).astype(np.float32) / math.sqrt(d) * 2.0, "bf16")
    wo = W.store(g.standard_normal((hp * 128, H)).astype(np.float32) / math.sqrt(hp * 128), "bf16")
    bias = (g.standard_normal(H) * 0.1).astype(np.float32)
    ctx = ag.Context(0, ag.gate_mha_workspace_bytes(B, L, d, hp, 128, H))
    logits = torch.empty(B, L, H, dtype=torch.float32, device=DEV)
    flags = torch.empty(B, H, L, dtype=torch.uint8, device=DEV)
    ag.ag_gate_mha(ctx, dev(x), dev(wqkv), hp, 128, dev(wo), dev(bias), tau, n_sink, logits, flags)
    torch.cuda.synchronize()
    ctx.close()
    ref_logits, ref_flags = oracle.gate_mha(x.f32, wqkv.f32, hp, 128, wo.f32, bias, tau, n_sink, store="bf16")
    exact_logits, exact_flags = oracle.gate_mha(x.f32, wqkv.f32, hp, 128, wo.f32, bias, tau, n_sink, store=None)
    _gate_mha_exact_check(logits.cpu().numpy(), flags.cpu().numpy(), exact_logits, exact_flags, tau, n_sink)
    return logits.cpu().numpy(), flags.cpu().numpy(), ref_logits, ref_flags


# Largest distance between a logit of the HIP gate module and the oracle's exact (fp64, nothing rounded in between)
# logit that its bf16 intermediates Q', K', V', A may cause: each of the h' d'_k = 512 features of A carries a
# relative error of a few 2^-9 (its own rounding plus those of Q', K', V' behind it), the projection sums them
# against weights of size 1/sqrt(512) with random signs, which gives about 1e-2 |A|; measured at most 7e-3.
GATE_MHA_LOGIT_TOL = 1.5e-2


def _gate_mha_exact_check(logits, flags, exact_logits, exact_flags, tau, n_sink):
    """The module against the oracle that rounds nothing between its steps (the definition of Sec. 3.3, Eq. 3,
    independent of where the kernel stores bf16): logits within GATE_MHA_LOGIT_TOL, flags equal wherever the exact
    logit is further than that from the threshold, sink tokens kept."""
    err = float(np.abs(logits - exact_logits).max())
    near = (np.abs(exact_logits - oracle.logit_threshold(tau)) < GATE_MHA_LOGIT_TOL).transpose(0, 2, 1)
    print("gate_mha vs exact oracle: logit max-abs err %.3g (bound %.3g); %d of %d logits within the bound of the "
          "threshold, %d of them differ" % (err, GATE_MHA_LOGIT_TOL, int(near.sum()), near.size,
                                            int((flags != exact_flags).sum())))
    assert err <= GATE_MHA_LOGIT_TOL
    assert np.array_equal(flags[~near], exact_flags[~near])
    assert (flags[:, :, :n_sink] == 1).all()


@pytest.mark.parametrize("B,L,d,hp,H,n_sink", [(1, 300, 256, 4, 8, 0), (2, 129, 512, 2, 32, 2), (1, 1000, 1024, 4, 32, 0),
                                               (3, 64, 128, 1, 4, 1)])
def test_gate_mha_against_oracle(B, L, d, hp, H, n_sink):
    """The paper's main gate (MHA' front end + projection).  Q', K', V' and the attention output are bf16 tensors
    on both sides; flags are compared where the oracle's logit is further than 2e-2 from the threshold (the
    band that the bf16 storage of those tensors can move a logit by), the rest is counted."""
    tau = 0.45
    logits, flags, ref_logits, ref_flags = _gate_mha_case(B, L, d, hp, H, 130 + L, tau, n_sink)
    err = np.abs(logits - ref_logits).max()
    scale = np.sqrt(np.mean(ref_logits ** 2))
    near = (np.abs(ref_logits - oracle.logit_threshold(tau)) < 2e-2).transpose(0, 2, 1)
    print("gate_mha B%d L%d d%d h'%d: logit max-abs err %.3g (logit RMS %.3g); %d of %d within the band, %d flags differ"
          % (B, L, d, hp, err, scale, int(near.sum()), near.size, int((flags != ref_flags).sum())))
    assert err <= 1e-2
    assert np.array_equal(flags[~near], ref_flags[~near])
    assert (flags[:, :, :n_sink] == 1).all()


def test_gate_mha_full_size_llama2_7b_shape():
    """The gate module at the paper's size (d = 4096, h' = 4, d'_k = 128, 32 flag columns) on a 4096-token prompt."""
    tau = 0.5
    logits, flags, ref_logits, ref_flags = _gate_mha_case(1, 4096, 4096, 4, 32, 140, tau, 0)
    err = np.abs(logits - ref_logits).max()
    near = (np.abs(ref_logits - oracle.logit_threshold(tau)) < 2e-2).transpose(0, 2, 1)
    print("gate_mha full size: logit max-abs err %.3g (logit RMS %.3g); %d of %d within the band, %d flags differ"
          % (err, np.sqrt(np.mean(ref_logits ** 2)), int(near.sum()), near.size, int((flags != ref_flags).sum())))
    assert err <= 1e-2 and np.array_equal(flags[~near], ref_flags[~near])


@pytest.mark.parametrize("dtype,B,Hq,Hkv,L,D", [("bf16", 1, 16, 16, 2048, 128), ("bf16", 2, 8, 2, 300, 64), ("f32", 1, 4, 4, 128, 64)])
def test_compact_prefill_in_one_call_equals_the_two_calls(dtype, B, Hq, Hkv, L, D):
    """ag_compact_prefill_attn (one flag scan) leaves the same cache and the same output, bit for bit, as
    ag_compact_kv followed by ag_prefill_attn."""
    g = np.random.default_rng(150 + L)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    q, k, v = (dev(W.store(g.standard_normal(s).astype(np.float32), dtype))
               for s in ((B, Hq, L, D), (B, Hkv, L, D), (B, Hkv, L, D)))
    flags = dev((g.random((B, Hkv, L)) < np.linspace(0.1, 0.9, Hkv)[None, :, None]).astype(np.uint8))
    scale = 1.0 / math.sqrt(D)
    ro = oracle.slab_row_off(B * Hkv, L)
    ctx = make_ctx(B, L, Hq, Hkv, D, ag.AG_BF16 if dtype == "bf16" else ag.AG_F32)
    c1, c2 = new_cache(B, Hkv, D, tdt, ro), new_cache(B, Hkv, D, tdt, ro)
    o1, o2 = torch.empty_like(q), torch.empty_like(q)
    ag.ag_compact_kv(ctx, k, v, flags, 7, c1)
    ag.ag_prefill_attn(ctx, q, k, v, flags, scale, c1, o1)
    ag.ag_compact_prefill_attn(ctx, q, k, v, flags, scale, 7, c2, o2)
    torch.cuda.synchronize()
    ctx.poll_error()
    ctx.close()
    assert torch.equal(o1, o2) and torch.equal(c1.len, c2.len) and torch.equal(c1.idx, c2.idx)
    assert torch.equal(c1.k, c2.k) and torch.equal(c1.v, c2.v)


@pytest.mark.parametrize("first_evicting_layer", [1, 2])
def test_gate_of_the_next_layer_overlaps_on_a_second_stream(first_evicting_layer):
    """Previous-layer gating (Table 3, settings (4-1) and (4-2)): layer l evicts by the flags that the PREVIOUS
    layer's gate computes from the previous layer's hidden states; eviction begins at the second layer in (4-1) and
    at the third in (4-2), the layers before keep everything.  The flags of layer l + 1 then do not depend on
    layer l's attention, so that gate runs on a second stream (own context, own workspace, default priority) while
    layer l compacts and attends.  Every layer of the overlapped run is checked against the oracle -- flags
    (outside the 1e-3 band around the threshold), compacted lengths and positions, sampled attention rows -- and
    the overlapped run equals the in-line run bit for bit."""
    B, H, L, D, d, layers = 1, 16, 2048, 128, 1024, 4
    g = np.random.default_rng(160)
    xs_h = [W.store(g.standard_normal((B, L, d)).astype(np.float32) * 0.5, "bf16") for _ in range(layers)]
    wg_h = [W.store(g.standard_normal((d, H)).astype(np.float32) / 32.0, "bf16") for _ in range(layers)]
    bias_h = (0.3 * g.standard_normal(H)).astype(np.float32)
    qkv_h = [[W.store(g.standard_normal((B, H, L, D)).astype(np.float32), "bf16") for _ in range(3)] for _ in range(layers)]
    xs, wg, bias = [dev(t) for t in xs_h], [dev(t) for t in wg_h], dev(bias_h)
    qkv = [[dev(t) for t in lay] for lay in qkv_h]
    scale = 1.0 / math.sqrt(D)
    ro = oracle.slab_row_off(B * H, L)

    def gate_into(ctx, l, flags_l):
        """flags of layer l: the gate of layer l - 1 on layer l - 1's hidden states, or all ones before eviction begins"""
        if l < first_evicting_layer:
            flags_l.fill_(1)
        else:
            ag.ag_gate(ctx, xs[l - 1], wg[l - 1], bias, 0.5, 0, None, flags_l)

    def run(overlap):
        main = torch.cuda.current_stream()
        side = torch.cuda.Stream() if overlap else main
        ctx_a = make_ctx(B, L, H, H, D, ag.AG_BF16, d_in=d)
        ctx_g = make_ctx(B, L, H, H, D, ag.AG_BF16, d_in=d) if overlap else ctx_a
        flags = [torch.empty(B, H, L, dtype=torch.uint8, device=DEV) for _ in range(layers)]
        outs = [torch.empty_like(qkv[0][0]) for _ in range(layers)]
        caches = [new_cache(B, H, D, torch.bfloat16, ro) for _ in range(layers)]
        ready = [torch.cuda.Event() for _ in range(layers)]
        side.wait_stream(main)
        with torch.cuda.stream(side):
            gate_into(ctx_g, 0, flags[0])
            ready[0].record(side)
        for l in range(layers):
            if l + 1 < layers:      # the flags of the next layer: enqueued before, run beside, this layer's attention
                with torch.cuda.stream(side):
                    gate_into(ctx_g, l + 1, flags[l + 1])
                    ready[l + 1].record(side)
            main.wait_event(ready[l])
            q, k, v = qkv[l]
            ag.ag_compact_prefill_attn(ctx_a, q, k, v, flags[l], scale, 0, caches[l], outs[l])
        main.wait_stream(side)
        torch.cuda.synchronize()
        ctx_a.poll_error()
        ctx_a.close()
        if overlap:
            ctx_g.close()
        return flags, outs, caches

    f0, o0, c0 = run(False)
    f1, o1, c1 = run(True)
    rows = sample_rows(L, 161, 6)
    for l in range(layers):
        assert torch.equal(f0[l], f1[l]) and torch.equal(o0[l], o1[l])
        assert torch.equal(c0[l].len, c1[l].len) and torch.equal(c0[l].k, c1[l].k)
        # the overlapped run against the oracle
        fl = f1[l].cpu().numpy()
        if l < first_evicting_layer:
            assert (fl == 1).all()
        else:
            ref_logits, ref_flags = oracle.gate(xs_h[l - 1].f32, wg_h[l - 1].f32, bias_h, 0.5, 0)
            near = (np.abs(ref_logits - oracle.logit_threshold(0.5)) < 1e-3).transpose(0, 2, 1)
            assert np.array_equal(fl[~near], ref_flags[~near])
            assert 0.2 < fl.mean() < 0.8
        q, k, v = qkv_h[l]
        rc, over = oracle.compact_kv(k.storage, v.storage, fl, ro)
        assert over == 0 and np.array_equal(c1[l].len.cpu().numpy(), rc.len)
        gi, gk = c1[l].idx.cpu().numpy(), host_bits(c1[l].k)
        for u in range(B * H):
            a, n = int(ro[u]), int(rc.len[u])
            assert np.array_equal(gi[a:a + n], rc.idx[a:a + n]) and np.array_equal(gk[a:a + n], rc.k[a:a + n])
        check_sampled_rows(host_f32(o1[l]), q, k, v, fl, scale, rows, "previous-layer gating, layer %d" % l)


# ------------------------------------------------------------------------------------------- seeded shape sweeps
def _sweep_cases(n, seed):
    g = np.random.default_rng(seed)
    cases = []
    for i in range(n):
        D = int(g.choice([64, 128, 128]))
        dtype = "f32" if (i % 5 == 4) else "bf16"
        G = int(g.choice([1, 1, 2, 4, 8]))
        Hkv = int(g.integers(1, 5))
        B = int(g.integers(1, 4))
        L = int(g.choice([int(g.integers(1, 70)), int(g.integers(70, 400)), int(g.integers(400, 900))]))
        if dtype == "f32":
            L = min(L, 200)
        keep = float(g.choice([0.0, 0.1, 0.5, 0.9, 1.0]))
        n_recent = int(g.choice([1, 1, 3, 17]))
        cases.append((dtype, B, Hkv * G, Hkv, L, D, keep, n_recent, bool(g.integers(0, 2))))
    return cases


@pytest.mark.parametrize("case", _sweep_cases(24, 170), ids=lambda c: "%s-B%d-Hq%d-Hkv%d-L%d-D%d-keep%.1f-w%d-%s" % (
    c[0], c[1], c[2], c[3], c[4], c[5], c[6], c[7], "cache" if c[8] else "nocache"))
def test_prefill_shape_sweep(case):
    """Seeded sweep over batch, group size, ragged lengths, keep ratios (incl. 0 and 1), window and both prefill
    entry forms, element by element against the oracle."""
    dtype, B, Hq, Hkv, L, D, keep, n_recent, with_cache = case
    g = np.random.default_rng(171 + L + Hq)
    q, k, v = (W.store(g.standard_normal(s).astype(np.float32), dtype)
               for s in ((B, Hq, L, D), (B, Hkv, L, D), (B, Hkv, L, D)))
    flags = (g.random((B, Hkv, L)) < keep).astype(np.uint8)
    scale = 1.0 / math.sqrt(D)
    got = host_f32(_prefill_recent(q, k, v, flags, scale, n_recent, with_cache))
    ref = oracle.prefill_attn(q.f32, k.f32, v.f32, flags, scale, n_recent=n_recent)
    err, tol = attn_error(dtype, got, ref), attn_tolerance(dtype, ref)
    assert np.isfinite(got).all() and err <= tol, "err %.3g > tol %.3g" % (err, tol)


@pytest.mark.parametrize("seed", range(8))
def test_decode_shape_sweep(seed):
    """Seeded sweep over ragged decode batches (group sizes, empty and one-row units, both dtypes and head sizes)."""
    from test_parity_gpu import check_decode
    g = np.random.default_rng(180 + seed)
    dtype = "f32" if seed % 4 == 3 else "bf16"
    D = int(g.choice([64, 128]))
    G = int(g.choice([1, 2, 4, 8]))
    Hkv, B = int(g.integers(1, 5)), int(g.integers(1, 4))
    max_len = int(g.choice([40, 300, 1200]))
    len0 = np.rint(max_len * g.random(B * Hkv)).astype(np.int32)
    len0[g.integers(0, B * Hkv)] = 0
    wl = W.decode_batch(40 + seed, "t", dtype, B, Hkv * G, Hkv, D, len0, 5, pos0=max_len + 1)
    check_decode(wl, 5, 0.5, dtype)


# ------------------------------------------------------------------ K/V projection fused with the compaction
@pytest.mark.parametrize("B,L,d,Hkv,keep,cap_extra", [(1, 300, 256, 2, 0.5, 4), (3, 100, 128, 4, 0.3, 0), (2, 257, 512, 1, 0.9, 2),
                                                      (1, 4096, 4096, 32, None, 8), (2, 640, 1024, 8, 0.0, 1),
                                                      (1, 200, 64, 3, 1.0, -50)])
def test_project_compact_kv(B, L, d, Hkv, keep, cap_extra):
    """ag_project_compact_kv against the oracle's projection (Eq. 2) followed by its compaction.  The full K, V agree
    with the fp64 product rounded to bf16 up to one bf16 spacing (the kernel accumulates in fp32); idx and len are
    bit-exact; every cache row is bit-identical to the row of the kernel's own K, V that it copies.  The last case
    gives the units less room than they keep: the surplus rows are dropped and reported."""
    D = 128
    g = np.random.default_rng(300 + L)
    x = W.store((0.5 * g.standard_normal((B, L, d))).astype(np.float32), "bf16")
    w = W.store((g.standard_normal((d, 2 * Hkv * D)) / math.sqrt(d)).astype(np.float32), "bf16")
    if keep is None:
        rho = 0.2 + 0.7 * g.random((1, Hkv, 1))
        flags = (g.random((B, Hkv, L)) < rho).astype(np.uint8)
    else:
        flags = (g.random((B, Hkv, L)) < keep).astype(np.uint8)
    U = B * Hkv
    cap = max(1, int(flags.reshape(U, L).sum(1).max()) + cap_extra)
    ro = oracle.slab_row_off(U, cap)
    cache = new_cache(B, Hkv, D, torch.bfloat16, ro)
    cache.idx.fill_(-7)
    kv = torch.zeros(2, B, Hkv, L, D, dtype=torch.bfloat16, device=DEV)
    ws = max(ag.project_compact_workspace_bytes(B, L, Hkv), 1 << 20)
    ctx = ag.Context(0, ws)
    ag.ag_project_compact_kv(ctx, dev(x), dev(w), dev(flags), 11, kv, cache)
    torch.cuda.synchronize()
    want_k, want_v = oracle.project_kv(x.f32, w.f32, Hkv, D, store="bf16")
    got_k, got_v = host_f32(kv[0]).astype(np.float64), host_f32(kv[1]).astype(np.float64)
    for got, want in ((got_k, want_k), (got_v, want_v)):
        # one bf16 spacing of the larger magnitude, plus the fp32 accumulation error of a d-term sum near zero
        tol = np.maximum(np.abs(want), np.abs(got)) * 2.0 ** -7 + 1e-5 * math.sqrt(d)
        assert np.all(np.abs(got - want) <= tol)
        assert np.mean(got != want) < 0.05   # the two roundings rarely disagree
    ref, over = oracle.compact_kv(host_bits(kv[0]), host_bits(kv[1]), flags, ro, pos0=11)
    if cap_extra >= 0:
        assert over == 0
        ctx.poll_error()
    else:
        assert over > 0
        with pytest.raises(ag.AgError):
            ctx.poll_error()
    assert np.array_equal(cache.len.cpu().numpy(), ref.len)
    gk, gv, gi = host_bits(cache.k), host_bits(cache.v), cache.idx.cpu().numpy()
    for u in range(U):
        a, n = int(ro[u]), int(ref.len[u])
        assert np.array_equal(gk[a:a + n], ref.k[a:a + n]) and np.array_equal(gv[a:a + n], ref.v[a:a + n])
        assert np.array_equal(gi[a:a + n], ref.idx[a:a + n])
        assert (gi[a + n:int(ro[u + 1])] == -7).all()   # nothing written behind the valid rows
    ctx.close()


def test_project_compact_kv_feeds_the_prefill():
    """The fused call's outputs are what ag_prefill_attn expects: same result as project -> ag_compact_kv."""
    B, L, d, H, D = 1, 512, 512, 4, 128
    g = np.random.default_rng(333)
    x = W.store((0.5 * g.standard_normal((B, L, d))).astype(np.float32), "bf16")
    w = W.store((g.standard_normal((d, 2 * H * D)) / math.sqrt(d)).astype(np.float32), "bf16")
    q = W.store(g.standard_normal((B, H, L, D)).astype(np.float32), "bf16")
    flags = (g.random((B, H, L)) < 0.5).astype(np.uint8)
    ro = oracle.slab_row_off(B * H, L)
    ctx = make_ctx(B, L, H, H, D, ag.AG_BF16)
    kv = torch.zeros(2, B, H, L, D, dtype=torch.bfloat16, device=DEV)
    c1 = new_cache(B, H, D, torch.bfloat16, ro)
    ag.ag_project_compact_kv(ctx, dev(x), dev(w), dev(flags), 0, kv, c1)
    c2 = new_cache(B, H, D, torch.bfloat16, ro)
    ag.ag_compact_kv(ctx, kv[0], kv[1], dev(flags), 0, c2)
    o1, o2 = (torch.empty(B, H, L, D, dtype=torch.bfloat16, device=DEV) for _ in range(2))
    ag.ag_prefill_attn(ctx, dev(q), kv[0], kv[1], dev(flags), 1 / math.sqrt(D), c1, o1)
    ag.ag_prefill_attn(ctx, dev(q), kv[0], kv[1], dev(flags), 1 / math.sqrt(D), c2, o2)
    torch.cuda.synchronize()
    assert torch.equal(c1.len, c2.len) and torch.equal(o1, o2)
    ref = oracle.prefill_attn(q.f32, host_f32(kv[0]), host_f32(kv[1]), flags, 1 / math.sqrt(D))
    assert attn_error("bf16", host_f32(o1), ref) <= attn_tolerance("bf16", ref)
    ctx.close()


# ------------------------------------------------------------------ normalisation + gate at full size
def test_rmsnorm_gate_full_size_llama2_7b_shape():
    """ag_rmsnorm_gate on a whole Llama2-7B-shaped layer (4096 tokens x 4096 features, 32 heads): x within one bf16
    spacing of the oracle's stored x and nearest-rounded up to the fp32 arithmetic; logits and flags against the
    oracle's gate of the x the kernel stored."""
    wl = W.config2(with_qkv=False)
    B, L, d, H = wl.B, wl.L, wl.d_model, wl.Hkv
    g0 = np.random.default_rng(95)
    h = W.store(wl.x.f32 * np.exp(g0.uniform(-1, 2, size=(B, L, 1))).astype(np.float32), "bf16")
    g = W.store(1.0 + 0.1 * g0.standard_normal(d).astype(np.float32), "bf16")
    ctx = make_ctx(B, L, H, H, 128, ag.AG_BF16, d_in=d)
    x = torch.empty(B, L, d, dtype=torch.bfloat16, device=DEV)
    logits = torch.empty(B, L, H, dtype=torch.float32, device=DEV)
    flags = torch.empty(B, H, L, dtype=torch.uint8, device=DEV)
    ag.ag_rmsnorm_gate(ctx, dev(h), dev(g), 1e-5, dev(wl.w_gate), dev(wl.bias), wl.tau, wl.n_sink, x, logits, flags)
    torch.cuda.synchronize()
    ctx.poll_error()
    ctx.close()
    got_x = host_f32(x).astype(np.float64)
    exact = oracle.rmsnorm(h.f32, g.f32, 1e-5)
    stored = oracle.rmsnorm(h.f32, g.f32, 1e-5, store="bf16")
    assert np.all(np.abs(got_x - exact) <= np.abs(exact) * (2.0 ** -8) * (1 + 2.0 ** -10) + 1e-30)
    assert np.all(np.abs(got_x - stored) <= np.abs(stored) * 2.0 ** -7)
    n_off = int((got_x != stored).sum())
    assert n_off <= 1e-3 * got_x.size
    ref_logits, ref_flags = oracle.gate(got_x.astype(np.float32), wl.w_gate.f32, wl.bias, wl.tau, wl.n_sink)
    assert np.abs(logits.cpu().numpy() - ref_logits).max() <= 1e-4
    near = (np.abs(ref_logits - oracle.logit_threshold(wl.tau)) < 1e-3).transpose(0, 2, 1)
    got_f = flags.cpu().numpy()
    assert np.array_equal(got_f[~near], ref_flags[~near])
    print("rmsnorm+gate cfg2 shape: %d of %d stored x differ from the fp64 rounding by one spacing; %d logits within "
          "1e-3 of the threshold, %d flags differ there" % (n_off, got_x.size, int(near.sum()),
                                                             int((got_f != ref_flags).sum())))


# ------------------------------------------------------------------------------------------ kernel timing
def test_kernel_timing_counts_launches_and_leaves_results_alone():
    """With timing on, the step's kernels each report the launches made and a duration that is positive and below
    the wall-clock time of the timed region; the outputs are the bits of the untimed run."""
    import time
    wl = W.config2(L=2048)                                            # long enough for the fused gate kernel
    B, L, Hq, Hkv, D, d = wl.B, wl.L, wl.Hq, wl.Hkv, wl.D, wl.d_model
    U, cap = B * Hkv, L + 8
    ro = oracle.slab_row_off(U, cap)
    dq, dk, dv, dx, dw, db = dev(wl.q), dev(wl.k), dev(wl.v), dev(wl.x), dev(wl.w_gate), dev(wl.bias)
    g = np.random.default_rng(91)
    q1 = dev(W.store(g.standard_normal((B, Hq, D)).astype(np.float32), "bf16"))
    k1 = dev(W.store(g.standard_normal((B, Hkv, D)).astype(np.float32), "bf16"))
    v1 = dev(W.store(g.standard_normal((B, Hkv, D)).astype(np.float32), "bf16"))
    keep1 = torch.ones(B, Hkv, dtype=torch.uint8, device=DEV)
    res, steps = [], 3
    for timed in (False, True):
        ctx = make_ctx(B, L, Hq, Hkv, D, ag.AG_BF16, d_in=d, cache_rows=U * cap)
        flags = torch.empty(B, Hkv, L, dtype=torch.uint8, device=DEV)
        out, o1 = torch.empty_like(dq), torch.empty_like(q1)
        ctx.timing_enable(timed)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            cache = new_cache(B, Hkv, D, torch.bfloat16, ro)
            ag.ag_gate(ctx, dx, dw, db, wl.tau, wl.n_sink, None, flags)
            ag.ag_compact_prefill_attn(ctx, dq, dk, dv, flags, wl.scale, 0, cache, out)
            ag.ag_decode_attn(ctx, q1, k1, v1, keep1, L, wl.scale, cache, o1)
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3
        if timed:
            times = ctx.timing_read()
            for name in ("gate", "compact", "prefill", "decode_partial", "decode_merge"):
                ms, n = times[name]
                assert n == steps, (name, n)
                assert 0.0 < ms < wall_ms, (name, ms, wall_ms)
            ctx.timing_enable(True)                                   # enabling again clears the counts
            assert all(n == 0 for _, n in ctx.timing_read().values())
        ctx.poll_error()
        res.append((flags, out, o1, cache.len.clone()))
        ctx.close()
    for a, b in zip(*res):
        assert torch.equal(a, b)


# ------------------------------------------------------------------ the benchmark's step, at full size
def test_config2_full_size_step_as_the_benchmark_runs_it():
    """ag_gate -> ag_compact_prefill_attn -> ag_decode_attn on the whole Llama2-7B-shaped layer (config 2), the calls
    and launch shapes that bench.py times: flags against the oracle's gate (logits within 1e-3 of the threshold
    excluded and counted), the cache bit for bit against the oracle's compaction of the flags the GPU produced,
    sampled query rows of every head against the definition, one decode step against the oracle on that cache."""
    wl = W.config2()
    B, L, Hq, Hkv, D, d = wl.B, wl.L, wl.Hq, wl.Hkv, wl.D, wl.d_model
    U, cap = B * Hkv, L + 8
    ro = oracle.slab_row_off(U, cap)
    ctx = make_ctx(B, L, Hq, Hkv, D, ag.AG_BF16, d_in=d, cache_rows=U * cap)
    cache = new_cache(B, Hkv, D, torch.bfloat16, ro)
    flags = torch.empty(B, Hkv, L, dtype=torch.uint8, device=DEV)
    dq, dk, dv = dev(wl.q), dev(wl.k), dev(wl.v)
    out = torch.empty_like(dq)
    ag.ag_gate(ctx, dev(wl.x), dev(wl.w_gate), dev(wl.bias), wl.tau, wl.n_sink, None, flags)
    ag.ag_compact_prefill_attn(ctx, dq, dk, dv, flags, wl.scale, 0, cache, out)
    torch.cuda.synchronize()
    ctx.poll_error()
    got_flags = flags.cpu().numpy()
    ref_logits, ref_flags = oracle.gate(wl.x.f32, wl.w_gate.f32, wl.bias, wl.tau, wl.n_sink)
    near = (np.abs(ref_logits - oracle.logit_threshold(wl.tau)) < 1e-3).transpose(0, 2, 1)
    assert np.array_equal(got_flags[~near], ref_flags[~near])
    ref, over = oracle.compact_kv(wl.k.storage, wl.v.storage, got_flags, ro)
    assert over == 0 and np.array_equal(cache.len.cpu().numpy(), ref.len)
    gk, gv, gi = host_bits(cache.k), host_bits(cache.v), cache.idx.cpu().numpy()
    for u in range(U):
        a, n = int(ro[u]), int(ref.len[u])
        assert np.array_equal(gk[a:a + n], ref.k[a:a + n]) and np.array_equal(gv[a:a + n], ref.v[a:a + n])
        assert np.array_equal(gi[a:a + n], ref.idx[a:a + n])
    check_sampled_rows(host_f32(out), wl.q, wl.k, wl.v, got_flags, wl.scale, sample_rows(L, 77), "cfg2 step")
    decode_and_check(ctx, wl, cache, ref, ro, 1, 78, None)
    print("cfg2 step: %d of %d logits within 1e-3 of the threshold, %d flags differ there" %
          (int(near.sum()), near.size, int((got_flags != ref_flags).sum())))
    ctx.close()


# ----------------------------------------------------------------- the whole path on drawn shapes, packed caches
def _pipeline_cases(n, seed):
    g = np.random.default_rng(seed)
    cases = []
    for i in range(n):
        dtype = "f32" if i % 4 == 3 else "bf16"
        D = int(g.choice([64, 128]))
        Hkv = int(g.choice([1, 2, 4]))
        G = int(g.choice([1, 2, 4]))
        cases.append(dict(dtype=dtype, D=D, B=int(g.integers(1, 4)), Hkv=Hkv, Hq=Hkv * G, L=int(g.integers(20, 420)),
                          d_in=64 * int(g.integers(1, 9)), n_recent=int(g.choice([1, 3, 17, 64])), tau=float(g.choice([0.3, 0.5, 0.7])),
                          n_sink=int(g.choice([0, 1])), steps=int(g.integers(3, 9)), seed=int(g.integers(1 << 30))))
    return cases


@pytest.mark.parametrize("case", _pipeline_cases(24, 900), ids=lambda c: "%s-D%d-B%d-Hq%d-Hkv%d-L%d-d%d-w%d" % (
    c["dtype"], c["D"], c["B"], c["Hq"], c["Hkv"], c["L"], c["d_in"], c["n_recent"]))
def test_whole_path_on_drawn_shapes_with_packed_caches_and_recent_window(case):
    """Gate -> packed cache layout -> compaction -> windowed prefill over the cache -> decode steps with the ring of
    recent tokens, every stage against the oracle, on drawn shapes (both dtypes and head dimensions, grouped heads,
    window widths 1 .. 64, ragged lengths).  The later stages run on the flags the HIP gate produced; the units'
    capacities are their kept rows + `steps`, so the decode fills the packed cache exactly when every token is kept."""
    c = case
    dtype, D, B, Hq, Hkv, L, d_in, n_recent, steps = c["dtype"], c["D"], c["B"], c["Hq"], c["Hkv"], c["L"], c["d_in"], c["n_recent"], c["steps"]
    g = np.random.default_rng(c["seed"])
    tdt = torch_dtype(dtype)
    code = ag.AG_BF16 if dtype == "bf16" else ag.AG_F32
    T = L + steps
    x = W.store((0.5 * g.standard_normal((B, L, d_in))).astype(np.float32), dtype)
    wg = W.store((g.standard_normal((d_in, Hkv)) / math.sqrt(d_in)).astype(np.float32), dtype)
    bias = (0.3 * g.standard_normal(Hkv)).astype(np.float32)
    q_all, k_all, v_all = (W.store(g.standard_normal((B, h, T, D)).astype(np.float32), dtype) for h in (Hq, Hkv, Hkv))
    f_new = (g.random((B, Hkv, steps)) < 0.6).astype(np.uint8)
    scale = 1.0 / math.sqrt(D)
    U = B * Hkv
    # gate
    ctx = make_ctx(B, L, Hq, Hkv, D, code, d_in=d_in, cache_rows=U * T)
    flags = torch.empty(B, Hkv, L, dtype=torch.uint8, device=DEV)
    logits = torch.empty(B, L, Hkv, dtype=torch.float32, device=DEV)
    ag.ag_gate(ctx, dev(x), dev(wg), torch.from_numpy(bias).to(DEV), c["tau"], c["n_sink"], logits, flags)
    torch.cuda.synchronize()
    ref_logits, ref_flags = oracle.gate(x.f32, wg.f32, bias, c["tau"], c["n_sink"])
    assert np.abs(logits.cpu().numpy() - ref_logits).max() <= 2e-4
    near = (np.abs(ref_logits - oracle.logit_threshold(c["tau"])) < 1e-3).transpose(0, 2, 1)
    fl = flags.cpu().numpy()
    if c["n_sink"]:
        near[:, :, :c["n_sink"]] = False
    assert np.array_equal(fl[~near], ref_flags[~near])
    f_all = np.concatenate([fl, f_new], axis=2)
    # packed layout
    want_ro, need = oracle.packed_row_off(fl, steps, 10 ** 9)
    total = int(need)
    row_off = torch.zeros(U + 1, dtype=torch.int64, device=DEV)
    ag.ag_pack_row_off(ctx, flags, steps, total, row_off)
    torch.cuda.synchronize()
    assert np.array_equal(row_off.cpu().numpy(), want_ro)
    cache = ag.KVCache(torch.full((max(total, 1), D), float("nan"), dtype=tdt, device=DEV),
                       torch.full((max(total, 1), D), float("nan"), dtype=tdt, device=DEV),
                       torch.full((max(total, 1),), -1, dtype=torch.int32, device=DEV), row_off,
                       torch.zeros(U, dtype=torch.int32, device=DEV), B, Hkv, D, total_rows=total)
    dq, dk, dv = dev(q_all), dev(k_all), dev(v_all)
    qp, kp, vp = dq[:, :, :L].contiguous(), dk[:, :, :L].contiguous(), dv[:, :, :L].contiguous()
    ag.ag_compact_kv(ctx, kp, vp, flags, 0, cache)
    torch.cuda.synchronize()
    ctx.poll_error()
    ref_cache, over = oracle.compact_kv(k_all.f32[:, :, :L], v_all.f32[:, :, :L], fl, want_ro)
    assert over == 0 and np.array_equal(cache.len.cpu().numpy(), ref_cache.len)
    gk, gi = host_f32(cache.k), cache.idx.cpu().numpy()
    for u in range(U):
        a, n = int(want_ro[u]), int(ref_cache.len[u])
        assert np.array_equal(gk[a:a + n], ref_cache.k[a:a + n]) and np.array_equal(gi[a:a + n], ref_cache.idx[a:a + n])
    # windowed prefill over the packed cache
    out = torch.empty_like(qp)
    ag.ag_prefill_attn_recent(ctx, qp, kp, vp, flags, scale, cache, n_recent, out)
    torch.cuda.synchronize()
    ctx.poll_error()
    want = oracle.prefill_attn(q_all.f32[:, :, :L], k_all.f32[:, :, :L], v_all.f32[:, :, :L], fl, scale, n_recent=n_recent)
    got = host_f32(out)
    assert np.isfinite(got).all() and attn_error(dtype, got, want) <= attn_tolerance(dtype, want)
    # decode with the ring
    ring = None            # a window of one token is the plain decode: the ring holds the tokens BEFORE the current one
    if n_recent > 1:
        ring = ag.RecentRing(torch.zeros(U, n_recent, D, dtype=tdt, device=DEV), torch.zeros(U, n_recent, D, dtype=tdt, device=DEV),
                             torch.zeros(U, n_recent, dtype=torch.uint8, device=DEV),
                             torch.zeros(U, n_recent, dtype=torch.int32, device=DEV), n_recent)
        ag.ag_recent_fill(ctx, kp, vp, flags, 0, ring)
    o1 = torch.empty(B, Hq, D, dtype=tdt, device=DEV)
    dfn = dev(f_new)
    for s_ in range(steps):
        p = L + s_
        args = (dq[:, :, p].contiguous(), dk[:, :, p].contiguous(), dv[:, :, p].contiguous(), dfn[:, :, s_].contiguous(), p, scale, cache)
        if ring is None:
            ag.ag_decode_attn(ctx, *args, o1)
        else:
            ag.ag_decode_attn_recent(ctx, *args, ring, o1)
        want1 = oracle.prefill_rows(q_all.f32[:, :, :p + 1], k_all.f32[:, :, :p + 1], v_all.f32[:, :, :p + 1],
                                    f_all[:, :, :p + 1], scale, np.array([p]), n_recent=n_recent)[:, :, 0]
        got1 = host_f32(o1)
        assert np.isfinite(got1).all() and attn_error(dtype, got1, want1) <= attn_tolerance(dtype, want1), "step %d" % s_
        _, dropped = oracle.decode_step(q_all.f32[:, :, p], k_all.f32[:, :, p], v_all.f32[:, :, p], f_new[:, :, s_], p, ref_cache, scale)
        assert dropped == 0 and np.array_equal(cache.len.cpu().numpy(), ref_cache.len)
    ctx.poll_error()
    gk, gi = host_f32(cache.k), cache.idx.cpu().numpy()
    for u in range(U):
        a, n = int(want_ro[u]), int(ref_cache.len[u])
        assert np.array_equal(gk[a:a + n], ref_cache.k[a:a + n]) and np.array_equal(gi[a:a + n], ref_cache.idx[a:a + n])
    ctx.close()


# ------------------------------------------------------------------------- the 64-queries-per-wave variant (experiment)
_Q64_CHILD = r"""
import math, sys
import numpy as np
sys.path.insert(0, %(tests)r); sys.path.insert(0, %(root)r)
import oracle, workloads as W
from test_parity_configs_gpu import _prefill_case, check_sampled_rows, sample_rows
from gpu_util import ensure_built, host_f32
ensure_built()
for name, B, Hq, Hkv, L in (("split, balanced order", 1, 16, 16, 2048), ("GQA, four heads per workgroup", 1, 8, 2, 1500),
                            ("two heads per workgroup, ragged", 2, 4, 2, 333), ("few heads, 4 chunks", 1, 3, 3, 4096),
                            ("many heads, head-major order", 4, 32, 32, 512)):
    g = np.random.default_rng(170)
    flags = (g.random((B, Hkv, L)) < np.linspace(1.0, 0.05, Hkv)[None, :, None]).astype(np.uint8)
    flags[:, 0] = 1
    flags[:, -1] = 0
    q, k, v, out = _prefill_case(B, Hq, Hkv, L, flags, 171)
    got = host_f32(out)
    if L <= 1500:
        ref = oracle.prefill_attn(q.f32, k.f32, v.f32, flags, 1.0 / math.sqrt(128))
        check_sampled_rows(got, q, k, v, flags, 1.0 / math.sqrt(128), np.arange(L, dtype=np.int32), name)
    else:
        check_sampled_rows(got, q, k, v, flags, 1.0 / math.sqrt(128), sample_rows(L, 172, 6), name)
    G = Hq // Hkv
    assert np.array_equal(got[:, -G:], np.repeat(v.f32[:, -1:], G, axis=1))      # fully evicted head: out == v
print("q64 ok")
"""


def test_prefill_64_queries_per_wave_variant_matches_the_oracle():
    """The experimental prefill kernel with 64 queries per wave (environment AG_PREFILL_Q64=1, read once per process,
    hence the child process): same plan, split and merge as the 4-wave kernel, checked against the oracle on launch
    shapes that cover one, two and four query heads per workgroup, the key-chunk split and the head-major order."""
    import os
    import subprocess
    import sys
    here = os.path.dirname(os.path.abspath(__file__))
    env = dict(os.environ, AG_PREFILL_Q64="1")
    r = subprocess.run([sys.executable, "-c", _Q64_CHILD % {"tests": here, "root": os.path.dirname(here)}], env=env,
                       capture_output=True, text=True, timeout=280)
    print(r.stdout[-1500:])
    assert r.returncode == 0 and "q64 ok" in r.stdout, r.stderr[-3000:]
