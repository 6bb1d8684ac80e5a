"""Edge cases of the masked attention that only show with hostile values: NaN planted in rows a query must not see.

Eq. 5 excludes a masked key exactly (its term is absent, not multiplied by a small weight), so whatever an evicted
token's K/V rows hold, every query that does not see that token must come out unchanged.  With the recent-token
window (Table 6 of the appendix) an evicted token IS seen by the next n_recent - 1 queries and by itself; those
rows legitimately turn non-finite, all others must equal the clean run bit for bit and match the oracle, which
decides visibility with an `if` and therefore never touches the planted values for them."""
import math

import numpy as np
import pytest
import torch

import oracle
import paper_2410_12876_amd as ag
import workloads as W
from gpu_util import DEV, attn_error, attn_tolerance, dev, ensure_built, host_f32, make_ctx, new_cache

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _lib():
    ensure_built()


def _run(q, k, v, flags, scale, n_recent, dtype, with_cache):
    B, Hq, L, D = q.f32.shape
    Hkv = k.f32.shape[1]
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    ctx = make_ctx(B, L, Hq, Hkv, D, ag.AG_BF16 if dtype == "bf16" else ag.AG_F32)
    dq, dk, dv, df = dev(q), dev(k), dev(v), dev(flags)
    out = torch.empty_like(dq)
    cache = None
    if with_cache:      # slack rows of the cache are NaN as well: nothing past a unit's length may be read
        cache = new_cache(B, Hkv, D, tdt, oracle.slab_row_off(B * Hkv, L + 3), fill=float("nan"))
        ag.ag_compact_kv(ctx, dk, dv, df, 0, cache)
    ag.ag_prefill_attn_recent(ctx, dq, dk, dv, df, scale, cache, n_recent, out)
    torch.cuda.synchronize()
    ctx.poll_error()
    ctx.close()
    return host_f32(out)


@pytest.mark.parametrize("dtype,Hq,Hkv,L,D,n_recent,with_cache", [
    ("bf16", 2, 2, 600, 128, 5, True),       # tuned D = 128 kernel, band tiles
    ("bf16", 2, 2, 600, 128, 64, True),      # widest window: three band tiles per workgroup
    ("bf16", 8, 2, 333, 128, 10, False),     # GQA, 32 queries per workgroup, internal compaction
    ("bf16", 2, 2, 300, 64, 5, True),        # generic MFMA kernel
    ("bf16", 2, 2, 300, 64, 64, True),
    ("f32", 2, 2, 150, 64, 5, True),         # plain-ALU kernel
    ("bf16", 2, 2, 600, 128, 1, True),       # no window: the evicted rows are never read by others
])
def test_poisoned_evicted_rows_reach_only_the_queries_that_see_them(dtype, Hq, Hkv, L, D, n_recent, with_cache):
    B = 1
    g = np.random.default_rng(200 + L + n_recent + D)
    q, k, v = (W.store(g.standard_normal(s).astype(np.float32), dtype)
               for s in ((B, Hq, L, D), (B, Hkv, L, D), (B, Hkv, L, D)))
    flags = (g.random((B, Hkv, L)) < 0.5).astype(np.uint8)
    scale = 1.0 / math.sqrt(D)
    # poison a sparse subset of the evicted tokens, so that most queries see none of them even with a wide window:
    # isolated tokens, one run of three in a row, and one just before a 64- and a 128-token tile edge
    poison = np.zeros((B, Hkv, L), dtype=bool)
    poison[:, :, 40::97] = True
    poison[:, :, 210:213] = True
    poison[:, :, [62, 63, 127, 128, L - 1]] = True
    poison &= flags == 0
    assert poison.sum() >= 6
    kp, vp = k.f32.copy(), v.f32.copy()
    kp[poison] = np.nan
    vp[poison] = np.nan
    clean = _run(q, k, v, flags, scale, n_recent, dtype, with_cache)
    got = _run(q, W.store(kp, dtype), W.store(vp, dtype), flags, scale, n_recent, dtype, with_cache)
    ref = oracle.prefill_attn(q.f32, kp, vp, flags, scale, n_recent=n_recent)
    G = Hq // Hkv
    # rows the definition leaves finite: those that see no poisoned token (computed here from the mask definition:
    # a poisoned token t is seen by itself and by queries j with 0 < j - t < n_recent)
    sees = np.zeros((B, Hkv, L), dtype=bool)
    for t in zip(*np.nonzero(poison)):
        b, h, pos = t
        sees[b, h, pos:min(L, pos + n_recent)] = True
    sees_q = np.repeat(sees, G, axis=1)
    assert np.array_equal(np.isfinite(ref).all(axis=-1), ~sees_q)          # the oracle agrees with that reading
    ok = ~sees_q
    assert ok.sum() > 0.3 * ok.size
    assert np.isfinite(got[ok]).all(), "%d clean rows came out non-finite" % int((~np.isfinite(got[ok]).all(axis=-1)).sum())
    assert np.array_equal(got[ok], clean[ok])                                # untouched by the planted values
    assert attn_error(dtype, got[ok], ref[ok]) <= attn_tolerance(dtype)
    # and the rows that do see a poisoned token show it instead of hiding it
    assert (~np.isfinite(got[sees_q])).any(axis=-1).all()


@pytest.mark.parametrize("dtype,Hq,Hkv,L,D,n_recent", [("bf16", 2, 2, 700, 128, 1), ("bf16", 8, 2, 300, 128, 1),
                                                       ("bf16", 2, 2, 300, 64, 1), ("f32", 2, 2, 250, 64, 1),
                                                       ("bf16", 2, 2, 500, 128, 5)])
def test_prefill_after_a_cache_overflow_attends_only_the_rows_that_fit(dtype, Hq, Hkv, L, D, n_recent):
    """A caller-sized cache that is too small: the kept rows beyond a unit's capacity are dropped (Sec. 3.3's cache
    simply does not hold them) and AG_ECAPACITY is reported.  The attention of the same call must then treat exactly
    those tokens as evicted -- visible to themselves only -- which is the oracle on flags with the dropped tokens'
    bits cleared; in particular the zero rows that pad the last key tile are never attended."""
    B, cap = 1, 100
    g = np.random.default_rng(300 + L + D)
    q, k, v = (W.store(g.standard_normal(s).astype(np.float32), dtype)
               for s in ((B, Hq, L, D), (B, Hkv, L, D), (B, Hkv, L, D)))
    flags = (g.random((B, Hkv, L)) < 0.6).astype(np.uint8)
    flags[0, 0, 120:] = 0            # unit 0 stays below its capacity, unit 1 overflows
    kept_before = np.cumsum(flags, axis=-1) - flags
    fits = flags & (kept_before < cap)
    assert fits[0, 0].sum() == flags[0, 0].sum() < cap and flags[0, 1].sum() > cap == fits[0, 1].sum()
    scale = 1.0 / math.sqrt(D)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    ctx = make_ctx(B, L, Hq, Hkv, D, ag.AG_BF16 if dtype == "bf16" else ag.AG_F32)
    dq, dk, dv, df = dev(q), dev(k), dev(v), dev(flags)
    out = torch.empty_like(dq)
    ro = oracle.slab_row_off(B * Hkv, cap)
    cache = new_cache(B, Hkv, D, tdt, ro, fill=float("nan"))
    ag.ag_compact_prefill_attn(ctx, dq, dk, dv, df, scale, 0, cache, out, n_recent=n_recent)
    torch.cuda.synchronize()
    with pytest.raises(ag.AgError) as e:
        ctx.poll_error()
    assert e.value.status == ag.AG_ECAPACITY
    ctx.close()
    rc, over = oracle.compact_kv(k.f32, v.f32, flags, ro)
    assert over > 0 and int(rc.len.sum()) == int(fits.sum()) < int(flags.sum())
    assert np.array_equal(np.minimum(cache.len.cpu().numpy(), cap), rc.len)
    got = host_f32(out)
    ref = oracle.prefill_attn(q.f32, k.f32, v.f32, fits, scale, n_recent=n_recent)
    assert np.isfinite(got).all()
    assert attn_error(dtype, got, ref) <= attn_tolerance(dtype)


# --------------------------------------------------------------------------------------------- packed cache layout
def test_packed_cache_layout_prefill_equals_slabs_and_decode_fills_the_spare_rows():
    """ag_pack_row_off (Sec. 3.3: only the retained rows take cache memory) on a cfg2-like layer: offsets and the
    needed-rows word against the oracle's plain loop, every unit's capacity = its kept rows + room, the compaction
    into the packed cache against the oracle's, the prefill over the packed cache bit-identical to the prefill over
    full-length slabs, then `room` decode steps that use up the spare rows exactly and one more that is dropped."""
    B, H, L, D, room = 1, 16, 2048, 128, 3
    g = np.random.default_rng(400)
    q, k, v = (W.store(g.standard_normal((B, H, L, D)).astype(np.float32), "bf16") for _ in range(3))
    flags = (g.random((B, H, L)) < np.linspace(0.9, 0.05, H)[None, :, None]).astype(np.uint8)
    flags[0, 5] = 0                    # a fully evicted unit: capacity = room
    scale = 1.0 / math.sqrt(D)
    want_ro, need = oracle.packed_row_off(flags, room, 10 ** 9)
    total = int(need)
    assert total < B * H * (L + room) * 0.6          # the layout is much smaller than slabs
    ctx = make_ctx(B, L, H, H, D, ag.AG_BF16, cache_rows=total)
    dq, dk, dv, df = dev(q), dev(k), dev(v), dev(flags)
    row_off = torch.full((B * H + 1,), -1, dtype=torch.int64, device=DEV)
    needed = torch.zeros(1, dtype=torch.int64, device=DEV)
    ag.ag_pack_row_off(ctx, df, room, total, row_off, needed)
    torch.cuda.synchronize()
    assert np.array_equal(row_off.cpu().numpy(), want_ro) and int(needed.item()) == need
    packed = ag.KVCache(torch.full((total, D), float("nan"), dtype=torch.bfloat16, device=DEV),
                        torch.full((total, D), float("nan"), dtype=torch.bfloat16, device=DEV),
                        torch.full((total,), -1, dtype=torch.int32, device=DEV), row_off,
                        torch.zeros(B * H, dtype=torch.int32, device=DEV), B, H, D, total_rows=total)
    out_p = torch.empty_like(dq)
    ag.ag_compact_prefill_attn(ctx, dq, dk, dv, df, scale, 0, packed, out_p)
    torch.cuda.synchronize()
    ctx.poll_error()
    rc, over = oracle.compact_kv(k.storage, v.storage, flags, want_ro)
    assert over == 0
    lens = packed.len.cpu().numpy()
    assert np.array_equal(lens, rc.len) and np.array_equal(np.diff(want_ro), lens + room)
    from gpu_util import host_bits
    gk, gv, gi = host_bits(packed.k), host_bits(packed.v), packed.idx.cpu().numpy()
    for u in range(B * H):
        a, n = int(want_ro[u]), int(rc.len[u])
        assert np.array_equal(gk[a:a + n], rc.k[a:a + n]) and np.array_equal(gv[a:a + n], rc.v[a:a + n])
        assert np.array_equal(gi[a:a + n], rc.idx[a:a + n])
    # the same attention over full-length slabs
    slabs = new_cache(B, H, D, torch.bfloat16, oracle.slab_row_off(B * H, L))
    out_s = torch.empty_like(dq)
    ag.ag_compact_prefill_attn(ctx, dq, dk, dv, df, scale, 0, slabs, out_s)
    torch.cuda.synchronize()
    assert torch.equal(out_p, out_s)
    # decoding into the spare rows
    ref = oracle.Cache(W.bf16_bits_to_f32(rc.k), W.bf16_bits_to_f32(rc.v), rc.idx.copy(), want_ro.copy(), rc.len.copy())
    o = torch.empty(B, H, D, dtype=torch.bfloat16, device=DEV)
    for s in range(room + 1):
        qs, kn, vn = (W.store(g.standard_normal((B, H, D)).astype(np.float32), "bf16") for _ in range(3))
        ag.ag_decode_attn(ctx, dev(qs), dev(kn), dev(vn), None, L + s, scale, packed, o)
        want, dropped = oracle.decode_step(qs.f32, kn.f32, vn.f32, None, L + s, ref, scale)
        got = host_f32(o)
        assert np.isfinite(got).all() and attn_error("bf16", got, want) <= attn_tolerance("bf16")
        assert np.array_equal(packed.len.cpu().numpy(), ref.len)
        assert dropped == (B * H if s == room else 0)
    with pytest.raises(ag.AgError) as e:
        ctx.poll_error()
    assert e.value.status == ag.AG_ECAPACITY
    assert np.array_equal(packed.len.cpu().numpy(), rc.len + room)
    ctx.close()


def test_packed_cache_layout_cut_off_at_the_allocation():
    """An allocation smaller than the layout needs: the offsets stop at total_rows, the units past the end get no
    rows, the compaction drops theirs (AG_ECAPACITY) exactly as the oracle's does with the same offsets, and the
    needed-rows word tells the caller what would have been enough."""
    B, H, L, D = 2, 4, 300, 64
    g = np.random.default_rng(401)
    k, v = (W.store(g.standard_normal((B, H, L, D)).astype(np.float32), "f32") for _ in range(2))
    flags = (g.random((B, H, L)) < 0.5).astype(np.uint8)
    want_all, need = oracle.packed_row_off(flags, 4, 10 ** 9)
    total = int(want_all[5]) + 7            # ends 7 rows into unit 5
    want_ro, _ = oracle.packed_row_off(flags, 4, total)
    ctx = make_ctx(B, L, H, H, D, ag.AG_F32, cache_rows=total)
    row_off = torch.zeros(B * H + 1, dtype=torch.int64, device=DEV)
    needed = torch.zeros(1, dtype=torch.int64, device=DEV)
    ag.ag_pack_row_off(ctx, dev(flags), 4, total, row_off, needed)
    cache = ag.KVCache(torch.zeros(total, D, device=DEV), torch.zeros(total, D, device=DEV),
                       torch.full((total,), -1, dtype=torch.int32, device=DEV), row_off,
                       torch.zeros(B * H, dtype=torch.int32, device=DEV), B, H, D, total_rows=total)
    ag.ag_compact_kv(ctx, dev(k), dev(v), dev(flags), 0, cache)
    torch.cuda.synchronize()
    assert np.array_equal(row_off.cpu().numpy(), want_ro) and int(needed.item()) == need > total
    with pytest.raises(ag.AgError) as e:
        ctx.poll_error()
    assert e.value.status == ag.AG_ECAPACITY
    rc, over = oracle.compact_kv(k.f32, v.f32, flags, want_ro)
    assert over == 3 and np.array_equal(cache.len.cpu().numpy(), rc.len) and rc.len[5] == 7 and (rc.len[6:] == 0).all()
    assert np.array_equal(cache.k.cpu().numpy()[:total], rc.k[:total])
    ctx.close()
