"""ag_decode_attn_static, the decode entry point that allocates nothing (its scratch is a static device array of
the library), against ag_decode_attn on the same inputs: same kernels, so outputs, lengths, positions and appended
rows must agree bit for bit.  Two calls in a row share the array; the second is the smaller problem, so whatever
the first left behind lies beyond what the second writes."""
import numpy as np
import pytest
import torch

import paper_2410_12876_amd as ag
import workloads as W
from gpu_util import DEV, cache_from_host, dev, ensure_built, host_bits, make_ctx

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _lib():
    ensure_built()


def run_steps(fn, ctx, wl, steps):
    """`steps` decode steps of workload wl through entry point fn; returns per-step output bits and the final cache."""
    cache = cache_from_host(wl.B, wl.Hkv, wl.D, wl.k_cache, wl.v_cache, wl.idx, wl.row_off, wl.len0)
    out = torch.empty(wl.B, wl.Hq, wl.D, dtype=torch.bfloat16 if wl.dtype == "bf16" else torch.float32, device=DEV)
    outs = []
    for s in range(steps):
        q, kn, vn, nf = wl.step_inputs(s, 0.5)
        fn(ctx, dev(q), dev(kn), dev(vn), dev(nf), wl.pos0 + s, wl.scale, cache, out)
        outs.append(host_bits(out).copy())
    ctx.poll_error()
    return outs, cache


def test_static_scratch_decode_equals_workspace_decode_on_two_calls_in_a_row():
    g = np.random.default_rng(7)
    big_len = np.rint(3000 * (0.1 + 0.9 * g.random(4 * 8))).astype(np.int32)
    big_len[3] = 0
    big_len[5] = 1
    small_len = np.rint(400 * (0.1 + 0.9 * g.random(2 * 2))).astype(np.int32)
    big = W.decode_batch(41, "static_big", "bf16", 4, 8, 8, 128, big_len, 3, pos0=3000)
    small = W.decode_batch(42, "static_small", "bf16", 2, 8, 2, 128, small_len, 2, pos0=400)   # GQA, fewer items
    bare = ag.Context(0, 0)          # no workspace at all: the static entry point must not need one
    assert ag.decode_static_scratch_bytes() == 16 << 20
    for wl, steps in ((big, 3), (small, 2)):
        print("static decode: %s, %d units, %d rows" % (wl.name, wl.B * wl.Hkv, int(wl.row_off[-1])), flush=True)
        ref_ctx = make_ctx(wl.B, 1, wl.Hq, wl.Hkv, wl.D, ag.AG_BF16, cache_rows=int(wl.row_off[-1]))
        want, want_cache = run_steps(ag.ag_decode_attn, ref_ctx, wl, steps)
        got, got_cache = run_steps(ag.ag_decode_attn_static, bare, wl, steps)
        assert 0 < ag.decode_scratch_bytes(got_cache, wl.Hq) <= ag.decode_static_scratch_bytes()
        for s in range(steps):
            assert np.array_equal(got[s], want[s]), "step %d of %s differs" % (s, wl.name)
        assert np.array_equal(got_cache.len.cpu().numpy(), want_cache.len.cpu().numpy())
        assert np.array_equal(got_cache.idx.cpu().numpy(), want_cache.idx.cpu().numpy())
        assert np.array_equal(host_bits(got_cache.k), host_bits(want_cache.k))
        assert np.array_equal(host_bits(got_cache.v), host_bits(want_cache.v))
        ref_ctx.close()
    bare.close()


def test_static_scratch_decode_rejects_a_cache_beyond_its_array():
    """A cache whose records would not fit the 16 MiB array is refused with AG_EWORKSPACE before anything is
    launched (the tensors behind the oversized row count are never touched)."""
    B, H, D = 1, 2, 128
    rows = 8 << 20            # 64 Ki items of 130 floats each: 34 MB of records
    k = torch.zeros(16, D, dtype=torch.bfloat16, device=DEV)
    cache = ag.KVCache(k, k.clone(), torch.zeros(16, dtype=torch.int32, device=DEV),
                       torch.zeros(B * H + 1, dtype=torch.int64, device=DEV),
                       torch.zeros(B * H, dtype=torch.int32, device=DEV), B, H, D, total_rows=rows)
    ctx = ag.Context(0, 0)
    assert ag.decode_scratch_bytes(cache, H) > ag.decode_static_scratch_bytes()
    q = torch.zeros(B, H, D, dtype=torch.bfloat16, device=DEV)
    with pytest.raises(ag.AgError) as e:
        ag.ag_decode_attn_static(ctx, q, q, q, None, 5, 0.1, cache, q.clone())
    assert e.value.status == ag.AG_EWORKSPACE and "static" in str(e.value)
    ctx.close()
