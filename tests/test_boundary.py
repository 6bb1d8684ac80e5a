"""The C-ABI boundary without a GPU: the library loads, exports what include/ag.h declares, and every
host-detectable error path answers with the documented status (context made with device = -1)."""
import os
import re

import pytest
import torch

import paper_2410_12876_amd as ag

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(ag.LIB_PATH):
        from paper_2410_12876_amd import build
        build.build()
    return ag.load()


def declared_functions():
    """every function declared in include/*.h (ag.h: the method's boundary; ag_bench.h: benchmark instrumentation)"""
    import glob
    names = set()
    for path in sorted(glob.glob(os.path.join(ROOT, "include", "*.h"))):
        text = re.sub(r"/\*.*?\*/", "", open(path).read(), flags=re.S)
        names |= set(re.findall(r"\b(ag_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


def test_the_method_header_declares_no_instrumentation():
    text = open(os.path.join(ROOT, "include", "ag.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    assert not re.search(r"ag_(timing|probe)_", text)


def test_library_exports_every_declared_symbol(lib):
    names = declared_functions()
    assert set(names) == set(ag.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_workspace_bytes_covers_configs(lib):
    w2 = ag.workspace_bytes(1, 4096, 32, 32, 128, ag.AG_BF16, 4096, 4096 * 32)
    assert w2 > 2 * 32 * 4096 * 128 * 2          # room for an internal compaction of K and V
    assert ag.workspace_bytes(0, 4096, 32, 32, 128, ag.AG_BF16, 4096, 0) == 0
    assert ag.workspace_bytes(1, 4096, 32, 5, 128, ag.AG_BF16, 4096, 0) == 0     # Hq % Hkv != 0


def make_cache(B=1, Hkv=2, D=64, rows=40, dtype=torch.float32):
    k = torch.zeros(rows, D, dtype=dtype)
    return ag.KVCache(k, k.clone(), torch.zeros(rows, dtype=torch.int32), torch.zeros(B * Hkv + 1, dtype=torch.int64),
                      torch.zeros(B * Hkv, dtype=torch.int32), B, Hkv, D)


def expect(status, fn, *a, **kw):
    with pytest.raises(ag.AgError) as e:
        fn(*a, **kw)
    assert e.value.status == status, str(e.value)


def test_error_paths_without_device(lib):
    ctx = ag.Context(device=-1, workspace=1 << 20)
    x = torch.zeros(1, 8, 64)
    w = torch.zeros(64, 4)
    bias = torch.zeros(4)
    flags = torch.zeros(1, 4, 8, dtype=torch.uint8)
    # a well-formed call passes validation and then reports that the context has no device
    expect(ag.AG_EHIP, ag.ag_gate, ctx, x, w, bias, 0.5, 0, None, flags, stream=0)
    expect(ag.AG_EINVAL, ag.ag_gate, ctx, x, w, bias, 1.0, 0, None, flags, stream=0)          # tau outside (0,1)
    expect(ag.AG_EINVAL, ag.ag_gate, ctx, x, w, bias, 0.5, -1, None, flags, stream=0)         # n_sink < 0
    expect(ag.AG_EINVAL, ag.ag_gate, ctx, x, w, None, 0.5, 0, None, flags, stream=0)          # null bias
    expect(ag.AG_EUNSUPPORTED, ag.ag_gate, ctx, x, torch.zeros(64, 33), torch.zeros(33), 0.5, 0, None, flags, stream=0)
    xb = torch.zeros(1, 8, 48, dtype=torch.bfloat16)
    expect(ag.AG_EUNSUPPORTED, ag.ag_gate, ctx, xb, torch.zeros(48, 4, dtype=torch.bfloat16), bias, 0.5, 0, None,
           flags, stream=0)                                                                      # bf16 d_in % 64

    hb, gb, wb = xb.new_zeros(1, 8, 64), xb.new_zeros(64), xb.new_zeros(64, 4)
    expect(ag.AG_EHIP, ag.ag_rmsnorm_gate, ctx, hb, gb, 1e-5, wb, bias, 0.5, 0, hb.clone(), None, flags, stream=0)
    expect(ag.AG_EINVAL, ag.ag_rmsnorm_gate, ctx, hb, gb, 0.0, wb, bias, 0.5, 0, hb.clone(), None, flags, stream=0)   # eps
    expect(ag.AG_EINVAL, ag.ag_rmsnorm_gate, ctx, hb, None, 1e-5, wb, bias, 0.5, 0, hb.clone(), None, flags, stream=0)
    expect(ag.AG_EUNSUPPORTED, ag.ag_rmsnorm_gate, ctx, x, w[:, 0].contiguous(), 1e-5, w, bias, 0.5, 0, x.clone(), None,
           flags, stream=0)                                                                      # fp32 is not built
    big = xb.new_zeros(1, 8, 8256)
    expect(ag.AG_EUNSUPPORTED, ag.ag_rmsnorm_gate, ctx, big, xb.new_zeros(8256), 1e-5, xb.new_zeros(8256, 4), bias, 0.5,
           0, big.clone(), None, flags, stream=0)                                                # d_in > 8192

    q = torch.zeros(1, 4, 8, 64)
    k = torch.zeros(1, 2, 8, 64)
    f2 = torch.zeros(1, 2, 8, dtype=torch.uint8)
    cache = make_cache()
    expect(ag.AG_EHIP, ag.ag_compact_kv, ctx, k, k, f2, 0, cache, stream=0)
    expect(ag.AG_EINVAL, ag.ag_compact_kv, ctx, k, None, f2, 0, cache, stream=0)
    ro = torch.zeros(3, dtype=torch.int64)
    expect(ag.AG_EHIP, ag.ag_pack_row_off, ctx, f2, 4, 100, ro, None, stream=0)
    expect(ag.AG_EINVAL, ag.ag_pack_row_off, ctx, f2, -1, 100, ro, None, stream=0)            # negative room
    expect(ag.AG_EINVAL, ag.ag_pack_row_off, ctx, f2, 4, 100, None, None, stream=0)           # null row_off
    expect(ag.AG_EHIP, ag.ag_prefill_attn, ctx, q, k, k, f2, 0.125, cache, q.clone(), stream=0)
    expect(ag.AG_EHIP, ag.ag_prefill_attn, ctx, q, k, k, f2, 0.125, None, q.clone(), stream=0)
    expect(ag.AG_EINVAL, ag.ag_prefill_attn, ctx, q, k, k, f2, 0.0, cache, q.clone(), stream=0)  # scale
    q3 = torch.zeros(1, 3, 8, 64)
    expect(ag.AG_EINVAL, ag.ag_prefill_attn, ctx, q3, k, k, f2, 0.125, cache, q3.clone(), stream=0)   # Hq % Hkv
    q48 = torch.zeros(1, 2, 8, 48)
    k48 = torch.zeros(1, 2, 8, 48)
    expect(ag.AG_EUNSUPPORTED, ag.ag_prefill_attn, ctx, q48, k48, k48, f2, 0.125, None, q48.clone(), stream=0)
    expect(ag.AG_EINVAL, ag.ag_prefill_attn, ctx, q, k, k, f2, 0.125, make_cache(D=128), q.clone(), stream=0)

    qd = torch.zeros(1, 4, 64)
    kn = torch.zeros(1, 2, 64)
    expect(ag.AG_EHIP, ag.ag_decode_attn, ctx, qd, kn, kn, None, 8, 0.125, cache, qd.clone(), stream=0)
    expect(ag.AG_EINVAL, ag.ag_decode_attn, ctx, torch.zeros(1, 3, 64), kn, kn, None, 8, 0.125, cache, qd.clone(), stream=0)
    expect(ag.AG_EINVAL, ag.ag_decode_attn, ctx, qd, kn, kn, None, 8, -1.0, cache, qd.clone(), stream=0)
    # the entry point that allocates nothing: same validation, and a cache beyond its static array is refused
    expect(ag.AG_EHIP, ag.ag_decode_attn_static, ctx, qd, kn, kn, None, 8, 0.125, cache, qd.clone(), stream=0)
    expect(ag.AG_EINVAL, ag.ag_decode_attn_static, ctx, qd, kn, None, None, 8, 0.125, cache, qd.clone(), stream=0)
    huge = make_cache()
    huge.c.total_rows = 1 << 24
    assert ag.decode_scratch_bytes(huge, 4) > ag.decode_static_scratch_bytes() == 16 << 20
    expect(ag.AG_EWORKSPACE, ag.ag_decode_attn_static, ctx, qd, kn, kn, None, 8, 0.125, huge, qd.clone(), stream=0)
    ctx.close()


def test_workspace_too_small_is_reported(lib):
    ctx = ag.Context(device=-1, workspace=1024)
    q = torch.zeros(1, 4, 256, 64)
    k = torch.zeros(1, 4, 256, 64)
    f = torch.zeros(1, 4, 256, dtype=torch.uint8)
    expect(ag.AG_EWORKSPACE, ag.ag_prefill_attn, ctx, q, k, k, f, 0.125, None, q.clone(), stream=0)
    x = torch.zeros(1, 4096, 64)
    expect(ag.AG_EWORKSPACE, ag.ag_gate, ctx, x, torch.zeros(64, 4), torch.zeros(4), 0.5, 0, None,
           torch.zeros(1, 4, 4096, dtype=torch.uint8), stream=0)
    ctx.close()


def test_missing_library_fails_loudly(monkeypatch, lib):
    monkeypatch.setattr(ag, "_lib", None)
    monkeypatch.setattr(ag, "LIB_PATH", "/nonexistent/libag.so")
    with pytest.raises(ImportError):
        ag.load()


def test_gate_presets_match_the_header():
    """(tau, gamma) of the two experiments (Sec. 4.1 training details, Sec. 4.2 implementation details)."""
    text = open(os.path.join(ROOT, "include", "ag.h")).read()
    val = {m.group(1): float(m.group(2)) for m in re.finditer(r"#define (AG_(?:TAU|GAMMA)_[A-Z]+) ([0-9.]+)f", text)}
    assert (val["AG_TAU_PRETRAIN"], val["AG_GAMMA_PRETRAIN"]) == ag.PRESET_PRETRAIN == (0.5, 2.0)
    assert (val["AG_TAU_FINETUNE"], val["AG_GAMMA_FINETUNE"]) == ag.PRESET_FINETUNE == (0.3, 0.0)


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU; --gpus N > 1 exits with a message instead of running."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_header_is_plain_c_and_the_library_links_from_c(lib, tmp_path):
    """include/ag.h compiled as C99 by gcc, linked against libag.so, run without a GPU."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    exe = str(tmp_path / "abi_from_c")
    libdir = os.path.dirname(ag.LIB_PATH)
    cmd = ["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
           os.path.join(ROOT, "tests", "abi_from_c.c"), "-o", exe, "-L", libdir, "-l:libag.so", "-Wl,-rpath," + libdir,
           "-Wl,-rpath,/opt/rocm/lib"]
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stderr
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0 and r.stdout.strip().endswith("ok"), r.stdout + r.stderr
