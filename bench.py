#!/usr/bin/env python3
"""Benchmark of the Attention-Gate hot path on one MI355X.

One "step" is one pass of the whole path over one Llama2-7B-shaped layer (config 2: bf16, B=1, L=4096,
d=4096, 32 heads x 128, per-head keep ratios U[0.2, 0.9]):
    ag_gate -> ag_compact_prefill_attn (= ag_compact_kv + ag_prefill_attn over the compacted cache, sharing one
    launch for the flag scan and the copy) -> one ag_decode_attn step.
`value` is prompt tokens per second through that step, inputs resident in HBM.  The same JSON line carries
  roofline      : the dominant kernel (masked prefill attention) against the bf16 MFMA peak,
  decode        : config 3 (B=32, ragged caches ~ round(4096 U[0.1,1]), Bernoulli(0.5) appends), 256 decode
                  steps, achieved HBM GB/s of the decode kernel against the 8 TB/s peak,
  cpu_baseline  : the CPU oracle timed on a bounded sample of the same workload on the host cores.
The step is timed over --steps launches without instrumentation (eager by default, --graph replays a checked HIP
graph).  Kernel durations for the roofline come from HIP event pairs that the library records around every
kernel on the launch stream (ag_timing_* of the C ABI) over the same number of steps right after.
  machine       : what this machine sustains (MFMA loop, streaming copy, vendor bf16 GEMM) beside the data-sheet peaks.
Optional legs: --config 4 / --config 5 --layer l (the other layer workloads), --keep, --seq-len, --config5-stack
(config 5 end to end: the prompt, then 256 decode steps, through all 32 layers), --project (the K/V projection
with the compaction in its epilogue), --norm-gate (the gate fused with the normalisation of its input), --power (package power under the prefill kernel),
next_layer_gate_overlap (the next layer's gate on a second stream).
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np

MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16
HBM_PEAK_GBS = 8000.0            # MI355X HBM3E


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def to_dev(t, torch):
    if t.is_bf16:
        return torch.from_numpy(t.bits.view(np.int16)).view(torch.bfloat16).cuda()
    return torch.from_numpy(t.f32).cuda()


def visible_pairs(flags: np.ndarray, G: int) -> int:
    """sum over (b, query head, row j) of (cnt[j] + 1): visible query-key pairs incl. the diagonal."""
    f = flags.astype(np.int64)
    cnt = np.cumsum(f, axis=-1) - f          # exclusive prefix count
    return int((cnt + 1).sum()) * G


def make_workload(args, W):
    """--config 2 (default, the headline workload), 4 (Llama-3-8B GQA shape, L = 32768, flags given as runs) or
    5 (one layer of the 32-layer stack, B = 16, L = 2048; --layer picks it)."""
    if args.config == 4:
        return W.config4(with_x=True)
    if args.config == 5:
        return W.config5_layer(args.layer)
    return W.config2(L=args.seq_len, keep=None if args.keep is None else np.full(32, args.keep))


def prefill_leg(args, torch, ag, W):
    wl = make_workload(args, W)
    B, L, Hq, Hkv, D, d = wl.B, wl.L, wl.Hq, wl.Hkv, wl.D, wl.d_model
    G = Hq // Hkv
    U = B * Hkv
    cap = L + 8
    rows = U * cap
    ctx = ag.Context(0, ag.workspace_bytes(B, L, Hq, Hkv, D, ag.AG_BF16, d, rows))
    x, wg, bias = to_dev(wl.x, torch), to_dev(wl.w_gate, torch), torch.from_numpy(wl.bias).cuda()
    q, k, v = to_dev(wl.q, torch), to_dev(wl.k, torch), to_dev(wl.v, torch)
    flags = torch.empty(B, Hkv, L, dtype=torch.uint8, device="cuda")
    # config 4 gives its flags (run-structured); the gate still runs in the step, into a buffer of its own
    given = None if wl.flags is None else torch.from_numpy(wl.flags).cuda()
    pf_flags = flags if given is None else given
    out = torch.empty_like(q)
    ro = np.arange(U + 1, dtype=np.int64) * cap
    cache = ag.KVCache(torch.zeros(rows, D, dtype=torch.bfloat16, device="cuda"),
                       torch.zeros(rows, D, dtype=torch.bfloat16, device="cuda"),
                       torch.zeros(rows, dtype=torch.int32, device="cuda"), torch.from_numpy(ro).cuda(),
                       torch.zeros(U, dtype=torch.int32, device="cuda"), B, Hkv, D)
    dq = torch.randn(B, Hq, D, device="cuda").to(torch.bfloat16)
    dk = torch.randn(B, Hkv, D, device="cuda").to(torch.bfloat16)
    dv = torch.randn(B, Hkv, D, device="cuda").to(torch.bfloat16)
    dout = torch.empty_like(dq)

    def step():
        ag.ag_gate(ctx, x, wg, bias, wl.tau, wl.n_sink, None, flags)
        ag.ag_compact_prefill_attn(ctx, q, k, v, pf_flags, wl.scale, 0, cache, out)   # scan + compaction in one launch, then attention
        ag.ag_decode_attn(ctx, dq, dk, dv, None, L, wl.scale, cache, dout)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    graph = None
    if args.graph:
        # The whole step (4 library calls, ~10 kernels, no allocation, no host sync) is captured once in a HIP
        # graph and replayed.  Replays are checked against the eager result first.
        ref_out, ref_dout, ref_len = out.clone(), dout.clone(), cache.len.clone()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
        for r in range(3):
            out.zero_(); dout.zero_()
            graph.replay()
            torch.cuda.synchronize()
            if not (torch.equal(out, ref_out) and torch.equal(dout, ref_dout) and torch.equal(cache.len, ref_len)):
                raise RuntimeError("graph replay %d differs from the eager step" % r)
            step()      # eager work between replays
            torch.cuda.synchronize()
    run = graph.replay if graph is not None else step
    for _ in range(2):
        run()
    torch.cuda.synchronize()
    block_s = []
    for _ in range(max(1, args.repeats)):       # the timed block, repeated: spread of one block of --steps steps
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            run()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        block_s.append(t1 - t0)
    block_s.sort()
    t0, t1 = 0.0, block_s[len(block_s) // 2]    # the median block is the one reported
    # per-kernel durations: HIP event pairs around every kernel, same steps launched eagerly
    ctx.timing_enable(True)
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t3 = time.perf_counter()
    times = ctx.timing_read()
    ctx.timing_enable(False)
    ctx.poll_error()

    # what the parity bar sets aside: gate logits within 1e-3 of the threshold (their flags may legitimately differ from
    # a reference computed in another precision), counted on one untimed gate call that also writes the logits
    logits = torch.empty(B, L, Hkv, dtype=torch.float32, device="cuda")
    ag.ag_gate(ctx, x, wg, bias, wl.tau, wl.n_sink, logits, flags)
    thr = math.log(wl.tau / (1.0 - wl.tau))
    near = int(((logits - thr).abs() < 1e-3).sum().item())
    gate_keep = flags.float().mean(dim=(0, 2)).cpu().numpy()
    fl = pf_flags.cpu().numpy()
    pairs = visible_pairs(fl, G)
    flops = 4.0 * D * pairs
    kept_rows = int(fl.sum())
    per_kernel = {n: (ms / c if c else None) for n, (ms, c) in times.items()}
    pf_ms = per_kernel["prefill"]
    ach = flops / (pf_ms * 1e-3) / 1e12
    res = {
        "seconds": t1 - t0,
        "ms_per_step_spread": {"min": block_s[0] / args.steps * 1e3, "median": block_s[len(block_s) // 2] / args.steps * 1e3,
                               "max": block_s[-1] / args.steps * 1e3, "blocks": len(block_s)},
        "seconds_instrumented": t3 - t2,
        "tokens": B * L * args.steps,
        "kernel_ms": per_kernel,
        "keep_ratio": float(fl.mean()),
        "keep_ratio_per_head": [round(float(r), 4) for r in fl.mean(axis=(0, 2))],
        "gate": {"near_threshold_logits": near, "logits": int(logits.numel()), "band": 1e-3,
                 "keep_ratio_per_head": [round(float(r), 4) for r in gate_keep]},
        "roofline": {"kernel": "ag_prefill_bf16_kernel<128, %d, false, 4>" % min(4, G), "bound": "mfma", "achieved": ach,
                     "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": ach / MFMA_BF16_PEAK_TFLOPS,
                     "traffic": TRAFFIC_BYTES.get(("prefill", L)) if args.keep is None and args.config == 2 else None, "flops_per_launch": flops, "visible_pairs": pairs,
                     "avg_launch_ms": pf_ms},
        "compact_gbs": (2 * 2 * kept_rows * D * 2 + fl.size + 4 * kept_rows) / (per_kernel["compact"] * 1e-3) / 1e9,
        "gate_gbs": (B * L * d * 2) / (per_kernel["gate"] * 1e-3) / 1e9,
        "config": {"workload": wl.name, "B": B, "L": L, "d_model": d, "Hq": Hq, "Hkv": Hkv, "D": D,
                   "keep": ("given as runs" if args.config == 4 else "per layer and head" if args.config == 5 else
                            "per-head U[0.2,0.9]" if args.keep is None else "every head %.2f" % args.keep) +
                           ", mean %.3f" % fl.mean(),
                   "launch": "hip graph replay" if graph is not None else "eager"},
    }
    ctx.close()
    return res, wl, fl


def decode_leg(args, torch, ag, W):
    """Config 3: `--decode-steps` decode steps (256) over B = 32 x 32 ragged caches, Bernoulli(0.5) appends.
    Three passes from the same starting lengths: (1) eager launches, no instrumentation: wall clock; (2) the same
    steps captured once into ONE HIP graph (every step's position and inputs are baked into its nodes) and replayed:
    wall clock -- the graph's result is first checked against the eager pass bit for bit; (3) eager with the library's
    per-launch events: kernel durations.  The headline of the leg is the whole step (both kernels and the gaps
    between them) of the faster of (1) and (2); the streaming kernel alone is reported beside it."""
    steps, warm = args.decode_steps, min(args.warmup, 8)
    wl = W.config3(B=args.decode_batch, steps=steps + warm)
    B, Hq, Hkv, D = wl.B, wl.Hq, wl.Hkv, wl.D
    total = int(wl.row_off[-1])
    ctx = ag.Context(0, ag.workspace_bytes(B, 1, Hq, Hkv, D, ag.AG_BF16, 0, total))
    cache = ag.KVCache(to_dev(wl.k_cache, torch), to_dev(wl.v_cache, torch), torch.from_numpy(wl.idx).cuda(),
                       torch.from_numpy(wl.row_off).cuda(), torch.from_numpy(wl.len0).cuda(), B, Hkv, D,
                       total_rows=total)
    n_in = 8
    ins = []
    for s in range(n_in):
        q, kn, vn, nf = wl.step_inputs(s, 0.5)
        ins.append((to_dev(q, torch), to_dev(kn, torch), to_dev(vn, torch), torch.from_numpy(nf).cuda()))
    out = torch.empty(B, Hq, D, dtype=torch.bfloat16, device="cuda")

    def step(s):
        q, kn, vn, nf = ins[s % n_in]
        ag.ag_decode_attn(ctx, q, kn, vn, nf, wl.pos0 + s, wl.scale, cache, out)

    def all_steps():
        for s in range(warm, warm + steps):
            step(s)

    for s in range(warm):
        step(s)
    torch.cuda.synchronize()
    len_start = cache.len.clone()
    len_before = len_start.cpu().numpy().astype(np.int64)

    def timed(run, repeats):
        """wall-clock seconds of `run` (all the steps) from len_start, `repeats` times"""
        secs = []
        for _ in range(repeats):
            cache.len.copy_(len_start)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            run()
            torch.cuda.synchronize()
            secs.append(time.perf_counter() - t0)
        return secs

    eager_s = timed(all_steps, args.repeats)
    ref_out, ref_len = out.clone(), cache.len.clone()
    len_after = ref_len.cpu().numpy().astype(np.int64)
    # one graph that holds all the steps; replays checked against the eager pass, with eager work in between
    graph_s = None
    if not args.no_decode_graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        cache.len.copy_(len_start)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            all_steps()
        torch.cuda.current_stream().wait_stream(side)
        for r in range(2):
            cache.len.copy_(len_start)
            out.zero_()
            graph.replay()
            torch.cuda.synchronize()
            if not (torch.equal(out, ref_out) and torch.equal(cache.len, ref_len)):
                raise RuntimeError("decode graph replay %d differs from the eager steps" % r)
            cache.len.copy_(len_start)
            for s in range(warm, warm + 4):     # eager work between replays
                step(s)
            torch.cuda.synchronize()
        graph_s = timed(graph.replay, args.repeats)
    # kernel durations: the library's events on each launch
    cache.len.copy_(len_start)
    ctx.timing_enable(True)
    torch.cuda.synchronize()
    all_steps()
    torch.cuda.synchronize()
    times = ctx.timing_read()
    ctx.timing_enable(False)
    ctx.poll_error()
    # rows read per step grow by the appends; appends are spread evenly, so use the mean of first and last
    rows_per_step = 0.5 * (len_before.sum() + len_after.sum())
    bytes_per_step = rows_per_step * D * 2 * 2
    part_ms = times["decode_partial"][0] / max(times["decode_partial"][1], 1)
    merge_ms = times["decode_merge"][0] / max(times["decode_merge"][1], 1)
    ach = bytes_per_step / (part_ms * 1e-3) / 1e9
    best = min(eager_s + (graph_s or []))
    use_graph = graph_s is not None and min(graph_s) <= min(eager_s)
    med = lambda xs: sorted(xs)[len(xs) // 2]
    step_ms = best / steps * 1e3
    res = {
        "metric": "decode attention HBM GB/s, whole step (both kernels, gaps included)",
        "value": bytes_per_step / (step_ms * 1e-3) / 1e9, "unit": "GB/s",
        "steps": steps, "ms_per_step": step_ms, "launch": "one hip graph of all steps" if use_graph else "eager",
        "ms_per_step_eager": {"min": min(eager_s) / steps * 1e3, "median": med(eager_s) / steps * 1e3,
                              "max": max(eager_s) / steps * 1e3},
        "ms_per_step_graph": None if graph_s is None else {"min": min(graph_s) / steps * 1e3,
                                                           "median": med(graph_s) / steps * 1e3,
                                                           "max": max(graph_s) / steps * 1e3},
        "kernel_ms": {"decode_partial": part_ms, "decode_merge": merge_ms},
        "roofline": {"kernel": "ag_decode_partial_kernel<bf16,128,1>", "bound": "hbm", "achieved": ach,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBS,
                     "frac_step": bytes_per_step / (step_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                     "traffic": TRAFFIC_BYTES.get(("decode", B, steps)),
                     "bytes_per_launch": bytes_per_step, "avg_launch_ms": part_ms},
        "config": {"workload": wl.name, "B": B, "Hq": Hq, "Hkv": Hkv, "D": D,
                   "mean_len": float(rows_per_step / (B * Hkv)), "keep_vs_4096": float(rows_per_step / (B * Hkv) / 4096)},
    }
    ctx.close()
    return res, wl


def config5_stack_leg(args, torch, ag, W):
    """Config 5 end to end: the 32-layer attention path (no MLPs), B = 16, prompt L = 2048, then 256 decode steps,
    with gate, compaction, masked attention and ragged decode on every layer.  Each layer has its own gate (the
    weights, per-head biases and dead heads of workloads.config5_layer; keep falls from 0.9 to 0.1 with depth) and
    its own activations, seeded N(0, 1) (x: 0.5 N(0, 1)) drawn on the device -- their values do not change the work,
    the flags the gate makes of them do.  The caches use the packed layout (ag_pack_row_off: retained rows + room
    for the generated tokens per unit), sized from an untimed pass of the gates.
    Timed: (1) the prompt through all 32 layers (gate -> packed offsets -> compaction + attention per layer);
    (2) `--stack-tokens` decode steps through all 32 layers (every generated token kept)."""
    layers, B, H, D, L, d = args.stack_layers, 16, 32, 128, 2048, 4096
    tokens = args.stack_tokens
    U, room = B * H, tokens + 8
    gen = torch.Generator(device="cuda")
    gen.manual_seed(5)
    scale = 1.0 / math.sqrt(D)
    ctx = ag.Context(0, ag.workspace_bytes(B, L, H, H, D, ag.AG_BF16, d, U * (L + room)))
    lay = []
    for l in range(layers):
        w, bias, keep, dead = W.config5_gate_params(l)
        x = (0.5 * torch.randn(B, L, d, device="cuda", generator=gen)).to(torch.bfloat16)
        q, k, v = (torch.randn(B, H, L, D, device="cuda", generator=gen).to(torch.bfloat16) for _ in range(3))
        flags = torch.empty(B, H, L, dtype=torch.uint8, device="cuda")
        ag.ag_gate(ctx, x, to_dev(w, torch), torch.from_numpy(bias).cuda(), 0.5, 0, None, flags)
        kept = int(flags.sum().item())               # untimed sizing pass: rows this layer's cache needs
        total = kept + U * room
        cache = ag.KVCache(torch.zeros(total, D, dtype=torch.bfloat16, device="cuda"),
                           torch.zeros(total, D, dtype=torch.bfloat16, device="cuda"),
                           torch.zeros(total, dtype=torch.int32, device="cuda"),
                           torch.zeros(U + 1, dtype=torch.int64, device="cuda"),
                           torch.zeros(U, dtype=torch.int32, device="cuda"), B, H, D, total_rows=total)
        lay.append(dict(x=x, w=to_dev(w, torch), bias=torch.from_numpy(bias).cuda(), q=q, k=k, v=v, flags=flags,
                        cache=cache, total=total, kept=kept, out=torch.empty_like(q), dead=int(dead.sum())))
    dq, dk, dv = (torch.randn(B, H, D, device="cuda", generator=gen).to(torch.bfloat16) for _ in range(3))
    dout = torch.empty(B, H, D, dtype=torch.bfloat16, device="cuda")

    def prompt():
        for a in lay:
            ag.ag_gate(ctx, a["x"], a["w"], a["bias"], 0.5, 0, None, a["flags"])
            ag.ag_pack_row_off(ctx, a["flags"], room, a["total"], a["cache"].row_off)
            ag.ag_compact_prefill_attn(ctx, a["q"], a["k"], a["v"], a["flags"], scale, 0, a["cache"], a["out"])

    def decode(n):
        for s in range(n):
            for a in lay:
                ag.ag_decode_attn(ctx, dq, dk, dv, None, L + s, scale, a["cache"], dout)

    prompt()
    torch.cuda.synchronize()
    ctx.poll_error()
    t0 = time.perf_counter()
    prompt()
    torch.cuda.synchronize()
    t_prompt = time.perf_counter() - t0
    ctx.poll_error()
    rows0 = sum(int(a["cache"].len.sum().item()) for a in lay)
    assert rows0 == sum(a["kept"] for a in lay)
    decode(2)       # warm-up steps (their rows stay in the caches; the timed steps follow on)
    torch.cuda.synchronize()
    rows1 = sum(int(a["cache"].len.sum().item()) for a in lay)
    t0 = time.perf_counter()
    decode(tokens)
    torch.cuda.synchronize()
    t_dec = time.perf_counter() - t0
    ctx.poll_error()
    rows2 = sum(int(a["cache"].len.sum().item()) for a in lay)
    assert rows2 == rows1 + tokens * U * layers
    byts = 0.5 * (rows1 + rows2) * D * 2 * 2      # K and V rows read per token, mean of first and last step
    ctx.close()
    return {"workload": "cfg5_stack_%d_layers_B16_L2048" % layers, "layers": layers, "prompt_tokens": B * L,
            "cache_layout": "packed (ag_pack_row_off), %d spare rows per unit" % room,
            "kept_rows_after_prompt": rows0, "keep_ratio_mean": rows0 / (layers * U * L),
            "cache_bytes": sum(a["total"] for a in lay) * D * 2 * 2, "slab_cache_bytes": layers * U * (L + room) * D * 2 * 2,
            "dead_heads": sum(a["dead"] for a in lay),
            "prompt_ms_all_layers": t_prompt * 1e3, "prompt_tokens_per_s": B * L / t_prompt,
            "decode_tokens": tokens, "decode_ms_per_token": t_dec / tokens * 1e3,
            "decode_tokens_per_s": B * tokens / t_dec, "decode_bytes_per_token": byts,
            "decode_gbs": byts * tokens / t_dec / 1e9, "decode_launches_per_token": 2 * layers,
            "seconds_prompt_plus_decode": t_prompt + t_dec}


def projection_leg(args, torch, ag, W, wl):
    """The layer's K/V projection with the compaction in its epilogue (ag_project_compact_kv) on the headline shape,
    beside the separate compaction it replaces.  Weights are seeded N(0, 1/d) drawn on the device."""
    B, L, d, H, D = wl.B, wl.L, wl.d_model, wl.Hkv, wl.D
    gen = torch.Generator(device="cuda")
    gen.manual_seed(2)
    x = to_dev(wl.x, torch)
    w = (torch.randn(d, 2 * H * D, device="cuda", generator=gen) / math.sqrt(d)).to(torch.bfloat16)
    flags = torch.empty(B, H, L, dtype=torch.uint8, device="cuda")
    U = B * H
    ro = torch.arange(U + 1, dtype=torch.int64, device="cuda") * L
    cache = ag.KVCache(torch.zeros(U * L, D, dtype=torch.bfloat16, device="cuda"),
                       torch.zeros(U * L, D, dtype=torch.bfloat16, device="cuda"),
                       torch.zeros(U * L, dtype=torch.int32, device="cuda"), ro,
                       torch.zeros(U, dtype=torch.int32, device="cuda"), B, H, D)
    kv = torch.zeros(2, B, H, L, D, dtype=torch.bfloat16, device="cuda")
    ctx = ag.Context(0, ag.workspace_bytes(B, L, H, H, D, ag.AG_BF16, d, 0))
    ag.ag_gate(ctx, x, to_dev(wl.w_gate, torch), torch.from_numpy(wl.bias).cuda(), wl.tau, wl.n_sink, None, flags)
    for _ in range(3):
        ag.ag_project_compact_kv(ctx, x, w, flags, 0, kv, cache)
    torch.cuda.synchronize()
    ctx.timing_enable(True)
    for _ in range(10):
        ag.ag_project_compact_kv(ctx, x, w, flags, 0, kv, cache)
    for _ in range(10):
        ag.ag_compact_kv(ctx, kv[0], kv[1], flags, 0, cache)
    torch.cuda.synchronize()
    t = ctx.timing_read()
    ctx.timing_enable(False)
    ctx.poll_error()
    ctx.close()
    proj_ms = t["mha_proj"][0] / t["mha_proj"][1]
    flops = 2.0 * B * L * d * 2 * H * D
    return {"workload": wl.name + " K/V projection, d -> 2 x %d x %d" % (H, D), "fused_projection_compaction_ms": proj_ms,
            "tflops": flops / (proj_ms * 1e-3) / 1e12, "separate_compaction_ms": t["compact"][0] / t["compact"][1]}


def power_leg(args, torch, ag, W, wl):
    """Package power while the prefill kernel of the workload runs back to back for about two seconds: the board's
    own sensor (hwmon power1_input, microwatts) sampled from a host thread, beside its cap (power1_cap) and the idle
    reading before the loop.  Shows whether the kernel runs into the power limit rather than an issue limit."""
    import glob
    import threading
    hw = sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*"))

    def read(name):
        for h in hw:
            try:
                return float(open(os.path.join(h, name)).read())
            except (OSError, ValueError):
                continue
        return None

    if read("power1_input") is None and read("power1_average") is None:
        return {"available": False}
    sensor = "power1_input" if read("power1_input") is not None else "power1_average"
    B, L, Hq, Hkv, D = wl.B, wl.L, wl.Hq, wl.Hkv, wl.D
    U, cap = B * Hkv, L
    q, k, v = to_dev(wl.q, torch), to_dev(wl.k, torch), to_dev(wl.v, torch)
    ctx = ag.Context(0, ag.workspace_bytes(B, L, Hq, Hkv, D, ag.AG_BF16, wl.d_model, 0))
    if wl.flags is not None:
        flags = torch.from_numpy(wl.flags).cuda()
    else:  # the workload's own flags, from its gate
        flags = torch.empty(B, Hkv, L, dtype=torch.uint8, device="cuda")
        ag.ag_gate(ctx, to_dev(wl.x, torch), to_dev(wl.w_gate, torch), torch.from_numpy(wl.bias).cuda(), wl.tau, wl.n_sink,
                   None, flags)
    cache = ag.KVCache(torch.zeros(U * cap, D, dtype=torch.bfloat16, device="cuda"),
                       torch.zeros(U * cap, D, dtype=torch.bfloat16, device="cuda"),
                       torch.zeros(U * cap, dtype=torch.int32, device="cuda"),
                       torch.arange(U + 1, dtype=torch.int64, device="cuda") * cap,
                       torch.zeros(U, dtype=torch.int32, device="cuda"), B, Hkv, D)
    out = torch.empty_like(q)
    ag.ag_compact_kv(ctx, k, v, flags, 0, cache)
    ag.ag_prefill_attn(ctx, q, k, v, flags, wl.scale, cache, out)
    torch.cuda.synchronize()
    time.sleep(0.5)
    idle = read(sensor)
    samples, stop = [], [False]

    def sampler():
        while not stop[0]:
            samples.append(read(sensor))
            time.sleep(0.02)

    th = threading.Thread(target=sampler)
    t0 = time.perf_counter()
    th.start()
    n = 0
    while time.perf_counter() - t0 < 2.0:
        for _ in range(200):
            ag.ag_prefill_attn(ctx, q, k, v, flags, wl.scale, cache, out)
        torch.cuda.synchronize()
        n += 200
    t1 = time.perf_counter()
    stop[0] = True
    th.join()
    ctx.close()
    body = [x for x in samples[len(samples) // 4:] if x is not None]      # skip the ramp at the start
    pcap = read("power1_cap")
    return {"available": True, "sensor": sensor, "workload": wl.name, "prefill_us_per_launch": (t1 - t0) / n * 1e6,
            "idle_w": idle / 1e6 if idle else None, "mean_w": sum(body) / len(body) / 1e6 if body else None,
            "max_w": max(body) / 1e6 if body else None, "cap_w": pcap / 1e6 if pcap else None}


def norm_gate_leg(args, torch, ag, W, wl):
    """The gate fused with the RMS normalisation that produces its input (ag_rmsnorm_gate) on the headline shape,
    beside the two separate passes it replaces: the framework's own rms_norm kernel, then ag_gate.  The residual
    stream h is the layer's x scaled by 3 (the normalisation removes the scale); weights 1 + 0.1 N(0, 1)."""
    B, L, d, H = wl.B, wl.L, wl.d_model, wl.Hkv
    gen = torch.Generator(device="cuda")
    gen.manual_seed(3)
    h = (to_dev(wl.x, torch).float() * 3.0).to(torch.bfloat16)
    g = (1.0 + 0.1 * torch.randn(d, device="cuda", generator=gen)).to(torch.bfloat16)
    wg, bias = to_dev(wl.w_gate, torch), torch.from_numpy(wl.bias).cuda()
    x = torch.empty_like(h)
    flags = torch.empty(B, H, L, dtype=torch.uint8, device="cuda")
    ctx = ag.Context(0, ag.workspace_bytes(B, L, H, H, wl.D, ag.AG_BF16, d, 0))
    n = 20

    def fused():
        ag.ag_rmsnorm_gate(ctx, h, g, 1e-5, wg, bias, wl.tau, wl.n_sink, x, None, flags)

    def separate():
        y = torch.nn.functional.rms_norm(h, (d,), g, 1e-5)
        ag.ag_gate(ctx, y, wg, bias, wl.tau, wl.n_sink, None, flags)

    def wall(fn):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / n * 1e3

    fused_ms, sep_ms = wall(fused), wall(separate)
    ctx.timing_enable(True)
    for _ in range(n):
        fused()
    torch.cuda.synchronize()
    t = ctx.timing_read()
    ctx.timing_enable(False)
    ctx.poll_error()
    ctx.close()
    k_ms = t["norm_gate"][0] / t["norm_gate"][1]
    nbytes = 2.0 * B * L * d * 2
    return {"workload": wl.name + " rms_norm + gate, d = %d, H_f = %d" % (d, H), "fused_kernel_ms": k_ms,
            "fused_gbs": nbytes / (k_ms * 1e-3) / 1e9, "fused_wall_ms": fused_ms,
            "framework_rms_norm_then_ag_gate_wall_ms": sep_ms}


def overlap_leg(args, torch, ag, W, wl):
    """Several layers back to back: the gate of layer l+1 takes its input from before layer l's attention
    (previous-layer gating, Table 3), so it can run on a second stream (own context and workspace) beside layer
    l's compaction + attention.  Reports ms per layer with the gates in line and with the gates on the side."""
    B, L, Hq, Hkv, D, d = wl.B, wl.L, wl.Hq, wl.Hkv, wl.D, wl.d_model
    layers, U, cap = 8, wl.B * wl.Hkv, wl.L + 8
    x, wg, bias = to_dev(wl.x, torch), to_dev(wl.w_gate, torch), torch.from_numpy(wl.bias).cuda()
    q, k, v = to_dev(wl.q, torch), to_dev(wl.k, torch), to_dev(wl.v, torch)
    out = torch.empty_like(q)
    ro = torch.from_numpy(np.arange(U + 1, dtype=np.int64) * cap).cuda()
    cache = ag.KVCache(torch.zeros(U * cap, D, dtype=torch.bfloat16, device="cuda"),
                       torch.zeros(U * cap, D, dtype=torch.bfloat16, device="cuda"),
                       torch.zeros(U * cap, dtype=torch.int32, device="cuda"), ro,
                       torch.zeros(U, dtype=torch.int32, device="cuda"), B, Hkv, D)
    flags = [torch.empty(B, Hkv, L, dtype=torch.uint8, device="cuda") for _ in range(2)]
    ws = ag.workspace_bytes(B, L, Hq, Hkv, D, ag.AG_BF16, d, U * cap)
    ctx_a, ctx_g = ag.Context(0, ws), ag.Context(0, ws)
    main, side = torch.cuda.current_stream(), torch.cuda.Stream()
    ready = [torch.cuda.Event() for _ in range(2)]
    used = [torch.cuda.Event() for _ in range(2)]

    def run(overlap):
        gs, gctx = (side, ctx_g) if overlap else (main, ctx_a)
        gs.wait_stream(main)
        with torch.cuda.stream(gs):
            ag.ag_gate(gctx, x, wg, bias, wl.tau, wl.n_sink, None, flags[0])
            ready[0].record(gs)
        for l in range(layers):
            if l + 1 < layers:
                with torch.cuda.stream(gs):
                    gs.wait_event(used[(l + 1) & 1]) if l >= 1 else None   # the flag buffer's previous reader is done
                    ag.ag_gate(gctx, x, wg, bias, wl.tau, wl.n_sink, None, flags[(l + 1) & 1])
                    ready[(l + 1) & 1].record(gs)
            main.wait_event(ready[l & 1])
            ag.ag_compact_prefill_attn(ctx_a, q, k, v, flags[l & 1], wl.scale, 0, cache, out)
            used[l & 1].record(main)
        main.wait_stream(gs)

    res = {}
    for name, ov in (("gates_in_line", False), ("gates_on_second_stream", True)):
        for _ in range(2):
            run(ov)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            run(ov)
        torch.cuda.synchronize()
        res[name + "_ms_per_layer"] = (time.perf_counter() - t0) / args.steps / layers * 1e3
    ctx_a.close()
    ctx_g.close()
    res["layers"] = layers
    return res


def cpu_baseline(wl, W):
    """The oracle, as it stands, on the whole config-2 step (gate over all tokens and heads, compaction, masked
    prefill, one decode step) on the host cores; its one OpenMP loop runs over the 32 (batch, head) units."""
    import oracle
    L, D, H = wl.L, wl.D, wl.Hkv
    ro = oracle.slab_row_off(H, L + 8)
    g = np.random.default_rng(0)
    dq, dk, dv = (g.standard_normal((1, H, D)).astype(np.float32) for _ in range(3))
    t0 = time.perf_counter()
    _, f = oracle.gate(wl.x.f32, wl.w_gate.f32, wl.bias, wl.tau, wl.n_sink)
    oracle.compact_kv(wl.k.bits, wl.v.bits, f, ro)
    oracle.prefill_attn(wl.q.f32, wl.k.f32, wl.v.f32, f, wl.scale)
    t_mid = time.perf_counter()
    c32, _ = oracle.compact_kv(wl.k.f32, wl.v.f32, f, ro)     # fp32 copy of the cache for the decode step: not timed
    t_mid2 = time.perf_counter()
    oracle.decode_step(dq, dk, dv, None, L, c32, wl.scale)
    t1 = time.perf_counter()
    t = (t_mid - t0) + (t1 - t_mid2)
    # one thread, on the masked prefill of 2 of the heads (the step's dominant part), scaled to all heads
    n_thr = oracle.threads()
    oracle.set_threads(1)
    s0 = time.perf_counter()
    oracle.prefill_attn(wl.q.f32[:, :2], wl.k.f32[:, :2], wl.v.f32[:, :2], f[:, :2], wl.scale)
    t_one = (time.perf_counter() - s0) * H / 2
    oracle.set_threads(n_thr)
    return {"value": wl.B * L / t, "unit": "tokens/s", "cores": min(n_thr, wl.B * H), "kind": "oracle",
            "sample": "one whole config-2 step (all %d heads, L=%d): %.2f s" % (H, L, t), "seconds_sample": t,
            "one_thread_prefill_tokens_per_s": wl.B * L / t_one,
            "one_thread_sample": "masked prefill of 2 heads on 1 thread, scaled to %d heads: %.1f s" % (H, t_one)}


# HBM bytes per launch from the rocprofv3 counter passes summarised in
# profiles/bench_cfg2_prefill_cfg3_decode_hbm_traffic.md (2.0 x FETCH_SIZE + 1.0 x WRITE_SIZE, in KiB, the
# factors calibrated on the 1 GiB copy kernel); they hold for the default workloads only.
TRAFFIC_BYTES = {
    ("prefill", 4096): int((2.0 * 66377 + 39503) * 1024),
    ("decode", 32, 256): int((2.0 * 576164 + 10405) * 1024),
}


def machine_context(torch, ag):
    """What this machine sustains, next to the data-sheet peaks: a register-only bf16 MFMA loop, a 1 GiB streaming
    copy, and the vendor library's bf16 GEMM (8192^3) as the practical MFMA ceiling under the power limit."""
    ctx = ag.Context(0, 2 << 30)
    mfma = ctx.probe_mfma(200000)
    mfma_data = ctx.probe_mfma_data(200000)
    # the matrix pipe alone at lower duty cycles (one wave per SIMD, data-like operands): duty -> TFLOP/s
    duty = {"%.2f" % (256.0 / (256 + 64 * idle)): ctx.probe_mfma_duty(idle, 200000 // (1 + idle // 2)) for idle in (0, 1, 2, 3, 4)}
    copy = ctx.probe_copy(1 << 30)
    ctx.close()
    a = torch.randn(8192, 8192, device="cuda", dtype=torch.bfloat16)
    b = torch.randn(8192, 8192, device="cuda", dtype=torch.bfloat16)
    for _ in range(3):
        a @ b
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(10):
        a @ b
    e1.record()
    torch.cuda.synchronize()
    gemm = 10 * 2 * 8192 ** 3 / (e0.elapsed_time(e1) * 1e-3) / 1e12
    return {"mfma_loop_tflops": mfma, "mfma_loop_random_operands_tflops": mfma_data,
            "mfma_loop_random_operands_tflops_by_duty": duty, "hbm_copy_gbs_1GiB": copy,
            "vendor_gemm_bf16_8192_tflops": gemm}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=2, choices=[2, 4, 5],
                    help="prefill workload: 2 = headline (default); 4, 5 = the other layer-shaped configurations")
    ap.add_argument("--layer", type=int, default=16, help="layer of config 5")
    ap.add_argument("--seq-len", type=int, default=4096)
    ap.add_argument("--keep", type=float, default=None,
                    help="one keep ratio for every head instead of config 2's per-head U[0.2, 0.9]")
    ap.add_argument("--decode-steps", type=int, default=256)
    ap.add_argument("--decode-batch", type=int, default=32)
    ap.add_argument("--project", action="store_true",
                    help="also time the K/V projection with the compaction in its epilogue (ag_project_compact_kv)")
    ap.add_argument("--norm-gate", action="store_true",
                    help="also time the gate fused with the RMS normalisation of its input (ag_rmsnorm_gate)")
    ap.add_argument("--power", action="store_true",
                    help="also sample the package power sensor while the prefill kernel runs back to back")
    ap.add_argument("--config5-stack", "--decode-stack", dest="config5_stack", action="store_true",
                    help="also run config 5 end to end: the prompt through all 32 layers, then --stack-tokens decode "
                         "steps through all 32 layers (about 45 GB of activations and caches on the device)")
    ap.add_argument("--stack-tokens", type=int, default=256)
    ap.add_argument("--stack-layers", type=int, default=32)
    ap.add_argument("--graph", action="store_true", help="replay the step from a HIP graph instead of launching it eagerly")
    ap.add_argument("--repeats", type=int, default=5,
                    help="times the timed block of --steps steps (and the decode leg's block) is repeated; the line "
                         "carries min / median / max, `value` is the median")
    ap.add_argument("--no-decode-graph", action="store_true", help="decode leg: eager launches only")
    ap.add_argument("--skip-decode", action="store_true")
    ap.add_argument("--skip-cpu-baseline", action="store_true")
    ap.add_argument("--skip-overlap", action="store_true", help="skip the multi-layer gate-overlap measurement")
    ap.add_argument("--skip-machine", action="store_true", help="skip the MFMA / copy / vendor-GEMM probes")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2410_12876_amd as ag
    import workloads as W
    if not os.path.exists(ag.LIB_PATH):
        from paper_2410_12876_amd import build
        build.build()
    if not torch.cuda.is_available():
        print("bench.py needs a GPU: the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)

    log("[bench] generating config %d ..." % args.config)
    pre, wl, flags = prefill_leg(args, torch, ag, W)
    log("[bench] prefill leg done: %.3f ms/step" % (pre["seconds"] / args.steps * 1e3))
    if args.config != 2:  # the other legs are defined on the headline workload
        args.skip_decode = args.skip_cpu_baseline = args.skip_overlap = True
    dec = None
    if not args.skip_decode:
        log("[bench] generating config 3 ...")
        dec, _ = decode_leg(args, torch, ag, W)
        log("[bench] decode leg done: %.1f GB/s" % dec["value"])
    cpu = None
    if not args.skip_cpu_baseline:
        log("[bench] timing the CPU oracle on one step ...")
        cpu = cpu_baseline(wl, W)
    overlap = None if args.skip_overlap else overlap_leg(args, torch, ag, W, wl)
    proj = projection_leg(args, torch, ag, W, wl) if args.project and wl.x is not None else None
    norm_gate = norm_gate_leg(args, torch, ag, W, wl) if args.norm_gate and wl.x is not None else None
    power = power_leg(args, torch, ag, W, wl) if args.power else None
    stack = None
    if args.config5_stack:
        log("[bench] config 5 end to end, %d layers ..." % args.stack_layers)
        stack = config5_stack_leg(args, torch, ag, W)
    machine = None if args.skip_machine else machine_context(torch, ag)
    if machine:
        pre["roofline"]["frac_of_vendor_gemm"] = pre["roofline"]["achieved"] / machine["vendor_gemm_bf16_8192_tflops"]
        if dec:
            dec["roofline"]["frac_of_copy"] = dec["roofline"]["achieved"] / machine["hbm_copy_gbs_1GiB"]

    line = {
        "metric": "prefill tokens/s (gate + compaction + masked prefill attention + 1 decode step per layer)",
        "value": pre["tokens"] / pre["seconds"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": pre["seconds"] / args.steps * 1e3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": pre["config"], "kernel_ms": pre["kernel_ms"],
        "ms_per_step_spread": pre["ms_per_step_spread"],
        "ms_per_step_with_kernel_events": pre["seconds_instrumented"] / args.steps * 1e3, "roofline": pre["roofline"],
        "compact_gbs": pre["compact_gbs"], "gate_gbs": pre["gate_gbs"], "keep_ratio_per_head": pre["keep_ratio_per_head"],
        "gate": pre["gate"], "decode": dec, "cpu_baseline": cpu,
        "next_layer_gate_overlap": overlap, "config5_stack": stack, "kv_projection": proj, "norm_gate": norm_gate, "prefill_power": power, "machine": machine,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
