"""Seeded synthetic inputs for the Attention-Gate (AG) hot path.

This module only *draws* tensors: it holds none of the method's arithmetic (no
gate, no mask, no softmax, no compaction).  Both the CPU oracle's tests and the
HIP path's tests/benchmarks take their inputs from here so that the two sides
see bit-identical values.  Everything is produced on the host by numpy's
counter-based Philox generator with key ``241012876 + 1000*config + tensor_id``
and rounded once to the storage dtype (fp32, or bf16 kept as uint16 bit
patterns).

The shapes follow the Llama2-7B / Llama-3-8B attention layers the paper's
experiments run on (Sec. 4.1), and the keep ratios follow the eviction ratios
its tables report (roughly 40-70 % evicted, Tables 1, 2 and 6); the paper's
datasets and trained gates are replaced by these synthetic draws.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, Optional

import numpy as np
from scipy.stats import norm as _norm

BASE_SEED = 241012876


# --------------------------------------------------------------------------
# raw draws and storage rounding
# --------------------------------------------------------------------------
def rng(config: int, tensor_id: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=BASE_SEED + 1000 * config + tensor_id))


def normal(config: int, tensor_id: int, shape, std: float = 1.0) -> np.ndarray:
    x = rng(config, tensor_id).standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        x *= np.float32(std)
    return x


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass
class Tensor:
    """A host tensor in its storage dtype plus the same values widened to fp32."""
    f32: np.ndarray                      # values as the kernels see them, widened
    bits: Optional[np.ndarray] = None    # uint16 bf16 patterns (None for fp32 storage)

    @property
    def is_bf16(self) -> bool:
        return self.bits is not None

    @property
    def storage(self) -> np.ndarray:
        return self.bits if self.bits is not None else self.f32


def store(x: np.ndarray, dtype: str) -> Tensor:
    if dtype == "f32":
        return Tensor(np.ascontiguousarray(x, dtype=np.float32))
    if dtype == "bf16":
        bits = f32_to_bf16_bits(x)
        return Tensor(bf16_bits_to_f32(bits), bits)
    raise ValueError(dtype)


# --------------------------------------------------------------------------
# flag patterns (inputs for the cases where flags are given, not gated)
# --------------------------------------------------------------------------
def bernoulli_flags(config: int, tensor_id: int, shape, keep: float) -> np.ndarray:
    return (rng(config, tensor_id).random(size=shape) < keep).astype(np.uint8)


def run_flags(config: int, tensor_id: int, n_units: int, L: int, mean_keep_run: float,
              keep_ratio: float) -> np.ndarray:
    """Alternating kept / evicted runs with geometric lengths, per unit.

    Kept runs have mean ``mean_keep_run``; evicted runs have mean
    ``mean_keep_run * (1-keep_ratio)/keep_ratio`` so the overall keep ratio is
    ``keep_ratio``.  Whole tiles of evicted tokens appear, as in the eviction
    maps of Fig. 1.
    """
    g = rng(config, tensor_id)
    out = np.zeros((n_units, L), dtype=np.uint8)
    mean_evict = mean_keep_run * (1.0 - keep_ratio) / keep_ratio
    for u in range(n_units):
        n_runs = int(2 * L / (mean_keep_run + mean_evict)) + 64
        while True:
            ka = g.geometric(1.0 / mean_keep_run, size=n_runs)
            ea = g.geometric(1.0 / mean_evict, size=n_runs)
            runs = np.empty(2 * n_runs, dtype=np.int64)
            runs[0::2] = ka
            runs[1::2] = ea
            ends = np.cumsum(runs)
            if ends[-1] >= L:
                break
            n_runs *= 2
        starts = ends - runs
        for s, e in zip(starts[0::2], ends[0::2]):
            if s >= L:
                break
            out[u, s:min(e, L)] = 1
    return out


def gate_bias_for_keep(w_gate_f32: np.ndarray, x_std: float, keep: np.ndarray, tau: float) -> np.ndarray:
    """Per-head bias that makes a N(0, x_std^2)-input linear gate keep ``keep[h]``.

    With inputs i.i.d. N(0, x_std^2) the logit of head h is N(0, (x_std*|w_h|)^2),
    so the bias that leaves a fraction keep[h] above logit(tau) follows from the
    normal quantile; no logit is evaluated here.
    """
    sigma = x_std * np.linalg.norm(w_gate_f32.astype(np.float64), axis=0)
    thr = math.log(tau / (1.0 - tau))
    return (thr - sigma * _norm.ppf(1.0 - np.asarray(keep, dtype=np.float64))).astype(np.float32)


# --------------------------------------------------------------------------
# layer workloads (gate -> compaction -> masked prefill [-> decode])
# --------------------------------------------------------------------------
@dataclass
class LayerWorkload:
    name: str
    config: int
    dtype: str
    B: int
    L: int
    d_model: int
    Hq: int
    Hkv: int
    D: int
    tau: float
    n_sink: int
    scale: float
    x: Optional[Tensor] = None        # [B, L, d_model]
    w_gate: Optional[Tensor] = None   # [d_model, Hkv]
    bias: Optional[np.ndarray] = None  # fp32 [Hkv]
    q: Optional[Tensor] = None        # [B, Hq, L, D]
    k: Optional[Tensor] = None        # [B, Hkv, L, D]
    v: Optional[Tensor] = None        # [B, Hkv, L, D]
    flags: Optional[np.ndarray] = None  # given flags u8 [B, Hkv, L] (None => from the gate)
    keep: Optional[np.ndarray] = None   # target keep ratio per head
    extra: Dict = field(default_factory=dict)


def _project(x_f32: np.ndarray, w: np.ndarray, H: int, D: int) -> np.ndarray:
    """[B,L,d] x [d,H*D] -> [B,H,L,D]; the model's own Q/K/V projection (Eq. 2),
    which sits outside the AG hot path and therefore counts as input preparation."""
    B, L, d = x_f32.shape
    y = (x_f32.reshape(B * L, d) @ w).reshape(B, L, H, D)
    return np.ascontiguousarray(y.transpose(0, 2, 1, 3))


def gated_layer(config: int, name: str, dtype: str, B: int, L: int, d_model: int, Hq: int, Hkv: int,
                D: int, x_std: float, keep, tau: float = 0.5, n_sink: int = 0,
                seed_shift: int = 0, with_qkv: bool = True) -> LayerWorkload:
    """A layer whose flags come from the linear gate (Sec. 3.4, linear variant)."""
    t0 = 100 * seed_shift
    wl = LayerWorkload(name, config, dtype, B, L, d_model, Hq, Hkv, D, tau, n_sink, 1.0 / math.sqrt(D))
    x = normal(config, t0 + 1, (B, L, d_model), x_std)
    wl.x = store(x, dtype)
    wl.w_gate = store(normal(config, t0 + 2, (d_model, Hkv), 1.0 / math.sqrt(d_model)), dtype)
    keep = np.broadcast_to(np.asarray(keep, dtype=np.float64), (Hkv,)).copy()
    wl.keep = keep
    wl.bias = gate_bias_for_keep(wl.w_gate.f32, x_std, keep, tau)
    if with_qkv:
        wstd = 1.0 / math.sqrt(d_model)
        wl.q = store(_project(wl.x.f32, normal(config, t0 + 3, (d_model, Hq * D), wstd), Hq, D), dtype)
        wl.k = store(_project(wl.x.f32, normal(config, t0 + 4, (d_model, Hkv * D), wstd), Hkv, D), dtype)
        wl.v = store(_project(wl.x.f32, normal(config, t0 + 5, (d_model, Hkv * D), wstd), Hkv, D), dtype)
    return wl


def config1() -> LayerWorkload:
    """Tiny fp32 layer: B=1, L=128, d=256, 4 heads x 64, ~50 % keep, token 0 kept."""
    return gated_layer(1, "cfg1_tiny_f32", "f32", 1, 128, 256, 4, 4, 64, 1.0, 0.5, tau=0.5, n_sink=1)


def config2(L: int = 4096, keep=None, with_qkv: bool = True) -> LayerWorkload:
    """Llama2-7B-shaped layer in bf16: d=4096, 32 heads x 128, keep ratios U[0.2, 0.9]."""
    if keep is None:
        keep = 0.2 + 0.7 * rng(2, 9).random(32)
    return gated_layer(2, "cfg2_llama2_7b_L%d" % L, "bf16", 1, L, 4096, 32, 32, 128, 0.5, keep,
                       tau=0.5, n_sink=0, with_qkv=with_qkv)


def config4(L: int = 32768, with_x: bool = False) -> LayerWorkload:
    """Llama-3-8B-shaped GQA layer: 32 query / 8 KV heads x 128, flags given as runs, keep 0.3."""
    Hq, Hkv, D = 32, 8, 128
    wl = LayerWorkload("cfg4_llama3_8b_gqa_L%d" % L, 4, "bf16", 1, L, 4096, Hq, Hkv, D, 0.5, 0,
                       1.0 / math.sqrt(D))
    wl.q = store(normal(4, 3, (1, Hq, L, D), 1.0), "bf16")
    wl.k = store(normal(4, 4, (1, Hkv, L, D), 1.0), "bf16")
    wl.v = store(normal(4, 5, (1, Hkv, L, D), 1.0), "bf16")
    wl.flags = run_flags(4, 6, Hkv, L, 16.0, 0.3).reshape(1, Hkv, L)
    wl.keep = np.full(Hkv, 0.3)
    if with_x:
        wl.x = store(normal(4, 1, (1, L, 4096), 0.5), "bf16")
        wl.w_gate = store(normal(4, 2, (4096, Hkv), 1.0 / 64.0), "bf16")
        wl.bias = gate_bias_for_keep(wl.w_gate.f32, 0.5, wl.keep, 0.5)
    return wl


def config5_layer(layer: int, B: int = 16, L: int = 2048, n_layers: int = 32) -> LayerWorkload:
    """One layer of the 32-layer 7B-shaped stack: keep falls linearly 0.9 -> 0.1 with
    depth, and in layers >= 24 about 10 % of heads are fully evicted (Fig. 1)."""
    H, D, d = 32, 128, 4096
    g = rng(5, 1000 + layer)
    rho = 0.9 - 0.8 * layer / (n_layers - 1)
    keep = np.clip(rho + 0.05 * (g.random(H) - 0.5), 0.02, 0.98)
    dead = (g.random(H) < 0.10) if layer >= 24 else np.zeros(H, dtype=bool)
    wl = gated_layer(5, "cfg5_layer%02d" % layer, "bf16", B, L, d, H, H, D, 0.5, keep, tau=0.5,
                     n_sink=0, seed_shift=layer + 1, with_qkv=False)
    # a fully evicted head: bias far below any reachable logit
    wl.bias = np.where(dead, np.float32(-1.0e4), wl.bias).astype(np.float32)
    wl.keep = np.where(dead, 0.0, keep)
    t0 = 100 * (layer + 1)
    wl.q = store(normal(5, t0 + 3, (B, H, L, D), 1.0), "bf16")
    wl.k = store(normal(5, t0 + 4, (B, H, L, D), 1.0), "bf16")
    wl.v = store(normal(5, t0 + 5, (B, H, L, D), 1.0), "bf16")
    wl.extra["dead_heads"] = dead
    return wl


# --------------------------------------------------------------------------
# decode workloads (ragged per-head caches)
# --------------------------------------------------------------------------
@dataclass
class DecodeWorkload:
    name: str
    config: int
    dtype: str
    B: int
    Hq: int
    Hkv: int
    D: int
    scale: float
    steps: int
    len0: np.ndarray          # int32 [B*Hkv] initial kept rows per unit
    row_off: np.ndarray       # int64 [B*Hkv+1] slab offsets (capacity = len0 + steps)
    k_cache: Tensor           # [total_rows, D]   (rows beyond len are slack)
    v_cache: Tensor
    idx: np.ndarray           # int32 [total_rows] original positions (slack = -1)
    pos0: int                 # position of the first decoded token

    def step_inputs(self, s: int, keep_prob: Optional[float] = 0.5):
        """q, k_new, v_new (N(0,1)) and Bernoulli new-token flags of decode step s."""
        c, t0 = self.config, 10000 + 10 * s
        q = store(normal(c, t0 + 1, (self.B, self.Hq, self.D)), self.dtype)
        kn = store(normal(c, t0 + 2, (self.B, self.Hkv, self.D)), self.dtype)
        vn = store(normal(c, t0 + 3, (self.B, self.Hkv, self.D)), self.dtype)
        nf = None if keep_prob is None else bernoulli_flags(c, t0 + 4, (self.B, self.Hkv), keep_prob)
        return q, kn, vn, nf


def decode_batch(config: int, name: str, dtype: str, B: int, Hq: int, Hkv: int, D: int, len0: np.ndarray,
                 steps: int, pos0: int, fill_slack: Optional[float] = None) -> DecodeWorkload:
    U = B * Hkv
    len0 = np.asarray(len0, dtype=np.int32).reshape(U)
    cap = len0.astype(np.int64) + steps
    row_off = np.zeros(U + 1, dtype=np.int64)
    np.cumsum(cap, out=row_off[1:])
    total = int(row_off[-1])
    k = normal(config, 21, (total, D))
    v = normal(config, 22, (total, D))
    idx = np.full(total, -1, dtype=np.int32)
    g = rng(config, 23)
    for u in range(U):
        n = int(len0[u])
        r0 = int(row_off[u])
        # sorted distinct original positions of the surviving prompt tokens
        idx[r0:r0 + n] = np.sort(g.choice(pos0, size=n, replace=False)) if n <= pos0 else np.arange(n)
        if fill_slack is not None:
            k[r0 + n:int(row_off[u + 1])] = fill_slack
            v[r0 + n:int(row_off[u + 1])] = fill_slack
    return DecodeWorkload(name, config, dtype, B, Hq, Hkv, D, 1.0 / math.sqrt(D), steps, len0, row_off,
                          store(k, dtype), store(v, dtype), idx, pos0)


def config5_gate_params(layer: int, n_layers: int = 32):
    """The gate of one layer of config 5 without the layer's activations: (w_gate, bias, target keep per head, dead
    heads), the same draws as config5_layer makes (for benchmarks that fill the activations on the device)."""
    H, d = 32, 4096
    g = rng(5, 1000 + layer)
    rho = 0.9 - 0.8 * layer / (n_layers - 1)
    keep = np.clip(rho + 0.05 * (g.random(H) - 0.5), 0.02, 0.98)
    dead = (g.random(H) < 0.10) if layer >= 24 else np.zeros(H, dtype=bool)
    w_gate = store(normal(5, 100 * (layer + 1) + 2, (d, H), 1.0 / math.sqrt(d)), "bf16")
    bias = gate_bias_for_keep(w_gate.f32, 0.5, keep, 0.5)
    bias = np.where(dead, np.float32(-1.0e4), bias).astype(np.float32)
    return w_gate, bias, np.where(dead, 0.0, keep), dead


def config5_decode_lens(layer: int, B: int = 16, L: int = 2048, n_layers: int = 32) -> np.ndarray:
    """Kept rows per (batch, head) unit of layer `layer` after a 2048-token prompt, for the 32-layer decode
    phase: the layer's per-head keep ratios are those of config5_layer (fully evicted heads included), each
    sequence of the batch deviates from them by a few rows."""
    H = 32
    g = rng(5, 1000 + layer)
    rho = 0.9 - 0.8 * layer / (n_layers - 1)
    keep = np.clip(rho + 0.05 * (g.random(H) - 0.5), 0.02, 0.98)
    dead = (g.random(H) < 0.10) if layer >= 24 else np.zeros(H, dtype=bool)
    gb = rng(5, 5000 + layer)
    lens = np.rint(keep[None, :] * L + 8.0 * gb.standard_normal((B, H)))
    lens = np.clip(lens, 1, L)
    lens[:, dead] = 0
    return lens.astype(np.int32).reshape(B * H)


def config3(B: int = 32, steps: int = 256, max_len: int = 4096, fill_slack: Optional[float] = None) -> DecodeWorkload:
    """Decode-heavy batch: 32 heads x 128, len ~ round(max_len * U[0.1, 1]), 5 % of units len 1."""
    H, D = 32, 128
    g = rng(3, 20)
    len0 = np.rint(max_len * (0.1 + 0.9 * g.random(B * H))).astype(np.int32)
    len0[g.random(B * H) < 0.05] = 1
    return decode_batch(3, "cfg3_decode_B%d" % B, "bf16", B, H, H, D, len0, steps, pos0=max_len, fill_slack=fill_slack)
