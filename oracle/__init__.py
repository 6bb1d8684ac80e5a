"""CPU oracle for the Attention-Gate hot path (ctypes wrapper around ag_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the benchmark's
cpu_baseline leg.  The product package never imports this module and this module never
imports the product package.  Inputs are fp32 numpy arrays (bf16 data widened by the
caller); floating-point results come back in fp64.

Each function cites the passage it follows in ag_oracle.c.  Every function here is pinned
by tests/test_oracle_pins.py against brute-force dense-mask attention, closed forms,
library routines and invariants; nothing is "parity unpinned".
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import numpy as np

from . import build as _build

_LIB = None


def lib() -> C.CDLL:
    global _LIB
    if _LIB is None:
        path = _build.build(force=False)
        L = C.CDLL(path)
        L.ag_oracle_threads.restype = C.c_int
        L.ag_oracle_logit_threshold.restype = C.c_double
        L.ag_oracle_logit_threshold.argtypes = [C.c_double]
        L.ag_oracle_compact_kv.restype = C.c_int
        L.ag_oracle_decode_step.restype = C.c_int
        _LIB = L
    return _LIB


def threads() -> int:
    return int(lib().ag_oracle_threads())


def set_threads(n: int) -> None:
    lib().ag_oracle_set_threads(C.c_int(n))


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def logit_threshold(tau: float) -> float:
    return float(lib().ag_oracle_logit_threshold(C.c_double(tau)))


def gate(feat, w, bias, tau: float, n_sink: int = 0):
    """feat [B,L,d_in], w [d_in,H_f], bias [H_f] -> (logits f64 [B,L,H_f], flags u8 [B,H_f,L])."""
    feat, w, bias = _f32(feat), _f32(w), _f32(bias)
    B, L, d_in = feat.shape
    H_f = w.shape[1]
    assert w.shape[0] == d_in and bias.shape == (H_f,)
    logits = np.empty((B, L, H_f), dtype=np.float64)
    flags = np.empty((B, H_f, L), dtype=np.uint8)
    lib().ag_oracle_gate(_p(feat), _p(w), _p(bias), C.c_int(B), C.c_int(L), C.c_int(d_in), C.c_int(H_f),
                         C.c_double(tau), C.c_int(n_sink), _p(logits), _p(flags))
    return logits, flags


def _round_to(x: np.ndarray, store) -> np.ndarray:
    """Value of x after being stored in `store` ("bf16": round to nearest even on the upper 16 bits of the fp32
    pattern; "f32"; None: left in fp64)."""
    if store is None:
        return np.asarray(x, dtype=np.float64)
    x32 = np.ascontiguousarray(x, dtype=np.float32)
    if store == "f32":
        return x32.astype(np.float64)
    assert store == "bf16"
    b = x32.view(np.uint32)
    b = (b + (np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1)))) & np.uint32(0xFFFF0000)
    return b.view(np.float32).astype(np.float64)


def gate_mha(x, w_qkv, h_prime: int, d_prime: int, w_o, bias, tau: float, n_sink: int = 0, store=None):
    """The main Attention-Gate module (Sec. 3.3, Eq. 3): MHA' over the hidden states, then the gate projection.

    x [B,L,d]; w_qkv [d, 3*h'*d'] with column blocks (Q'|K'|V'), heads side by side inside a block;
    w_o [h'*d', H_f]; bias [H_f].  Steps, in the paper's order:
      Q',K',V' = X W'                                   (library matmul in fp64)
      A_h      = causal softmax(Q'_h K'_h^T / sqrt d') V'_h    (prefill_attn with every flag set = no eviction)
      logits   = concat_h(A_h) W^{O'} + bias;  flags by Eq. 4  (gate)
    `store` names the dtype in which the module's tensors Q',K',V' and A are held between the steps ("bf16" for
    a bf16 model, None = exact); the arithmetic itself stays fp64.
    Returns (logits f64 [B,L,H_f], flags u8 [B,H_f,L])."""
    x, w_qkv = np.asarray(_f32(x), dtype=np.float64), np.asarray(_f32(w_qkv), dtype=np.float64)
    B, L, d = x.shape
    hd = h_prime * d_prime
    assert w_qkv.shape == (d, 3 * hd)
    proj = _round_to(x.reshape(B * L, d) @ w_qkv, store).reshape(B, L, 3, h_prime, d_prime)
    qp, kp, vp = (np.ascontiguousarray(proj[:, :, i].transpose(0, 2, 1, 3)) for i in range(3))  # [B,h',L,d']
    ones = np.ones((B, h_prime, L), dtype=np.uint8)
    a = prefill_attn(qp, kp, vp, ones, 1.0 / np.sqrt(d_prime))                                  # [B,h',L,d']
    feat = _round_to(a, store).transpose(0, 2, 1, 3).reshape(B, L, hd)
    return gate(feat, w_o, bias, tau, n_sink)


def rmsnorm(h, g, eps: float, store=None):
    """Root-mean-square normalisation of the hidden states, the step that precedes the attention block (and with it
    the gate of Eq. 3, whose input X is the block's input) in the decoder models of Sec. 4.  The paper does not
    restate it; this is the definition those models use:
        x[b,t,c] = h[b,t,c] / sqrt( (1/d) sum_c' h[b,t,c']^2 + eps ) * g[c]
    h [B,L,d], g [d]; arithmetic in fp64; `store` names the dtype x is then held in ("bf16" rounds to nearest even,
    None = exact).  Returns x f64 [B,L,d]."""
    h, g = np.asarray(_f32(h), dtype=np.float64), np.asarray(_f32(g), dtype=np.float64)
    assert h.ndim == 3 and g.shape == (h.shape[2],) and eps > 0.0
    ms = np.empty(h.shape[:2], dtype=np.float64)
    for b in range(h.shape[0]):
        for t in range(h.shape[1]):
            ms[b, t] = np.sum(h[b, t] * h[b, t]) / h.shape[2]
    return _round_to(h / np.sqrt(ms + eps)[:, :, None] * g[None, None, :], store)


def rmsnorm_gate(h, g, eps: float, w, bias, tau: float, n_sink: int = 0, store=None):
    """rmsnorm, then the gate (Eq. 3, Eq. 4) on the stored x.  Returns (x, logits, flags)."""
    x = rmsnorm(h, g, eps, store)
    logits, flags = gate(x, w, bias, tau, n_sink)  # (gate reads its features as fp32: exact for a stored x)
    return x, logits, flags


def project_kv(x, w_kv, Hkv: int, D: int, store=None):
    """The layer's own key/value projection (Eq. 2: K_i = X W_i^K, V_i = X W_i^V) in the layout the path consumes.

    x [B,L,d]; w_kv [d, 2*Hkv*D] with the K columns of all heads first (head h at columns h*D .. h*D+D-1), then the
    V columns in the same order.  The product is a library matmul in fp64; `store` names the dtype in which K and V
    are then held ("bf16" rounds to nearest even, None = exact).  Returns (k, v), each f64 [B,Hkv,L,D]."""
    x, w_kv = np.asarray(_f32(x), dtype=np.float64), np.asarray(_f32(w_kv), dtype=np.float64)
    B, L, d = x.shape
    assert w_kv.shape == (d, 2 * Hkv * D)
    proj = _round_to(x.reshape(B * L, d) @ w_kv, store).reshape(B, L, 2, Hkv, D)
    k, v = (np.ascontiguousarray(proj[:, :, i].transpose(0, 2, 1, 3)) for i in range(2))
    return k, v


def prefill_attn(q, k, v, flags, scale: float, n_recent: int = 1) -> np.ndarray:
    """q [B,Hq,L,D], k/v [B,Hkv,L,D], flags u8 [B,Hkv,L] -> out f64 [B,Hq,L,D]."""
    q, k, v = _f32(q), _f32(k), _f32(v)
    flags = np.ascontiguousarray(flags, dtype=np.uint8)
    B, Hq, L, D = q.shape
    Hkv = k.shape[1]
    assert k.shape == (B, Hkv, L, D) and v.shape == k.shape and flags.shape == (B, Hkv, L)
    assert Hq % Hkv == 0 and n_recent >= 1
    out = np.empty((B, Hq, L, D), dtype=np.float64)
    lib().ag_oracle_prefill_attn(_p(q), _p(k), _p(v), _p(flags), C.c_int(B), C.c_int(L), C.c_int(Hq),
                                 C.c_int(Hkv), C.c_int(D), C.c_double(scale), C.c_int(n_recent), _p(out))
    return out


def prefill_rows(q, k, v, flags, scale: float, rows, n_recent: int = 1) -> np.ndarray:
    """prefill_attn restricted to the query positions `rows` (same for every head):
    out f64 [B,Hq,len(rows),D].  For sampled checks of problems too large to compute whole."""
    q, k, v = _f32(q), _f32(k), _f32(v)
    flags = np.ascontiguousarray(flags, dtype=np.uint8)
    rows = np.ascontiguousarray(rows, dtype=np.int32)
    B, Hq, L, D = q.shape
    Hkv = k.shape[1]
    assert k.shape == (B, Hkv, L, D) and v.shape == k.shape and flags.shape == (B, Hkv, L)
    assert Hq % Hkv == 0 and n_recent >= 1 and rows.ndim == 1
    assert rows.size == 0 or (rows.min() >= 0 and rows.max() < L)
    out = np.empty((B, Hq, rows.size, D), dtype=np.float64)
    lib().ag_oracle_prefill_rows(_p(q), _p(k), _p(v), _p(flags), C.c_int(B), C.c_int(L), C.c_int(Hq),
                                 C.c_int(Hkv), C.c_int(D), C.c_double(scale), C.c_int(n_recent), _p(rows),
                                 C.c_int(rows.size), _p(out))
    return out


@dataclass
class Cache:
    """Ragged per-(batch, KV head) cache.  k/v hold rows in the storage dtype given to
    compact_kv (any dtype); decode_step needs fp32 rows."""
    k: np.ndarray          # [total_rows, D]
    v: np.ndarray
    idx: np.ndarray        # int32 [total_rows]
    row_off: np.ndarray    # int64 [U+1]
    len: np.ndarray        # int32 [U]

    def copy(self) -> "Cache":
        return Cache(self.k.copy(), self.v.copy(), self.idx.copy(), self.row_off.copy(), self.len.copy())


def slab_row_off(n_units: int, capacity) -> np.ndarray:
    cap = np.broadcast_to(np.asarray(capacity, dtype=np.int64), (n_units,))
    ro = np.zeros(n_units + 1, dtype=np.int64)
    np.cumsum(cap, out=ro[1:])
    return ro


def compact_kv(k, v, flags, row_off, pos0: int = 0, fill=0):
    """k/v [B,Hkv,L,D] (any dtype, copied byte for byte), flags u8 [B,Hkv,L] -> (Cache, overflow)."""
    k = np.ascontiguousarray(k)
    v = np.ascontiguousarray(v)
    flags = np.ascontiguousarray(flags, dtype=np.uint8)
    B, Hkv, L, D = k.shape
    U = B * Hkv
    row_off = np.ascontiguousarray(row_off, dtype=np.int64)
    assert row_off.shape == (U + 1,) and v.shape == k.shape and v.dtype == k.dtype
    total = int(row_off[-1])
    kc = np.full((total, D), fill, dtype=k.dtype)
    vc = np.full((total, D), fill, dtype=k.dtype)
    idx = np.full(total, -1, dtype=np.int32)
    ln = np.zeros(U, dtype=np.int32)
    over = lib().ag_oracle_compact_kv(_p(k), _p(v), _p(flags), C.c_int(U), C.c_int(L),
                                      C.c_size_t(D * k.dtype.itemsize), C.c_int(pos0), _p(row_off),
                                      _p(kc), _p(vc), _p(idx), _p(ln))
    return Cache(kc, vc, idx, row_off, ln), int(over)


def decode_step(q, k_new, v_new, new_flags, pos: int, cache: Cache, scale: float):
    """One decode step over `cache` (fp32 rows; updated in place) -> (out f64 [B,Hq,D], dropped)."""
    q, k_new, v_new = _f32(q), _f32(k_new), _f32(v_new)
    B, Hq, D = q.shape
    Hkv = k_new.shape[1]
    assert cache.k.dtype == np.float32 and cache.v.dtype == np.float32
    assert cache.k.flags.c_contiguous and cache.v.flags.c_contiguous
    assert cache.len.shape == (B * Hkv,) and cache.k.shape[1] == D
    if new_flags is not None:
        new_flags = np.ascontiguousarray(new_flags, dtype=np.uint8).reshape(B * Hkv)
    out = np.empty((B, Hq, D), dtype=np.float64)
    dropped = lib().ag_oracle_decode_step(_p(q), _p(k_new), _p(v_new), _p(new_flags), C.c_int(pos),
                                          C.c_int(B), C.c_int(Hq), C.c_int(Hkv), C.c_int(D),
                                          C.c_double(scale), _p(cache.k), _p(cache.v), _p(cache.idx),
                                          _p(cache.row_off), _p(cache.len), _p(out))
    return out, int(dropped)


def packed_row_off(flags, room: int, total_rows: int):
    """Slab offsets of the packed cache layout (Sec. 3.3: only the retained rows take cache memory): unit u gets its
    kept rows plus `room` spare rows, units back to back, the layout cut off at total_rows.  Plain loop over the
    units.  Returns (row_off i64 [units + 1], rows the layout needs)."""
    f = np.asarray(flags)
    f = f.reshape(-1, f.shape[-1])
    row_off = np.zeros(f.shape[0] + 1, dtype=np.int64)
    need = 0
    for u in range(f.shape[0]):
        kept = 0
        for t in range(f.shape[1]):
            kept += 1 if f[u, t] != 0 else 0
        need += kept + room
        row_off[u + 1] = min(need, total_rows)
    return row_off, need
