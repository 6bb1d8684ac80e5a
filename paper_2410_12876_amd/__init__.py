"""Python binding of libag (include/ag.h): argument marshalling only.

Every step of the Attention-Gate path runs in the HIP kernels of libag.so; PyTorch is used
for device memory and streams.  There is no CPU fallback: importing the library on a machine
where libag.so has not been built raises, and every call returns the library's status as an
exception.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libag.so")

AG_OK, AG_EINVAL, AG_EUNSUPPORTED, AG_ECAPACITY, AG_EWORKSPACE, AG_EHIP = range(6)
AG_F32, AG_BF16 = 0, 1
# (tau, gamma) of the paper's two experiments (Sec. 4.1 training details; Sec. 4.2 implementation details); gamma is
# the constant of Sec. 3.5 inside the sigmoid and enters ag_gate as a bias of gamma in every head
PRESET_PRETRAIN = (0.5, 2.0)
PRESET_FINETUNE = (0.3, 0.0)
STATUS_NAMES = ["AG_OK", "AG_EINVAL", "AG_EUNSUPPORTED", "AG_ECAPACITY", "AG_EWORKSPACE", "AG_EHIP"]

EXPORTS = ["ag_create", "ag_destroy", "ag_last_error", "ag_workspace_bytes", "ag_poll_error",
           "ag_timing_kernels", "ag_timing_kernel_name", "ag_timing_enable", "ag_timing_read",
           "ag_probe_mfma", "ag_probe_mfma_data", "ag_probe_mfma_duty", "ag_probe_copy", "ag_gate", "ag_rmsnorm_gate", "ag_compact_kv", "ag_pack_row_off", "ag_prefill_attn", "ag_prefill_attn_recent",
           "ag_compact_prefill_attn", "ag_project_compact_kv", "ag_project_compact_workspace_bytes", "ag_decode_attn", "ag_decode_attn_static", "ag_decode_static_scratch_bytes", "ag_decode_scratch_bytes", "ag_recent_fill", "ag_decode_attn_recent", "ag_gate_mha", "ag_gate_mha_workspace_bytes"]


class ag_recent_ring(C.Structure):
    _fields_ = [("k", C.c_void_p), ("v", C.c_void_p), ("flags", C.c_void_p), ("pos", C.c_void_p),
                ("n_recent", C.c_int32)]


class AgError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__("%s: %s" % (STATUS_NAMES[status] if 0 <= status < 6 else status, message))
        self.status = status


class ag_kv_cache(C.Structure):
    _fields_ = [("k", C.c_void_p), ("v", C.c_void_p), ("idx", C.c_void_p), ("row_off", C.c_void_p),
                ("len", C.c_void_p), ("total_rows", C.c_int64), ("B", C.c_int32), ("Hkv", C.c_int32),
                ("D", C.c_int32), ("dtype", C.c_int)]


_lib = None


def load() -> C.CDLL:
    """Load libag.so (built by paper_2410_12876_amd/build.py); raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError("libag.so is not built: run `python -m paper_2410_12876_amd.build` "
                          "(or __graft_entry__.build()) first; there is no fallback path")
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64, f32 = C.c_void_p, C.c_int, C.c_int64, C.c_float
    lib.ag_create.restype = C.c_int
    lib.ag_create.argtypes = [C.POINTER(vp), i32, C.c_size_t]
    lib.ag_destroy.restype = None
    lib.ag_destroy.argtypes = [vp]
    lib.ag_last_error.restype = C.c_char_p
    lib.ag_last_error.argtypes = [vp]
    lib.ag_workspace_bytes.restype = C.c_size_t
    lib.ag_workspace_bytes.argtypes = [i32, i32, i32, i32, i32, i32, i32, i64]
    lib.ag_poll_error.restype = C.c_int
    lib.ag_poll_error.argtypes = [vp, vp]
    lib.ag_timing_kernels.restype = C.c_int
    lib.ag_timing_kernel_name.restype = C.c_char_p
    lib.ag_timing_kernel_name.argtypes = [i32]
    lib.ag_timing_enable.restype = C.c_int
    lib.ag_timing_enable.argtypes = [vp, i32]
    lib.ag_timing_read.restype = C.c_int
    lib.ag_timing_read.argtypes = [vp, i32, C.POINTER(C.c_double), C.POINTER(C.c_int)]
    lib.ag_probe_mfma.restype = C.c_int
    lib.ag_probe_mfma.argtypes = [vp, vp, i32, C.POINTER(C.c_double)]
    lib.ag_probe_mfma_data.restype = C.c_int
    lib.ag_probe_mfma_data.argtypes = [vp, vp, i32, C.POINTER(C.c_double)]
    lib.ag_probe_mfma_duty.restype = C.c_int
    lib.ag_probe_mfma_duty.argtypes = [vp, vp, i32, i32, C.POINTER(C.c_double)]
    lib.ag_probe_copy.restype = C.c_int
    lib.ag_probe_copy.argtypes = [vp, vp, C.c_size_t, C.POINTER(C.c_double)]
    lib.ag_gate.restype = C.c_int
    lib.ag_gate.argtypes = [vp, vp, vp, i32, i32, i32, i32, vp, vp, i32, f32, i32, vp, vp]
    lib.ag_rmsnorm_gate.restype = C.c_int
    lib.ag_rmsnorm_gate.argtypes = [vp, vp, vp, i32, i32, i32, i32, vp, f32, vp, vp, i32, f32, i32, vp, vp, vp]
    lib.ag_compact_kv.restype = C.c_int
    lib.ag_compact_kv.argtypes = [vp, vp, vp, vp, vp, i32, i32, C.POINTER(ag_kv_cache)]
    lib.ag_pack_row_off.restype = C.c_int
    lib.ag_pack_row_off.argtypes = [vp, vp, vp, i32, i32, i32, i32, i64, vp, vp]
    lib.ag_prefill_attn.restype = C.c_int
    lib.ag_prefill_attn.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, f32,
                                    C.POINTER(ag_kv_cache), vp]
    lib.ag_prefill_attn_recent.restype = C.c_int
    lib.ag_prefill_attn_recent.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, f32,
                                           C.POINTER(ag_kv_cache), i32, vp]
    lib.ag_compact_prefill_attn.restype = C.c_int
    lib.ag_compact_prefill_attn.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, f32, i32,
                                            C.POINTER(ag_kv_cache), i32, vp]
    lib.ag_project_compact_workspace_bytes.restype = C.c_size_t
    lib.ag_project_compact_workspace_bytes.argtypes = [i32, i32, i32]
    lib.ag_project_compact_kv.restype = C.c_int
    lib.ag_project_compact_kv.argtypes = [vp, vp, vp, i32, i32, i32, i32, vp, vp, i32, vp, C.POINTER(ag_kv_cache)]
    lib.ag_decode_attn.restype = C.c_int
    lib.ag_decode_attn.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, f32, C.POINTER(ag_kv_cache), vp]
    lib.ag_decode_attn_static.restype = C.c_int
    lib.ag_decode_attn_static.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, f32, C.POINTER(ag_kv_cache), vp]
    lib.ag_decode_static_scratch_bytes.restype = C.c_size_t
    lib.ag_decode_static_scratch_bytes.argtypes = []
    lib.ag_decode_scratch_bytes.restype = C.c_size_t
    lib.ag_decode_scratch_bytes.argtypes = [C.POINTER(ag_kv_cache), i32]
    lib.ag_gate_mha_workspace_bytes.restype = C.c_size_t
    lib.ag_gate_mha_workspace_bytes.argtypes = [i32, i32, i32, i32, i32, i32]
    lib.ag_gate_mha.restype = C.c_int
    lib.ag_gate_mha.argtypes = [vp, vp, vp, i32, i32, i32, i32, vp, i32, i32, vp, vp, i32, f32, i32, vp, vp]
    lib.ag_recent_fill.restype = C.c_int
    lib.ag_recent_fill.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, C.POINTER(ag_recent_ring)]
    lib.ag_decode_attn_recent.restype = C.c_int
    lib.ag_decode_attn_recent.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, f32, C.POINTER(ag_kv_cache),
                                          C.POINTER(ag_recent_ring), vp]
    _lib = lib
    return lib


def _ptr(t) -> Optional[int]:
    """Device (or raw integer) pointer of a tensor argument; None stays NULL."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_contiguous():
        raise ValueError("tensor arguments must be contiguous")
    return t.data_ptr()


def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.bfloat16:
        return AG_BF16
    if t.dtype == torch.float32:
        return AG_F32
    raise ValueError("unsupported tensor dtype %s" % t.dtype)


def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def workspace_bytes(B: int, L: int, Hq: int, Hkv: int, D: int, dtype: int, d_in: int = 0,
                    cache_rows: int = 0) -> int:
    return int(load().ag_workspace_bytes(B, L, Hq, Hkv, D, dtype, d_in, cache_rows))


class Context:
    """ag_ctx.  device = -1 gives a context that validates arguments but cannot launch."""

    def __init__(self, device: int = 0, workspace: int = 0):
        self._lib = load()
        h = C.c_void_p()
        st = self._lib.ag_create(C.byref(h), device, workspace)
        if st != AG_OK:
            raise AgError(st, "ag_create(device=%d, workspace=%d) failed" % (device, workspace))
        self._h = h
        self.device = device

    def close(self) -> None:
        if getattr(self, "_h", None):
            self._lib.ag_destroy(self._h)
            self._h = None

    __del__ = close

    def _check(self, st: int) -> None:
        if st != AG_OK:
            raise AgError(st, self._lib.ag_last_error(self._h).decode())

    def poll_error(self, stream=None) -> None:
        self._check(self._lib.ag_poll_error(self._h, _stream_ptr(stream)))

    def timing_enable(self, on: bool = True) -> None:
        self._check(self._lib.ag_timing_enable(self._h, 1 if on else 0))

    def timing_read(self) -> dict:
        """{kernel name: (total ms, launches)} of the launches recorded since timing_enable(True)."""
        out = {}
        for kid in range(self._lib.ag_timing_kernels()):
            ms, n = C.c_double(), C.c_int()
            self._check(self._lib.ag_timing_read(self._h, kid, C.byref(ms), C.byref(n)))
            out[self._lib.ag_timing_kernel_name(kid).decode()] = (ms.value, n.value)
        return out


    def probe_mfma(self, iters: int = 20000, stream=None) -> float:
        """Sustained dense bf16 MFMA TFLOP/s of this GPU (register-only loop)."""
        out = C.c_double()
        self._check(self._lib.ag_probe_mfma(self._h, _stream_ptr(stream), iters, C.byref(out)))
        return out.value

    def probe_mfma_data(self, iters: int = 20000, stream=None) -> float:
        """The same loop on operands that change per MFMA and look like data (the ceiling under the power cap)."""
        out = C.c_double()
        self._check(self._lib.ag_probe_mfma_data(self._h, _stream_ptr(stream), iters, C.byref(out)))
        return out.value

    def probe_mfma_duty(self, idle: int, iters: int = 20000, stream=None) -> float:
        """The data-operand MFMA loop at one wave per SIMD, sleeping idle x 64 cycles after every 8 MFMAs; TFLOP/s."""
        out = C.c_double(0.0)
        self._check(self._lib.ag_probe_mfma_duty(self._h, _stream_ptr(stream), iters, idle, C.byref(out)))
        return out.value

    def probe_copy(self, nbytes: int, stream=None) -> float:
        """Sustained HBM read+write GB/s of a streaming copy of nbytes inside the workspace."""
        out = C.c_double()
        self._check(self._lib.ag_probe_copy(self._h, _stream_ptr(stream), nbytes, C.byref(out)))
        return out.value


class KVCache:
    """ag_kv_cache over caller-made device tensors (k, v [rows, D]; idx i32; row_off i64; len i32)."""

    def __init__(self, k, v, idx, row_off, len_, B: int, Hkv: int, D: int, dtype: Optional[int] = None,
                 total_rows: Optional[int] = None):
        self.k, self.v, self.idx, self.row_off, self.len = k, v, idx, row_off, len_
        self.B, self.Hkv, self.D = B, Hkv, D
        self.c = ag_kv_cache(_ptr(k), _ptr(v), _ptr(idx), _ptr(row_off), _ptr(len_),
                             int(k.shape[0]) if total_rows is None else total_rows, B, Hkv, D,
                             _dtype_code(k) if dtype is None else dtype)


def ag_gate(ctx: Context, feat, w_gate, bias, tau: float, n_sink: int, logits_out, flags_out, stream=None) -> None:
    """feat [B, L, d_in], w_gate [d_in, H_f], bias f32 [H_f] -> logits_out f32 [B, L, H_f] (or None),
    flags_out u8 [B, H_f, L]."""
    B, L, d_in = feat.shape
    H_f = w_gate.shape[1]
    ctx._check(ctx._lib.ag_gate(ctx._h, _stream_ptr(stream), _ptr(feat), _dtype_code(feat), B, L, d_in,
                                _ptr(w_gate), _ptr(bias), H_f, tau, n_sink, _ptr(logits_out), _ptr(flags_out)))


def ag_rmsnorm_gate(ctx: Context, h, norm_w, eps: float, w_gate, bias, tau: float, n_sink: int, x_out, logits_out,
                    flags_out, stream=None) -> None:
    """h [B, L, d_in], norm_w [d_in], w_gate [d_in, H_f], bias f32 [H_f] -> x_out [B, L, d_in] (may be h),
    logits_out f32 [B, L, H_f] (or None), flags_out u8 [B, H_f, L]."""
    B, L, d_in = h.shape
    H_f = w_gate.shape[1]
    ctx._check(ctx._lib.ag_rmsnorm_gate(ctx._h, _stream_ptr(stream), _ptr(h), _dtype_code(h), B, L, d_in,
                                        _ptr(norm_w), eps, _ptr(w_gate), _ptr(bias), H_f, tau, n_sink, _ptr(x_out),
                                        _ptr(logits_out), _ptr(flags_out)))


def ag_compact_kv(ctx: Context, k, v, flags, pos0: int, cache: KVCache, stream=None) -> None:
    """k, v [B, Hkv, L, D], flags u8 [B, Hkv, L] -> cache (k, v, idx, len written)."""
    L = k.shape[2]
    ctx._check(ctx._lib.ag_compact_kv(ctx._h, _stream_ptr(stream), _ptr(k), _ptr(v), _ptr(flags), L, pos0,
                                      C.byref(cache.c)))


def ag_pack_row_off(ctx: Context, flags, room: int, total_rows: int, row_off, rows_needed=None, stream=None) -> None:
    """flags u8 [B, Hkv, L] -> row_off i64 [B*Hkv + 1] of the packed layout (retained rows + room per unit, cut off at
    total_rows); rows_needed i64 [1] (or None) receives the rows the layout needs."""
    B, Hkv, L = flags.shape
    ctx._check(ctx._lib.ag_pack_row_off(ctx._h, _stream_ptr(stream), _ptr(flags), B, Hkv, L, room, total_rows,
                                        _ptr(row_off), _ptr(rows_needed)))


def project_compact_workspace_bytes(B: int, L: int, Hkv: int) -> int:
    return int(load().ag_project_compact_workspace_bytes(B, L, Hkv))


def ag_project_compact_kv(ctx: Context, x, w_kv, flags, pos0: int, kv_out, cache: KVCache, stream=None) -> None:
    """x [B, L, d] bf16, w_kv [d, 2*Hkv*128] bf16 (K columns, then V columns), flags u8 [B, Hkv, L] ->
    kv_out [2, B, Hkv, L, 128] (k, v of every token) and cache (kept rows, idx, len)."""
    B, L, d = x.shape
    ctx._check(ctx._lib.ag_project_compact_kv(ctx._h, _stream_ptr(stream), _ptr(x), _dtype_code(x), B, L, d, _ptr(w_kv),
                                              _ptr(flags), pos0, _ptr(kv_out), C.byref(cache.c)))


def ag_prefill_attn(ctx: Context, q, k, v, flags, scale: float, cache: Optional[KVCache], out, stream=None) -> None:
    """q, out [B, Hq, L, D]; k, v [B, Hkv, L, D]; flags u8 [B, Hkv, L]; cache from ag_compact_kv or None."""
    B, Hq, L, D = q.shape
    Hkv = k.shape[1]
    ctx._check(ctx._lib.ag_prefill_attn(ctx._h, _stream_ptr(stream), _ptr(q), _ptr(k), _ptr(v), _ptr(flags),
                                        B, L, Hq, Hkv, D, _dtype_code(q), scale,
                                        C.byref(cache.c) if cache is not None else None, _ptr(out)))


def ag_prefill_attn_recent(ctx: Context, q, k, v, flags, scale: float, cache: Optional[KVCache], n_recent: int, out,
                           stream=None) -> None:
    """ag_prefill_attn with the n_recent - 1 tokens before each query visible whatever their flag."""
    B, Hq, L, D = q.shape
    Hkv = k.shape[1]
    ctx._check(ctx._lib.ag_prefill_attn_recent(ctx._h, _stream_ptr(stream), _ptr(q), _ptr(k), _ptr(v), _ptr(flags),
                                               B, L, Hq, Hkv, D, _dtype_code(q), scale,
                                               C.byref(cache.c) if cache is not None else None, n_recent, _ptr(out)))


def ag_compact_prefill_attn(ctx: Context, q, k, v, flags, scale: float, pos0: int, cache: KVCache, out,
                            n_recent: int = 1, stream=None) -> None:
    """ag_compact_kv + ag_prefill_attn in one call (one flag scan): fills `cache` and `out`."""
    B, Hq, L, D = q.shape
    Hkv = k.shape[1]
    ctx._check(ctx._lib.ag_compact_prefill_attn(ctx._h, _stream_ptr(stream), _ptr(q), _ptr(k), _ptr(v), _ptr(flags),
                                                B, L, Hq, Hkv, D, _dtype_code(q), scale, pos0, C.byref(cache.c),
                                                n_recent, _ptr(out)))


def ag_decode_attn(ctx: Context, q, k_new, v_new, new_flags, pos: int, scale: float, cache: KVCache, out,
                   stream=None) -> None:
    """q, out [B, Hq, D]; k_new, v_new [B, Hkv, D]; new_flags u8 [B, Hkv] or None; cache updated in place."""
    Hq = q.shape[1]
    ctx._check(ctx._lib.ag_decode_attn(ctx._h, _stream_ptr(stream), _ptr(q), _ptr(k_new), _ptr(v_new),
                                       _ptr(new_flags), pos, Hq, scale, C.byref(cache.c), _ptr(out)))


def ag_decode_attn_static(ctx: Context, q, k_new, v_new, new_flags, pos: int, scale: float, cache: KVCache, out,
                          stream=None) -> None:
    """ag_decode_attn out of the library's static per-GPU scratch array: allocates nothing, needs no workspace."""
    Hq = q.shape[1]
    ctx._check(ctx._lib.ag_decode_attn_static(ctx._h, _stream_ptr(stream), _ptr(q), _ptr(k_new), _ptr(v_new),
                                              _ptr(new_flags), pos, Hq, scale, C.byref(cache.c), _ptr(out)))


def decode_static_scratch_bytes() -> int:
    return int(load().ag_decode_static_scratch_bytes())


def decode_scratch_bytes(cache: KVCache, Hq: int) -> int:
    return int(load().ag_decode_scratch_bytes(C.byref(cache.c), Hq))


class RecentRing:
    """The last n_recent tokens of every (batch, KV head) unit for the recent-token window; tensors are the
    caller's: k, v [B*Hkv, n_recent, D], flags u8 [B*Hkv, n_recent], pos i32 [B*Hkv, n_recent]."""

    def __init__(self, k, v, flags, pos, n_recent: int):
        self.k, self.v, self.flags, self.pos, self.n_recent = k, v, flags, pos, n_recent
        self.c = ag_recent_ring(_ptr(k), _ptr(v), _ptr(flags), _ptr(pos), n_recent)


def ag_recent_fill(ctx: Context, k, v, flags, pos0: int, ring: RecentRing, stream=None) -> None:
    """k, v [B, Hkv, L, D], flags u8 [B, Hkv, L]: the ring takes the last prompt tokens."""
    B, Hkv, L, D = k.shape
    ctx._check(ctx._lib.ag_recent_fill(ctx._h, _stream_ptr(stream), _ptr(k), _ptr(v), _ptr(flags), B, L, Hkv, D,
                                       _dtype_code(k), pos0, C.byref(ring.c)))


def ag_decode_attn_recent(ctx: Context, q, k_new, v_new, new_flags, pos: int, scale: float, cache: KVCache,
                          ring: Optional[RecentRing], out, stream=None) -> None:
    """ag_decode_attn with the evicted tokens of the ring's window visible; the ring then takes the new token."""
    Hq = q.shape[1]
    ctx._check(ctx._lib.ag_decode_attn_recent(ctx._h, _stream_ptr(stream), _ptr(q), _ptr(k_new), _ptr(v_new),
                                              _ptr(new_flags), pos, Hq, scale, C.byref(cache.c),
                                              C.byref(ring.c) if ring is not None else None, _ptr(out)))


def gate_mha_workspace_bytes(B: int, L: int, d_model: int, h_prime: int, d_prime: int, H_f: int) -> int:
    return int(load().ag_gate_mha_workspace_bytes(B, L, d_model, h_prime, d_prime, H_f))


def ag_gate_mha(ctx: Context, x, w_qkv, h_prime: int, d_prime: int, w_o, bias, tau: float, n_sink: int, logits_out,
                flags_out, stream=None) -> None:
    """The paper's main gate: x [B, L, d]; w_qkv [d, 3*h'*d'] (Q'|K'|V', head-major inside); w_o [h'*d', H_f];
    bias f32 [H_f]; logits_out f32 [B, L, H_f] or None; flags_out u8 [B, H_f, L]."""
    B, L, d = x.shape
    H_f = w_o.shape[1]
    ctx._check(ctx._lib.ag_gate_mha(ctx._h, _stream_ptr(stream), _ptr(x), _dtype_code(x), B, L, d, _ptr(w_qkv),
                                    h_prime, d_prime, _ptr(w_o), _ptr(bias), H_f, tau, n_sink, _ptr(logits_out),
                                    _ptr(flags_out)))
