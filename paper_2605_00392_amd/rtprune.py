"""ctypes binding of the RTPrune C ABI (``include/rtprune.h``).

Argument marshalling only: every function below has the name and the argument
order of the C entry point it forwards to, takes torch tensors (or raw integer
addresses) for device pointers, and returns the C status code.  All arithmetic
runs in the HIP library; torch is used for device memory and streams.  If the
library has not been built the first call raises: there is no fallback.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Dict, Optional

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "librtprune.so")

RTP_OK, RTP_EINVAL, RTP_EUNSUPPORTED, RTP_EWORKSPACE, RTP_EHIP = range(5)
RTP_F32, RTP_BF16 = 0, 1
RTP_METRIC_L2NORM, RTP_METRIC_VARIANCE = 0, 1
RTP_POSITIONS_CONSECUTIVE, RTP_POSITIONS_ORIGINAL = 0, 1
RTP_DEV_BAD_OFFSETS, RTP_DEV_IMAGE_TOO_LONG, RTP_DEV_BAD_IMAGE, RTP_DEV_SYNC_TIMEOUT = 1, 2, 4, 8

EXPORTS = (
    "rtprune_status_string", "rtprune_workspace_bytes", "rtprune_dynamic_ratio",
    "rtprune_norms_topk", "rtprune_ot_pair", "rtprune_merge", "rtprune_prune", "rtprune_prune_splice",
    "rtprune_profile_enable", "rtprune_profile_summary", "rtprune_profile_only", "rtprune_copy_bytes",
    "rtprune_text_density_workspace_bytes", "rtprune_text_density", "rtprune_prune_static",
)
RTPRUNE_STATIC_SCRATCH_BYTES = 64 << 20


class RtpruneError(RuntimeError):
    pass


class rtprune_params(ctypes.Structure):
    _fields_ = [
        ("z", ctypes.c_float), ("alpha", ctypes.c_float), ("eps", ctypes.c_float),
        ("iters", ctypes.c_int32), ("dynamic", ctypes.c_int32),
        ("ratio", ctypes.c_float), ("ratio_min", ctypes.c_float), ("ratio_max", ctypes.c_float),
        ("phi_lo", ctypes.c_float), ("phi_hi", ctypes.c_float),
        ("metric", ctypes.c_int32), ("mid_merge_min_images", ctypes.c_int32),
    ]


class rtprune_text_spans(ctypes.Structure):
    _fields_ = [
        ("prefix", ctypes.c_void_p), ("prefix_offsets", ctypes.c_void_p), ("prefix_rows", ctypes.c_int64),
        ("suffix", ctypes.c_void_p), ("suffix_offsets", ctypes.c_void_p), ("suffix_rows", ctypes.c_int64),
    ]


class rtprune_batch(ctypes.Structure):
    _fields_ = [
        ("tokens", ctypes.c_void_p), ("offsets", ctypes.c_void_p),
        ("total_tokens", ctypes.c_int64), ("B", ctypes.c_int32), ("D", ctypes.c_int32),
        ("max_tokens", ctypes.c_int32), ("dtype", ctypes.c_int32),
    ]


_lib = None


def load_library(path: Optional[str] = None) -> ctypes.CDLL:
    """Open ``librtprune.so`` (once) and declare the prototypes."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    p = path or LIB_PATH
    if not os.path.exists(p):
        raise RtpruneError(
            f"{p} is missing: build it with `python -m paper_2605_00392_amd.build` "
            "(there is no CPU fallback)")
    lib = ctypes.CDLL(p)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    pp, pb = ctypes.POINTER(rtprune_params), ctypes.POINTER(rtprune_batch)
    lib.rtprune_status_string.restype = ctypes.c_char_p
    lib.rtprune_status_string.argtypes = [ctypes.c_int]
    lib.rtprune_workspace_bytes.restype = ctypes.c_int
    lib.rtprune_workspace_bytes.argtypes = [i32, i64, i32, i32, i32, pp, ctypes.POINTER(ctypes.c_size_t)]
    lib.rtprune_dynamic_ratio.restype = ctypes.c_int
    lib.rtprune_dynamic_ratio.argtypes = [pb, vp, pp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.rtprune_norms_topk.restype = ctypes.c_int
    lib.rtprune_norms_topk.argtypes = [pb, vp, pp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.rtprune_ot_pair.restype = ctypes.c_int
    lib.rtprune_ot_pair.argtypes = [pb, vp, vp, vp, pp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.rtprune_merge.restype = ctypes.c_int
    lib.rtprune_merge.argtypes = [pb, vp, vp, vp, vp, vp, pp, vp, vp, ctypes.c_size_t, vp]
    lib.rtprune_prune.restype = ctypes.c_int
    lib.rtprune_prune.argtypes = [pb, vp, pp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.rtprune_prune_splice.restype = ctypes.c_int
    lib.rtprune_prune_splice.argtypes = [pb, vp, pp, ctypes.POINTER(rtprune_text_spans), i32, vp, ctypes.c_int64,
                                         vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.rtprune_prune_static.restype = ctypes.c_int
    lib.rtprune_prune_static.argtypes = [pb, vp, pp, vp, vp, vp, vp, vp, vp, vp]
    lib.rtprune_profile_enable.restype = ctypes.c_int
    lib.rtprune_profile_enable.argtypes = [ctypes.c_int]
    lib.rtprune_profile_only.restype = ctypes.c_int
    lib.rtprune_profile_only.argtypes = [ctypes.c_char_p]
    lib.rtprune_profile_summary.restype = ctypes.c_int
    lib.rtprune_profile_summary.argtypes = [ctypes.c_char_p, ctypes.c_size_t]
    lib.rtprune_text_density_workspace_bytes.restype = ctypes.c_int
    lib.rtprune_text_density_workspace_bytes.argtypes = [i32, i32, i32, i32, i32, ctypes.POINTER(ctypes.c_size_t)]
    lib.rtprune_text_density.restype = ctypes.c_int
    lib.rtprune_text_density.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, i32, ctypes.c_float, vp, vp, vp,
                                         vp, ctypes.c_size_t, vp]
    lib.rtprune_copy_bytes.restype = ctypes.c_int
    lib.rtprune_copy_bytes.argtypes = [vp, vp, ctypes.c_size_t, vp]
    if path is None:
        _lib = lib
    return lib


def make_params(d: Optional[Dict[str, float]] = None, **kw) -> rtprune_params:
    """Fill the C parameter struct from a dict / keywords (paper defaults otherwise)."""
    v = dict(z=0.2, alpha=0.1, eps=0.05, iters=100, dynamic=0, ratio=0.84,
             ratio_min=0.6, ratio_max=1.0, phi_lo=0.0, phi_hi=1.0, metric=RTP_METRIC_L2NORM,
             mid_merge_min_images=0)
    if d:
        v.update(d)
    v.update(kw)
    return rtprune_params(v["z"], v["alpha"], v["eps"], int(v["iters"]), int(v["dynamic"]),
                          v["ratio"], v["ratio_min"], v["ratio_max"], v["phi_lo"], v["phi_hi"],
                          int(v["metric"]), int(v["mid_merge_min_images"]))


def _addr(x) -> Optional[int]:
    """Device address of a torch tensor (or pass an int / None through)."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if not x.is_contiguous():
        raise RtpruneError("device arrays must be contiguous")
    return x.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


@dataclass
class DeviceBatch:
    """A packed ragged batch resident on the device (see ``rtprune_batch`` in the header)."""
    tokens: object          # torch tensor [total, D], float32 or bfloat16
    offsets: object         # torch int32 [B + 1]
    total_tokens: int
    max_tokens: int
    B: int
    D: int
    dtype: int

    def desc(self) -> rtprune_batch:
        return rtprune_batch(_addr(self.tokens), _addr(self.offsets), self.total_tokens,
                             self.B, self.D, self.max_tokens, self.dtype)


def upload(batch, device="cuda:0") -> DeviceBatch:
    """Copy a host ``synth.Batch`` to the device (plumbing, no arithmetic)."""
    import numpy as np
    import torch
    if batch.dtype == "bf16":
        t = torch.from_numpy(batch.tokens.view(np.int16)).to(device).view(torch.bfloat16)
        dt = RTP_BF16
    else:
        t = torch.from_numpy(batch.tokens).to(device)
        dt = RTP_F32
    off = torch.from_numpy(batch.offsets).to(device)
    d = batch.tokens.shape[1]
    return DeviceBatch(t.contiguous(), off, batch.total_tokens, batch.max_tokens, batch.batch, d, dt)


def status_string(status: int) -> str:
    return load_library().rtprune_status_string(int(status)).decode()


def check(status: int) -> None:
    if status != RTP_OK:
        raise RtpruneError(status_string(status))


# --- the C entry points, name for name ---------------------------------------

def rtprune_workspace_bytes(B: int, total_tokens: int, max_tokens: int, D: int, dtype: int,
                            params: Optional[rtprune_params] = None):
    """Returns ``(status, bytes)``; ``params`` None asks for the worst case over all parameters."""
    n = ctypes.c_size_t(0)
    rc = load_library().rtprune_workspace_bytes(B, total_tokens, max_tokens, D, dtype,
                                                ctypes.byref(params) if params is not None else None,
                                                ctypes.byref(n))
    return rc, int(n.value)


def rtprune_dynamic_ratio(batch: DeviceBatch, density, params: rtprune_params, phi, ratio,
                          keep_counts, workspace, stream=None) -> int:
    d = batch.desc()
    return load_library().rtprune_dynamic_ratio(
        ctypes.byref(d), _addr(density), ctypes.byref(params), _addr(phi), _addr(ratio),
        _addr(keep_counts), _addr(workspace), workspace.numel() if workspace is not None else 0,
        _stream(stream))


def rtprune_norms_topk(batch: DeviceBatch, keep_counts_in, params: rtprune_params, norms, sel_idx,
                       keep_counts, out_offsets, plan_offsets, workspace, stream=None) -> int:
    d = batch.desc()
    return load_library().rtprune_norms_topk(
        ctypes.byref(d), _addr(keep_counts_in), ctypes.byref(params), _addr(norms), _addr(sel_idx),
        _addr(keep_counts), _addr(out_offsets), _addr(plan_offsets), _addr(workspace),
        workspace.numel() if workspace is not None else 0, _stream(stream))


def rtprune_ot_pair(batch: DeviceBatch, sel_idx, keep_counts, plan_offsets, params: rtprune_params,
                    scores, plan, pair, workspace, stream=None) -> int:
    d = batch.desc()
    return load_library().rtprune_ot_pair(
        ctypes.byref(d), _addr(sel_idx), _addr(keep_counts), _addr(plan_offsets),
        ctypes.byref(params), _addr(scores), _addr(plan), _addr(pair), _addr(workspace),
        workspace.numel() if workspace is not None else 0, _stream(stream))


def rtprune_merge(batch: DeviceBatch, sel_idx, keep_counts, out_offsets, plan, plan_offsets,
                  params: rtprune_params, out, workspace=None, stream=None) -> int:
    d = batch.desc()
    return load_library().rtprune_merge(
        ctypes.byref(d), _addr(sel_idx), _addr(keep_counts), _addr(out_offsets), _addr(plan),
        _addr(plan_offsets), ctypes.byref(params), _addr(out), _addr(workspace),
        workspace.numel() if workspace is not None else 0, _stream(stream))


def rtprune_prune(batch: DeviceBatch, density, params: rtprune_params, out, out_offsets,
                  keep_counts, sel_idx, pair, ratio, workspace, stream=None) -> int:
    d = batch.desc()
    return load_library().rtprune_prune(
        ctypes.byref(d), _addr(density), ctypes.byref(params), _addr(out), _addr(out_offsets),
        _addr(keep_counts), _addr(sel_idx), _addr(pair), _addr(ratio), _addr(workspace),
        workspace.numel() if workspace is not None else 0, _stream(stream))


def make_text_spans(prefix=None, prefix_offsets=None, prefix_rows: int = 0,
                    suffix=None, suffix_offsets=None, suffix_rows: int = 0) -> rtprune_text_spans:
    """Fill the C text-span struct from device arrays (or None for an absent side)."""
    return rtprune_text_spans(_addr(prefix), _addr(prefix_offsets), int(prefix_rows),
                              _addr(suffix), _addr(suffix_offsets), int(suffix_rows))


def rtprune_prune_splice(batch: DeviceBatch, density, params: rtprune_params, text: rtprune_text_spans,
                         position_mode: int, seq, seq_capacity_rows: int, seq_offsets, position_ids,
                         keep_counts, sel_idx, pair, ratio, workspace, stream=None) -> int:
    d = batch.desc()
    return load_library().rtprune_prune_splice(
        ctypes.byref(d), _addr(density), ctypes.byref(params), ctypes.byref(text), int(position_mode),
        _addr(seq), int(seq_capacity_rows), _addr(seq_offsets), _addr(position_ids), _addr(keep_counts),
        _addr(sel_idx), _addr(pair), _addr(ratio), _addr(workspace),
        workspace.numel() if workspace is not None else 0, _stream(stream))


def rtprune_prune_static(batch: DeviceBatch, density, params: rtprune_params, out, out_offsets,
                         keep_counts, sel_idx, pair, ratio, stream=None) -> int:
    d = batch.desc()
    return load_library().rtprune_prune_static(
        ctypes.byref(d), _addr(density), ctypes.byref(params), _addr(out), _addr(out_offsets),
        _addr(keep_counts), _addr(sel_idx), _addr(pair), _addr(ratio), _stream(stream))


def rtprune_profile_enable(on: int) -> int:
    return load_library().rtprune_profile_enable(int(on))


def rtprune_profile_only(kernel: Optional[str]) -> int:
    return load_library().rtprune_profile_only(kernel.encode() if kernel else None)


def rtprune_profile_summary():
    """Returns ``(status, list of {kernel, launches, total_ms})``."""
    import json
    buf = ctypes.create_string_buffer(1 << 14)
    rc = load_library().rtprune_profile_summary(buf, len(buf))
    return rc, (json.loads(buf.value.decode()) if rc == RTP_OK else [])


def rtprune_copy_bytes(dst, src, nbytes: int, stream=None) -> int:
    return load_library().rtprune_copy_bytes(_addr(dst), _addr(src), nbytes, _stream(stream))


def rtprune_text_density_workspace_bytes(B: int, max_height: int, max_width: int, patch_h: int, patch_w: int):
    """Returns ``(status, bytes)``."""
    n = ctypes.c_size_t(0)
    rc = load_library().rtprune_text_density_workspace_bytes(B, max_height, max_width, patch_h, patch_w,
                                                             ctypes.byref(n))
    return rc, int(n.value)


def rtprune_text_density(pixels, pixel_offsets, heights, widths, B: int, max_height: int, max_width: int,
                         patch_h: int, patch_w: int, tau: float, density, patch_density, patch_offsets,
                         workspace, stream=None) -> int:
    return load_library().rtprune_text_density(
        _addr(pixels), _addr(pixel_offsets), _addr(heights), _addr(widths), B, max_height, max_width,
        patch_h, patch_w, tau, _addr(density), _addr(patch_density), _addr(patch_offsets),
        _addr(workspace), workspace.numel() if workspace is not None else 0, _stream(stream))


def alloc_workspace(batch: DeviceBatch, params: Optional[rtprune_params] = None):
    """A uint8 device tensor of the size ``rtprune_workspace_bytes`` asks for (``params`` None:
    enough for every call)."""
    import torch
    rc, n = rtprune_workspace_bytes(batch.B, batch.total_tokens, batch.max_tokens, batch.D, batch.dtype, params)
    check(rc)
    return torch.empty(n, dtype=torch.uint8, device=batch.tokens.device)
