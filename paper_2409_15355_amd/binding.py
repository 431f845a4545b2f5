"""Thin ctypes face of the HIP library: argument marshalling only.

Function names and argument order follow ``include/ba.h``.  Tensors are torch CUDA
tensors (PyTorch is used for device memory and streams, nothing else); metadata are
host sequences of ints.  Every step of the hot path runs inside ``libba_hip.so``; if
the library is missing, loading fails loudly -- there is no fallback.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libba_hip.so")

BA_OK = 0
DTYPE_BF16, DTYPE_F32 = 0, 1
ROPE_INTERLEAVED, ROPE_HALF = 0, 1
ROPE_NONE, ROPE_APPLY = 0, 1
REENC_SHIFT, REENC_ABSOLUTE = 0, 1

EXPORTS = ["ba_version", "ba_status_string", "ba_last_error", "ba_profile_begin", "ba_profile_end",
           "ba_encode_blocks",
           "ba_encode_blocks_workspace_bytes", "ba_reencode_positions",
           "ba_final_block_attention", "ba_final_block_attention_workspace_bytes",
           "ba_final_block_attention_static",
           "ba_final_block_attention_cached", "ba_final_block_attention_cached_workspace_bytes",
           "ba_block_attention_prompts", "ba_block_attention_prompts_workspace_bytes", "ba_set_gather_below",
           "ba_block_attention_prompts_backward", "ba_block_attention_prompts_backward_workspace_bytes"]


class BaTensor(ctypes.Structure):
    _fields_ = [("ptr", ctypes.c_void_p), ("stride_tok", ctypes.c_int64),
                ("stride_head", ctypes.c_int64), ("dtype", ctypes.c_int32)]


class BaHeads(ctypes.Structure):
    _fields_ = [("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("q_to_kv", ctypes.POINTER(ctypes.c_int32)),
                ("softmax_scale", ctypes.c_float), ("rope_base", ctypes.c_double),
                ("inv_freq", ctypes.POINTER(ctypes.c_double)), ("rope_layout", ctypes.c_int32)]


class BaError(RuntimeError):
    def __init__(self, status: int, name: str, detail: str):
        super().__init__(f"{name} ({status}): {detail}")
        self.status = status


_lib = None
_I32P = ctypes.c_void_p  # const int32_t*: host arrays travel as plain addresses (numpy's typed pointers cost microseconds each)
_TP = ctypes.POINTER(BaTensor)
_HP = ctypes.POINTER(BaHeads)


def load():
    """dlopen libba_hip.so (built by ``paper_2409_15355_amd.build``)."""
    global _lib
    if _lib is not None:
        return _lib
    # PyTorch ships its own HIP runtime; the process must use exactly one, and the device
    # memory handed to this library is torch's, so torch's runtime has to be loaded first.
    import torch  # noqa: F401
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2409_15355_amd.build`")
    lib = ctypes.CDLL(LIB_PATH)
    lib.ba_version.restype = ctypes.c_int32
    lib.ba_status_string.restype = ctypes.c_char_p
    lib.ba_status_string.argtypes = [ctypes.c_int32]
    lib.ba_last_error.restype = ctypes.c_char_p
    lib.ba_profile_begin.restype = ctypes.c_int32
    lib.ba_profile_begin.argtypes = [ctypes.c_int32]
    lib.ba_profile_end.restype = ctypes.c_int32
    lib.ba_profile_end.argtypes = [ctypes.POINTER(ctypes.c_double), _I32P]
    lib.ba_encode_blocks.restype = ctypes.c_int32
    lib.ba_encode_blocks.argtypes = [_HP, _TP, _TP, _TP, _TP, _TP, ctypes.c_int32, _I32P, ctypes.c_int32,
                                     ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    lib.ba_encode_blocks_workspace_bytes.restype = ctypes.c_size_t
    lib.ba_encode_blocks_workspace_bytes.argtypes = [_HP, ctypes.c_int32, _I32P, ctypes.c_int32, ctypes.c_int32]
    lib.ba_reencode_positions.restype = ctypes.c_int32
    lib.ba_reencode_positions.argtypes = [_HP, _TP, _TP, ctypes.c_int32, ctypes.c_int64, ctypes.c_int64,
                                          ctypes.c_int32, _I32P, _I32P, _I32P, _I32P, _I32P, ctypes.c_int32,
                                          ctypes.c_void_p]
    lib.ba_final_block_attention.restype = ctypes.c_int32
    lib.ba_final_block_attention.argtypes = [_HP, _TP, _TP, _TP, _TP, _TP, _TP, _TP, ctypes.c_int32, _I32P,
                                             _I32P, _I32P, ctypes.c_int32, ctypes.c_void_p, ctypes.c_size_t,
                                             ctypes.c_void_p]
    lib.ba_final_block_attention_static.restype = ctypes.c_int32
    lib.ba_final_block_attention_static.argtypes = [_HP, _TP, _TP, _TP, _TP, _TP, _TP, _TP, ctypes.c_int32, _I32P,
                                                    _I32P, _I32P, ctypes.c_int32, ctypes.c_void_p]
    lib.ba_final_block_attention_workspace_bytes.restype = ctypes.c_size_t
    lib.ba_final_block_attention_workspace_bytes.argtypes = [_HP, ctypes.c_int32, _I32P, _I32P, ctypes.c_int32,
                                                             ctypes.c_int32]
    lib.ba_final_block_attention_cached.restype = ctypes.c_int32
    lib.ba_final_block_attention_cached.argtypes = [_HP, _TP, _TP, _TP, _TP, _TP, _TP, _TP, ctypes.c_int32, _I32P,
                                                    _I32P, _I32P, _I32P, _I32P, _I32P, _I32P, ctypes.c_void_p,
                                                    ctypes.c_size_t, ctypes.c_void_p]
    lib.ba_final_block_attention_cached_workspace_bytes.restype = ctypes.c_size_t
    lib.ba_final_block_attention_cached_workspace_bytes.argtypes = [_HP, ctypes.c_int32, _I32P, _I32P, _I32P,
                                                                    ctypes.c_int32]
    lib.ba_block_attention_prompts_backward.restype = ctypes.c_int32
    lib.ba_block_attention_prompts_backward.argtypes = [_HP, _TP, _TP, _TP, _TP, ctypes.c_void_p, _TP, _TP, _TP, _TP,
                                                        ctypes.c_int32, _I32P, _I32P, ctypes.c_void_p, ctypes.c_size_t,
                                                        ctypes.c_void_p]
    lib.ba_block_attention_prompts_backward_workspace_bytes.restype = ctypes.c_size_t
    lib.ba_block_attention_prompts_backward_workspace_bytes.argtypes = [_HP, ctypes.c_int32, _I32P, _I32P]
    lib.ba_set_gather_below.restype = ctypes.c_int32
    lib.ba_set_gather_below.argtypes = [ctypes.c_int32]
    lib.ba_block_attention_prompts.restype = ctypes.c_int32
    lib.ba_block_attention_prompts.argtypes = [_HP, _TP, _TP, _TP, _TP, _TP, ctypes.c_void_p, ctypes.c_int32, _I32P,
                                               _I32P, ctypes.c_int32, ctypes.c_void_p, ctypes.c_size_t,
                                               ctypes.c_void_p]
    lib.ba_block_attention_prompts_workspace_bytes.restype = ctypes.c_size_t
    lib.ba_block_attention_prompts_workspace_bytes.argtypes = [_HP, ctypes.c_int32, _I32P, _I32P, ctypes.c_int32,
                                                               ctypes.c_int32]
    _lib = lib
    return lib


def _check(status: int) -> None:
    if status != BA_OK:
        lib = load()
        raise BaError(status, lib.ba_status_string(status).decode(), lib.ba_last_error().decode())


class Heads:
    """Host-side head description (ba_heads) that keeps its arrays alive."""

    def __init__(self, n_q_heads: int, n_kv_heads: int, head_dim: int, rope_base: float = 10000.0,
                 rope_layout: int = ROPE_INTERLEAVED, softmax_scale: float = 0.0,
                 q_to_kv: Optional[Sequence[int]] = None, inv_freq: Optional[Sequence[float]] = None):
        self._q_to_kv = None if q_to_kv is None else np.ascontiguousarray(q_to_kv, dtype=np.int32)
        self._inv_freq = None if inv_freq is None else np.ascontiguousarray(inv_freq, dtype=np.float64)
        self.c = BaHeads(n_q_heads, n_kv_heads, head_dim,
                         None if self._q_to_kv is None else self._q_to_kv.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                         float(softmax_scale), float(rope_base),
                         None if self._inv_freq is None else self._inv_freq.ctypes.data_as(ctypes.POINTER(ctypes.c_double)),
                         rope_layout)
        self.n_q_heads, self.n_kv_heads, self.head_dim = n_q_heads, n_kv_heads, head_dim


_dtype_codes = None  # torch dtype -> BA_DTYPE_*, filled on first use (torch is imported lazily)


def _tensor(t, dtype_code: Optional[int] = None) -> Optional[BaTensor]:
    """[tokens, heads, D] torch tensor (any token / head strides, D contiguous)."""
    global _dtype_codes
    if t is None:
        return None
    st = t.stride()
    if len(st) != 3 or st[2] != 1:
        raise ValueError("expected a [tokens, heads, head_dim] tensor with contiguous head_dim")
    if dtype_code is None:
        if _dtype_codes is None:
            import torch
            _dtype_codes = {torch.float32: DTYPE_F32, torch.bfloat16: DTYPE_BF16}
        dtype_code = _dtype_codes.get(t.dtype)
        if dtype_code is None:
            raise ValueError(f"dtype {t.dtype} not supported")
    return BaTensor(t.data_ptr(), st[0], st[1], dtype_code)


def _ref(x):
    return None if x is None else ctypes.byref(x)


def _ints(a) -> Optional[np.ndarray]:
    return None if a is None else np.ascontiguousarray(a, dtype=np.int32)


def _ip(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data


_raw_stream = None  # fast path to the current stream's handle, looked up once


def _stream_handle(stream) -> int:
    global _raw_stream
    if stream is not None:
        return int(stream.cuda_stream)
    import torch
    if _raw_stream is None:
        _raw_stream = getattr(torch._C, "_cuda_getCurrentRawStream", False)
    if _raw_stream:
        return int(_raw_stream(torch.cuda.current_device()))
    return int(torch.cuda.current_stream().cuda_stream)


def _ws(ws):
    if ws is None:
        return None, 0
    return ctypes.c_void_p(ws.data_ptr()), ws.numel() * ws.element_size()


def ba_version() -> int:
    return int(load().ba_version())


PROFILE_ATTENTION, PROFILE_REENCODE, PROFILE_COMBINE, PROFILE_CLASSES = 0, 1, 2, 3


def ba_profile_begin(max_records: int = 65536) -> None:
    _check(load().ba_profile_begin(max_records))


def ba_profile_end():
    """Returns (ms_sum[3], launches[3]) indexed by PROFILE_*."""
    ms = (ctypes.c_double * PROFILE_CLASSES)()
    n = (ctypes.c_int32 * PROFILE_CLASSES)()
    _check(load().ba_profile_end(ms, n))
    return list(ms), list(n)


def ba_encode_blocks_workspace_bytes(heads: Heads, block_offsets, rope_mode: int = ROPE_APPLY,
                                     have_k_local_out: bool = False) -> int:
    offs = _ints(block_offsets)
    return int(load().ba_encode_blocks_workspace_bytes(ctypes.byref(heads.c), len(offs) - 1, _ip(offs),
                                                       rope_mode, int(have_k_local_out)))


def ba_encode_blocks(heads: Heads, q, k, v, o_out, k_local_out, block_offsets, rope_mode: int = ROPE_APPLY,
                     ws=None, stream=None) -> None:
    offs = _ints(block_offsets)
    wp, wb = _ws(ws)
    tq, tk, tv, to, tkl = _tensor(q), _tensor(k), _tensor(v), _tensor(o_out), _tensor(k_local_out)
    _check(load().ba_encode_blocks(ctypes.byref(heads.c), _ref(tq), _ref(tk), _ref(tv), _ref(to), _ref(tkl),
                                   len(offs) - 1, _ip(offs), rope_mode, wp, wb, _stream_handle(stream)))


def ba_reencode_positions(heads: Heads, k_src, k_dst, src_tok_off, dst_tok_off, lens, old_pos0=None,
                          new_pos0=None, mode: int = REENC_SHIFT, stream=None) -> None:
    """k_src / k_dst: [layers, tokens, heads, D] (or [tokens, heads, D] for one layer)."""
    if k_src.dim() == 3:
        k_src, k_dst = k_src[None], k_dst[None]
    n_layers = k_src.shape[0]
    ts, td = _tensor(k_src[0]), _tensor(k_dst[0])
    so, do, ln = _ints(src_tok_off), _ints(dst_tok_off), _ints(lens)
    op, npos = _ints(old_pos0), _ints(new_pos0)
    _check(load().ba_reencode_positions(ctypes.byref(heads.c), _ref(ts), _ref(td), n_layers, k_src.stride(0),
                                        k_dst.stride(0), len(ln), _ip(so), _ip(do), _ip(ln), _ip(op), _ip(npos),
                                        mode, _stream_handle(stream)))


def ba_final_block_attention_workspace_bytes(heads: Heads, cu_q, cu_ctx, rope_mode: int = ROPE_APPLY,
                                             have_k_f_rot_out: bool = False) -> int:
    cq, cc = _ints(cu_q), _ints(cu_ctx)
    return int(load().ba_final_block_attention_workspace_bytes(ctypes.byref(heads.c), len(cq) - 1, _ip(cq),
                                                               _ip(cc), rope_mode, int(have_k_f_rot_out)))


def ba_final_block_attention(heads: Heads, q_f, k_ctx, v_ctx, k_f, v_f, o_out, k_f_rot_out, cu_q, cu_ctx,
                             q_pos0=None, rope_mode: int = ROPE_APPLY, ws=None, stream=None) -> None:
    cq, cc, qp = _ints(cu_q), _ints(cu_ctx), _ints(q_pos0)
    wp, wb = _ws(ws)
    tq, tkc, tvc = _tensor(q_f), _tensor(k_ctx), _tensor(v_ctx)
    tkf, tvf, to, tkr = _tensor(k_f), _tensor(v_f), _tensor(o_out), _tensor(k_f_rot_out)
    _check(load().ba_final_block_attention(ctypes.byref(heads.c), _ref(tq), _ref(tkc), _ref(tvc), _ref(tkf),
                                           _ref(tvf), _ref(to), _ref(tkr), len(cq) - 1, _ip(cq), _ip(cc),
                                           _ip(qp), rope_mode, wp, wb, _stream_handle(stream)))


STATIC_SCRATCH_BYTES = 32 << 20


def ba_final_block_attention_static(heads: Heads, q_f, k_ctx, v_ctx, k_f, v_f, o_out, k_f_rot_out, cu_q, cu_ctx,
                                    q_pos0=None, rope_mode: int = ROPE_APPLY, stream=None) -> None:
    """ba_final_block_attention with the workspace in the library's static device array (no allocation)."""
    cq, cc, qp = _ints(cu_q), _ints(cu_ctx), _ints(q_pos0)
    tq, tkc, tvc = _tensor(q_f), _tensor(k_ctx), _tensor(v_ctx)
    tkf, tvf, to, tkr = _tensor(k_f), _tensor(v_f), _tensor(o_out), _tensor(k_f_rot_out)
    _check(load().ba_final_block_attention_static(ctypes.byref(heads.c), _ref(tq), _ref(tkc), _ref(tvc), _ref(tkf),
                                                  _ref(tvf), _ref(to), _ref(tkr), len(cq) - 1, _ip(cq), _ip(cc),
                                                  _ip(qp), rope_mode, _stream_handle(stream)))


def ba_final_block_attention_cached_workspace_bytes(heads: Heads, cu_q, cu_blk, blk_len,
                                                    have_k_f_rot_out: bool = False) -> int:
    cq, cb, bl = _ints(cu_q), _ints(cu_blk), _ints(blk_len)
    return int(load().ba_final_block_attention_cached_workspace_bytes(ctypes.byref(heads.c), len(cq) - 1, _ip(cq),
                                                                      _ip(cb), _ip(bl), int(have_k_f_rot_out)))


def ba_final_block_attention_cached(heads: Heads, q_f, k_cache, v_cache, k_f, v_f, o_out, k_f_rot_out, cu_q, cu_blk,
                                    blk_tok_off, blk_len, blk_old_pos0=None, blk_new_pos0=None, q_pos0=None,
                                    ws=None, stream=None) -> None:
    cq, cb = _ints(cu_q), _ints(cu_blk)
    bo, bl, op, npos, qp = _ints(blk_tok_off), _ints(blk_len), _ints(blk_old_pos0), _ints(blk_new_pos0), _ints(q_pos0)
    wp, wb = _ws(ws)
    tq, tkc, tvc = _tensor(q_f), _tensor(k_cache), _tensor(v_cache)
    tkf, tvf, to, tkr = _tensor(k_f), _tensor(v_f), _tensor(o_out), _tensor(k_f_rot_out)
    _check(load().ba_final_block_attention_cached(ctypes.byref(heads.c), _ref(tq), _ref(tkc), _ref(tvc), _ref(tkf),
                                                  _ref(tvf), _ref(to), _ref(tkr), len(cq) - 1, _ip(cq), _ip(cb),
                                                  _ip(bo), _ip(bl), _ip(op), _ip(npos), _ip(qp), wp, wb,
                                                  _stream_handle(stream)))


def ba_block_attention_prompts_workspace_bytes(heads: Heads, cu_blk, block_offsets, rope_mode: int = ROPE_APPLY,
                                               have_k_rot_out: bool = False) -> int:
    cb, offs = _ints(cu_blk), _ints(block_offsets)
    return int(load().ba_block_attention_prompts_workspace_bytes(ctypes.byref(heads.c), len(cb) - 1, _ip(cb),
                                                                 _ip(offs), rope_mode, int(have_k_rot_out)))


def ba_block_attention_prompts(heads: Heads, q, k, v, o_out, k_rot_out, lse_out, cu_blk, block_offsets,
                               rope_mode: int = ROPE_APPLY, ws=None, stream=None) -> None:
    """lse_out: float32 tensor [T, n_q_heads] (contiguous) or None."""
    cb, offs = _ints(cu_blk), _ints(block_offsets)
    wp, wb = _ws(ws)
    tq, tk, tv, to, tkr = _tensor(q), _tensor(k), _tensor(v), _tensor(o_out), _tensor(k_rot_out)
    lse_p = None if lse_out is None else ctypes.c_void_p(lse_out.data_ptr())
    _check(load().ba_block_attention_prompts(ctypes.byref(heads.c), _ref(tq), _ref(tk), _ref(tv), _ref(to), _ref(tkr),
                                             lse_p, len(cb) - 1, _ip(cb), _ip(offs), rope_mode, wp, wb,
                                             _stream_handle(stream)))


def ba_set_gather_below(mean_block_tokens: int) -> int:
    """Mean cached-block length below which ba_final_block_attention_cached gathers; returns the old value."""
    return int(load().ba_set_gather_below(int(mean_block_tokens)))


def ba_block_attention_prompts_backward_workspace_bytes(heads: Heads, cu_blk, block_offsets) -> int:
    cb, offs = _ints(cu_blk), _ints(block_offsets)
    return int(load().ba_block_attention_prompts_backward_workspace_bytes(ctypes.byref(heads.c), len(cb) - 1, _ip(cb),
                                                                          _ip(offs)))


def ba_block_attention_prompts_backward(heads: Heads, q, k, v, o, lse, d_out, dq_out, dk_out, dv_out, cu_blk,
                                        block_offsets, ws=None, stream=None) -> None:
    """lse: the forward call's float32 [T, n_q_heads] tensor."""
    cb, offs = _ints(cu_blk), _ints(block_offsets)
    wp, wb = _ws(ws)
    ts = [_tensor(x) for x in (q, k, v, o, d_out, dq_out, dk_out, dv_out)]
    _check(load().ba_block_attention_prompts_backward(ctypes.byref(heads.c), _ref(ts[0]), _ref(ts[1]), _ref(ts[2]),
                                                      _ref(ts[3]), ctypes.c_void_p(lse.data_ptr()), _ref(ts[4]),
                                                      _ref(ts[5]), _ref(ts[6]), _ref(ts[7]), len(cb) - 1, _ip(cb),
                                                      _ip(offs), wp, wb, _stream_handle(stream)))
