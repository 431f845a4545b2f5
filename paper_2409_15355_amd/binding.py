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
           "ba_block_attention_prompts", "ba_block_attention_prompts_workspace_bytes",
           "ba_block_attention_prompts_backward", "ba_block_attention_prompts_backward_workspace_bytes",
           "ba_schedule_final_block", "ba_schedule_encode_blocks", "ba_schedule_prompts",
           "ba_measure_xcd_speed", "ba_measure_xcd_speed_workspace_bytes", "ba_diag_final_block_phases",
           "ba_diag_mfma_ceiling", "ba_diag_mfma_ceiling_workspace_bytes"]


class BaTensor(ctypes.Structure):
    _fields_ = [("ptr", ctypes.c_void_p), ("stride_tok", ctypes.c_int64),
                ("stride_head", ctypes.c_int64), ("dtype", ctypes.c_int32)]


class BaHeads(ctypes.Structure):
    _fields_ = [("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("q_to_kv", ctypes.POINTER(ctypes.c_int32)),
                ("softmax_scale", ctypes.c_float), ("rope_base", ctypes.c_double),
                ("inv_freq", ctypes.POINTER(ctypes.c_double)), ("rope_layout", ctypes.c_int32),
                ("xcd_speed", ctypes.POINTER(ctypes.c_float))]


class BaWorkItem(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("launch", "problem", "first_token", "tile_rows", "tile_keys", "row_begin",
                                               "row_end", "split", "n_splits", "ctx_begin", "ctx_end", "self_begin",
                                               "self_end", "kv_head", "xcd")]


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
                                                    _I32P, _I32P, _I32P, _I32P, _I32P, _I32P, ctypes.c_int32,
                                                    ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    lib.ba_final_block_attention_cached_workspace_bytes.restype = ctypes.c_size_t
    lib.ba_final_block_attention_cached_workspace_bytes.argtypes = [_HP, ctypes.c_int32, _I32P, _I32P, _I32P,
                                                                    ctypes.c_int32, ctypes.c_int32]
    lib.ba_block_attention_prompts_backward.restype = ctypes.c_int32
    lib.ba_block_attention_prompts_backward.argtypes = [_HP, _TP, _TP, _TP, _TP, ctypes.c_void_p, _TP, _TP, _TP, _TP,
                                                        ctypes.c_int32, _I32P, _I32P, ctypes.c_void_p, ctypes.c_size_t,
                                                        ctypes.c_void_p]
    lib.ba_block_attention_prompts_backward_workspace_bytes.restype = ctypes.c_size_t
    lib.ba_block_attention_prompts_backward_workspace_bytes.argtypes = [_HP, ctypes.c_int32, _I32P, _I32P]
    lib.ba_block_attention_prompts.restype = ctypes.c_int32
    lib.ba_block_attention_prompts.argtypes = [_HP, _TP, _TP, _TP, _TP, _TP, ctypes.c_void_p, ctypes.c_int32, _I32P,
                                               _I32P, ctypes.c_int32, ctypes.c_void_p, ctypes.c_size_t,
                                               ctypes.c_void_p]
    lib.ba_block_attention_prompts_workspace_bytes.restype = ctypes.c_size_t
    lib.ba_block_attention_prompts_workspace_bytes.argtypes = [_HP, ctypes.c_int32, _I32P, _I32P, ctypes.c_int32,
                                                               ctypes.c_int32]
    _WP = ctypes.POINTER(BaWorkItem)
    lib.ba_schedule_final_block.restype = ctypes.c_int64
    lib.ba_schedule_final_block.argtypes = [_HP, ctypes.c_int32, _I32P, _I32P, ctypes.c_int32, _WP, ctypes.c_int64]
    lib.ba_schedule_encode_blocks.restype = ctypes.c_int64
    lib.ba_schedule_encode_blocks.argtypes = [_HP, ctypes.c_int32, _I32P, _WP, ctypes.c_int64]
    lib.ba_schedule_prompts.restype = ctypes.c_int64
    lib.ba_schedule_prompts.argtypes = [_HP, ctypes.c_int32, _I32P, _I32P, _WP, ctypes.c_int64]
    lib.ba_diag_mfma_ceiling.restype = ctypes.c_int32
    lib.ba_diag_mfma_ceiling.argtypes = [ctypes.c_int32, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double),
                                         ctypes.POINTER(ctypes.c_double), ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    lib.ba_diag_mfma_ceiling_workspace_bytes.restype = ctypes.c_size_t
    lib.ba_diag_mfma_ceiling_workspace_bytes.argtypes = []
    lib.ba_measure_xcd_speed.restype = ctypes.c_int32
    lib.ba_measure_xcd_speed.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    lib.ba_diag_final_block_phases.restype = ctypes.c_int32
    lib.ba_diag_final_block_phases.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_float), ctypes.c_void_p,
                                               ctypes.c_size_t, ctypes.c_void_p]
    lib.ba_measure_xcd_speed_workspace_bytes.restype = ctypes.c_size_t
    lib.ba_measure_xcd_speed_workspace_bytes.argtypes = []
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
                 q_to_kv: Optional[Sequence[int]] = None, inv_freq: Optional[Sequence[float]] = None,
                 xcd_speed: Optional[Sequence[float]] = None):
        self._q_to_kv = None if q_to_kv is None else np.ascontiguousarray(q_to_kv, dtype=np.int32)
        self._inv_freq = None if inv_freq is None else np.ascontiguousarray(inv_freq, dtype=np.float64)
        self._xcd_speed = None if xcd_speed is None else np.ascontiguousarray(xcd_speed, dtype=np.float32)
        if self._xcd_speed is not None and self._xcd_speed.shape != (8,):
            raise ValueError("xcd_speed: eight numbers, one per XCD")
        self.c = BaHeads(n_q_heads, n_kv_heads, head_dim,
                         None if self._q_to_kv is None else self._q_to_kv.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                         float(softmax_scale), float(rope_base),
                         None if self._inv_freq is None else self._inv_freq.ctypes.data_as(ctypes.POINTER(ctypes.c_double)),
                         rope_layout,
                         None if self._xcd_speed is None else self._xcd_speed.ctypes.data_as(ctypes.POINTER(ctypes.c_float)))
        self.n_q_heads, self.n_kv_heads, self.head_dim = n_q_heads, n_kv_heads, head_dim


_dtype_codes = None  # torch dtype -> BA_DTYPE_*, filled on first use (torch is imported lazily)


def _tensor(t, name: str = "tensor", n_heads: Optional[int] = None, head_dim: Optional[int] = None,
            min_tokens: int = 0, allow_f32: bool = False) -> Optional[BaTensor]:
    """[tokens, heads, D] torch tensor on the GPU (any token / head strides, D contiguous).

    The C boundary sees a pointer and two strides, not an extent: everything it cannot check is
    checked here, before anything is launched -- the device, the dtype, heads and head_dim against
    the call's head description, and that the tensor has at least the rows the call's offset
    arrays reach."""
    global _dtype_codes
    if t is None:
        return None
    if _dtype_codes is None:
        import torch
        _dtype_codes = {torch.float32: DTYPE_F32, torch.bfloat16: DTYPE_BF16}
    if not getattr(t, "is_cuda", False):
        raise ValueError(f"{name}: expected a tensor in GPU memory, got one on {getattr(t, 'device', '?')}")
    dtype_code = _dtype_codes.get(t.dtype)
    if dtype_code is None or (dtype_code == DTYPE_F32 and not allow_f32):
        raise ValueError(f"{name}: dtype {t.dtype} not supported here")
    st, shp = t.stride(), tuple(t.shape)
    if len(st) != 3 or (shp[2] > 1 and st[2] != 1):
        raise ValueError(f"{name}: expected a [tokens, heads, head_dim] tensor with contiguous head_dim")
    if n_heads is not None and shp[1] != n_heads:
        raise ValueError(f"{name}: {shp[1]} heads, the call's head description says {n_heads}")
    if head_dim is not None and shp[2] != head_dim:
        raise ValueError(f"{name}: head_dim {shp[2]}, the call's head description says {head_dim}")
    if shp[0] < min_tokens:
        raise ValueError(f"{name}: {shp[0]} tokens, the call's offsets reach {min_tokens}")
    return BaTensor(t.data_ptr(), st[0], st[1], dtype_code)


def _last(a: Optional[np.ndarray]) -> int:
    """Rows a cumulative offset array reaches (0 for none)."""
    return int(a[-1]) if a is not None and len(a) else 0


def _reach(off: Optional[np.ndarray], ln: Optional[np.ndarray]) -> int:
    """Rows that blocks [off[b], off[b] + len[b]) reach (empty blocks touch nothing)."""
    if off is None or ln is None or not len(ln):
        return 0
    if len(off) != len(ln):
        raise ValueError("per-block arrays of different lengths")
    live = ln > 0
    return int((off[live].astype(np.int64) + ln[live]).max()) if live.any() else 0


def _same_len(n: int, **arrays) -> None:
    for name, a in arrays.items():
        if a is not None and len(a) != n:
            raise ValueError(f"{name}: {len(a)} entries, expected {n}")


def _lse(t, name: str, tokens: int, n_q_heads: int):
    """float32 [tokens, n_q_heads], contiguous, on the GPU -> pointer (None stays None)."""
    if t is None:
        return None
    import torch
    if not t.is_cuda or t.dtype != torch.float32 or t.dim() != 2 or not t.is_contiguous():
        raise ValueError(f"{name}: expected a contiguous float32 [tokens, n_q_heads] tensor in GPU memory")
    if t.shape[1] != n_q_heads or t.shape[0] < tokens:
        raise ValueError(f"{name}: shape {tuple(t.shape)}, the call needs [{tokens}, {n_q_heads}]")
    return ctypes.c_void_p(t.data_ptr())


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
    if not getattr(ws, "is_cuda", False) or not ws.is_contiguous():
        raise ValueError("workspace: expected a contiguous tensor in GPU memory")
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
    T, hq, hkv, d = _last(offs), heads.n_q_heads, heads.n_kv_heads, heads.head_dim
    tq, tk, tv = _tensor(q, "q", hq, d, T), _tensor(k, "k", hkv, d, T), _tensor(v, "v", hkv, d, T)
    to, tkl = _tensor(o_out, "o_out", hq, d, T), _tensor(k_local_out, "k_local_out", hkv, d, T)
    _check(load().ba_encode_blocks(ctypes.byref(heads.c), _ref(tq), _ref(tk), _ref(tv), _ref(to), _ref(tkl),
                                   len(offs) - 1, _ip(offs), rope_mode, wp, wb, _stream_handle(stream)))


def ba_reencode_positions(heads: Heads, k_src, k_dst, src_tok_off, dst_tok_off, lens, old_pos0=None,
                          new_pos0=None, mode: int = REENC_SHIFT, stream=None) -> None:
    """k_src / k_dst: [layers, tokens, heads, D] (or [tokens, heads, D] for one layer)."""
    if k_src.dim() == 3:
        k_src, k_dst = k_src[None], k_dst[None]
    if k_src.dim() != 4 or k_dst.dim() != 4 or k_src.shape[0] != k_dst.shape[0]:
        raise ValueError("k_src / k_dst: expected [layers, tokens, heads, head_dim] with equal layer counts")
    n_layers = k_src.shape[0]
    so, do, ln = _ints(src_tok_off), _ints(dst_tok_off), _ints(lens)
    op, npos = _ints(old_pos0), _ints(new_pos0)
    _same_len(len(ln), src_tok_off=so, dst_tok_off=do, old_pos0=op, new_pos0=npos)
    hkv, d = heads.n_kv_heads, heads.head_dim
    if n_layers == 0:
        return
    ts = _tensor(k_src[0], "k_src", hkv, d, _reach(so, ln), allow_f32=True)
    td = _tensor(k_dst[0], "k_dst", hkv, d, _reach(do, ln), allow_f32=True)
    _check(load().ba_reencode_positions(ctypes.byref(heads.c), _ref(ts), _ref(td), n_layers, k_src.stride(0),
                                        k_dst.stride(0), len(ln), _ip(so), _ip(do), _ip(ln), _ip(op), _ip(npos),
                                        mode, _stream_handle(stream)))


def _final_tensors(heads: Heads, q_f, k_ctx, v_ctx, k_f, v_f, o_out, k_f_rot_out, cq, cc, qp):
    if len(cq) != len(cc):
        raise ValueError("cu_q and cu_ctx: one entry per prompt plus one, each")
    _same_len(len(cq) - 1, q_pos0=qp)
    hq, hkv, d, tq_, tc_ = heads.n_q_heads, heads.n_kv_heads, heads.head_dim, _last(cq), _last(cc)
    return (_tensor(q_f, "q_f", hq, d, tq_), _tensor(k_ctx, "k_ctx", hkv, d, tc_), _tensor(v_ctx, "v_ctx", hkv, d, tc_),
            _tensor(k_f, "k_f", hkv, d, tq_), _tensor(v_f, "v_f", hkv, d, tq_), _tensor(o_out, "o_out", hq, d, tq_),
            _tensor(k_f_rot_out, "k_f_rot_out", hkv, d, tq_))


def ba_final_block_attention_workspace_bytes(heads: Heads, cu_q, cu_ctx, rope_mode: int = ROPE_APPLY,
                                             have_k_f_rot_out: bool = False) -> int:
    cq, cc = _ints(cu_q), _ints(cu_ctx)
    return int(load().ba_final_block_attention_workspace_bytes(ctypes.byref(heads.c), len(cq) - 1, _ip(cq),
                                                               _ip(cc), rope_mode, int(have_k_f_rot_out)))


def ba_final_block_attention(heads: Heads, q_f, k_ctx, v_ctx, k_f, v_f, o_out, k_f_rot_out, cu_q, cu_ctx,
                             q_pos0=None, rope_mode: int = ROPE_APPLY, ws=None, stream=None) -> None:
    cq, cc, qp = _ints(cu_q), _ints(cu_ctx), _ints(q_pos0)
    wp, wb = _ws(ws)
    tq, tkc, tvc, tkf, tvf, to, tkr = _final_tensors(heads, q_f, k_ctx, v_ctx, k_f, v_f, o_out, k_f_rot_out, cq, cc, qp)
    _check(load().ba_final_block_attention(ctypes.byref(heads.c), _ref(tq), _ref(tkc), _ref(tvc), _ref(tkf),
                                           _ref(tvf), _ref(to), _ref(tkr), len(cq) - 1, _ip(cq), _ip(cc),
                                           _ip(qp), rope_mode, wp, wb, _stream_handle(stream)))


STATIC_SCRATCH_BYTES = 32 << 20


def ba_final_block_attention_static(heads: Heads, q_f, k_ctx, v_ctx, k_f, v_f, o_out, k_f_rot_out, cu_q, cu_ctx,
                                    q_pos0=None, rope_mode: int = ROPE_APPLY, stream=None) -> None:
    """ba_final_block_attention with the workspace in the library's static device array (no allocation)."""
    cq, cc, qp = _ints(cu_q), _ints(cu_ctx), _ints(q_pos0)
    tq, tkc, tvc, tkf, tvf, to, tkr = _final_tensors(heads, q_f, k_ctx, v_ctx, k_f, v_f, o_out, k_f_rot_out, cq, cc, qp)
    _check(load().ba_final_block_attention_static(ctypes.byref(heads.c), _ref(tq), _ref(tkc), _ref(tvc), _ref(tkf),
                                                  _ref(tvf), _ref(to), _ref(tkr), len(cq) - 1, _ip(cq), _ip(cc),
                                                  _ip(qp), rope_mode, _stream_handle(stream)))


GATHER_DEFAULT = -1


def ba_final_block_attention_cached_workspace_bytes(heads: Heads, cu_q, cu_blk, blk_len,
                                                    have_k_f_rot_out: bool = False,
                                                    gather_below: int = GATHER_DEFAULT) -> int:
    cq, cb, bl = _ints(cu_q), _ints(cu_blk), _ints(blk_len)
    return int(load().ba_final_block_attention_cached_workspace_bytes(ctypes.byref(heads.c), len(cq) - 1, _ip(cq),
                                                                      _ip(cb), _ip(bl), int(have_k_f_rot_out),
                                                                      int(gather_below)))


def ba_final_block_attention_cached(heads: Heads, q_f, k_cache, v_cache, k_f, v_f, o_out, k_f_rot_out, cu_q, cu_blk,
                                    blk_tok_off, blk_len, blk_old_pos0=None, blk_new_pos0=None, q_pos0=None,
                                    ws=None, stream=None, gather_below: int = GATHER_DEFAULT) -> None:
    """gather_below: mean cached-block length (tokens) below which the context is gathered first
    (GATHER_DEFAULT: 256; 0: never); pass the same value to the workspace query."""
    cq, cb = _ints(cu_q), _ints(cu_blk)
    bo, bl, op, npos, qp = _ints(blk_tok_off), _ints(blk_len), _ints(blk_old_pos0), _ints(blk_new_pos0), _ints(q_pos0)
    wp, wb = _ws(ws)
    if len(cq) != len(cb):
        raise ValueError("cu_q and cu_blk: one entry per prompt plus one, each")
    _same_len(_last(cb), blk_tok_off=bo, blk_len=bl, blk_old_pos0=op, blk_new_pos0=npos)
    _same_len(len(cq) - 1, q_pos0=qp)
    hq, hkv, d, tq_, tc_ = heads.n_q_heads, heads.n_kv_heads, heads.head_dim, _last(cq), _reach(bo, bl)
    tq, tkc, tvc = _tensor(q_f, "q_f", hq, d, tq_), _tensor(k_cache, "k_cache", hkv, d, tc_), _tensor(v_cache, "v_cache", hkv, d, tc_)
    tkf, tvf = _tensor(k_f, "k_f", hkv, d, tq_), _tensor(v_f, "v_f", hkv, d, tq_)
    to, tkr = _tensor(o_out, "o_out", hq, d, tq_), _tensor(k_f_rot_out, "k_f_rot_out", hkv, d, tq_)
    _check(load().ba_final_block_attention_cached(ctypes.byref(heads.c), _ref(tq), _ref(tkc), _ref(tvc), _ref(tkf),
                                                  _ref(tvf), _ref(to), _ref(tkr), len(cq) - 1, _ip(cq), _ip(cb),
                                                  _ip(bo), _ip(bl), _ip(op), _ip(npos), _ip(qp), int(gather_below),
                                                  wp, wb, _stream_handle(stream)))


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
    if _last(cb) != len(offs) - 1:
        raise ValueError("block_offsets: one entry per block of cu_blk plus one")
    T, hq, hkv, d = _last(offs), heads.n_q_heads, heads.n_kv_heads, heads.head_dim
    tq, tk, tv = _tensor(q, "q", hq, d, T), _tensor(k, "k", hkv, d, T), _tensor(v, "v", hkv, d, T)
    to, tkr = _tensor(o_out, "o_out", hq, d, T), _tensor(k_rot_out, "k_rot_out", hkv, d, T)
    lse_p = _lse(lse_out, "lse_out", T, hq)
    _check(load().ba_block_attention_prompts(ctypes.byref(heads.c), _ref(tq), _ref(tk), _ref(tv), _ref(to), _ref(tkr),
                                             lse_p, len(cb) - 1, _ip(cb), _ip(offs), rope_mode, wp, wb,
                                             _stream_handle(stream)))


def ba_block_attention_prompts_backward_workspace_bytes(heads: Heads, cu_blk, block_offsets) -> int:
    cb, offs = _ints(cu_blk), _ints(block_offsets)
    return int(load().ba_block_attention_prompts_backward_workspace_bytes(ctypes.byref(heads.c), len(cb) - 1, _ip(cb),
                                                                          _ip(offs)))


def ba_block_attention_prompts_backward(heads: Heads, q, k, v, o, lse, d_out, dq_out, dk_out, dv_out, cu_blk,
                                        block_offsets, ws=None, stream=None) -> None:
    """lse: the forward call's float32 [T, n_q_heads] tensor."""
    cb, offs = _ints(cu_blk), _ints(block_offsets)
    wp, wb = _ws(ws)
    if _last(cb) != len(offs) - 1:
        raise ValueError("block_offsets: one entry per block of cu_blk plus one")
    T, hq, hkv, d = _last(offs), heads.n_q_heads, heads.n_kv_heads, heads.head_dim
    if lse is None:
        raise ValueError("lse: the forward call's log-sum-exps are needed")
    ts = [_tensor(x, nm, nh, d, T) for x, nm, nh in ((q, "q", hq), (k, "k", hkv), (v, "v", hkv), (o, "o", hq),
                                                     (d_out, "d_out", hq), (dq_out, "dq_out", hq),
                                                     (dk_out, "dk_out", hkv), (dv_out, "dv_out", hkv))]
    _check(load().ba_block_attention_prompts_backward(ctypes.byref(heads.c), _ref(ts[0]), _ref(ts[1]), _ref(ts[2]),
                                                      _ref(ts[3]), _lse(lse, "lse", T, hq), _ref(ts[4]),
                                                      _ref(ts[5]), _ref(ts[6]), _ref(ts[7]), len(cb) - 1, _ip(cb),
                                                      _ip(offs), wp, wb, _stream_handle(stream)))


def _schedule(fn, *args):
    """Two calls: count the work items, then fetch them.  Returns a list of BaWorkItem."""
    n = int(fn(*args, None, 0))
    if n < 0:
        _check(n)
    items = (BaWorkItem * max(n, 1))()
    got = int(fn(*args, items, n))
    if got < 0:
        _check(got)
    return list(items[:got])


def ba_schedule_final_block(heads: Heads, cu_q, cu_ctx, n_compute_units: int = 256):
    """Work items of ba_final_block_attention (host only; see include/ba.h)."""
    cq, cc = _ints(cu_q), _ints(cu_ctx)
    return _schedule(load().ba_schedule_final_block, ctypes.byref(heads.c), len(cq) - 1, _ip(cq), _ip(cc),
                     int(n_compute_units))


def ba_schedule_encode_blocks(heads: Heads, block_offsets):
    offs = _ints(block_offsets)
    return _schedule(load().ba_schedule_encode_blocks, ctypes.byref(heads.c), len(offs) - 1, _ip(offs))


def ba_schedule_prompts(heads: Heads, cu_blk, block_offsets):
    cb, offs = _ints(cu_blk), _ints(block_offsets)
    return _schedule(load().ba_schedule_prompts, ctypes.byref(heads.c), len(cb) - 1, _ip(cb), _ip(offs))


def ba_measure_xcd_speed_workspace_bytes() -> int:
    return int(load().ba_measure_xcd_speed_workspace_bytes())


def ba_measure_xcd_speed(ws, stream=None):
    """Eight relative XCD speeds (mean 1) for Heads(xcd_speed=...); synchronises the stream."""
    out = (ctypes.c_float * 8)()
    wp, wb = _ws(ws)
    _check(load().ba_measure_xcd_speed(out, wp, wb, _stream_handle(stream)))
    return [float(x) for x in out]


DIAG_PHASES = ("entry_to_first_copies_issued", "to_first_tiles_and_queries_landed", "to_loop_entered", "walk",
               "walk_end_to_partials_stored", "workgroup_lifetime", "launch_first_entry_to_last_store", "longest_walk")


def ba_diag_final_block_phases(ws, xcd_speed=None, stream=None) -> dict:
    """Microseconds per phase of one final-block launch (see include/ba.h); ws as for ba_measure_xcd_speed."""
    out = (ctypes.c_double * len(DIAG_PHASES))()
    wp, wb = _ws(ws)
    sp = None
    if xcd_speed is not None:
        if len(xcd_speed) != 8:
            raise ValueError("xcd_speed: eight numbers")
        sp = (ctypes.c_float * 8)(*[float(x) for x in xcd_speed])
    _check(load().ba_diag_final_block_phases(out, sp, wp, wb, _stream_handle(stream)))
    return {k: float(v) for k, v in zip(DIAG_PHASES, out)}


def ba_diag_mfma_ceiling(lds_reads_per_two_mfma: int, stream=None) -> dict:
    """Sustained MFMA rate on data-like operands (see include/ba.h); synchronises the stream."""
    import torch
    ws = torch.empty(int(load().ba_diag_mfma_ceiling_workspace_bytes()), dtype=torch.uint8, device="cuda")
    t, c, b = ctypes.c_double(), ctypes.c_double(), ctypes.c_double()
    wp, wb = _ws(ws)
    _check(load().ba_diag_mfma_ceiling(int(lds_reads_per_two_mfma), ctypes.byref(t), ctypes.byref(c), ctypes.byref(b), wp, wb,
                                       _stream_handle(stream)))
    return {"TFLOPs": t.value, "clock_GHz": c.value, "pipe_busy": b.value}
