"""Block-attention oracle (CPU, fp64) -- TEST INFRASTRUCTURE ONLY.

Python face of ``ba_oracle.c`` plus two NumPy-only functions (a dense brute-force
masked attention and the split-softmax merge).  Only ``tests/``, the smoke check and
the benchmark's ``cpu_baseline`` leg may import this package; the product package
never does, and this package never imports the product.

Every tensor is a NumPy float64 array, packed token-major ``[tokens, heads, D]``.
bf16 inputs are up-cast exactly with :func:`bf16_bits_to_f64` first.

What each function follows in arXiv 2409.15355:

* :func:`theta`, :func:`rope` -- Eq. 1 (and its transpose, Eq. 2).
* :func:`encode_blocks` -- Section 1 step 1, Section 2.1: per-block causal attention
  at local positions (first token of a block at position 0, Section 2.3).
* :func:`reencode` -- Section 2.3, Eq. 2 then Eq. 3, no rounding in between.
* :func:`final_block` -- Section 1 step 3, Section 2.5.
* :func:`masked_attention_bruteforce` -- Section 2.4: the lower-triangular mask
  modified so that only the last block sees other blocks; dense softmax.
* :func:`masked_attention_backward_bruteforce` -- the gradient of the same function
  (Section 2.4's mask inside a block fine-tune step), by the chain rule written out.
* :func:`merge_partials` -- softmax associativity (not in the paper; pins the
  split-KV combine).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ba_oracle.c")
_LIB = os.path.join(_HERE, "libba_oracle.so")

LAYOUT_INTERLEAVED = 0
LAYOUT_HALF = 1
ROPE_NONE = 0
ROPE_APPLY = 1
REENC_SHIFT = 0
REENC_ABSOLUTE = 1

_lib = None


def build(force: bool = False) -> str:
    """Compile ba_oracle.c with gcc (OpenMP).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_D = ctypes.POINTER(ctypes.c_double)
_I = ctypes.POINTER(ctypes.c_int)


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build()
    lib = ctypes.CDLL(_LIB)
    lib.bao_num_threads.restype = ctypes.c_int
    lib.bao_theta.argtypes = [ctypes.c_double, ctypes.c_int, _D]
    lib.bao_theta.restype = None
    lib.bao_rope.argtypes = [_D, ctypes.c_int, ctypes.c_double, _D, ctypes.c_int, ctypes.c_int, _D]
    lib.bao_rope.restype = None
    lib.bao_encode_blocks.argtypes = [_D, _D, _D, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                      ctypes.c_int, _I, ctypes.c_double, _D, ctypes.c_int,
                                      ctypes.c_int, _I, ctypes.c_int, _I, ctypes.c_int, _D, _D]
    lib.bao_encode_blocks.restype = ctypes.c_int
    lib.bao_reencode.argtypes = [_D, _D, ctypes.c_int, ctypes.c_int64, ctypes.c_int64, ctypes.c_int,
                                 ctypes.c_int, _D, ctypes.c_int, ctypes.c_int, _I, _I, _I, _I, _I,
                                 ctypes.c_int]
    lib.bao_reencode.restype = ctypes.c_int
    lib.bao_final_block.argtypes = [_D, _D, _D, _D, _D, ctypes.c_int, ctypes.c_int, ctypes.c_int, _I,
                                    ctypes.c_double, _D, ctypes.c_int, ctypes.c_int, _I, _I, _I,
                                    ctypes.c_int, _I, ctypes.c_int, _D, _D, _D]
    lib.bao_final_block.restype = ctypes.c_int
    _lib = lib
    return lib


def num_threads() -> int:
    return int(_load().bao_num_threads())


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _i32(a) -> Optional[np.ndarray]:
    return None if a is None else np.ascontiguousarray(a, dtype=np.int32)


def _pd(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(_D)


def _pi(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(_I)


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact up-cast of bfloat16 bit patterns (uint16) to float64."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def theta(base: float, D: int) -> np.ndarray:
    """theta_j = base^(-2j/D), j = 0..D/2-1."""
    out = np.empty(D // 2, dtype=np.float64)
    _load().bao_theta(float(base), int(D), _pd(out))
    return out


def rope(x, pos: float, th, layout: int = LAYOUT_INTERLEAVED, inverse: bool = False) -> np.ndarray:
    """Eq. 1 (inverse=False) or Eq. 2 (inverse=True) on one vector of length D."""
    x = _f64(x)
    th = _f64(th)
    y = np.empty_like(x)
    _load().bao_rope(_pd(x), x.shape[-1], float(pos), _pd(th), int(layout), int(bool(inverse)), _pd(y))
    return y


def encode_blocks(q, k, v, offs: Sequence[int], th, *, scale: Optional[float] = None,
                  layout: int = LAYOUT_INTERLEAVED, rope_mode: int = ROPE_APPLY,
                  q_to_kv=None, rows=None, want_k_local: bool = True):
    """Per-block causal attention at local positions.  Returns (o, k_local)."""
    q, k, v, th = _f64(q), _f64(k), _f64(v), _f64(th)
    T, Hq, D = q.shape
    Hkv = k.shape[1]
    assert k.shape == (T, Hkv, D) and v.shape == (T, Hkv, D)
    offs_a = _i32(offs)
    rows_a = _i32(rows)
    n_out = T if rows_a is None else len(rows_a)
    o = np.empty((n_out, Hq, D), dtype=np.float64)
    k_local = np.empty((T, Hkv, D), dtype=np.float64) if want_k_local else None
    sc = float(scale) if scale is not None else 1.0 / np.sqrt(D)
    rc = _load().bao_encode_blocks(_pd(q), _pd(k), _pd(v), T, Hq, Hkv, D, _pi(_i32(q_to_kv)), sc,
                                   _pd(th), int(layout), len(offs_a) - 1, _pi(offs_a),
                                   int(rope_mode), _pi(rows_a), 0 if rows_a is None else len(rows_a),
                                   _pd(o), _pd(k_local))
    if rc != 0:
        raise ValueError("bao_encode_blocks: bad arguments")
    return o, k_local


def reencode(k_src, src_off, dst_off, lens, th, *, old_pos0=None, new_pos0=None,
             mode: int = REENC_SHIFT, layout: int = LAYOUT_INTERLEAVED, out=None) -> np.ndarray:
    """Eq. 2 then Eq. 3 on cached keys.  k_src: [layers, tokens, Hkv, D] (or 3-D for one
    layer).  Returns the destination array (same token extent as ``out`` if given,
    else as k_src); rows no block writes keep their previous contents (zeros if
    freshly allocated)."""
    k_src = _f64(k_src)
    squeeze = k_src.ndim == 3
    if squeeze:
        k_src = k_src[None]
    n_layers, Tsrc, Hkv, D = k_src.shape
    if out is None:
        out = np.zeros_like(k_src)
    else:
        assert out.dtype == np.float64 and out.flags.c_contiguous
        if out.ndim == 3:
            out = out[None]
    th = _f64(th)
    so, do, ln = _i32(src_off), _i32(dst_off), _i32(lens)
    rc = _load().bao_reencode(_pd(k_src), _pd(out), n_layers, Tsrc * Hkv * D,
                              out.shape[1] * Hkv * D, Hkv, D, _pd(th), int(layout), len(ln),
                              _pi(so), _pi(do), _pi(ln), _pi(_i32(old_pos0)), _pi(_i32(new_pos0)),
                              int(mode))
    if rc != 0:
        raise ValueError("bao_reencode: bad arguments")
    return out[0] if squeeze else out


def final_block(q_f, k_ctx, v_ctx, k_f, v_f, cu_q, cu_ctx, th, *, scale: Optional[float] = None,
                layout: int = LAYOUT_INTERLEAVED, rope_mode: int = ROPE_APPLY, q_pos0=None,
                q_to_kv=None, rows=None, want_stats: bool = False):
    """Final-block attention.  Returns o, or (o, m, l) with want_stats."""
    q_f, k_f, v_f, th = _f64(q_f), _f64(k_f), _f64(v_f), _f64(th)
    Lq, Hq, D = q_f.shape
    Hkv = k_f.shape[1]
    k_ctx = _f64(k_ctx).reshape(-1, Hkv, D)
    v_ctx = _f64(v_ctx).reshape(-1, Hkv, D)
    cq, cc = _i32(cu_q), _i32(cu_ctx)
    assert cq[-1] == Lq and cc[-1] <= k_ctx.shape[0]
    rows_a = _i32(rows)
    n_out = Lq if rows_a is None else len(rows_a)
    o = np.empty((n_out, Hq, D), dtype=np.float64)
    m = np.empty((n_out, Hq), dtype=np.float64) if want_stats else None
    l = np.empty((n_out, Hq), dtype=np.float64) if want_stats else None
    sc = float(scale) if scale is not None else 1.0 / np.sqrt(D)
    # keep 1-element dummies alive so that empty contexts still give valid pointers
    kc = k_ctx if k_ctx.size else np.zeros((1, Hkv, D))
    vc = v_ctx if v_ctx.size else np.zeros((1, Hkv, D))
    rc = _load().bao_final_block(_pd(q_f), _pd(kc), _pd(vc), _pd(k_f), _pd(v_f), Hq, Hkv, D,
                                 _pi(_i32(q_to_kv)), sc, _pd(th), int(layout), len(cq) - 1, _pi(cq),
                                 _pi(cc), _pi(_i32(q_pos0)), int(rope_mode), _pi(rows_a),
                                 0 if rows_a is None else len(rows_a), _pd(o), _pd(m), _pd(l))
    if rc != 0:
        raise ValueError("bao_final_block: bad arguments")
    return (o, m, l) if want_stats else o


# --------------------------------------------------------------------------------------
# NumPy-only second implementation: explicit mask, absolute positions, dense softmax.
# --------------------------------------------------------------------------------------

def block_mask(offs: Sequence[int]) -> np.ndarray:
    """M[t, s] = (s <= t) and (block(s) == block(t) or block(t) is the last block)."""
    offs = np.asarray(offs, dtype=np.int64)
    T = int(offs[-1])
    blk = np.zeros(T, dtype=np.int64)
    for b in range(len(offs) - 1):
        blk[offs[b]:offs[b + 1]] = b
    last = len(offs) - 2
    t = np.arange(T)[:, None]
    s = np.arange(T)[None, :]
    return (s <= t) & ((blk[None, :] == blk[:, None]) | (blk[:, None] == last))


def rope_dense(x: np.ndarray, pos: np.ndarray, th: np.ndarray, layout: int) -> np.ndarray:
    """Eq. 1 for a whole [T, H, D] tensor at integer positions pos[T] (vectorised)."""
    x = np.asarray(x, dtype=np.float64)
    T, H, D = x.shape
    ang = np.asarray(pos, dtype=np.float64)[:, None] * np.asarray(th)[None, :]  # [T, D/2]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    y = np.empty_like(x)
    if layout == LAYOUT_HALF:
        a, b = x[..., : D // 2], x[..., D // 2:]
        y[..., : D // 2] = c * a - s * b
        y[..., D // 2:] = s * a + c * b
    else:
        a, b = x[..., 0::2], x[..., 1::2]
        y[..., 0::2] = c * a - s * b
        y[..., 1::2] = s * a + c * b
    return y


def masked_attention_bruteforce(q, k, v, offs, th, *, scale=None, layout=LAYOUT_INTERLEAVED,
                                q_to_kv=None) -> np.ndarray:
    """Whole-sequence Block-attention from the explicit T x T mask, q and k rotated at
    ABSOLUTE positions 0..T-1.  Tiny inputs only (O(T^2) memory per head)."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    T, Hq, D = q.shape
    Hkv = k.shape[1]
    sc = float(scale) if scale is not None else 1.0 / np.sqrt(D)
    pos = np.arange(T)
    qr = rope_dense(q, pos, th, layout)
    kr = rope_dense(k, pos, th, layout)
    M = block_mask(offs)
    out = np.empty_like(q)
    for h in range(Hq):
        g = int(q_to_kv[h]) if q_to_kv is not None else h // (Hq // Hkv)
        S = sc * (qr[:, h, :] @ kr[:, g, :].T)
        S = np.where(M, S, -np.inf)
        S = S - S.max(axis=1, keepdims=True)
        P = np.exp(S)
        P = P / P.sum(axis=1, keepdims=True)
        out[:, h, :] = P @ v[:, g, :]
    return out


def masked_attention_backward_bruteforce(q, k, v, d_out, offs, th, *, scale=None, layout=LAYOUT_INTERLEAVED):
    """Gradients of sum(out * d_out), out = masked_attention_bruteforce(q, k, v, ...), with respect
    to q, k, v (all un-rotated).  With P the masked softmax of S = scale * q^ k^T:
    dV = P^T dO;  dP = dO V^T;  dS = P * (dP - rowsum(dO * O));  dq^ = scale * dS k^;
    dk^ = scale * dS^T q^;  and Eq. 1 is an orthogonal map, so dq = R(pos)^T dq^ = R(-pos) dq^.
    Heads that share a KV head add up in dk and dv.  Returns (dq, dk, dv, lse) with lse the row
    log-sum-exp of the masked scaled scores.  Tiny inputs only."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    d_out = np.asarray(d_out, dtype=np.float64)
    T, Hq, D = q.shape
    Hkv = k.shape[1]
    G = Hq // Hkv
    sc = float(scale) if scale is not None else 1.0 / np.sqrt(D)
    pos = np.arange(T)
    qr = rope_dense(q, pos, th, layout)
    kr = rope_dense(k, pos, th, layout)
    M = block_mask(offs)
    dqr = np.zeros_like(q)
    dkr = np.zeros_like(k)
    dv = np.zeros_like(v)
    lse = np.empty((T, Hq))
    for h in range(Hq):
        g = h // G
        S = np.where(M, sc * (qr[:, h, :] @ kr[:, g, :].T), -np.inf)
        m = S.max(axis=1, keepdims=True)
        E = np.exp(S - m)
        l = E.sum(axis=1, keepdims=True)
        P = E / l
        lse[:, h] = (m + np.log(l))[:, 0]
        O = P @ v[:, g, :]
        dO = d_out[:, h, :]
        dv[:, g, :] += P.T @ dO
        dP = dO @ v[:, g, :].T
        dS = P * (dP - (dO * O).sum(axis=1, keepdims=True))
        dqr[:, h, :] = sc * (dS @ kr[:, g, :])
        dkr[:, g, :] += sc * (dS.T @ qr[:, h, :])
    return rope_dense(dqr, -pos, th, layout), rope_dense(dkr, -pos, th, layout), dv, lse


def masked_attention_backward_term_sums(q, k, v, d_out, offs, th, *, scale=None, layout=LAYOUT_INTERLEAVED):
    """For every element of the gradients that masked_attention_backward_bruteforce returns, the sum
    of the ABSOLUTE values of the products it is the sum of: dV = sum_i P_ij dO_i; dq^ = scale sum_j
    dS_ij k^_j and dk^ = scale sum_i dS_ij q^_i, where dS_ij = P_ij (sum_d dO_id v_jd - sum_d dO_id
    O_id) is itself a sum of products, so that its share is P_ij (sum_d |dO_id v_jd| + sum_d |dO_id
    O_id|): what does not cancel when the two inner sums nearly do (a row that sees one key has
    dS = 0 exactly, and an error in either inner sum still reaches dq in full).  Not a gradient: the
    scale a rounding-error bound is stated against (|fl(sum a_i b_i) - sum a_i b_i| <= eps sum
    |a_i b_i|).  dq and dk are turned back by an orthogonal map of each dimension pair, so both
    members of a pair get the pair's Euclidean norm of the rotated-frame sums.  Returns (aq, ak, av).
    Tiny inputs only."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    d_out = np.asarray(d_out, dtype=np.float64)
    T, Hq, D = q.shape
    Hkv = k.shape[1]
    G = Hq // Hkv
    sc = float(scale) if scale is not None else 1.0 / np.sqrt(D)
    pos = np.arange(T)
    qr = rope_dense(q, pos, th, layout)
    kr = rope_dense(k, pos, th, layout)
    M = block_mask(offs)
    aq = np.zeros_like(q)
    ak = np.zeros_like(k)
    av = np.zeros_like(v)
    for h in range(Hq):
        g = h // G
        S = np.where(M, sc * (qr[:, h, :] @ kr[:, g, :].T), -np.inf)
        E = np.exp(S - S.max(axis=1, keepdims=True))
        P = E / E.sum(axis=1, keepdims=True)
        dO = d_out[:, h, :]
        O = P @ v[:, g, :]
        abs_dS = P * (np.abs(dO) @ np.abs(v[:, g, :]).T + (np.abs(dO) * np.abs(O)).sum(axis=1, keepdims=True))
        av[:, g, :] += P.T @ np.abs(dO)
        aq[:, h, :] = sc * (abs_dS @ np.abs(kr[:, g, :]))
        ak[:, g, :] += sc * (abs_dS.T @ np.abs(qr[:, h, :]))

    def pair_norm(a):
        if layout == LAYOUT_HALF:
            n = np.sqrt(a[..., :D // 2] ** 2 + a[..., D // 2:] ** 2)
            return np.concatenate([n, n], axis=-1)
        return np.repeat(np.sqrt(a[..., 0::2] ** 2 + a[..., 1::2] ** 2), 2, axis=-1)

    return pair_norm(aq), pair_norm(ak), av


def merge_partials(o_parts, m_parts, l_parts) -> np.ndarray:
    """Merge softmax partials over disjoint key sets.  o_parts[i] is the normalised
    output over key set i, m_parts[i] its max scaled score, l_parts[i] its sum of
    exponentials: m = max m_i; l = sum l_i e^(m_i - m); o = sum o_i l_i e^(m_i - m) / l."""
    m = np.max(np.stack(m_parts), axis=0)
    num = 0.0
    den = 0.0
    for o_i, m_i, l_i in zip(o_parts, m_parts, l_parts):
        w = l_i * np.exp(m_i - m)
        num = num + o_i * w[..., None]
        den = den + w
    return num / den[..., None]
