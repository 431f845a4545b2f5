"""Host-side checks of the C boundary that need no GPU: the shared library loads, exports
every symbol include/ba.h declares, and turns bad arguments into status codes before any
device work is attempted."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2409_15355_amd import binding as ba

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(ba.LIB_PATH):
        from paper_2409_15355_amd import build
        build.build()
    return ba.load()


def test_library_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "ba.h")).read()
    declared = set(re.findall(r"\b(ba_[a-z_0-9]+)\s*\(", header))
    assert declared == set(ba.EXPORTS), declared ^ set(ba.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name
    assert lib.ba_version() >= 100
    assert lib.ba_status_string(0) == b"BA_OK"
    assert lib.ba_status_string(-4) == b"BA_ERR_WORKSPACE"


def fake(ptr=0x1000, st=1024, sh=128, dtype=0):
    return ba.BaTensor(ptr, st, sh, dtype)


def call_encode(lib, heads, q, k, v, o, kl, offs, rope=1, ws=None, wsb=0):
    offs = np.asarray(offs, dtype=np.int32)
    r = lambda t: None if t is None else ctypes.byref(t)
    return lib.ba_encode_blocks(ctypes.byref(heads.c), r(q), r(k), r(v), r(o), r(kl), len(offs) - 1,
                                offs.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), rope, ws, wsb, None)


def test_encode_rejects_bad_arguments(lib):
    h = ba.Heads(8, 2, 128)
    t = fake()
    assert call_encode(lib, h, None, t, t, t, None, [0, 4]) == -1
    assert b"q" in lib.ba_last_error()
    assert call_encode(lib, h, t, t, t, t, None, [1, 4]) == -1          # c[0] != 0
    assert call_encode(lib, h, t, t, t, t, None, [0, 5, 4]) == -1       # decreasing
    assert call_encode(lib, ba.Heads(8, 3, 128), t, t, t, t, None, [0, 4]) == -1   # Hq % Hkv
    assert call_encode(lib, ba.Heads(8, 2, 96), t, t, t, t, None, [0, 4]) == -2    # head_dim
    assert call_encode(lib, h, fake(ptr=0x1004), t, t, t, None, [0, 4]) == -3      # alignment
    assert call_encode(lib, h, fake(st=1028), t, t, t, None, [0, 4]) == -3
    assert call_encode(lib, h, fake(dtype=1), t, t, t, None, [0, 4]) == -2         # fp32 attention
    assert call_encode(lib, h, t, t, t, t, None, [0, 4], rope=1, ws=None, wsb=0) == -4  # workspace
    assert call_encode(lib, h, t, t, t, t, fake(), [0, 4], rope=0) == -1           # k_local_out without rope
    assert call_encode(lib, ba.Heads(8, 2, 128, q_to_kv=[0, 1, 0, 1, 0, 1, 0, 1]), t, t, t, t, None, [0, 4]) == -2
    # empty input is a legal no-op that never reaches the device
    assert call_encode(lib, h, t, t, t, t, None, [0, 0, 0], rope=0) == 0
    assert call_encode(lib, ba.Heads(8, 2, 128, q_to_kv=[0, 0, 0, 0, 1, 1, 1, 1]), t, t, t, t, None, [0], rope=0) == 0


def call_reenc(lib, heads, src, dst, layers, sls, sld, so, do, ln, old=None, new=None, mode=0):
    a = lambda x: None if x is None else np.asarray(x, dtype=np.int32)
    so, do, ln, old, new = a(so), a(do), a(ln), a(old), a(new)
    p = lambda x: None if x is None else x.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
    return lib.ba_reencode_positions(ctypes.byref(heads.c), ctypes.byref(src), ctypes.byref(dst), layers, sls, sld,
                                     len(ln), p(so), p(do), p(ln), p(old), p(new), mode, None)


def test_reencode_rejects_bad_arguments(lib):
    h = ba.Heads(8, 8, 128)
    src, dst = fake(0x100000), fake(0x900000)
    assert call_reenc(lib, h, src, dst, 1, 0, 0, [0], [0], [-1]) == -1
    assert call_reenc(lib, h, src, dst, 1, 0, 0, [0], [0], [4], mode=7) == -1
    assert call_reenc(lib, h, src, fake(0x900000, dtype=1), 1, 0, 0, [0], [0], [4]) == -2   # dtype mismatch
    # aliasing: same buffer but moved offsets is not "exactly in place"
    assert call_reenc(lib, h, src, src, 1, 0, 0, [0], [8], [4]) == -1
    # partial overlap of distinct pointers
    assert call_reenc(lib, h, src, fake(0x100000 + 2048), 1, 0, 0, [0], [0], [4]) == -1
    # overlapping destination blocks
    assert call_reenc(lib, h, src, dst, 1, 0, 0, [0, 4], [0, 2], [4, 4]) == -1
    assert call_reenc(lib, h, src, dst, 2, 1028, 1024, [0], [0], [4]) == -3
    # nothing to do
    assert call_reenc(lib, h, src, dst, 0, 0, 0, [0], [0], [4]) == 0
    assert call_reenc(lib, h, src, dst, 1, 0, 0, [], [], []) == 0


def test_final_rejects_bad_arguments_and_sizes_workspace(lib):
    h = ba.Heads(32, 8, 128, 500000.0)
    t = fake()
    i32 = lambda x: np.asarray(x, dtype=np.int32)
    p = lambda x: x.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))

    def call(cu_q, cu_ctx, ws=None, wsb=0, q=t):
        cq, cc = i32(cu_q), i32(cu_ctx)
        return lib.ba_final_block_attention(ctypes.byref(h.c), ctypes.byref(q), ctypes.byref(t), ctypes.byref(t),
                                            ctypes.byref(t), ctypes.byref(t), ctypes.byref(t), None, len(cq) - 1,
                                            p(cq), p(cc), None, 1, ws, wsb, None)

    assert call([0, 0], [0, 10]) == -1        # empty final block
    assert call([1, 5], [0, 10]) == -1        # cu_q[0] != 0
    assert call([0, 5], [10, 3]) == -1        # cu_ctx decreases
    assert call([0, 256], [0, 31744]) == -4   # workspace missing
    need = ba.ba_final_block_attention_workspace_bytes(h, [0, 256], [0, 31744])
    # config 5: 8 KV splits x 8192 packed rows x (128 fp16 + 2 fp32) + rotated final-block keys and queries
    assert need == 8 * 8192 * 128 * 2 + 8 * 8192 * 2 * 4 + 8192 * 4 + 256 * 8 * 128 * 2 + 256 * 32 * 128 * 2
    assert call([0, 256], [0, 31744], ws=ctypes.c_void_p(0x10000), wsb=need - 1) == -4
    # zero prompts: legal no-op
    cq = i32([0])
    assert lib.ba_final_block_attention(ctypes.byref(h.c), None, None, None, None, None, None, None, 0, p(cq),
                                        p(cq), None, 1, None, 0, None) == 0


def test_workspace_queries(lib):
    h = ba.Heads(32, 8, 128)
    # rotated keys (unless the caller takes them) and the table of rotation factors (2 floats per token and pair)
    assert ba.ba_encode_blocks_workspace_bytes(h, [0, 200, 400], ba.ROPE_APPLY, False) == 400 * 8 * 128 * 2 + 400 * 64 * 8
    assert ba.ba_encode_blocks_workspace_bytes(h, [0, 200, 400], ba.ROPE_APPLY, True) == 400 * 64 * 8
    assert ba.ba_encode_blocks_workspace_bytes(h, [0, 200, 400], ba.ROPE_NONE, False) == 0
    # a single small prompt needs no split partials
    assert ba.ba_final_block_attention_workspace_bytes(ba.Heads(4, 4, 64), [0, 64], [0, 128], ba.ROPE_NONE) == 0


def test_final_cached_rejects_bad_arguments_and_sizes_workspace(lib):
    h = ba.Heads(32, 8, 128, 500000.0)
    t = fake()
    i32 = lambda x: np.asarray(x, dtype=np.int32)
    p = lambda x: x.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))

    def call(cu_q, cu_blk, off, ln, ws=None, wsb=0, gather_below=-1):
        cq, cb, bo, bl = i32(cu_q), i32(cu_blk), i32(off), i32(ln)
        return lib.ba_final_block_attention_cached(ctypes.byref(h.c), ctypes.byref(t), ctypes.byref(t), ctypes.byref(t),
                                                   ctypes.byref(t), ctypes.byref(t), ctypes.byref(t), None, len(cq) - 1,
                                                   p(cq), p(cb), p(bo), p(bl), None, None, None, gather_below, ws, wsb,
                                                   None)

    assert call([0, 0], [0, 1], [0], [10]) == -1          # empty final block
    assert call([0, 5], [1, 2], [0, 0], [10, 10]) == -1   # cu_blk[0] != 0
    assert call([0, 5], [0, 1], [0], [-3]) == -1          # negative block length
    assert call([0, 5], [0, 1100], [0] * 1100, [300] * 1100) == -2  # more blocks in one prompt than the kernel's table takes
    assert call([0, 5], [0, 1100], [0] * 1100, [1] * 1100) == -4    # short blocks are gathered: no such limit; workspace missing
    # the gathered route's workspace: K and V of the context, then the final-block step's own
    small = ba.ba_final_block_attention_cached_workspace_bytes(h, [0, 5], [0, 1100], [1] * 1100)
    assert small == 2 * ((1100 * 8 * 128 * 2 + 255) // 256 * 256) + \
        ba.ba_final_block_attention_workspace_bytes(h, [0, 5], [0, 1100], ba.ROPE_APPLY)
    # never gather: the table limit is back; the threshold is the call's own argument, nothing is kept
    assert call([0, 5], [0, 1100], [0] * 1100, [1] * 1100, gather_below=0) == -2
    assert call([0, 5], [0, 1100], [0] * 1100, [1] * 1100) == -4
    assert call([0, 5], [0, 1100], [0] * 1100, [1] * 1100, gather_below=-7) == -1  # neither a count nor the default
    # 300-token blocks are gathered when the caller's threshold says so, and sized accordingly
    assert ba.ba_final_block_attention_cached_workspace_bytes(h, [0, 5], [0, 3], [300] * 3, gather_below=301) == \
        2 * (900 * 8 * 128 * 2) + ba.ba_final_block_attention_workspace_bytes(h, [0, 5], [0, 900], ba.ROPE_APPLY)
    assert call([0, 256], [0, 31], [1024 * b for b in range(31)], [1024] * 31) == -4  # workspace missing
    need = ba.ba_final_block_attention_cached_workspace_bytes(h, [0, 256], [0, 31], [1024] * 31)
    # config 5 as 31 cached blocks: split partials + rotated final-block keys and queries + 31 rows of rotations
    assert need == 8 * 8192 * 128 * 2 + 8 * 8192 * 2 * 4 + 8192 * 4 + 256 * 8 * 128 * 2 + 256 * 32 * 128 * 2 + 31 * 128 * 4
    # zero prompts: legal no-op
    z = i32([0])
    assert lib.ba_final_block_attention_cached(ctypes.byref(h.c), None, None, None, None, None, None, None, 0, p(z),
                                               p(z), None, None, None, None, None, -1, None, 0, None) == 0


def test_whole_prompts_rejects_bad_arguments_and_sizes_workspace(lib):
    h = ba.Heads(32, 8, 128, 500000.0)
    t = fake()
    i32 = lambda x: np.asarray(x, dtype=np.int32)
    p = lambda x: x.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))

    def call(heads, cu_blk, offs, rope=1, ws=None, wsb=0):
        cb, of = i32(cu_blk), i32(offs)
        return lib.ba_block_attention_prompts(ctypes.byref(heads.c), ctypes.byref(t), ctypes.byref(t), ctypes.byref(t),
                                              ctypes.byref(t), None, None, len(cb) - 1, p(cb), p(of), rope, ws, wsb, None)

    assert call(h, [1, 2], [0, 5, 9]) == -1                 # cu_blk[0] != 0
    assert call(h, [0, 2, 2], [0, 5, 9]) == -1              # a prompt without a block
    assert call(h, [0, 2], [0, 9, 5]) == -1                 # offsets decrease
    assert call(h, [0, 2], [0, 5, 9], rope=7) == -1         # unknown rope mode
    assert call(ba.Heads(4, 4, 64), [0, 2], [0, 5, 9]) == -4   # (fewer than four query heads per KV head: run padded) workspace missing
    assert call(h, [0, 2], [0, 5, 9]) == -4                 # workspace missing
    assert b"workspace" in lib.ba_last_error()
    # rotated keys + the table of factors (one (cos, sin) pair per token and dimension pair)
    assert ba.ba_block_attention_prompts_workspace_bytes(h, [0, 2], [0, 100, 164]) == \
        164 * 8 * 128 * 2 + (164 * 128 * 4 + 255) // 256 * 256
    assert ba.ba_block_attention_prompts_workspace_bytes(h, [0, 2], [0, 100, 164], have_k_rot_out=True) == \
        (164 * 128 * 4 + 255) // 256 * 256
    assert ba.ba_block_attention_prompts_workspace_bytes(h, [0, 2], [0, 100, 164], ba.ROPE_NONE) == 0
    # two query heads per KV head run as groups of four: padded q and o (4 heads per KV head), padded log-sum-exps
    a256 = lambda n: (n + 255) // 256 * 256
    h2 = ba.Heads(16, 8, 128, 500000.0)
    assert ba.ba_block_attention_prompts_workspace_bytes(h2, [0, 2], [0, 100, 164], ba.ROPE_NONE) == \
        2 * a256(164 * 32 * 128 * 2) + a256(164 * 32 * 4)
    assert ba.ba_block_attention_prompts_workspace_bytes(h2, [0, 2], [0, 100, 164]) == \
        2 * a256(164 * 32 * 128 * 2) + a256(164 * 32 * 4) + 164 * 8 * 128 * 2 + a256(164 * 128 * 4)
    assert call(h, [0, 2], [0, 0, 0]) == 0                  # no tokens: legal no-op
    # a block whose row offsets would not fit the kernel's 32-bit arithmetic: 3,000 tokens at a token
    # stride of 2^19 elements
    wide = fake()
    wide.stride_tok = 1 << 19
    cb, of = i32([0, 2]), i32([0, 3000, 3064])
    rc = lib.ba_block_attention_prompts(ctypes.byref(h.c), ctypes.byref(wide), ctypes.byref(t), ctypes.byref(t),
                                        ctypes.byref(wide), None, None, 1, p(cb), p(of), 1, None, 0, None)
    assert rc == -2 and b"too long" in lib.ba_last_error()


def test_whole_prompts_backward_rejects_bad_arguments_and_sizes_workspace(lib):
    h = ba.Heads(32, 8, 128, 500000.0)
    t = fake()
    i32 = lambda x: np.asarray(x, dtype=np.int32)
    p = lambda x: x.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
    lse = ctypes.c_void_p(256)

    def call(heads, cu_blk, offs, lse_p=lse, ws=None, wsb=0):
        cb, of = i32(cu_blk), i32(offs)
        r = ctypes.byref(t)
        return lib.ba_block_attention_prompts_backward(ctypes.byref(heads.c), r, r, r, r, lse_p, r, r, r, r, len(cb) - 1,
                                                       p(cb), p(of), ws, wsb, None)

    assert call(h, [1, 2], [0, 5, 9]) == -1                   # cu_blk[0] != 0
    assert call(h, [0, 2], [0, 9, 5]) == -1                   # offsets decrease
    assert call(h, [0, 2], [0, 5, 9], lse_p=None) == -1       # no log-sum-exps
    assert call(ba.Heads(4, 4, 64), [0, 2], [0, 5, 9]) == -4  # (fewer than four query heads per KV head: run padded) workspace missing
    assert call(h, [0, 2], [0, 5, 9]) == -4                   # workspace missing
    # rotated q, rotated k, the table of rotation factors, (log-sum-exp, delta) per row + padding
    T = 164
    a256 = lambda n: (n + 255) // 256 * 256
    assert ba.ba_block_attention_prompts_backward_workspace_bytes(h, [0, 2], [0, 100, T]) == \
        a256(T * 32 * 128 * 2) + a256(T * 8 * 128 * 2) + a256(T * 128 * 4) + a256(T * 32 * 8 + 16)
    assert call(h, [0, 2], [0, 0, 0]) == 0                    # no tokens: legal no-op


def test_header_is_plain_c(tmp_path):
    """include/ba.h is the boundary of a C-ABI library: a C99 compiler takes it as it is, with
    warnings as errors, and the structs it declares have the layout the Python face assumes."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler here")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    src = tmp_path / "use_header.c"
    src.write_text('#include <stdio.h>\n#include <stddef.h>\n#include "ba.h"\n'
                   'int main(void) {\n'
                   '  printf("%zu %zu %zu %zu\\n", sizeof(ba_tensor), sizeof(ba_heads),\n'
                   '         offsetof(ba_heads, rope_base), offsetof(ba_heads, rope_layout));\n'
                   '  return 0;\n}\n')
    exe = tmp_path / "use_header"
    subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(root, "include"),
                    str(src), "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    assert [int(x) for x in out] == [ctypes.sizeof(ba.BaTensor), ctypes.sizeof(ba.BaHeads),
                                     ba.BaHeads.rope_base.offset, ba.BaHeads.rope_layout.offset]


def test_reencode_rejects_overlapping_blocks_in_place(lib):
    """A token listed in two blocks of an in-place call would be rotated twice (or by two workgroups
    at once): rejected like overlapping destinations of a gathered call."""
    h = ba.Heads(8, 8, 128)
    src = fake(0x100000)
    assert call_reenc(lib, h, src, src, 1, 0, 0, [0, 2], [0, 2], [4, 4]) == -1
    assert b"overlap" in lib.ba_last_error()


def test_final_cached_rejects_negative_cache_offsets_on_both_routes(lib):
    h = ba.Heads(32, 8, 128, 500000.0)
    t = fake()
    i32 = lambda x: np.asarray(x, dtype=np.int32)
    p = lambda x: x.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
    cq, cb, bo, bl = i32([0, 5]), i32([0, 2]), i32([0, -8]), i32([300, 300])
    for gather_below in (0, 1 << 30):  # the kernel that reads the table; the gathered copy
        need = ba.ba_final_block_attention_cached_workspace_bytes(h, cq, cb, bl, gather_below=gather_below)
        rc = lib.ba_final_block_attention_cached(ctypes.byref(h.c), ctypes.byref(t), ctypes.byref(t), ctypes.byref(t),
                                                 ctypes.byref(t), ctypes.byref(t), ctypes.byref(t), None, 1, p(cq), p(cb),
                                                 p(bo), p(bl), None, None, None, gather_below, ctypes.c_void_p(0x10000),
                                                 need, None)
        assert rc == -1 and b"negative cache offset" in lib.ba_last_error()


def test_workspace_queries_reject_what_the_calls_reject(lib):
    """The size queries read their host arrays with the checks of the calls: a bad array gives 0,
    never an index out of range or a size wrapped from a negative number."""
    h = ba.Heads(32, 8, 128)
    assert ba.ba_encode_blocks_workspace_bytes(h, [0, 200, 100]) == 0          # offsets decrease
    assert ba.ba_encode_blocks_workspace_bytes(h, [5, 200]) == 0               # offsets do not start at 0
    assert ba.ba_encode_blocks_workspace_bytes(ba.Heads(32, 8, 96), [0, 200]) == 0
    assert ba.ba_block_attention_prompts_workspace_bytes(h, [0, -1], [0, 10]) == 0    # a prompt without blocks
    assert ba.ba_block_attention_prompts_workspace_bytes(h, [1, 2], [0, 10, 20]) == 0
    assert ba.ba_block_attention_prompts_workspace_bytes(h, [0, 2], [0, 10, 5]) == 0
    assert ba.ba_block_attention_prompts_backward_workspace_bytes(h, [0, -1], [0, 10]) == 0
    assert ba.ba_block_attention_prompts_backward_workspace_bytes(h, [0, 2], [0, 10, 5]) == 0


class FakeGpuTensor:
    """What the Python face reads of a torch tensor; claims to live on the GPU so that the checks
    behind the device check can be reached without one.  Every call below is rejected before
    anything is launched."""

    def __init__(self, shape, dtype=None, strides=None, is_cuda=True):
        import torch
        self.shape = tuple(shape)
        self.dtype = dtype or torch.bfloat16
        if strides is None:
            strides, acc = [], 1
            for n in reversed(self.shape):
                strides.insert(0, acc)
                acc *= n
        self._strides = tuple(strides)
        self.is_cuda = is_cuda
        self.device = "cuda:0" if is_cuda else "cpu"

    def stride(self, i=None):
        return self._strides if i is None else self._strides[i]

    def dim(self):
        return len(self.shape)

    def data_ptr(self):
        return 0x10000

    def is_contiguous(self):
        return True

    def numel(self):
        return int(np.prod(self.shape))

    def element_size(self):
        return 2

    def __getitem__(self, i):
        assert i == 0 or i is None
        if i is None:
            return FakeGpuTensor((1,) + self.shape, self.dtype, (0,) + self._strides, self.is_cuda)
        return FakeGpuTensor(self.shape[1:], self.dtype, self._strides[1:], self.is_cuda)


def test_python_face_rejects_tensors_the_boundary_cannot_check(lib):
    import torch
    h = ba.Heads(32, 8, 128, 500000.0)
    F = FakeGpuTensor
    q, kv = F((64, 32, 128)), F((64, 8, 128))
    ctx = F((1000, 8, 128))
    cu_q, cu_ctx = [0, 64], [0, 1000]
    ok = dict(heads=h, q_f=q, k_ctx=ctx, v_ctx=ctx, k_f=kv, v_f=kv, o_out=q, k_f_rot_out=None, cu_q=cu_q, cu_ctx=cu_ctx)

    def rejected(match, **over):
        with pytest.raises(ValueError, match=match):
            ba.ba_final_block_attention(**{**ok, **over})

    rejected("GPU memory", q_f=torch.zeros(64, 32, 128, dtype=torch.bfloat16))           # a CPU tensor
    rejected("GPU memory", k_ctx=torch.zeros(1000, 8, 128, dtype=torch.bfloat16))
    rejected("head_dim 64", q_f=F((64, 32, 64)))                                          # D = 64 tensor, Heads(..., 128)
    rejected("32 heads", k_f=F((64, 32, 128)))                                            # query-shaped keys
    rejected("tokens", k_ctx=F((999, 8, 128)))                                            # context shorter than cu_ctx[-1]
    rejected("tokens", o_out=F((63, 32, 128)))                                            # output shorter than cu_q[-1]
    rejected("dtype", v_ctx=F((1000, 8, 128), dtype=torch.float16))
    rejected("dtype", q_f=F((64, 32, 128), dtype=torch.float32))                          # fp32 attention is not built
    rejected("contiguous head_dim", q_f=F((64, 32, 128), strides=(32 * 256, 256, 2)))
    rejected("workspace", ws=torch.zeros(16, dtype=torch.uint8))                          # a CPU workspace
    rejected("q_pos0", q_pos0=[0, 1])
    # the other entry points go through the same checks
    with pytest.raises(ValueError, match="tokens"):
        ba.ba_encode_blocks(h, F((399, 32, 128)), F((400, 8, 128)), F((400, 8, 128)), F((400, 32, 128)), None, [0, 200, 400])
    with pytest.raises(ValueError, match="tokens"):   # the last block's last row lies outside the destination
        ba.ba_reencode_positions(ba.Heads(8, 8, 128), F((2, 500, 8, 128)), F((2, 450, 8, 128)), [0, 200], [0, 300],
                                 [200, 200])
    with pytest.raises(ValueError, match="entries"):
        ba.ba_reencode_positions(ba.Heads(8, 8, 128), F((2, 500, 8, 128)), F((2, 500, 8, 128)), [0, 200], [0], [200, 200])
    with pytest.raises(ValueError, match="tokens"):   # a cached block reaches beyond the cache
        ba.ba_final_block_attention_cached(h, q, F((1000, 8, 128)), F((1000, 8, 128)), kv, kv, q, None, cu_q, [0, 2],
                                           [0, 900], [300, 101])
    with pytest.raises(ValueError, match="entries"):
        ba.ba_final_block_attention_cached(h, q, ctx, ctx, kv, kv, q, None, cu_q, [0, 2], [0], [300, 100])
    lse_bad = F((164, 32), dtype=torch.float16)
    t164q, t164k = F((164, 32, 128)), F((164, 8, 128))
    with pytest.raises(ValueError, match="lse_out"):
        ba.ba_block_attention_prompts(h, t164q, t164k, t164k, t164q, None, lse_bad, [0, 2], [0, 100, 164])
    with pytest.raises(ValueError, match="lse"):
        ba.ba_block_attention_prompts_backward(h, t164q, t164k, t164k, t164q, F((100, 32), dtype=torch.float32), t164q,
                                               t164q, t164k, t164k, [0, 2], [0, 100, 164])
    with pytest.raises(ValueError, match="block_offsets"):
        ba.ba_block_attention_prompts(h, t164q, t164k, t164k, t164q, None, None, [0, 3], [0, 100, 164])


def test_probes_and_diagnostics_reject_bad_arguments_before_any_device_work(lib):
    speeds = (ctypes.c_float * 8)()
    phases = (ctypes.c_double * 8)()
    need = lib.ba_measure_xcd_speed_workspace_bytes()
    assert need > 2 * 31744 * 8 * 128 * 2  # (the probe's synthetic keys and values live in the workspace)
    assert lib.ba_measure_xcd_speed(None, None, 0, None) == -1
    assert lib.ba_measure_xcd_speed(speeds, None, 0, None) == -4
    assert lib.ba_measure_xcd_speed(speeds, ctypes.c_void_p(0x1000), need - 1, None) == -4
    assert lib.ba_measure_xcd_speed(speeds, ctypes.c_void_p(0x1010), need, None) == -4  # not 256-byte aligned
    assert [float(x) for x in speeds] == [1.0] * 8  # (equal speeds whenever nothing was measured)
    assert lib.ba_diag_final_block_phases(None, None, None, 0, None) == -1
    assert lib.ba_diag_final_block_phases(phases, None, None, 0, None) == -4
    assert lib.ba_diag_final_block_phases(phases, None, ctypes.c_void_p(0x1000), need - 1, None) == -4
    assert b"workspace" in lib.ba_last_error()
    t = ctypes.c_double()
    assert lib.ba_diag_mfma_ceiling(3, ctypes.byref(t), ctypes.byref(t), ctypes.byref(t), None, 0, None) == -1
