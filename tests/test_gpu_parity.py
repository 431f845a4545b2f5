"""GPU parity: the HIP library, called through its C boundary, against the CPU oracle on
the same seeded inputs.  Element by element at sizes the oracle finishes in seconds;
on sampled rows at the full benchmark sizes (every output row depends only on its own
query and its visible keys, so any subset of rows can be checked exactly)."""
import numpy as np
import pytest

import oracle
from paper_2409_15355_amd import workloads as wl
from gpu_util import (REENC_F32_REL_TOL, assert_attention_close, assert_reencode_bf16, dev_bf16, host_bits,
                      host_f64, pair_norm_rel_err)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ba():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2409_15355_amd import binding
    binding.load()
    return binding


def torch_mod():
    import torch
    return torch


def heads_of(ba, w: wl.Workload, layout=0):
    return ba.Heads(w.n_q_heads, w.n_kv_heads, w.head_dim, w.rope_base, rope_layout=layout)


def gen_qkv(seed0, T, hq, hkv, d):
    return (wl.normal_bf16_bits(seed0, (T, hq, d)), wl.normal_bf16_bits(seed0 + 1, (T, hkv, d)),
            wl.normal_bf16_bits(seed0 + 2, (T, hkv, d)))


def gpu_encode(ba, heads, qb, kb, vb, offs, rope_mode=1, want_k_local=True):
    torch = torch_mod()
    q, k, v = dev_bf16(qb), dev_bf16(kb), dev_bf16(vb)
    o = torch.full_like(q, float("nan"))
    k_local = torch.full_like(k, float("nan")) if (want_k_local and rope_mode == 1) else None
    nbytes = ba.ba_encode_blocks_workspace_bytes(heads, offs, rope_mode, k_local is not None)
    ws = torch.empty(max(nbytes, 1), dtype=torch.uint8, device="cuda")
    ba.ba_encode_blocks(heads, q, k, v, o, k_local, offs, rope_mode, ws)
    torch.cuda.synchronize()
    return o, k_local


def gpu_final(ba, heads, qf, kc, vc, kf, vf, cu_q, cu_ctx, q_pos0=None, rope_mode=1):
    torch = torch_mod()
    o = torch.full_like(qf, float("nan"))
    nbytes = ba.ba_final_block_attention_workspace_bytes(heads, cu_q, cu_ctx, rope_mode, False)
    ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")
    ba.ba_final_block_attention(heads, qf, kc, vc, kf, vf, o, None, cu_q, cu_ctx, q_pos0, rope_mode, ws)
    torch.cuda.synchronize()
    return o


# --------------------------------------------------------------------------------------------
# a-2: position re-encoding
# --------------------------------------------------------------------------------------------
@pytest.mark.parametrize("layout", [0, 1])
@pytest.mark.parametrize("d,hkv", [(64, 4), (128, 8)])
def test_reencode_bf16_shift_gather_and_inplace(ba, layout, d, hkv):
    torch = torch_mod()
    lens = [128, 1, 37, 200, 0, 64]
    src_off = np.concatenate([[0], np.cumsum(lens)[:-1]]).astype(np.int32)
    T = int(np.sum(lens))
    order = [3, 0, 5, 1, 2, 4]  # destination order of the blocks (gather form)
    dst_off = np.zeros(len(lens), dtype=np.int32)
    acc = 0
    for b in order:
        dst_off[b] = acc
        acc += lens[b]
    new_pos0 = np.array([0, 31999, 128, 7, 5, 100000], dtype=np.int32)
    n_layers = 3
    kb = wl.normal_bf16_bits(11 + d + layout, (n_layers, T, hkv, d))
    th = oracle.theta(500000.0, d)
    heads = ba.Heads(hkv, hkv, d, 500000.0, rope_layout=layout)
    ref = oracle.reencode(oracle.bf16_bits_to_f64(kb), src_off, dst_off, lens, th, new_pos0=new_pos0, layout=layout)
    src = dev_bf16(kb)
    dst = torch.zeros_like(src)
    ba.ba_reencode_positions(heads, src, dst, src_off, dst_off, lens, None, new_pos0, ba.REENC_SHIFT)
    torch.cuda.synchronize()
    assert_reencode_bf16(host_bits(dst), ref, layout, "gather")
    # block 0 has shift 0: bit-for-bit copy
    assert np.array_equal(host_bits(dst)[:, dst_off[0]:dst_off[0] + lens[0]], kb[:, :lens[0]])
    # in place (dst == src, same offsets)
    ref_ip = oracle.reencode(oracle.bf16_bits_to_f64(kb), src_off, src_off, lens, th, new_pos0=new_pos0, layout=layout)
    ba.ba_reencode_positions(heads, src, src, src_off, src_off, lens, None, new_pos0, ba.REENC_SHIFT)
    torch.cuda.synchronize()
    assert_reencode_bf16(host_bits(src), ref_ip, layout, "in place")


@pytest.mark.parametrize("layout", [0, 1])
@pytest.mark.parametrize("mode", [0, 1])
def test_reencode_f32_relative_error(ba, layout, mode):
    torch = torch_mod()
    d, hkv, lens = 128, 8, [77, 300, 5]
    src_off = np.array([0, 77, 377], dtype=np.int32)
    T = 382
    old = np.array([0, 0, 0] if mode == 1 else [3, 0, 1000], dtype=np.int32)
    new = np.array([31744, 250, 7], dtype=np.int32)
    k = wl.normal_f32(21 + layout + 2 * mode, (2, T, hkv, d))
    th = oracle.theta(500000.0, d)
    heads = ba.Heads(hkv, hkv, d, 500000.0, rope_layout=layout)
    ref = oracle.reencode(k.astype(np.float64), src_off, src_off, lens, th, old_pos0=old, new_pos0=new, mode=mode,
                          layout=layout)
    src = torch.from_numpy(k).cuda()
    dst = torch.zeros_like(src)
    ba.ba_reencode_positions(heads, src, dst, src_off, src_off, lens, old, new, mode)
    torch.cuda.synchronize()
    rel = pair_norm_rel_err(host_f64(dst), ref, layout)
    assert rel <= REENC_F32_REL_TOL, f"relative error {rel:.3e}"


def test_reencode_2500_blocks_in_one_call(ba):
    """More blocks than the larger of the two block tables holds (three launches), gathered into the
    reverse order, two layers."""
    torch = torch_mod()
    d, hkv, nb = 64, 2, 2500
    lens = [(3 * i) % 7 for i in range(nb)]  # some empty
    src_off = np.concatenate([[0], np.cumsum(lens)[:-1]]).astype(np.int32)
    T = int(np.sum(lens))
    dst_off = (T - src_off - np.array(lens)).astype(np.int32)
    new_pos0 = ((np.arange(nb) * 37) % 9000).astype(np.int32)
    kb = wl.normal_bf16_bits(41, (2, T, hkv, d))
    th = oracle.theta(10000.0, d)
    heads = ba.Heads(hkv, hkv, d, 10000.0)
    ref = oracle.reencode(oracle.bf16_bits_to_f64(kb), src_off, dst_off, lens, th, new_pos0=new_pos0)
    src = dev_bf16(kb)
    dst = torch.zeros_like(src)
    ba.ba_reencode_positions(heads, src, dst, src_off, dst_off, lens, None, new_pos0, ba.REENC_SHIFT)
    torch.cuda.synchronize()
    assert_reencode_bf16(host_bits(dst), ref, 0, "2500 blocks")


def test_reencode_negative_shift_and_strided_layers(ba):
    """Moving a block to a smaller position (negative shift) and a destination whose layer
    stride differs from the source's."""
    torch = torch_mod()
    d, hkv, L = 128, 2, 50
    kb = wl.normal_bf16_bits(31, (2, L, hkv, d))
    th = oracle.theta(10000.0, d)
    heads = ba.Heads(hkv, hkv, d, 10000.0)
    ref = oracle.reencode(oracle.bf16_bits_to_f64(kb), [0], [0], [L], th, old_pos0=[900], new_pos0=[10])
    src = dev_bf16(kb)
    big = torch.zeros((2, L + 13, hkv, d), dtype=torch.bfloat16, device="cuda")
    ba.ba_reencode_positions(heads, src, big, [0], [13], [L], [900], [10], ba.REENC_SHIFT)
    torch.cuda.synchronize()
    assert_reencode_bf16(host_bits(big[:, 13:]), ref, 0, "negative shift")
    assert float(big[:, :13].abs().max()) == 0.0


# --------------------------------------------------------------------------------------------
# a-1: per-block encoding
# --------------------------------------------------------------------------------------------
ENC_CASES = [
    # (name, Hq, Hkv, D, base, block lengths)
    ("cfg1-shape", 4, 4, 64, 10000.0, [128, 128]),
    ("cfg2-shape", 32, 8, 128, 500000.0, [200] * 10),
    ("ragged-gqa4", 8, 2, 128, 500000.0, [1, 63, 64, 65, 0, 130, 257, 2]),
    ("ragged-mha-d64", 2, 2, 64, 10000.0, [300, 5, 0, 0, 511, 256]),
    ("gqa8-d128", 8, 1, 128, 10000.0, [33, 100]),
    ("gqa3-odd-group", 6, 2, 64, 10000.0, [90, 171]),
    # groups of fewer than four query heads take the main core whatever the block length
    ("long-mha-d64", 2, 2, 64, 10000.0, [530, 300, 5]),
    ("gqa2", 4, 2, 128, 10000.0, [512, 31]),
    # medium blocks: many key tiles per work item of the short-block schedule
    ("medium-gqa4", 8, 2, 128, 500000.0, [700, 1, 63, 130]),
    ("medium-gqa8-d64", 8, 1, 64, 10000.0, [1000, 333]),
    # more blocks than one launch's table holds, on either schedule
    ("700-blocks-gqa4", 4, 1, 64, 10000.0, [1 + (7 * i) % 23 for i in range(700)]),
    ("700-blocks-mha", 2, 2, 64, 10000.0, [1 + (5 * i) % 17 for i in range(700)]),
    # the longest block lies in the second launch, and is longer than the whole first launch: the table of
    # rotation factors (a row per position inside a block) is written by the first launch for all of them
    ("long-block-in-second-launch", 4, 1, 64, 10000.0, [1 + i % 2 for i in range(320)] + [700, 3, 64]),
]


@pytest.mark.parametrize("case", ENC_CASES, ids=[c[0] for c in ENC_CASES])
@pytest.mark.parametrize("layout", [0, 1])
def test_encode_blocks_matches_oracle(ba, case, layout):
    name, hq, hkv, d, base, lens = case
    offs = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    T = int(offs[-1])
    qb, kb, vb = gen_qkv(100 + len(name) + layout, T, hq, hkv, d)
    th = oracle.theta(base, d)
    ref_o, ref_k = oracle.encode_blocks(oracle.bf16_bits_to_f64(qb), oracle.bf16_bits_to_f64(kb),
                                        oracle.bf16_bits_to_f64(vb), offs, th, layout=layout)
    heads = ba.Heads(hq, hkv, d, base, rope_layout=layout)
    o, k_local = gpu_encode(ba, heads, qb, kb, vb, offs)
    assert_attention_close(host_f64(o), ref_o, name)
    assert_reencode_bf16(host_bits(k_local), ref_k, layout, name + " k_local")


def test_encode_blocks_rope_none_and_workspace_path(ba):
    """q, k already rotated by the caller (ROPE_NONE); and ROPE_APPLY without k_local_out
    (rotated keys live in the workspace) gives the same output as with it."""
    hq, hkv, d, lens = 8, 2, 128, [70, 129]
    offs = np.array([0, 70, 199], dtype=np.int32)
    qb, kb, vb = gen_qkv(200, 199, hq, hkv, d)
    th = oracle.theta(10000.0, d)
    heads = ba.Heads(hq, hkv, d, 10000.0)
    ref_none, _ = oracle.encode_blocks(oracle.bf16_bits_to_f64(qb), oracle.bf16_bits_to_f64(kb),
                                       oracle.bf16_bits_to_f64(vb), offs, th, rope_mode=oracle.ROPE_NONE)
    o_none, _ = gpu_encode(ba, heads, qb, kb, vb, offs, rope_mode=0)
    assert_attention_close(host_f64(o_none), ref_none, "rope none")
    o_a, _ = gpu_encode(ba, heads, qb, kb, vb, offs, rope_mode=1, want_k_local=True)
    o_b, _ = gpu_encode(ba, heads, qb, kb, vb, offs, rope_mode=1, want_k_local=False)
    assert np.array_equal(host_bits(o_a), host_bits(o_b))


def test_encode_first_token_of_block_returns_v_exactly(ba):
    hq, hkv, d = 4, 2, 64
    offs = np.array([0, 40, 41, 300], dtype=np.int32)
    qb, kb, vb = gen_qkv(210, 300, hq, hkv, d)
    heads = ba.Heads(hq, hkv, d, 10000.0)
    o, _ = gpu_encode(ba, heads, qb, kb, vb, offs)
    ob = host_bits(o)
    for start in (0, 40, 41):
        for h in range(hq):
            assert np.array_equal(ob[start, h], vb[start, h // 2])


def test_encode_strided_views(ba):
    """q, k, v, o as views into one fused [T, Hq + 2 Hkv, D] projection buffer."""
    torch = torch_mod()
    hq, hkv, d, T = 8, 2, 128, 150
    offs = np.array([0, 64, 150], dtype=np.int32)
    qb, kb, vb = gen_qkv(220, T, hq, hkv, d)
    fused = torch.zeros((T, hq + 2 * hkv, d), dtype=torch.bfloat16, device="cuda")
    fused[:, :hq] = dev_bf16(qb)
    fused[:, hq:hq + hkv] = dev_bf16(kb)
    fused[:, hq + hkv:] = dev_bf16(vb)
    q, k, v = fused[:, :hq], fused[:, hq:hq + hkv], fused[:, hq + hkv:]
    o = torch.empty((T, hq, d), dtype=torch.bfloat16, device="cuda")
    k_local = torch.empty((T, hkv, d), dtype=torch.bfloat16, device="cuda")
    heads = ba.Heads(hq, hkv, d, 10000.0)
    ws = torch.empty(ba.ba_encode_blocks_workspace_bytes(heads, offs, 1, True), dtype=torch.uint8, device="cuda")
    ba.ba_encode_blocks(heads, q, k, v, o, k_local, offs, 1, ws)
    torch.cuda.synchronize()
    th = oracle.theta(10000.0, d)
    ref_o, _ = oracle.encode_blocks(oracle.bf16_bits_to_f64(qb), oracle.bf16_bits_to_f64(kb),
                                    oracle.bf16_bits_to_f64(vb), offs, th)
    assert_attention_close(host_f64(o), ref_o, "strided")


def test_encode_with_token_strides_too_wide_for_the_short_block_schedule(ba):
    """q and o as views with a token stride of 2^18 elements: the short-block schedule keeps 32-bit row
    offsets inside a block, which such strides would overflow at its longest blocks, so the call takes
    the main schedule (64-bit row addresses) whatever the block lengths; same results."""
    torch = torch_mod()
    hq, hkv, d, base = 8, 2, 128, 500000.0
    lens = [150, 64, 33]
    offs = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    T, stride = int(offs[-1]), 1 << 18
    qb, kb, vb = gen_qkv(240, T, hq, hkv, d)
    q_big = torch.zeros(T * stride, dtype=torch.bfloat16, device="cuda")
    o_big = torch.zeros(T * stride, dtype=torch.bfloat16, device="cuda")
    q = q_big.as_strided((T, hq, d), (stride, d, 1))
    o = o_big.as_strided((T, hq, d), (stride, d, 1))
    q.copy_(dev_bf16(qb))
    k, v = dev_bf16(kb), dev_bf16(vb)
    k_local = torch.empty_like(k)
    heads = ba.Heads(hq, hkv, d, base)
    ws = torch.empty(max(1, ba.ba_encode_blocks_workspace_bytes(heads, offs, ba.ROPE_APPLY, True)), dtype=torch.uint8, device="cuda")
    ba.ba_encode_blocks(heads, q, k, v, o, k_local, offs, ba.ROPE_APPLY, ws)
    torch.cuda.synchronize()
    f = oracle.bf16_bits_to_f64
    ref_o, ref_k = oracle.encode_blocks(f(qb), f(kb), f(vb), offs, oracle.theta(base, d))
    assert_attention_close(host_f64(o), ref_o, "wide token strides")
    assert_reencode_bf16(host_bits(k_local), ref_k, 0, "wide token strides, k_local")
    del q_big, o_big, q, o
    torch.cuda.empty_cache()


def test_encode_short_block_schedule_near_the_end_of_its_row_offsets(ba):
    """A 6,000-token block with q and o at a token stride of 2^17 elements: the largest row offsets
    the short-block schedule accepts (1.5 GB from the block's first row), checked on sampled rows
    including the last ones."""
    torch = torch_mod()
    hq, hkv, d, base = 4, 1, 64, 10000.0
    L, stride = 6000, 1 << 17
    offs = np.array([0, L], dtype=np.int32)
    qb, kb, vb = gen_qkv(250, L, hq, hkv, d)
    q_big = torch.zeros(L * stride, dtype=torch.bfloat16, device="cuda")
    o_big = torch.zeros(L * stride, dtype=torch.bfloat16, device="cuda")
    q = q_big.as_strided((L, hq, d), (stride, d, 1))
    o = o_big.as_strided((L, hq, d), (stride, d, 1))
    q.copy_(dev_bf16(qb))
    k, v = dev_bf16(kb), dev_bf16(vb)
    heads = ba.Heads(hq, hkv, d, base)
    ws = torch.empty(max(1, ba.ba_encode_blocks_workspace_bytes(heads, offs, ba.ROPE_APPLY, False)), dtype=torch.uint8, device="cuda")
    ba.ba_encode_blocks(heads, q, k, v, o, None, offs, ba.ROPE_APPLY, ws)
    torch.cuda.synchronize()
    rows = sorted(set([0, 1, 31, 32, 127, 128, 2999, 4095, 4096, L - 129, L - 2, L - 1] +
                      np.random.default_rng(5).integers(0, L, 40).tolist()))
    f = oracle.bf16_bits_to_f64
    ref, _ = oracle.encode_blocks(f(qb), f(kb), f(vb), offs, oracle.theta(base, d), rows=rows, want_k_local=False)
    assert_attention_close(host_f64(o[rows]), ref, "row offsets up to 1.5 GB")
    del q_big, o_big, q, o
    torch.cuda.empty_cache()


# --------------------------------------------------------------------------------------------
# a-3: final-block attention
# --------------------------------------------------------------------------------------------
FIN_CASES = [
    # (name, Hq, Hkv, D, base, [(t_ctx, l_q), ...])
    ("cfg1-shape", 4, 4, 64, 10000.0, [(256, 64)]),
    ("cfg2-shape-split", 32, 8, 128, 500000.0, [(2000, 64)]),
    ("no-context", 8, 2, 128, 10000.0, [(0, 100)]),
    ("ragged-batch", 8, 2, 128, 500000.0, [(130, 33), (0, 5), (1, 1), (700, 128), (63, 65)]),
    ("long-query-mha-d64", 2, 2, 64, 10000.0, [(100, 300), (5, 257)]),
    ("deep-split", 8, 8, 128, 500000.0, [(4100, 17)]),
    # more than eight splits (the merge's four-group form), a row count that does not fill its last workgroup
    ("many-splits-d64-odd-rows", 6, 2, 64, 10000.0, [(5000, 7)]),
    ("many-splits-d128-batch", 8, 2, 128, 500000.0, [(3000, 3), (2500, 9)]),
    # more prompts than one launch's table holds
    ("seventy-prompts", 4, 1, 64, 10000.0, [(20 + (3 * i) % 50, 1 + i % 5) for i in range(70)]),
]


@pytest.mark.parametrize("case", FIN_CASES, ids=[c[0] for c in FIN_CASES])
@pytest.mark.parametrize("layout", [0, 1])
def test_final_block_matches_oracle(ba, case, layout):
    name, hq, hkv, d, base, shapes = case
    cu_ctx = np.concatenate([[0], np.cumsum([s[0] for s in shapes])]).astype(np.int32)
    cu_q = np.concatenate([[0], np.cumsum([s[1] for s in shapes])]).astype(np.int32)
    seed = 300 + len(name) + layout
    qb, kfb, vfb = gen_qkv(seed, int(cu_q[-1]), hq, hkv, d)
    kcb = wl.normal_bf16_bits(seed + 3, (max(int(cu_ctx[-1]), 1), hkv, d))
    vcb = wl.normal_bf16_bits(seed + 4, (max(int(cu_ctx[-1]), 1), hkv, d))
    th = oracle.theta(base, d)
    ref = oracle.final_block(oracle.bf16_bits_to_f64(qb), oracle.bf16_bits_to_f64(kcb)[:cu_ctx[-1]],
                             oracle.bf16_bits_to_f64(vcb)[:cu_ctx[-1]], oracle.bf16_bits_to_f64(kfb),
                             oracle.bf16_bits_to_f64(vfb), cu_q, cu_ctx, th, layout=layout)
    heads = ba.Heads(hq, hkv, d, base, rope_layout=layout)
    o = gpu_final(ba, heads, dev_bf16(qb), dev_bf16(kcb), dev_bf16(vcb), dev_bf16(kfb), dev_bf16(vfb), cu_q, cu_ctx)
    assert_attention_close(host_f64(o), ref, name)


def test_final_block_query_heads_a_gigabyte_apart(ba):
    """Queries laid out head-major in a 4 GB buffer (head stride 2^29 elements), used as given
    (no rotary embedding): a group's rows then span 2^32 bytes, which the attention core's whole-row
    fetch of the query rows (32-bit offsets from the wave's first row) cannot address, so it takes its
    other way of loading them; same result either way."""
    torch = torch_mod()
    hq, hkv, d, lq, tc = 4, 1, 128, 70, 900
    qb, kfb, vfb = gen_qkv(960, lq, hq, hkv, d)
    kcb, vcb = wl.normal_bf16_bits(963, (tc, hkv, d)), wl.normal_bf16_bits(964, (tc, hkv, d))
    cu_q, cu_ctx = np.array([0, lq], dtype=np.int32), np.array([0, tc], dtype=np.int32)
    f = oracle.bf16_bits_to_f64
    th = oracle.theta(10000.0, d)
    ref = oracle.final_block(f(qb), f(kcb), f(vcb), f(kfb), f(vfb), cu_q, cu_ctx, th, rope_mode=oracle.ROPE_NONE)
    heads = ba.Heads(hq, hkv, d, 10000.0)
    big = torch.empty(hq << 29, dtype=torch.bfloat16, device="cuda")
    q_far = big.as_strided((lq, hq, d), (d, 1 << 29, 1))
    q_far.copy_(dev_bf16(qb))
    assert q_far.stride(1) * 2 * hq >= 1 << 32
    o_far = gpu_final(ba, heads, q_far, dev_bf16(kcb), dev_bf16(vcb), dev_bf16(kfb), dev_bf16(vfb), cu_q, cu_ctx, rope_mode=0)
    assert_attention_close(host_f64(o_far), ref, "head-major queries, heads 1 GB apart")
    o_near = gpu_final(ba, heads, dev_bf16(qb), dev_bf16(kcb), dev_bf16(vcb), dev_bf16(kfb), dev_bf16(vfb), cu_q, cu_ctx, rope_mode=0)
    assert np.array_equal(host_bits(o_far.contiguous()), host_bits(o_near)), "the two ways of loading the query rows differ"
    del big


@pytest.mark.parametrize("route", ["contiguous", "block-table"])
def test_final_block_context_rows_beyond_four_gigabytes(ba, route):
    """The context's rows lie 16 MB apart (views with a token stride of 2^23 elements into 5 GB
    buffers), so the byte offsets of the later key tiles do not fit 32 bits; through
    ba_final_block_attention on a re-encoded context, and through the block table on two cached
    blocks stored in the opposite order."""
    torch = torch_mod()
    hq, hkv, d, base = 4, 1, 128, 10000.0
    tc, lq, stride = 300, 40, 1 << 23
    cu_q, cu_ctx = np.array([0, lq], dtype=np.int32), np.array([0, tc], dtype=np.int32)
    qb, kfb, vfb = gen_qkv(950, lq, hq, hkv, d)
    k_raw, vcb = wl.normal_bf16_bits(953, (tc, hkv, d)), wl.normal_bf16_bits(954, (tc, hkv, d))
    th = oracle.theta(base, d)
    f = oracle.bf16_bits_to_f64
    heads = ba.Heads(hq, hkv, d, base)

    def spread(bits):
        big = torch.empty(tc * stride, dtype=torch.bfloat16, device="cuda")
        view = big.as_strided((tc, hkv, d), (stride, d, 1))
        view.copy_(dev_bf16(bits))
        assert view.stride(0) * 2 * (tc - 1) > 1 << 32
        return view

    if route == "contiguous":
        k_view, v_view = spread(k_raw), spread(vcb)
        ref = oracle.final_block(f(qb), f(k_raw), f(vcb), f(kfb), f(vfb), cu_q, cu_ctx, th)
        o = gpu_final(ba, heads, dev_bf16(qb), k_view, v_view, dev_bf16(kfb), dev_bf16(vfb), cu_q, cu_ctx)
    else:
        # prompt = block 0 (tokens 0..149) then block 1 (150..299); the cache holds block 1 first,
        # each block's keys rotated at its local positions
        lens, cache_off = [150, 150], np.array([150, 0], dtype=np.int32)
        k_cache, v_cache, k_ctx = np.zeros_like(k_raw), np.zeros_like(vcb), np.zeros((tc, hkv, d))
        for b, (p0, L) in enumerate(((0, 150), (150, 150))):
            k_local = wl.f32_to_bf16_bits(oracle.rope_dense(f(k_raw[p0:p0 + L]), np.arange(L), th, 0).astype(np.float32))
            k_cache[cache_off[b]:cache_off[b] + L] = k_local
            v_cache[cache_off[b]:cache_off[b] + L] = vcb[p0:p0 + L]
            k_ctx[p0:p0 + L] = oracle.reencode(f(k_local), [0], [0], [L], th, old_pos0=[0], new_pos0=[p0])
        ref = oracle.final_block(f(qb), k_ctx, f(vcb), f(kfb), f(vfb), cu_q, cu_ctx, th)
        k_view, v_view = spread(k_cache), spread(v_cache)
        cu_blk, bl = np.array([0, 2], dtype=np.int32), np.array(lens, dtype=np.int32)
        o = torch.full((lq, hq, d), float("nan"), dtype=torch.bfloat16, device="cuda")
        ws = torch.empty(max(256, ba.ba_final_block_attention_cached_workspace_bytes(heads, cu_q, cu_blk, bl,
                                                                                     gather_below=0)),
                         dtype=torch.uint8, device="cuda")
        ba.ba_final_block_attention_cached(heads, dev_bf16(qb), k_view, v_view, dev_bf16(kfb), dev_bf16(vfb), o, None,
                                           cu_q, cu_blk, cache_off, bl, None, None, None, ws, gather_below=0)
        torch.cuda.synchronize()
    assert_attention_close(host_f64(o), ref, "context rows 16 MB apart, " + route)
    del k_view, v_view
    torch.cuda.empty_cache()


def test_final_block_over_300k_context_tokens_sampled(ba):
    """300,007 context tokens (4,688 key tiles, the last one ragged) behind 33 query tokens: the most
    splits the host plans, long walks per split; every fourth query row against the oracle."""
    hq, hkv, d, base = 4, 1, 128, 500000.0
    tc, lq = 300_007, 33
    cu_q, cu_ctx = np.array([0, lq], dtype=np.int32), np.array([0, tc], dtype=np.int32)
    qb, kfb, vfb = gen_qkv(960, lq, hq, hkv, d)
    kcb, vcb = wl.normal_bf16_bits(963, (tc, hkv, d)), wl.normal_bf16_bits(964, (tc, hkv, d))
    heads = ba.Heads(hq, hkv, d, base)
    o = gpu_final(ba, heads, dev_bf16(qb), dev_bf16(kcb), dev_bf16(vcb), dev_bf16(kfb), dev_bf16(vfb), cu_q, cu_ctx)
    rows = list(range(0, lq, 4)) + [lq - 1]
    f = oracle.bf16_bits_to_f64
    ref = oracle.final_block(f(qb), f(kcb), f(vcb), f(kfb), f(vfb), cu_q, cu_ctx, oracle.theta(base, d), rows=rows)
    assert_attention_close(host_f64(o)[rows], ref, "300,007 context tokens")


def _with_component(bits, rows, dim, value):
    """Copy of a bf16 tensor with one head dimension of some rows set to a value (exact in bf16)."""
    x = wl.bf16_bits_to_f32(bits).copy()
    x[rows, :, dim] = np.float32(value)
    return wl.f32_to_bf16_bits(x)


@pytest.mark.parametrize("where", ["final", "encode", "encode-short-blocks-schedule", "whole-prompt"])
def test_late_keys_far_above_first_tile_move_the_reference(ba, where):
    """Every query carries +8 and the first 64 keys carry -32 in a slowly rotating head dimension, so
    the first key tile scores about 46 (log2 units) below the later ones: a reference taken from
    the first tile has to move when the second arrives, and across KV splits the partials carry
    very different references.  The keys that matter have ordinary scores, so the usual
    tolerance applies."""
    # (two query heads per KV head take the main schedule in per-block encoding, four the short-block one)
    hq, hkv, d = (4, 2, 64) if where in ("final", "encode") else (8, 2, 64)
    th = oracle.theta(10000.0, d)
    f = oracle.bf16_bits_to_f64
    heads = ba.Heads(hq, hkv, d, 10000.0)
    slow = d - 2  # first element of the last interleaved pair: 1.3e-4 rad per position
    if where == "final":
        tc, lq = 1000, 70
        cu_q, cu_ctx = np.array([0, lq], dtype=np.int32), np.array([0, tc], dtype=np.int32)
        qb, kfb, vfb = gen_qkv(900, lq, hq, hkv, d)
        kcb, vcb = wl.normal_bf16_bits(903, (tc, hkv, d)), wl.normal_bf16_bits(904, (tc, hkv, d))
        qb = _with_component(qb, slice(None), slow, 8.0)
        kcb = _with_component(_with_component(kcb, slice(None), slow, 0.0), slice(0, 64), slow, -32.0)
        kfb = _with_component(kfb, slice(None), slow, 0.0)
        ref = oracle.final_block(f(qb), f(kcb), f(vcb), f(kfb), f(vfb), cu_q, cu_ctx, th)
        o = gpu_final(ba, heads, dev_bf16(qb), dev_bf16(kcb), dev_bf16(vcb), dev_bf16(kfb), dev_bf16(vfb), cu_q, cu_ctx)
    else:
        offs = np.array([0, 600, 900], dtype=np.int32)
        qb, kb, vb = gen_qkv(910, 900, hq, hkv, d)
        qb = _with_component(qb, slice(None), slow, 8.0)
        kb = _with_component(kb, slice(None), slow, 0.0)
        kb = _with_component(_with_component(kb, slice(0, 64), slow, -32.0), slice(600, 664), slow, -32.0)
        if where == "whole-prompt":  # one prompt: a passage and a last block that sees it
            ref = oracle.masked_attention_bruteforce(f(qb), f(kb), f(vb), offs, th)
            o, _, _ = gpu_prompts(ba, heads, qb, kb, vb, np.array([0, 2], dtype=np.int32), offs, want_k_rot=False)
        else:
            ref, _ = oracle.encode_blocks(f(qb), f(kb), f(vb), offs, th)
            o, _ = gpu_encode(ba, heads, qb, kb, vb, offs)
    assert_attention_close(host_f64(o), ref, "late keys far above the first tile, " + where)


def test_final_block_rope_none_qpos_override_and_rot_out(ba):
    torch = torch_mod()
    hq, hkv, d = 8, 2, 128
    cu_q, cu_ctx = np.array([0, 40], dtype=np.int32), np.array([0, 333], dtype=np.int32)
    qb, kfb, vfb = gen_qkv(400, 40, hq, hkv, d)
    kcb, vcb = wl.normal_bf16_bits(403, (333, hkv, d)), wl.normal_bf16_bits(404, (333, hkv, d))
    th = oracle.theta(10000.0, d)
    f = oracle.bf16_bits_to_f64
    heads = ba.Heads(hq, hkv, d, 10000.0)
    ref_none = oracle.final_block(f(qb), f(kcb), f(vcb), f(kfb), f(vfb), cu_q, cu_ctx, th, rope_mode=oracle.ROPE_NONE)
    o = gpu_final(ba, heads, dev_bf16(qb), dev_bf16(kcb), dev_bf16(vcb), dev_bf16(kfb), dev_bf16(vfb), cu_q, cu_ctx,
                  rope_mode=0)
    assert_attention_close(host_f64(o), ref_none, "rope none")
    ref_pos = oracle.final_block(f(qb), f(kcb), f(vcb), f(kfb), f(vfb), cu_q, cu_ctx, th, q_pos0=[5000])
    o = gpu_final(ba, heads, dev_bf16(qb), dev_bf16(kcb), dev_bf16(vcb), dev_bf16(kfb), dev_bf16(vfb), cu_q, cu_ctx,
                  q_pos0=[5000])
    assert_attention_close(host_f64(o), ref_pos, "q_pos0")
    # rotated final-block keys handed back for later decoding
    kf = dev_bf16(kfb)
    rot = torch.zeros_like(kf)
    out = torch.empty((40, hq, d), dtype=torch.bfloat16, device="cuda")
    nbytes = ba.ba_final_block_attention_workspace_bytes(heads, cu_q, cu_ctx, 1, True)
    ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")
    ba.ba_final_block_attention(heads, dev_bf16(qb), dev_bf16(kcb), dev_bf16(vcb), kf, dev_bf16(vfb), out, rot, cu_q,
                                cu_ctx, None, 1, ws)
    torch.cuda.synchronize()
    ref_rot = oracle.rope_dense(f(kfb), 333 + np.arange(40), th, 0)
    assert_reencode_bf16(host_bits(rot), ref_rot, 0, "k_f_rot_out")


# --------------------------------------------------------------------------------------------
# whole pipeline on the benchmark workloads
# --------------------------------------------------------------------------------------------
def run_pipeline_gpu(ba, w: wl.Workload, seed_cfg: int, layout=0):
    """encode passages -> re-encode to prompt positions -> final block.  Returns device
    outputs plus the host bit patterns of the inputs."""
    torch = torch_mod()
    hq, hkv, d = w.n_q_heads, w.n_kv_heads, w.head_dim
    offs = w.passage_block_offsets()
    cu_ctx, cu_q = w.cu_ctx(), w.cu_q()
    Tp, Tq = int(offs[-1]), int(cu_q[-1])
    qb, kb, vb = gen_qkv(wl.tensor_seed(seed_cfg, 0), Tp, hq, hkv, d)
    qfb, kfb, vfb = gen_qkv(wl.tensor_seed(seed_cfg, 10), Tq, hq, hkv, d)
    heads = heads_of(ba, w, layout)
    o_p, k_local = gpu_encode(ba, heads, qb, kb, vb, offs)
    lens = np.diff(offs)
    new_pos0 = w.passage_new_pos0()
    k_ctx = torch.empty_like(k_local)
    ba.ba_reencode_positions(heads, k_local, k_ctx, offs[:-1], offs[:-1], lens, None, new_pos0, ba.REENC_SHIFT)
    o_f = gpu_final(ba, heads, dev_bf16(qfb), k_ctx, dev_bf16(vb), dev_bf16(kfb), dev_bf16(vfb), cu_q, cu_ctx)
    return dict(o_p=o_p, k_local=k_local, k_ctx=k_ctx, o_f=o_f, qb=qb, kb=kb, vb=vb, qfb=qfb, kfb=kfb, vfb=vfb,
                offs=offs, lens=lens, new_pos0=new_pos0, cu_q=cu_q, cu_ctx=cu_ctx)


def bf16_round(x: np.ndarray) -> np.ndarray:
    """fp64 -> nearest bf16 -> fp64: the storage precision of the KV cache (bfloat16)."""
    return oracle.bf16_bits_to_f64(wl.f32_to_bf16_bits(x.astype(np.float32)))


def oracle_pipeline(w: wl.Workload, r, layout=0, enc_rows=None, fin_rows=None):
    """The three steps on the oracle alone, from the seeded inputs; the cache and the
    prompt's K buffer hold bf16, so the oracle rounds its own keys where they are stored."""
    f = oracle.bf16_bits_to_f64
    th = oracle.theta(w.rope_base, w.head_dim)
    o_p, k_local = oracle.encode_blocks(f(r["qb"]), f(r["kb"]), f(r["vb"]), r["offs"], th, layout=layout, rows=enc_rows)
    k_ctx = oracle.reencode(bf16_round(k_local), r["offs"][:-1], r["offs"][:-1], r["lens"], th,
                            new_pos0=r["new_pos0"], layout=layout)
    o_f = oracle.final_block(f(r["qfb"]), bf16_round(k_ctx), f(r["vb"]), f(r["kfb"]), f(r["vfb"]), r["cu_q"],
                             r["cu_ctx"], th, layout=layout, rows=fin_rows)
    return o_p, k_local, k_ctx, o_f


@pytest.mark.parametrize("cfg", [1, 2])
def test_pipeline_config_1_and_2(ba, cfg):
    w = wl.config1() if cfg == 1 else wl.config2()
    r = run_pipeline_gpu(ba, w, cfg)
    o_p, k_local, k_ctx, o_f = oracle_pipeline(w, r)
    assert_attention_close(host_f64(r["o_p"]), o_p, f"cfg{cfg} encode")
    assert_reencode_bf16(host_bits(r["k_local"]), k_local, 0, f"cfg{cfg} k_local")
    assert_reencode_bf16(host_bits(r["k_ctx"]), k_ctx, 0, f"cfg{cfg} re-encode", roundings=2)
    assert_attention_close(host_f64(r["o_f"]), o_f, f"cfg{cfg} final")
    # passage 0 moves by zero positions: copied bit for bit
    L0 = int(r["lens"][0])
    assert np.array_equal(host_bits(r["k_ctx"])[:L0], host_bits(r["k_local"])[:L0])


def test_pipeline_config_3_ragged_batch_sampled_rows(ba):
    """Config 3 at full size (8 prompts x 20 ragged passages); the oracle checks a sample of
    rows: block starts, block ends, tile edges and random tokens."""
    w = wl.config3()
    r = run_pipeline_gpu(ba, w, 3)
    offs = r["offs"]
    rng = np.random.default_rng(3)
    enc_rows = sorted(set(offs[:-1].tolist() + (offs[1:] - 1).tolist()
                          + [int(o) + 63 for o in offs[:-1]] + [int(o) + 64 for o in offs[:-1]]
                          + rng.integers(0, offs[-1], 200).tolist()))
    enc_rows = [t for t in enc_rows if 0 <= t < offs[-1]]
    o_p, k_local, k_ctx, o_f = oracle_pipeline(w, r, enc_rows=enc_rows)
    assert_attention_close(host_f64(r["o_p"])[enc_rows], o_p, "cfg3 encode (sampled rows)")
    assert_reencode_bf16(host_bits(r["k_local"]), k_local, 0, "cfg3 k_local")
    assert_reencode_bf16(host_bits(r["k_ctx"]), k_ctx, 0, "cfg3 re-encode", roundings=2)
    assert_attention_close(host_f64(r["o_f"]), o_f, "cfg3 final")


def test_config_4_reencode_full_size_sampled(ba):
    """Config 4 at full size in the benchmark's launch configuration (32 layers x 32 passages
    x 1000 tokens, permuted slots), in place and gather form; sampled tokens vs the oracle."""
    torch = torch_mod()
    w = wl.config4()
    hkv, d, L, P, nl = w.n_kv_heads, w.head_dim, 1000, 32, w.n_layers
    gen = torch.Generator(device="cuda").manual_seed(wl.tensor_seed(4, 0))
    cache = torch.randn((nl, P * L, hkv, d), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    src_off = (np.arange(P) * L).astype(np.int32)
    lens = np.full(P, L, dtype=np.int32)
    new_pos0 = w.extra["new_pos0"]
    heads = heads_of(ba, w)
    dst = torch.zeros_like(cache)
    ba.ba_reencode_positions(heads, cache, dst, src_off, new_pos0, lens, None, new_pos0, ba.REENC_SHIFT)
    torch.cuda.synchronize()
    th = oracle.theta(w.rope_base, d)
    rng = np.random.default_rng(4)
    for layer in [0, 13, nl - 1]:
        for b in rng.integers(0, P, 4).tolist() + [int(np.argmin(new_pos0)), int(np.argmax(new_pos0))]:
            us = sorted(set([0, 1, 31, 32, 63, 64, L - 1] + rng.integers(0, L, 8).tolist()))
            src_rows = host_bits(cache[layer, b * L:(b + 1) * L])[us]
            # a uniform shift: the oracle's Eq. 2 -> Eq. 3 on the sampled tokens, whose in-block
            # index cancels between the two rotations
            ref = oracle.reencode(oracle.bf16_bits_to_f64(src_rows), [0], [0], [len(us)], th,
                                  new_pos0=[int(new_pos0[b])])
            got = host_bits(dst[layer, new_pos0[b]:new_pos0[b] + L])[us]
            assert_reencode_bf16(got, ref, 0, f"cfg4 layer {layer} block {b}")
    # in place gives the same bits at the source offsets
    inplace = cache.clone()
    ba.ba_reencode_positions(heads, inplace, inplace, src_off, src_off, lens, None, new_pos0, ba.REENC_SHIFT)
    torch.cuda.synchronize()
    for b in [0, 7, 31]:
        assert torch.equal(inplace[:, b * L:(b + 1) * L], dst[:, new_pos0[b]:new_pos0[b] + L])
    # norm preservation holds at any size: pair norms of the output equal those of the input
    a = cache[5].float()
    o = inplace[5].float()
    na = (a[..., 0::2] ** 2 + a[..., 1::2] ** 2).sqrt()
    no = (o[..., 0::2] ** 2 + o[..., 1::2] ** 2).sqrt()
    assert float(((na - no).abs() / (na + 1e-3)).max()) < 2e-2


def test_config_5_final_block_full_size_sampled(ba):
    """Config 5 (31 x 1024 context + 256-token final block, Llama-3-8B heads), one layer, in the
    benchmark's launch configuration; the oracle computes sampled final-block rows."""
    torch = torch_mod()
    w = wl.config5(n_layers=1)
    hq, hkv, d = w.n_q_heads, w.n_kv_heads, w.head_dim
    Tc, Lq = w.prompts[0].t_ctx, w.prompts[0].final_len
    kcb = wl.normal_bf16_bits(wl.tensor_seed(5, 0), (Tc, hkv, d))
    vcb = wl.normal_bf16_bits(wl.tensor_seed(5, 1), (Tc, hkv, d))
    qb, kfb, vfb = gen_qkv(wl.tensor_seed(5, 2), Lq, hq, hkv, d)
    heads = heads_of(ba, w)
    cu_q, cu_ctx = w.cu_q(), w.cu_ctx()
    o = gpu_final(ba, heads, dev_bf16(qb), dev_bf16(kcb), dev_bf16(vcb), dev_bf16(kfb), dev_bf16(vfb), cu_q, cu_ctx)
    rows = sorted(set([0, 1, 15, 16, 63, 64, 65, 127, 128, 255] + np.random.default_rng(5).integers(0, Lq, 10).tolist()))
    f = oracle.bf16_bits_to_f64
    ref = oracle.final_block(f(qb), f(kcb), f(vcb), f(kfb), f(vfb), cu_q, cu_ctx, oracle.theta(w.rope_base, d), rows=rows)
    assert_attention_close(host_f64(o)[rows], ref, "cfg5 final (sampled rows)")
    # ... and as bench.py launches it: KV splits sized by the XCD speeds measured on this device (another
    # order of the work items, unequal splits), then by a skewed set that moves every cut
    wsp = torch.empty(ba.ba_measure_xcd_speed_workspace_bytes(), dtype=torch.uint8, device="cuda")
    for speeds in (ba.ba_measure_xcd_speed(wsp), [1.06, 0.97, 1.03, 0.99, 1.02, 0.98, 1.03, 0.92]):
        sized = ba.Heads(hq, hkv, d, w.rope_base, xcd_speed=speeds)
        o2 = gpu_final(ba, sized, dev_bf16(qb), dev_bf16(kcb), dev_bf16(vcb), dev_bf16(kfb), dev_bf16(vfb), cu_q, cu_ctx)
        assert_attention_close(host_f64(o2)[rows], ref, f"cfg5 final, splits sized by {speeds} (sampled rows)")


def test_config_5_final_block_from_block_cache_full_size_sampled(ba):
    """Config 5 through the block-cache entry point: the 31 cached passages stay at local positions
    (stored in shuffled order in the cache), the kernel turns the queries instead; sampled rows against
    the oracle's re-encode + final block."""
    torch = torch_mod()
    w = wl.config5(n_layers=1)
    hq, hkv, d = w.n_q_heads, w.n_kv_heads, w.head_dim
    Tc, Lq = w.prompts[0].t_ctx, w.prompts[0].final_len
    L = 1024
    nb = Tc // L
    kcache_b = wl.normal_bf16_bits(wl.tensor_seed(5, 40), (Tc, hkv, d))
    vcache_b = wl.normal_bf16_bits(wl.tensor_seed(5, 41), (Tc, hkv, d))
    qb, kfb, vfb = gen_qkv(wl.tensor_seed(5, 42), Lq, hq, hkv, d)
    order = np.random.default_rng(55).permutation(nb)  # prompt slot s holds cache block order[s]
    b_off = (order * L).astype(np.int32)
    b_len = np.full(nb, L, dtype=np.int32)
    heads = heads_of(ba, w)
    cu_q, cu_blk = np.array([0, Lq], dtype=np.int32), np.array([0, nb], dtype=np.int32)
    o = torch.full((Lq, hq, d), float("nan"), dtype=torch.bfloat16, device="cuda")
    ws = torch.empty(ba.ba_final_block_attention_cached_workspace_bytes(heads, cu_q, cu_blk, b_len), dtype=torch.uint8,
                     device="cuda")
    ba.ba_final_block_attention_cached(heads, dev_bf16(qb), dev_bf16(kcache_b), dev_bf16(vcache_b), dev_bf16(kfb),
                                       dev_bf16(vfb), o, None, cu_q, cu_blk, b_off, b_len, None, None, None, ws)
    torch.cuda.synchronize()
    f = oracle.bf16_bits_to_f64
    th = oracle.theta(w.rope_base, d)
    dst = (np.arange(nb) * L).astype(np.int32)
    k_ctx = oracle.reencode(f(kcache_b), b_off, dst, b_len, th, new_pos0=dst)
    v_ctx = f(vcache_b).reshape(nb, L, hkv, d)[order].reshape(Tc, hkv, d)
    rows = sorted(set([0, 1, 63, 64, 128, 255] + np.random.default_rng(6).integers(0, Lq, 8).tolist()))
    ref = oracle.final_block(f(qb), k_ctx, v_ctx, f(kfb), f(vfb), cu_q, [0, Tc], th, rows=rows)
    assert_attention_close(host_f64(o)[rows], ref, "cfg5 final from block cache (sampled rows)")
    # ... and with the KV splits sized by a skewed set of XCD speeds (as bench.py passes measured ones)
    sized = ba.Heads(hq, hkv, d, w.rope_base, xcd_speed=[1.06, 0.97, 1.03, 0.99, 1.02, 0.98, 1.03, 0.92])
    o2 = torch.full((Lq, hq, d), float("nan"), dtype=torch.bfloat16, device="cuda")
    ws2 = torch.empty(ba.ba_final_block_attention_cached_workspace_bytes(sized, cu_q, cu_blk, b_len), dtype=torch.uint8,
                      device="cuda")
    ba.ba_final_block_attention_cached(sized, dev_bf16(qb), dev_bf16(kcache_b), dev_bf16(vcache_b), dev_bf16(kfb),
                                       dev_bf16(vfb), o2, None, cu_q, cu_blk, b_off, b_len, None, None, None, ws2)
    torch.cuda.synchronize()
    assert_attention_close(host_f64(o2)[rows], ref, "cfg5 final from block cache, sized splits (sampled rows)")


def test_config_5_single_block_full_attention_sampled(ba):
    """The same 32,000 tokens as ONE block through ba_encode_blocks (full-attention mode);
    sampled rows (first rows, tile edges, last row, random) against the oracle."""
    w = wl.config5(n_layers=1)
    hq, hkv, d = w.n_q_heads, w.n_kv_heads, w.head_dim
    T = w.prompts[0].t_ctx + w.prompts[0].final_len
    qb, kb, vb = gen_qkv(wl.tensor_seed(5, 20), T, hq, hkv, d)
    heads = heads_of(ba, w)
    offs = np.array([0, T], dtype=np.int32)
    o, k_local = gpu_encode(ba, heads, qb, kb, vb, offs)
    rows = sorted(set([0, 1, 63, 64, 65, 4095, 4096, 16383, T - 1] + np.random.default_rng(6).integers(0, T, 7).tolist()))
    f = oracle.bf16_bits_to_f64
    ref, _ = oracle.encode_blocks(f(qb), f(kb), f(vb), offs, oracle.theta(w.rope_base, d), rows=rows, want_k_local=False)
    assert_attention_close(host_f64(o)[rows], ref, "cfg5 single block (sampled rows)")


def test_encode_long_and_short_blocks_in_one_call_sampled(ba):
    """One call whose blocks fall on both sides of the length at which per-block encoding changes
    schedule (one launch of each kernel), the long ones right at that length and well beyond it;
    sampled rows of every block against the oracle, and the cached keys of all rows."""
    hq, hkv, d, base = 4, 1, 128, 500000.0
    lens = [6144, 100, 6145, 3, 9000, 257]
    offs = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    T = int(offs[-1])
    qb, kb, vb = gen_qkv(230, T, hq, hkv, d)
    heads = ba.Heads(hq, hkv, d, base)
    o, k_local = gpu_encode(ba, heads, qb, kb, vb, offs)
    rng = np.random.default_rng(7)
    rows = []
    for b, L in enumerate(lens):
        inside = sorted(set([0, 1, min(31, L - 1), min(32, L - 1), L // 2, L - 1] + rng.integers(0, L, 3).tolist()))
        rows += [int(offs[b]) + r for r in inside]
    f = oracle.bf16_bits_to_f64
    th = oracle.theta(base, d)
    ref, ref_k = oracle.encode_blocks(f(qb), f(kb), f(vb), offs, th, rows=rows)
    assert_attention_close(host_f64(o)[rows], ref, "long and short blocks (sampled rows)")
    assert_reencode_bf16(host_bits(k_local), ref_k, 0, "long and short blocks k_local")


# --------------------------------------------------------------------------------------------
# final block straight from the block cache (re-encoding folded into the attention kernel)
def _cached_case(name):
    """Returns hq, hkv, d, base, cache block table (offset, len, old_pos0) and prompts
    [(block ids, final len, explicit new positions or None, explicit q_pos0 or None)]."""
    if name == "rag-shared-blocks":
        blocks = [(700, 100, 0), (0, 257, 0), (300, 64, 0), (1100, 1, 0), (400, 300, 0), (900, 129, 0), (1150, 0, 0)]
        prompts = [([3, 0, 6, 4], 33, None, None), ([4, 1, 2, 5, 0], 70, None, None), ([], 9, None, None)]
        return 8, 2, 128, 500000.0, 1200, blocks, prompts
    if name == "deep-split-d64":
        blocks = [(b * 210, 200 + (b % 3), 0) for b in range(20)]
        prompts = [(list(range(19, -1, -1)), 17, None, None)]
        return 2, 2, 64, 10000.0, 4300, blocks, prompts
    if name == "moved-cache-positions":
        # keys cached at other positions than 0, explicit (gapped) new positions and query position
        blocks = [(0, 150, 1000), (150, 90, 37), (240, 64, 0)]
        prompts = [([1, 2, 0], 40, [5, 200, 300], 777), ([0], 3, [10], None)]
        return 8, 8, 128, 10000.0, 310, blocks, prompts
    if name == "seventy-prompts-shared-cache":
        # more prompts than one launch's tables hold (and more than the small tables: the large ones);
        # every prompt picks three of twelve cached blocks, so blocks are shared between prompts
        blocks = [(b * 130, 100 + 7 * (b % 5), 0) for b in range(12)]
        prompts = [([(5 * n) % 12, (5 * n + 3) % 12, (7 * n + 1) % 12], 1 + n % 4, None, None) for n in range(70)]
        return 4, 1, 64, 10000.0, 12 * 130, blocks, prompts
    raise KeyError(name)


@pytest.fixture(params=["table", "gathered"])
def cached_route(request):
    """Both routes of ba_final_block_attention_cached: the kernel that reads the block table, and
    the gathered copy it takes for short blocks (forced either way through the call's gather_below)."""
    return 0 if request.param == "table" else 1 << 30


@pytest.mark.parametrize("name", ["rag-shared-blocks", "deep-split-d64", "moved-cache-positions",
                                  "seventy-prompts-shared-cache"])
@pytest.mark.parametrize("layout", [0, 1])
def test_final_block_from_block_cache_matches_oracle(ba, name, layout, cached_route):
    torch = torch_mod()
    hq, hkv, d, base, t_cache, blocks, prompts = _cached_case(name)
    th = oracle.theta(base, d)
    f = oracle.bf16_bits_to_f64
    seed = 1200 + len(name) + layout
    kcache_b = wl.normal_bf16_bits(seed, (t_cache, hkv, d))
    vcache_b = wl.normal_bf16_bits(seed + 1, (t_cache, hkv, d))
    lq_total = sum(p[1] for p in prompts)
    qb, kfb, vfb = gen_qkv(seed + 2, lq_total, hq, hkv, d)
    # block table in prompt order + the oracle's route: re-encode each use of a block (fp64), concatenate
    cu_q, cu_blk, b_off, b_len, b_old, b_new, q_pos0 = [0], [0], [], [], [], [], []
    k_ctx, v_ctx, cu_ctx = [], [], [0]
    explicit_new = any(p[2] is not None for p in prompts)
    for ids, lq, new_pos, qp in prompts:
        run = 0
        for j, b in enumerate(ids):
            off, ln, old = blocks[b]
            new0 = new_pos[j] if new_pos is not None else run
            b_off.append(off); b_len.append(ln); b_old.append(old); b_new.append(new0)
            if ln:
                k_ctx.append(oracle.reencode(f(kcache_b), [off], [0], [ln], th, old_pos0=[old], new_pos0=[new0],
                                             layout=layout, out=np.zeros((ln, hkv, d)))[:ln])
                v_ctx.append(f(vcache_b)[off:off + ln])
            run += ln
        cu_q.append(cu_q[-1] + lq); cu_blk.append(len(b_off)); cu_ctx.append(cu_ctx[-1] + run)
        q_pos0.append(qp if qp is not None else run)
    k_ctx = np.concatenate(k_ctx) if k_ctx else np.zeros((1, hkv, d))
    v_ctx = np.concatenate(v_ctx) if v_ctx else np.zeros((1, hkv, d))
    ref = oracle.final_block(f(qb), k_ctx, v_ctx, f(kfb), f(vfb), cu_q, cu_ctx, th, layout=layout, q_pos0=q_pos0)
    heads = ba.Heads(hq, hkv, d, base, rope_layout=layout)
    o = torch.full((lq_total, hq, d), float("nan"), dtype=torch.bfloat16, device="cuda")
    kf_rot = torch.full((lq_total, hkv, d), float("nan"), dtype=torch.bfloat16, device="cuda")
    nbytes = ba.ba_final_block_attention_cached_workspace_bytes(heads, cu_q, cu_blk, b_len, True, gather_below=cached_route)
    ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")
    ba.ba_final_block_attention_cached(heads, dev_bf16(qb), dev_bf16(kcache_b), dev_bf16(vcache_b), dev_bf16(kfb),
                                       dev_bf16(vfb), o, kf_rot, cu_q, cu_blk, b_off, b_len,
                                       b_old if any(b_old) else None, b_new if explicit_new else None,
                                       q_pos0 if any(p[3] is not None for p in prompts) else None, ws,
                                       gather_below=cached_route)
    torch.cuda.synchronize()
    assert_attention_close(host_f64(o), ref, "block cache, " + name)
    # the rotated final-block keys come out as in the plain entry point
    kf_ref = np.concatenate([oracle.rope_dense(f(kfb)[cu_q[n]:cu_q[n + 1]], np.arange(cu_q[n + 1] - cu_q[n]) + q_pos0[n], th,
                                               layout=layout) for n in range(len(prompts))])
    assert_reencode_bf16(host_bits(kf_rot), kf_ref, layout, "k_f_rot_out, " + name)


def test_final_block_from_block_cache_agrees_with_two_step_path(ba, cached_route):
    """Same inputs through ba_reencode_positions + ba_final_block_attention: the two GPU routes differ
    only by where the extra bf16 rounding falls (re-encoded keys there, re-turned queries here)."""
    torch = torch_mod()
    hq, hkv, d, base = 8, 2, 128, 500000.0
    lens = [300, 128, 77, 513]
    offs = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    T, lq = int(offs[-1]), 50
    kcache_b, vcache_b = wl.normal_bf16_bits(1300, (T, hkv, d)), wl.normal_bf16_bits(1301, (T, hkv, d))
    qb, kfb, vfb = gen_qkv(1302, lq, hq, hkv, d)
    heads = ba.Heads(hq, hkv, d, base)
    kc, vc = dev_bf16(kcache_b), dev_bf16(vcache_b)
    cu_q, cu_ctx = np.array([0, lq], dtype=np.int32), np.array([0, T], dtype=np.int32)
    k_ctx = torch.empty_like(kc)
    ba.ba_reencode_positions(heads, kc, k_ctx, offs[:-1], offs[:-1], lens, None, offs[:-1], ba.REENC_SHIFT)
    o2 = gpu_final(ba, heads, dev_bf16(qb), k_ctx, vc, dev_bf16(kfb), dev_bf16(vfb), cu_q, cu_ctx)
    o1 = torch.full_like(o2, float("nan"))
    cu_blk = np.array([0, len(lens)], dtype=np.int32)
    ws = torch.empty(max(ba.ba_final_block_attention_cached_workspace_bytes(heads, cu_q, cu_blk, lens,
                                                                            gather_below=cached_route), 256),
                     dtype=torch.uint8, device="cuda")
    ba.ba_final_block_attention_cached(heads, dev_bf16(qb), kc, vc, dev_bf16(kfb), dev_bf16(vfb), o1, None, cu_q,
                                       cu_blk, offs[:-1], lens, None, None, None, ws, gather_below=cached_route)
    torch.cuda.synchronize()
    assert_attention_close(host_f64(o1), host_f64(o2), "block cache vs two-step")


def test_many_small_blocks_incremental_frame_update(ba, cached_route):
    """Appendix A's workload in miniature: a prompt of 320 small state blocks, of which one changes
    (and changes length) from one frame to the next.  Only the changed block is encoded again
    (ba_encode_blocks, cacheable keys at local positions); every other block is reused from the
    cache as it is, although all blocks behind the changed one move; both frames against the oracle."""
    torch = torch_mod()
    hq, hkv, d, base = 8, 2, 64, 10000.0
    th = oracle.theta(base, d)
    f = oracle.bf16_bits_to_f64
    heads = ba.Heads(hq, hkv, d, base)
    rng = np.random.default_rng(77)
    n_blk = 320
    lens = rng.integers(20, 61, n_blk).astype(np.int32)
    slot = 64  # cache rows reserved per block
    cap = (n_blk + 1) * slot
    # un-rotated q, k, v of every block's tokens, laid out in their cache slots
    qb, kb, vb = gen_qkv(1400, cap, hq, hkv, d)
    offs = (np.arange(n_blk) * slot).astype(np.int32)
    kcache = torch.zeros((cap, hkv, d), dtype=torch.bfloat16, device="cuda")
    vcache = dev_bf16(vb)
    k_local_ref = np.zeros((cap, hkv, d))

    def encode_into_cache(b_ids):
        """ba_encode_blocks on the given blocks (each its own call list entry), k_local written to the slots"""
        for b in b_ids:
            o0, ln = int(offs[b]), int(lens[b])
            blk = np.array([0, ln], dtype=np.int32)
            q, k, v = dev_bf16(qb[o0:o0 + ln]), dev_bf16(kb[o0:o0 + ln]), dev_bf16(vb[o0:o0 + ln])
            o = torch.empty_like(q)
            ws = torch.empty(ba.ba_encode_blocks_workspace_bytes(heads, blk, 1, True), dtype=torch.uint8, device="cuda")
            ba.ba_encode_blocks(heads, q, k, v, o, kcache[o0:o0 + ln], blk, 1, ws)
            k_local_ref[o0:o0 + ln] = oracle.rope_dense(f(kb[o0:o0 + ln]), np.arange(ln), th, 0)

    lq = 30
    qf, kff, vff = gen_qkv(1410, lq, hq, hkv, d)
    cu_q, cu_blk = np.array([0, lq], dtype=np.int32), np.array([0, n_blk], dtype=np.int32)

    def frame(order):
        b_off, b_len = offs[order], lens[order]
        ws = torch.empty(ba.ba_final_block_attention_cached_workspace_bytes(heads, cu_q, cu_blk, b_len,
                                                                            gather_below=cached_route),
                         dtype=torch.uint8, device="cuda")
        o = torch.full((lq, hq, d), float("nan"), dtype=torch.bfloat16, device="cuda")
        ba.ba_final_block_attention_cached(heads, dev_bf16(qf), kcache, vcache, dev_bf16(kff), dev_bf16(vff), o, None,
                                           cu_q, cu_blk, b_off, b_len, None, None, None, ws, gather_below=cached_route)
        torch.cuda.synchronize()
        # oracle: its own cache (its fp64 rotation of the seeded keys, rounded to bf16 as a cache stores it),
        # re-encoded in fp64, then the final block
        kc64 = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(k_local_ref.astype(np.float32))).astype(np.float64)
        new0 = np.concatenate([[0], np.cumsum(b_len)[:-1]]).astype(np.int32)
        T = int(b_len.sum())
        k_ctx = oracle.reencode(kc64, b_off, new0, b_len, th, new_pos0=new0, out=np.zeros((T, hkv, d)))
        v_ctx = np.concatenate([f(vb)[o0:o0 + ln] for o0, ln in zip(b_off, b_len)])
        ref = oracle.final_block(f(qf), k_ctx, v_ctx, f(kff), f(vff), cu_q, [0, T], th)
        assert_attention_close(host_f64(o), ref, "many small blocks")

    order = np.arange(n_blk)
    encode_into_cache(range(n_blk))
    torch.cuda.synchronize()
    # the cached keys themselves against the oracle's rotation at local positions
    for b in (0, 17, n_blk - 1):
        o0, ln = int(offs[b]), int(lens[b])
        assert_reencode_bf16(host_bits(kcache[o0:o0 + ln]), k_local_ref[o0:o0 + ln], 0, "cached block %d" % b)
    frame(order)
    # next frame: block 100 is replaced by new content of another length, stored in the spare slot
    spare = n_blk
    offs2 = np.concatenate([offs, [spare * slot]]).astype(np.int32)
    lens2 = np.concatenate([lens, [int(lens[100]) + 9]]).astype(np.int32)
    offs, lens = offs2, lens2
    encode_into_cache([spare])
    order2 = order.copy()
    order2[100] = spare
    frame(order2)


def test_determinism_bitwise(ba):
    """Same inputs -> bitwise-same outputs across runs (the split merge has a fixed order)."""
    hq, hkv, d = 32, 8, 128
    cu_q, cu_ctx = np.array([0, 64], dtype=np.int32), np.array([0, 2000], dtype=np.int32)
    qb, kfb, vfb = gen_qkv(500, 64, hq, hkv, d)
    kcb, vcb = wl.normal_bf16_bits(503, (2000, hkv, d)), wl.normal_bf16_bits(504, (2000, hkv, d))
    heads = ba.Heads(hq, hkv, d, 500000.0)
    args = (dev_bf16(qb), dev_bf16(kcb), dev_bf16(vcb), dev_bf16(kfb), dev_bf16(vfb), cu_q, cu_ctx)
    a = host_bits(gpu_final(ba, heads, *args))
    for _ in range(3):
        assert np.array_equal(a, host_bits(gpu_final(ba, heads, *args)))


# --------------------------------------------------------------------------------------------
# whole prompts in one call (the mask of Section 2.4)
# --------------------------------------------------------------------------------------------
def gpu_prompts(ba, heads, qb, kb, vb, cu_blk, offs, rope_mode=1, want_k_rot=True):
    torch = torch_mod()
    T, hq, d = qb.shape
    q, k, v = dev_bf16(qb), dev_bf16(kb), dev_bf16(vb)
    o = torch.full_like(q, float("nan"))
    k_rot = torch.full_like(k, float("nan")) if (want_k_rot and rope_mode == 1) else None
    lse = torch.full((T, hq), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(max(1, ba.ba_block_attention_prompts_workspace_bytes(heads, cu_blk, offs, rope_mode, k_rot is not None)),
                     dtype=torch.uint8, device="cuda")
    ba.ba_block_attention_prompts(heads, q, k, v, o, k_rot, lse, cu_blk, offs, rope_mode, ws)
    torch.cuda.synchronize()
    return o, k_rot, lse


def oracle_prompt_lse(q, k, offs, th, layout, scale):
    """log-sum-exp of the scaled scores over each row's visible keys, from the explicit mask."""
    T, hq, d = q.shape
    hkv = k.shape[1]
    pos = np.arange(T)
    qr, kr = oracle.rope_dense(q, pos, th, layout), oracle.rope_dense(k, pos, th, layout)
    M = oracle.block_mask(offs)
    out = np.empty((T, hq))
    for h in range(hq):
        S = scale * (qr[:, h, :] @ kr[:, h // (hq // hkv), :].T)
        S = np.where(M, S, -np.inf)
        m = S.max(axis=1)
        out[:, h] = m + np.log(np.exp(S - m[:, None]).sum(axis=1))
    return out


PROMPT_CASES = [
    # (name, Hq, Hkv, D, base, per-prompt block lengths; the last block of a prompt sees the others)
    ("two-prompts-gqa4", 8, 2, 128, 500000.0, [[40, 33, 1, 70, 50], [5, 64, 31]]),
    ("one-block-prompts", 4, 1, 64, 10000.0, [[90], [1], [33]]),
    ("empty-blocks-gqa8", 8, 1, 64, 10000.0, [[0, 65, 0, 20], [32, 0, 96]]),
    ("ragged-gqa4-d128", 4, 1, 128, 10000.0, [[129, 64, 63, 130], [200, 57]]),
    # fewer than four query heads per KV head (run as groups of four with zero phantom heads)
    ("config1-mha-d64", 4, 4, 64, 10000.0, [[128, 128, 64]]),
    ("gqa2-d128", 4, 2, 128, 500000.0, [[40, 0, 97, 33], [1, 70]]),
    ("mha-one-head-d128", 1, 1, 128, 10000.0, [[65, 31], [130]]),
    ("gqa3-d64", 6, 2, 64, 10000.0, [[50, 77, 20]]),
]


@pytest.mark.parametrize("case", PROMPT_CASES, ids=[c[0] for c in PROMPT_CASES])
@pytest.mark.parametrize("layout", [0, 1])
def test_whole_prompts_match_the_masked_attention_definition(ba, case, layout):
    """ba_block_attention_prompts against dense softmax under the explicit Block-attention mask
    (positions inside the prompt), prompt by prompt; the row log-sum-exps and the rotated keys too."""
    name, hq, hkv, d, base, prompts = case
    lens = [l for p in prompts for l in p]
    offs = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    cu_blk = np.concatenate([[0], np.cumsum([len(p) for p in prompts])]).astype(np.int32)
    T = int(offs[-1])
    qb, kb, vb = gen_qkv(300 + len(name) + layout, T, hq, hkv, d)
    heads = ba.Heads(hq, hkv, d, base, rope_layout=layout)
    o, k_rot, lse = gpu_prompts(ba, heads, qb, kb, vb, cu_blk, offs)
    f = oracle.bf16_bits_to_f64
    th = oracle.theta(base, d)
    og, lg, kg = host_f64(o), lse.cpu().numpy().astype(np.float64), host_bits(k_rot)
    for n in range(len(prompts)):
        t0, t1 = int(offs[cu_blk[n]]), int(offs[cu_blk[n + 1]])
        if t1 == t0:
            continue
        po = offs[cu_blk[n]:cu_blk[n + 1] + 1] - t0
        q, k, v = f(qb[t0:t1]), f(kb[t0:t1]), f(vb[t0:t1])
        ref = oracle.masked_attention_bruteforce(q, k, v, po, th, layout=layout)
        assert_attention_close(og[t0:t1], ref, f"{name} prompt {n}")
        ref_lse = oracle_prompt_lse(q, k, po, th, layout, 1.0 / np.sqrt(d))
        assert np.max(np.abs(lg[t0:t1] - ref_lse)) < 2e-2, name  # bf16 q^ and k^ in the scores
        ref_k = oracle.rope_dense(k, np.arange(t1 - t0), th, layout)
        assert_reencode_bf16(kg[t0:t1], ref_k, layout, f"{name} rotated keys, prompt {n}")


def test_whole_prompts_agree_with_the_three_step_path(ba):
    """Passage rows of the one-call path equal ba_encode_blocks' (the same kernel at other
    positions) and last-block rows equal the re-encode + final-block route, both within the
    output tolerance; rope_mode NONE on pre-rotated inputs gives the one-call result bit for bit."""
    torch = torch_mod()
    hq, hkv, d, base = 8, 2, 128, 500000.0
    prompts = [[100, 37, 64], [70, 129, 20]]
    lens = [l for p in prompts for l in p]
    offs = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    cu_blk = np.array([0, 3, 6], dtype=np.int32)
    T = int(offs[-1])
    qb, kb, vb = gen_qkv(320, T, hq, hkv, d)
    heads = ba.Heads(hq, hkv, d, base)
    o, k_rot, _ = gpu_prompts(ba, heads, qb, kb, vb, cu_blk, offs)
    o_enc, _ = gpu_encode(ba, heads, qb, kb, vb, offs)
    og, oe = host_f64(o), host_f64(o_enc)
    for n in range(2):
        for b in range(cu_blk[n], cu_blk[n + 1] - 1):  # passages: every block but the prompt's last
            sl = slice(int(offs[b]), int(offs[b + 1]))
            assert np.max(np.abs(og[sl] - oe[sl])) <= 2e-2
    # pre-rotated route: rotate q with the oracle at prompt positions, take the kernel's own rotated keys
    f = oracle.bf16_bits_to_f64
    th = oracle.theta(base, d)
    pos = np.concatenate([np.arange(int(offs[cu_blk[n + 1]]) - int(offs[cu_blk[n]])) for n in range(2)])
    q_rot_bits = wl.f32_to_bf16_bits(oracle.rope_dense(f(qb), pos, th, 0).astype(np.float32))
    o2, _, _ = gpu_prompts(ba, heads, q_rot_bits, host_bits(k_rot), vb, cu_blk, offs, rope_mode=0)
    assert np.max(np.abs(host_f64(o2) - og)) <= 2e-2


def test_whole_prompts_config_3_sampled(ba):
    """Config 3's eight prompts (20 ragged passages each) with their query blocks appended, in one
    call; sampled rows against the oracle's per-block encoding (passages) and final-block attention
    over keys rotated at prompt positions (query blocks)."""
    w = wl.config3()
    hq, hkv, d = w.n_q_heads, w.n_kv_heads, w.head_dim
    prompts = [list(p.passage_lens) + [p.final_len] for p in w.prompts]
    lens = [l for p in prompts for l in p]
    offs = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    cu_blk = np.concatenate([[0], np.cumsum([len(p) for p in prompts])]).astype(np.int32)
    T = int(offs[-1])
    qb, kb, vb = gen_qkv(wl.tensor_seed(3, 60), T, hq, hkv, d)
    heads = heads_of(ba, w)
    o, k_rot, lse = gpu_prompts(ba, heads, qb, kb, vb, cu_blk, offs)
    og = host_f64(o)
    f = oracle.bf16_bits_to_f64
    th = oracle.theta(w.rope_base, d)
    rng = np.random.default_rng(11)
    # passages: the oracle's per-block encoding at local positions (relative positions are what count)
    rows = sorted(set(offs[:-1].tolist() + (offs[1:] - 1).tolist() + rng.integers(0, T, 150).tolist()))
    last_blocks = set(int(cu_blk[n + 1]) - 1 for n in range(len(prompts)))
    blk_of = np.searchsorted(offs, np.arange(T), side="right") - 1
    prow = [t for t in rows if 0 <= t < T and int(blk_of[t]) not in last_blocks]
    ref_p, _ = oracle.encode_blocks(f(qb), f(kb), f(vb), offs, th, rows=prow, want_k_local=False)
    assert_attention_close(og[prow], ref_p, "whole prompts, passage rows")
    # query blocks: context keys rotated at their position in the prompt
    for n in (0, 3, 7):
        t0, tf, t1 = int(offs[cu_blk[n]]), int(offs[cu_blk[n + 1] - 1]), int(offs[cu_blk[n + 1]])
        k_ctx = oracle.rope_dense(f(kb[t0:tf]), np.arange(tf - t0), th, 0)
        ref_f = oracle.final_block(f(qb[tf:t1]), k_ctx, f(vb[t0:tf]), f(kb[tf:t1]), f(vb[tf:t1]), [0, t1 - tf],
                                   [0, tf - t0], th)
        assert_attention_close(og[tf:t1], ref_f, f"whole prompts, query block of prompt {n}")
    assert np.isfinite(lse.cpu().numpy()).all()


# --------------------------------------------------------------------------------------------
# backward of whole prompts
# --------------------------------------------------------------------------------------------
# Every gradient element is a sum of products a_i * b_i that the kernels form from bf16 factors (P and dS
# rounded to bf16 for the MFMA, relative 2^-9; the rotated q^ and k^ rounded once, 2^-9; P and dS also
# carry the score error of those roundings, about 1.6e-3 relative) and add up in fp32, then round the
# sum to bf16 once (2^-9 of the element): at worst about 6e-3 * sum |a_i b_i| + 2^-9 |element|.  dS is
# itself a difference of two sums, dS = P * (dP - delta) with delta = rowsum(dO * O) taken from the
# bf16 output the caller hands back: the rounding of O (2^-9 |O| per element) moves delta by up to
# 2^-9 sum_d |dO_d O_d| whatever dP - delta comes to, so the scale of dq and dk counts dS with
# P * (sum_d |dO_d v_d| + sum_d |dO_d O_d|), not with |dS| (a row that sees one key has dS = 0 and still
# an error of 1e-2 to 2e-2 in dq).  The bound is therefore the forward pass's pair of numbers, per
# element, against A = max(1, sum of the absolute values of all products) (the oracle's
# masked_attention_backward_term_sums) instead of the tensor's largest entry.
GRAD_MAX_TOL = 2e-2
GRAD_MEAN_TOL = 2e-3


def assert_grad_close(got, ref, mag, what):
    scale = np.maximum(1.0, mag)
    err = np.abs(got - ref) / scale
    assert np.isfinite(got).all(), f"{what}: non-finite gradient"
    i = int(np.argmax(err))
    assert float(err.max()) <= GRAD_MAX_TOL, (f"{what}: err {np.abs(got - ref).flat[i]:.4g} on an entry of {ref.flat[i]:.4g} "
                                              f"whose terms add up to {mag.flat[i]:.4g} in absolute value")
    assert float(err.mean()) <= GRAD_MEAN_TOL, f"{what}: mean scaled err {err.mean():.4g}"


def oracle_grads(q, k, v, do, offs, th, layout=0):
    """(dq, dk, dv) and the per-element sums of absolute terms they are compared against."""
    rq, rk, rv, _ = oracle.masked_attention_backward_bruteforce(q, k, v, do, offs, th, layout=layout)
    return (rq, rk, rv), oracle.masked_attention_backward_term_sums(q, k, v, do, offs, th, layout=layout)


@pytest.mark.parametrize("case", PROMPT_CASES, ids=[c[0] for c in PROMPT_CASES])
@pytest.mark.parametrize("layout", [0, 1])
def test_whole_prompts_backward_matches_the_gradient_of_the_definition(ba, case, layout):
    torch = torch_mod()
    name, hq, hkv, d, base, prompts = case
    lens = [l for p in prompts for l in p]
    offs = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    cu_blk = np.concatenate([[0], np.cumsum([len(p) for p in prompts])]).astype(np.int32)
    T = int(offs[-1])
    qb, kb, vb = gen_qkv(400 + len(name) + layout, T, hq, hkv, d)
    dob = wl.normal_bf16_bits(440 + len(name) + layout, (T, hq, d))
    heads = ba.Heads(hq, hkv, d, base, rope_layout=layout)
    o, _, lse = gpu_prompts(ba, heads, qb, kb, vb, cu_blk, offs, want_k_rot=False)
    q, k, v, do = dev_bf16(qb), dev_bf16(kb), dev_bf16(vb), dev_bf16(dob)
    dq, dk, dv = (torch.full_like(x, float("nan")) for x in (q, k, v))
    ws = torch.empty(ba.ba_block_attention_prompts_backward_workspace_bytes(heads, cu_blk, offs), dtype=torch.uint8, device="cuda")
    ba.ba_block_attention_prompts_backward(heads, q, k, v, o, lse, do, dq, dk, dv, cu_blk, offs, ws)
    torch.cuda.synchronize()
    f = oracle.bf16_bits_to_f64
    th = oracle.theta(base, d)
    gq, gk, gv = host_f64(dq), host_f64(dk), host_f64(dv)
    for n in range(len(prompts)):
        t0, t1 = int(offs[cu_blk[n]]), int(offs[cu_blk[n + 1]])
        if t1 == t0:
            continue
        po = offs[cu_blk[n]:cu_blk[n + 1] + 1] - t0
        (rq, rk, rv), (aq, ak, av) = oracle_grads(f(qb[t0:t1]), f(kb[t0:t1]), f(vb[t0:t1]), f(dob[t0:t1]),
                                                                   po, th, layout=layout)
        assert_grad_close(gq[t0:t1], rq, aq, f"{name} dq, prompt {n}")
        assert_grad_close(gk[t0:t1], rk, ak, f"{name} dk, prompt {n}")
        assert_grad_close(gv[t0:t1], rv, av, f"{name} dv, prompt {n}")


def test_whole_prompts_backward_medium_prompts(ba):
    """Blocks of several key tiles and row tiles (a 700-token passage, a 300-token last block), a
    second prompt that is one block; every gradient entry against the oracle.  The call is repeated
    and must give the same bits (no atomics, every sum has one owner)."""
    torch = torch_mod()
    hq, hkv, d, base = 8, 2, 128, 500000.0
    prompts = [[700, 129, 5, 300], [450]]
    lens = [l for p in prompts for l in p]
    offs = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    cu_blk = np.array([0, 4, 5], dtype=np.int32)
    T = int(offs[-1])
    qb, kb, vb = gen_qkv(460, T, hq, hkv, d)
    dob = wl.normal_bf16_bits(463, (T, hq, d))
    heads = ba.Heads(hq, hkv, d, base)
    o, _, lse = gpu_prompts(ba, heads, qb, kb, vb, cu_blk, offs, want_k_rot=False)
    q, k, v, do = dev_bf16(qb), dev_bf16(kb), dev_bf16(vb), dev_bf16(dob)
    ws = torch.empty(ba.ba_block_attention_prompts_backward_workspace_bytes(heads, cu_blk, offs), dtype=torch.uint8, device="cuda")
    outs = []
    for _ in range(2):
        dq, dk, dv = (torch.full_like(x, float("nan")) for x in (q, k, v))
        ba.ba_block_attention_prompts_backward(heads, q, k, v, o, lse, do, dq, dk, dv, cu_blk, offs, ws)
        torch.cuda.synchronize()
        outs.append((host_bits(dq), host_bits(dk), host_bits(dv)))
    for a, b in zip(outs[0], outs[1]):
        assert np.array_equal(a, b)
    f = oracle.bf16_bits_to_f64
    th = oracle.theta(base, d)
    gq, gk, gv = (oracle.bf16_bits_to_f64(x) for x in outs[0])
    for n in range(2):
        t0, t1 = int(offs[cu_blk[n]]), int(offs[cu_blk[n + 1]])
        po = offs[cu_blk[n]:cu_blk[n + 1] + 1] - t0
        (rq, rk, rv), (aq, ak, av) = oracle_grads(f(qb[t0:t1]), f(kb[t0:t1]), f(vb[t0:t1]), f(dob[t0:t1]), po, th)
        assert_grad_close(gq[t0:t1], rq, aq, f"dq, prompt {n}")
        assert_grad_close(gk[t0:t1], rk, ak, f"dk, prompt {n}")
        assert_grad_close(gv[t0:t1], rv, av, f"dv, prompt {n}")


def test_whole_prompts_forward_and_backward_on_strided_views(ba):
    """q, k, v as views into one fused [T, Hq + 2 Hkv, D] projection buffer, the gradients written
    into views of a buffer of the same shape, o and d_out with padded head strides: every tensor of
    both calls has token and head strides of its own.  Memory outside the views must stay untouched."""
    torch = torch_mod()
    hq, hkv, d, base = 8, 2, 128, 500000.0
    prompts = [[150, 64, 33], [200]]
    lens = [l for p in prompts for l in p]
    offs = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    cu_blk = np.array([0, 3, 4], dtype=np.int32)
    T = int(offs[-1])
    qb, kb, vb = gen_qkv(480, T, hq, hkv, d)
    dob = wl.normal_bf16_bits(483, (T, hq, d))
    fused = torch.zeros((T, hq + 2 * hkv, d), dtype=torch.bfloat16, device="cuda")
    fused[:, :hq], fused[:, hq:hq + hkv], fused[:, hq + hkv:] = dev_bf16(qb), dev_bf16(kb), dev_bf16(vb)
    q, k, v = fused[:, :hq], fused[:, hq:hq + hkv], fused[:, hq + hkv:]
    o_big = torch.full((T, hq, 2, d), 7.0, dtype=torch.bfloat16, device="cuda")
    o = o_big[:, :, 1]
    do_big = torch.zeros((T + 3, hq + 1, d), dtype=torch.bfloat16, device="cuda")
    do_big[3:, 1:] = dev_bf16(dob)
    do = do_big[3:, 1:]
    grads = torch.full((T, hq + 2 * hkv, d), 5.0, dtype=torch.bfloat16, device="cuda")
    dv, dq, dk = grads[:, :hkv], grads[:, hkv:hkv + hq], grads[:, hkv + hq:]  # (another order than the inputs')
    lse = torch.full((T, hq), float("nan"), dtype=torch.float32, device="cuda")
    heads = ba.Heads(hq, hkv, d, base)
    ws_f = torch.empty(ba.ba_block_attention_prompts_workspace_bytes(heads, cu_blk, offs, 1, False), dtype=torch.uint8, device="cuda")
    ba.ba_block_attention_prompts(heads, q, k, v, o, None, lse, cu_blk, offs, 1, ws_f)
    ws_b = torch.empty(ba.ba_block_attention_prompts_backward_workspace_bytes(heads, cu_blk, offs), dtype=torch.uint8, device="cuda")
    ba.ba_block_attention_prompts_backward(heads, q, k, v, o, lse, do, dq, dk, dv, cu_blk, offs, ws_b)
    torch.cuda.synchronize()
    assert float((o_big[:, :, 0] - 7.0).abs().max()) == 0.0
    f = oracle.bf16_bits_to_f64
    th = oracle.theta(base, d)
    og, gq, gk, gv = host_f64(o), host_f64(dq), host_f64(dk), host_f64(dv)
    for n in range(2):
        t0, t1 = int(offs[cu_blk[n]]), int(offs[cu_blk[n + 1]])
        po = offs[cu_blk[n]:cu_blk[n + 1] + 1] - t0
        ref = oracle.masked_attention_bruteforce(f(qb[t0:t1]), f(kb[t0:t1]), f(vb[t0:t1]), po, th)
        assert_attention_close(og[t0:t1], ref, f"strided o, prompt {n}")
        (rq, rk, rv), (aq, ak, av) = oracle_grads(f(qb[t0:t1]), f(kb[t0:t1]), f(vb[t0:t1]), f(dob[t0:t1]), po, th)
        assert_grad_close(gq[t0:t1], rq, aq, f"strided dq, prompt {n}")
        assert_grad_close(gk[t0:t1], rk, ak, f"strided dk, prompt {n}")
        assert_grad_close(gv[t0:t1], rv, av, f"strided dv, prompt {n}")


def test_whole_prompts_backward_near_the_end_of_its_row_offsets(ba):
    """o, d_out and dq_out at a token stride of 2^19 elements with a 2,000-token passage: row offsets
    of almost 2^31 bytes inside a block, the most the two calls accept."""
    torch = torch_mod()
    hq, hkv, d, base = 4, 1, 64, 10000.0
    prompts, stride = [[2000, 1000]], 1 << 19
    offs, cu_blk = np.array([0, 2000, 3000], dtype=np.int32), np.array([0, 2], dtype=np.int32)
    T = 3000
    qb, kb, vb = gen_qkv(490, T, hq, hkv, d)
    dob = wl.normal_bf16_bits(493, (T, hq, d))

    def wide():
        big = torch.zeros(T * stride, dtype=torch.bfloat16, device="cuda")
        return big, big.as_strided((T, hq, d), (stride, d, 1))

    (o_big, o), (do_big, do), (dq_big, dq) = wide(), wide(), wide()
    do.copy_(dev_bf16(dob))
    q, k, v = dev_bf16(qb), dev_bf16(kb), dev_bf16(vb)
    dk, dv = torch.empty_like(k), torch.empty_like(v)
    lse = torch.empty((T, hq), dtype=torch.float32, device="cuda")
    heads = ba.Heads(hq, hkv, d, base)
    ws_f = torch.empty(ba.ba_block_attention_prompts_workspace_bytes(heads, cu_blk, offs, 1, False), dtype=torch.uint8, device="cuda")
    ba.ba_block_attention_prompts(heads, q, k, v, o, None, lse, cu_blk, offs, 1, ws_f)
    ws_b = torch.empty(ba.ba_block_attention_prompts_backward_workspace_bytes(heads, cu_blk, offs), dtype=torch.uint8, device="cuda")
    ba.ba_block_attention_prompts_backward(heads, q, k, v, o, lse, do, dq, dk, dv, cu_blk, offs, ws_b)
    torch.cuda.synchronize()
    f = oracle.bf16_bits_to_f64
    th = oracle.theta(base, d)
    ref = oracle.masked_attention_bruteforce(f(qb), f(kb), f(vb), offs, th)
    assert_attention_close(host_f64(o), ref, "wide strides, forward")
    (rq, rk, rv), (aq, ak, av) = oracle_grads(f(qb), f(kb), f(vb), f(dob), offs, th)
    assert_grad_close(host_f64(dq), rq, aq, "wide strides, dq")
    assert_grad_close(host_f64(dk), rk, ak, "wide strides, dk")
    assert_grad_close(host_f64(dv), rv, av, "wide strides, dv")
    del o_big, do_big, dq_big, o, do, dq
    torch.cuda.empty_cache()


def test_calls_on_two_streams_at_once_do_not_disturb_each_other(ba):
    """Two independent final-block problems (their own tensors and workspaces) issued alternately on
    two streams, thirty calls each without a synchronisation in between, give the bits of the same
    calls issued alone: the library keeps no state between calls that two streams could share."""
    torch = torch_mod()
    hq, hkv, d = 8, 2, 128
    heads = ba.Heads(hq, hkv, d, 500000.0)
    probs = []
    for j, (tc, lq) in enumerate(((3000, 70), (1111, 130))):
        cu_q, cu_ctx = np.array([0, lq], dtype=np.int32), np.array([0, tc], dtype=np.int32)
        qb, kfb, vfb = gen_qkv(1500 + 10 * j, lq, hq, hkv, d)
        kcb, vcb = wl.normal_bf16_bits(1503 + 10 * j, (tc, hkv, d)), wl.normal_bf16_bits(1504 + 10 * j, (tc, hkv, d))
        t = [dev_bf16(x) for x in (qb, kcb, vcb, kfb, vfb)]
        ws = torch.empty(max(256, ba.ba_final_block_attention_workspace_bytes(heads, cu_q, cu_ctx, 1, False)), dtype=torch.uint8,
                         device="cuda")
        probs.append((t, cu_q, cu_ctx, ws, torch.empty((lq, hq, d), dtype=torch.bfloat16, device="cuda")))

    def call(j, stream=None):
        t, cu_q, cu_ctx, ws, o = probs[j]
        ba.ba_final_block_attention(heads, t[0], t[1], t[2], t[3], t[4], o, None, cu_q, cu_ctx, None, 1, ws, stream=stream)

    alone = []
    for j in range(2):
        call(j)
        torch.cuda.synchronize()
        alone.append(host_bits(probs[j][4]).copy())
        probs[j][4].fill_(float("nan"))
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    torch.cuda.synchronize()
    for _ in range(30):
        for j in range(2):
            call(j, streams[j])
    torch.cuda.synchronize()
    for j in range(2):
        assert np.array_equal(host_bits(probs[j][4]), alone[j]), f"problem {j}"


def test_calls_can_be_captured_in_a_hip_graph(ba):
    """The library only enqueues kernels on the caller's stream (no allocation, no copy, no
    synchronisation), so a sequence of calls can be captured and replayed: several replays, with
    eager work and synchronisations in between, give the eager result bit for bit."""
    torch = torch_mod()
    w = wl.config2()
    hq, hkv, d = w.n_q_heads, w.n_kv_heads, w.head_dim
    offs = w.passage_block_offsets()
    T, lq = int(offs[-1]), w.prompts[0].final_len
    qb, kb, vb = gen_qkv(500, T, hq, hkv, d)
    qfb, kfb, vfb = gen_qkv(503, lq, hq, hkv, d)
    heads = heads_of(ba, w)
    q, k, v, qf, kf, vf = (dev_bf16(x) for x in (qb, kb, vb, qfb, kfb, vfb))
    o_p, k_local, k_ctx = torch.empty_like(q), torch.empty_like(k), torch.empty_like(k)
    o_f = torch.empty_like(qf)
    cu_q, cu_ctx = w.cu_q(), w.cu_ctx()
    ws_e = torch.empty(ba.ba_encode_blocks_workspace_bytes(heads, offs, 1, True), dtype=torch.uint8, device="cuda")
    ws_f = torch.empty(ba.ba_final_block_attention_workspace_bytes(heads, cu_q, cu_ctx), dtype=torch.uint8, device="cuda")
    lens, new_pos0 = np.diff(offs), w.passage_new_pos0()

    def pipeline():
        ba.ba_encode_blocks(heads, q, k, v, o_p, k_local, offs, 1, ws_e)
        ba.ba_reencode_positions(heads, k_local, k_ctx, offs[:-1], offs[:-1], lens, None, new_pos0, ba.REENC_SHIFT)
        ba.ba_final_block_attention(heads, qf, k_ctx, v, kf, vf, o_f, None, cu_q, cu_ctx, None, 1, ws_f)

    pipeline()
    torch.cuda.synchronize()
    ref = (o_p.clone(), k_ctx.clone(), o_f.clone())
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        pipeline()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        pipeline()
    for rep in range(3):
        for t in (o_p, k_ctx, o_f):
            t.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, want in zip((o_p, k_ctx, o_f), ref):
            assert torch.equal(got, want), f"replay {rep}"
        pipeline()  # eager work between the replays
        torch.cuda.synchronize()


def test_whole_prompts_many_tiny_blocks_forward_and_backward(ba):
    """More blocks than one launch's table holds (two prompts of 230 blocks of 1 to 9 tokens each):
    the host cuts the list into several launches; outputs and gradients against the oracle."""
    torch = torch_mod()
    hq, hkv, d, base = 4, 1, 64, 10000.0
    rng = np.random.default_rng(91)
    prompts = [rng.integers(1, 10, 230).tolist(), rng.integers(1, 10, 230).tolist()]
    lens = [l for p in prompts for l in p]
    offs = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    cu_blk = np.array([0, 230, 460], dtype=np.int32)
    T = int(offs[-1])
    qb, kb, vb = gen_qkv(520, T, hq, hkv, d)
    dob = wl.normal_bf16_bits(523, (T, hq, d))
    heads = ba.Heads(hq, hkv, d, base)
    o, _, lse = gpu_prompts(ba, heads, qb, kb, vb, cu_blk, offs, want_k_rot=False)
    q, k, v, do = dev_bf16(qb), dev_bf16(kb), dev_bf16(vb), dev_bf16(dob)
    dq, dk, dv = (torch.full_like(x, float("nan")) for x in (q, k, v))
    ws = torch.empty(ba.ba_block_attention_prompts_backward_workspace_bytes(heads, cu_blk, offs), dtype=torch.uint8, device="cuda")
    ba.ba_block_attention_prompts_backward(heads, q, k, v, o, lse, do, dq, dk, dv, cu_blk, offs, ws)
    torch.cuda.synchronize()
    f = oracle.bf16_bits_to_f64
    th = oracle.theta(base, d)
    og, gq, gk, gv = host_f64(o), host_f64(dq), host_f64(dk), host_f64(dv)
    for n in range(2):
        t0, t1 = int(offs[cu_blk[n]]), int(offs[cu_blk[n + 1]])
        po = offs[cu_blk[n]:cu_blk[n + 1] + 1] - t0
        ref = oracle.masked_attention_bruteforce(f(qb[t0:t1]), f(kb[t0:t1]), f(vb[t0:t1]), po, th)
        assert_attention_close(og[t0:t1], ref, f"many tiny blocks, prompt {n}")
        (rq, rk, rv), (aq, ak, av) = oracle_grads(f(qb[t0:t1]), f(kb[t0:t1]), f(vb[t0:t1]), f(dob[t0:t1]), po, th)
        assert_grad_close(gq[t0:t1], rq, aq, f"dq, prompt {n}")
        assert_grad_close(gk[t0:t1], rk, ak, f"dk, prompt {n}")
        assert_grad_close(gv[t0:t1], rv, av, f"dv, prompt {n}")


# --------------------------------------------------------------------------------------------
# drawn shapes: every entry point on shapes nobody picked by hand
# --------------------------------------------------------------------------------------------
def _drawn_lengths(rng, k, hi):
    kind = int(rng.integers(0, 3))
    if kind == 0:
        return [int(x) for x in rng.integers(0, hi, k)]
    if kind == 1:  # around the tile sizes
        return [int(x) for x in rng.choice([1, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 257], k)]
    return [int(x) for x in rng.integers(1, 40, k)]


@pytest.mark.parametrize("seed", [11, 12, 13, 14])
def test_drawn_shapes_match_the_oracle(ba, seed):
    """Twelve cases per seed, drawn from: head_dim 64 / 128, 1-3 KV heads, 1-8 query heads per KV head,
    both pair layouts, two RoPE bases; per-block encoding, batched final blocks, whole prompts forward
    and backward, and the final block over a permuted block cache on both of its routes."""
    torch = torch_mod()
    rng = np.random.default_rng(seed)
    f = oracle.bf16_bits_to_f64
    for case in range(12):
        d, hkv, g = int(rng.choice([64, 128])), int(rng.choice([1, 2, 3])), int(rng.choice([1, 2, 3, 4, 5, 8]))
        base, layout = float(rng.choice([1e4, 5e5])), int(rng.integers(0, 2))
        kind, s0 = case % 4, int(rng.integers(0, 10 ** 6))
        hq = hkv * g
        th = oracle.theta(base, d)
        speeds = [float(x) for x in rng.uniform(0.8, 1.25, 8)] if kind in (1, 3) and rng.integers(0, 2) else None
        heads = ba.Heads(hq, hkv, d, base, rope_layout=layout, xcd_speed=speeds)
        tag = f"seed {seed} case {case}: D {d}, {hq}/{hkv} heads, layout {layout}" + (", XCD speeds" if speeds else "")
        if kind == 0:
            lens = _drawn_lengths(rng, int(rng.integers(1, 7)), 400)
            offs = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
            if offs[-1] == 0:
                continue
            qb, kb, vb = gen_qkv(s0, int(offs[-1]), hq, hkv, d)
            ref_o, ref_k = oracle.encode_blocks(f(qb), f(kb), f(vb), offs, th, layout=layout)
            o, k_local = gpu_encode(ba, heads, qb, kb, vb, offs)
            assert_attention_close(host_f64(o), ref_o, f"{tag}, encode {lens}")
            assert_reencode_bf16(host_bits(k_local), ref_k, layout, f"{tag}, k_local {lens}")
        elif kind == 1:
            shapes = [(int(rng.choice([0, 1, 63, 64, 65, 200, 700, 1500, 3000])), int(rng.choice([1, 2, 17, 64, 65, 130])))
                      for _ in range(int(rng.integers(1, 5)))]
            cu_ctx = np.concatenate([[0], np.cumsum([s[0] for s in shapes])]).astype(np.int32)
            cu_q = np.concatenate([[0], np.cumsum([s[1] for s in shapes])]).astype(np.int32)
            qb, kfb, vfb = gen_qkv(s0, int(cu_q[-1]), hq, hkv, d)
            kcb = wl.normal_bf16_bits(s0 + 3, (max(int(cu_ctx[-1]), 1), hkv, d))
            vcb = wl.normal_bf16_bits(s0 + 4, (max(int(cu_ctx[-1]), 1), hkv, d))
            ref = oracle.final_block(f(qb), f(kcb)[:cu_ctx[-1]], f(vcb)[:cu_ctx[-1]], f(kfb), f(vfb), cu_q, cu_ctx, th,
                                     layout=layout)
            o = gpu_final(ba, heads, dev_bf16(qb), dev_bf16(kcb), dev_bf16(vcb), dev_bf16(kfb), dev_bf16(vfb), cu_q, cu_ctx)
            assert_attention_close(host_f64(o), ref, f"{tag}, final {shapes}")
        elif kind == 2:
            prompts = [_drawn_lengths(rng, int(rng.integers(1, 5)), 150) for _ in range(int(rng.integers(1, 4)))]
            prompts = [p if sum(p) > 0 else p + [5] for p in prompts]
            lens = [l for p in prompts for l in p]
            offs = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
            cu_blk = np.concatenate([[0], np.cumsum([len(p) for p in prompts])]).astype(np.int32)
            T = int(offs[-1])
            qb, kb, vb = gen_qkv(s0, T, hq, hkv, d)
            dob = wl.normal_bf16_bits(s0 + 9, (T, hq, d))
            o, _, lse = gpu_prompts(ba, heads, qb, kb, vb, cu_blk, offs, want_k_rot=False)
            q, k, v, do = dev_bf16(qb), dev_bf16(kb), dev_bf16(vb), dev_bf16(dob)
            dq, dk, dv = (torch.full_like(x, float("nan")) for x in (q, k, v))
            ws = torch.empty(ba.ba_block_attention_prompts_backward_workspace_bytes(heads, cu_blk, offs), dtype=torch.uint8,
                             device="cuda")
            ba.ba_block_attention_prompts_backward(heads, q, k, v, o, lse, do, dq, dk, dv, cu_blk, offs, ws)
            torch.cuda.synchronize()
            og, gq, gk, gv = host_f64(o), host_f64(dq), host_f64(dk), host_f64(dv)
            for n in range(len(prompts)):
                t0, t1 = int(offs[cu_blk[n]]), int(offs[cu_blk[n + 1]])
                po = offs[cu_blk[n]:cu_blk[n + 1] + 1] - t0
                ref = oracle.masked_attention_bruteforce(f(qb[t0:t1]), f(kb[t0:t1]), f(vb[t0:t1]), po, th, layout=layout)
                assert_attention_close(og[t0:t1], ref, f"{tag}, prompts {prompts}")
                (rq, rk, rv), (aq, ak, av) = oracle_grads(f(qb[t0:t1]), f(kb[t0:t1]), f(vb[t0:t1]),
                                                                           f(dob[t0:t1]), po, th, layout=layout)
                assert_grad_close(gq[t0:t1], rq, aq, f"{tag}, dq {prompts}")
                assert_grad_close(gk[t0:t1], rk, ak, f"{tag}, dk {prompts}")
                assert_grad_close(gv[t0:t1], rv, av, f"{tag}, dv {prompts}")
        else:
            nb, lq, gathered = int(rng.integers(1, 9)), int(rng.choice([1, 17, 64, 90])), bool(rng.integers(0, 2))
            lens = [max(1, x) for x in _drawn_lengths(rng, nb, 300)]
            Tc, order = int(sum(lens)), rng.permutation(nb)
            k_raw, vb = wl.normal_bf16_bits(s0, (Tc, hkv, d)), wl.normal_bf16_bits(s0 + 1, (Tc, hkv, d))
            qb, kfb, vfb = gen_qkv(s0 + 2, lq, hq, hkv, d)
            cache_off, at = np.zeros(nb, dtype=np.int32), 0
            for b in order:  # the cache holds the blocks in another order than the prompt
                cache_off[b] = at
                at += lens[b]
            k_cache, v_cache = np.zeros((Tc, hkv, d), dtype=np.uint16), np.zeros((Tc, hkv, d), dtype=np.uint16)
            k_ctx, pos = np.zeros((Tc, hkv, d)), 0
            for b in range(nb):
                L = lens[b]
                k_local = wl.f32_to_bf16_bits(oracle.rope_dense(f(k_raw[pos:pos + L]), np.arange(L), th, layout).astype(np.float32))
                k_cache[cache_off[b]:cache_off[b] + L] = k_local
                v_cache[cache_off[b]:cache_off[b] + L] = vb[pos:pos + L]
                k_ctx[pos:pos + L] = oracle.reencode(f(k_local), [0], [0], [L], th, layout=layout, old_pos0=[0], new_pos0=[pos])
                pos += L
            ref = oracle.final_block(f(qb), k_ctx, f(vb), f(kfb), f(vfb), [0, lq], [0, Tc], th, layout=layout)
            cu_q, cu_blk, bl = np.array([0, lq], dtype=np.int32), np.array([0, nb], dtype=np.int32), np.array(lens, dtype=np.int32)
            gb = 10 ** 6 if gathered else 0
            o = torch.full((lq, hq, d), float("nan"), dtype=torch.bfloat16, device="cuda")
            ws = torch.empty(max(256, ba.ba_final_block_attention_cached_workspace_bytes(heads, cu_q, cu_blk, bl,
                                                                                         gather_below=gb)),
                             dtype=torch.uint8, device="cuda")
            ba.ba_final_block_attention_cached(heads, dev_bf16(qb), dev_bf16(k_cache), dev_bf16(v_cache), dev_bf16(kfb),
                                               dev_bf16(vfb), o, None, cu_q, cu_blk, cache_off, bl, None, None, None, ws,
                                               gather_below=gb)
            torch.cuda.synchronize()
            assert_attention_close(host_f64(o), ref, f"{tag}, cached {lens} x {lq}, {'gathered' if gathered else 'table'}")


@pytest.mark.parametrize("seed", [21, 22, 23])
def test_drawn_reencode_cases_match_the_oracle(ba, seed):
    """Sixteen re-encode cases per seed: 1-3 layers, 1-6 blocks (some empty) gathered into a permuted
    destination, both dtypes, both modes, both layouts, old and new positions anywhere in 0..131071
    (so shifts of either sign), head counts that take the kernel's different head splits, and for
    half of the bf16 cases a head-strided source (a view into a wider cache)."""
    torch = torch_mod()
    rng = np.random.default_rng(seed)
    for case in range(16):
        d, hkv = int(rng.choice([64, 128])), int(rng.choice([1, 2, 8]))
        layout, mode, f32 = int(rng.integers(0, 2)), int(rng.integers(0, 2)), bool(rng.integers(0, 2))
        base, n_layers, nb = float(rng.choice([1e4, 5e5])), int(rng.integers(1, 4)), int(rng.integers(1, 7))
        lens = [int(x) for x in rng.choice([0, 1, 7, 64, 100, 257, 600], nb)]
        src_off = np.concatenate([[0], np.cumsum(lens)[:-1]]).astype(np.int32)
        T = max(int(np.sum(lens)), 1)
        dst_off, at = np.zeros(nb, dtype=np.int32), 0
        for b in rng.permutation(nb):
            dst_off[b] = at
            at += lens[b]
        old = (np.zeros(nb) if mode == 1 else rng.integers(0, 131072, nb)).astype(np.int32)
        new = rng.integers(0, 131072, nb).astype(np.int32)
        th = oracle.theta(base, d)
        heads = ba.Heads(hkv, hkv, d, base, rope_layout=layout)
        tag = f"seed {seed} case {case}: D {d}, {hkv} heads, layout {layout}, mode {mode}, {'f32' if f32 else 'bf16'}, {lens}"
        if f32:
            k = wl.normal_f32(seed * 100 + case, (n_layers, T, hkv, d))
            ref = oracle.reencode(k.astype(np.float64), src_off, dst_off, lens, th, old_pos0=old, new_pos0=new, mode=mode,
                                  layout=layout)
            src = torch.from_numpy(k).cuda()
            dst = torch.zeros_like(src)
            ba.ba_reencode_positions(heads, src, dst, src_off, dst_off, lens, old, new, mode)
            torch.cuda.synchronize()
            rel = pair_norm_rel_err(host_f64(dst), ref, layout)
            assert rel <= REENC_F32_REL_TOL, f"{tag}: relative error {rel:.3e}"
        else:
            kb = wl.normal_bf16_bits(seed * 100 + case, (n_layers, T, hkv, d))
            ref = oracle.reencode(oracle.bf16_bits_to_f64(kb), src_off, dst_off, lens, th, old_pos0=old, new_pos0=new,
                                  mode=mode, layout=layout)
            if case % 2:  # the source as a view into a cache with twice the heads
                wide = torch.zeros((n_layers, T, 2 * hkv, d), dtype=torch.bfloat16, device="cuda")
                wide[:, :, hkv:] = dev_bf16(kb)
                src = wide[:, :, hkv:]
            else:
                src = dev_bf16(kb)
            dst = torch.zeros((n_layers, T, hkv, d), dtype=torch.bfloat16, device="cuda")
            ba.ba_reencode_positions(heads, src, dst, src_off, dst_off, lens, old, new, mode)
            torch.cuda.synchronize()
            assert_reencode_bf16(host_bits(dst), ref, layout, tag)


def test_final_block_with_splits_sized_by_xcd_speed(ba):
    """ba_heads.xcd_speed: unequal KV splits (here with strongly skewed speeds, so that every split
    boundary moves) give the oracle's result like the equal ones; and the probe that measures the
    speeds returns eight numbers with mean 1 that lie within what XCD clocks differ by."""
    torch = torch_mod()
    hq, hkv, d, lq, tc = 8, 2, 128, 70, 9000
    qb, kfb, vfb = gen_qkv(8100, lq, hq, hkv, d)
    kcb, vcb = wl.normal_bf16_bits(8103, (tc, hkv, d)), wl.normal_bf16_bits(8104, (tc, hkv, d))
    cu_q, cu_ctx = np.array([0, lq], dtype=np.int32), np.array([0, tc], dtype=np.int32)
    f = oracle.bf16_bits_to_f64
    ref = oracle.final_block(f(qb), f(kcb), f(vcb), f(kfb), f(vfb), cu_q, cu_ctx, oracle.theta(500000.0, d))
    outs = []
    for speeds in (None, [0.6, 1.9, 0.8, 1.2, 0.5, 2.0, 1.0, 1.0], [1.03, 0.97, 1.0, 1.0, 1.02, 0.98, 1.01, 0.99]):
        heads = ba.Heads(hq, hkv, d, 500000.0, xcd_speed=speeds)
        o = gpu_final(ba, heads, dev_bf16(qb), dev_bf16(kcb), dev_bf16(vcb), dev_bf16(kfb), dev_bf16(vfb), cu_q, cu_ctx)
        assert_attention_close(host_f64(o), ref, f"speeds {speeds}")
        outs.append(host_bits(o))
    assert len(ba.ba_schedule_final_block(ba.Heads(hq, hkv, d), cu_q, cu_ctx)) > 2  # (several splits, or the test is idle)
    ws = torch.empty(ba.ba_measure_xcd_speed_workspace_bytes(), dtype=torch.uint8, device="cuda")
    sp = ba.ba_measure_xcd_speed(ws)
    assert len(sp) == 8 and abs(sum(sp) / 8 - 1.0) < 1e-3 and all(0.8 < x < 1.25 for x in sp), sp
    # measured speeds are accepted as they come
    heads = ba.Heads(hq, hkv, d, 500000.0, xcd_speed=sp)
    o = gpu_final(ba, heads, dev_bf16(qb), dev_bf16(kcb), dev_bf16(vcb), dev_bf16(kfb), dev_bf16(vfb), cu_q, cu_ctx)
    assert_attention_close(host_f64(o), ref, "measured speeds")


@pytest.mark.gpu
def test_phase_marks_of_a_final_block_launch_are_consistent(ba):
    """The diagnostic's phases are positive, add up to the workgroup lifetime, and fit inside the launch."""
    torch = torch_mod()
    ws = torch.empty(ba.ba_measure_xcd_speed_workspace_bytes(), dtype=torch.uint8, device="cuda")
    ph = ba.ba_diag_final_block_phases(ws, xcd_speed=[1.02, 0.98, 1.0, 1.0, 1.01, 0.99, 1.0, 1.0])
    parts = [ph[k] for k in ba.DIAG_PHASES[:5]]
    assert all(x > 0.0 for x in parts), ph
    assert abs(sum(parts) - ph["workgroup_lifetime"]) < 0.05, ph
    assert ph["walk"] <= ph["longest_walk"] <= ph["launch_first_entry_to_last_store"], ph
    assert ph["workgroup_lifetime"] <= ph["launch_first_entry_to_last_store"] < 1000.0, ph
    # the walk is most of a workgroup's life at this shape (62 or 63 key tiles)
    assert ph["walk"] > 0.8 * ph["workgroup_lifetime"], ph
