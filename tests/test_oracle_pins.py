"""Pins for the CPU oracle: each test ties an oracle function to something other than
itself -- a library routine, a closed form, an invariant, a brute-force second
implementation -- chosen so that a dropped term, a wrong sign or index, or a
transposed operand fails at least one of them.  (arXiv 2409.15355: Section 1's three
steps, Section 2.3 Eq. 1-3, Section 2.4's mask, Section 2.5, and the statements that a
single block is ordinary full attention in Sections 3.2-3.3.)
"""
import math

import numpy as np
import pytest
import torch
from hypothesis import given, settings, strategies as st

import oracle

TOL = 1e-12


def rnd(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape)


def sdpa_causal(q, k, v, scale):
    """Library routine: PyTorch CPU scaled_dot_product_attention, fp64, causal."""
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]
    tk = torch.from_numpy(k).permute(1, 0, 2)[None]
    tv = torch.from_numpy(v).permute(1, 0, 2)[None]
    out = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True, scale=scale)
    return out[0].permute(1, 0, 2).numpy()


# ---- P1: one block == ordinary causal attention ------------------------------------
@pytest.mark.parametrize("layout", [oracle.LAYOUT_INTERLEAVED, oracle.LAYOUT_HALF])
def test_p1_single_block_is_causal_attention(layout):
    T, H, D = 37, 3, 16
    q, k, v = rnd(1, T, H, D), rnd(2, T, H, D), rnd(3, T, H, D)
    th = oracle.theta(10000.0, D)
    # library reference on tensors rotated by the independent NumPy rope
    pos = np.arange(T)
    qr, kr = oracle.rope_dense(q, pos, th, layout), oracle.rope_dense(k, pos, th, layout)
    ref = sdpa_causal(qr, kr, v, 1.0 / math.sqrt(D))
    o, k_local = oracle.encode_blocks(q, k, v, [0, T], th, layout=layout)
    assert np.abs(o - ref).max() < TOL
    assert np.abs(k_local - kr).max() < TOL
    # final block with no context is the same thing
    o2 = oracle.final_block(q, np.zeros((0, H, D)), np.zeros((0, H, D)), k, v, [0, T], [0, 0], th,
                            layout=layout)
    assert np.abs(o2 - ref).max() < TOL
    # and without rotation (rope_mode NONE) it is plain SDPA on the raw tensors
    o3, _ = oracle.encode_blocks(q, k, v, [0, T], th, rope_mode=oracle.ROPE_NONE)
    assert np.abs(o3 - sdpa_causal(q, k, v, 1.0 / math.sqrt(D))).max() < TOL


# ---- P2: rotation algebra ------------------------------------------------------------
def test_p2_rope_closed_form_small_case():
    # D = 2, theta_0 = 1: rotation of (1, 0) by pos is (cos pos, sin pos): sign pin.
    th = oracle.theta(10000.0, 2)
    assert th[0] == 1.0
    y = oracle.rope(np.array([1.0, 0.0]), 0.5, th)
    assert abs(y[0] - math.cos(0.5)) < 1e-15 and abs(y[1] - math.sin(0.5)) < 1e-15
    y = oracle.rope(np.array([0.0, 1.0]), 0.5, th)
    assert abs(y[0] + math.sin(0.5)) < 1e-15 and abs(y[1] - math.cos(0.5)) < 1e-15
    # theta_j = base^(-2j/D)
    th = oracle.theta(500000.0, 128)
    assert abs(th[1] - 500000.0 ** (-2.0 / 128)) < 1e-15 and abs(th[63] - 500000.0 ** (-126.0 / 128)) < 1e-18


@pytest.mark.parametrize("layout", [oracle.LAYOUT_INTERLEAVED, oracle.LAYOUT_HALF])
def test_p2_rotation_composition_and_inverse(layout):
    D = 32
    th = oracle.theta(500000.0, D)
    x = rnd(5, D)
    a, b = 123.0, 4567.0
    ab = oracle.rope(oracle.rope(x, b, th, layout), a, th, layout)
    assert np.abs(ab - oracle.rope(x, a + b, th, layout)).max() < 1e-11
    back = oracle.rope(oracle.rope(x, a, th, layout), a, th, layout, inverse=True)
    assert np.abs(back - x).max() < TOL
    # the C rope agrees with the independent vectorised NumPy rope
    dense = oracle.rope_dense(x[None, None, :], np.array([a]), th, layout)[0, 0]
    assert np.abs(dense - oracle.rope(x, a, th, layout)).max() < TOL


@pytest.mark.parametrize("layout", [oracle.LAYOUT_INTERLEAVED, oracle.LAYOUT_HALF])
def test_p2_reencode_equals_direct_encoding(layout):
    """Keys encoded at local positions 0..L-1 then re-encoded to start p equal keys
    encoded directly at absolute positions p..p+L-1; and the two-step Eq. 2 -> Eq. 3
    equals the single rotation by the shift."""
    L, H, D = 9, 2, 16
    th = oracle.theta(10000.0, D)
    k_raw = rnd(7, 2 * L, H, D)
    lens = [L, L]
    local_pos = np.concatenate([np.arange(L), np.arange(L)])
    k_cache = oracle.rope_dense(k_raw, local_pos, th, layout)
    new0 = [700, 31]
    dst_off = [L, 0]  # also swaps the two blocks (gather form)
    got = oracle.reencode(k_cache, [0, L], dst_off, lens, th, new_pos0=new0, layout=layout)
    for b in range(2):
        direct = oracle.rope_dense(k_raw[b * L:(b + 1) * L], new0[b] + np.arange(L), th, layout)
        assert np.abs(got[dst_off[b]:dst_off[b] + L] - direct).max() < 1e-11
        shift = oracle.rope_dense(k_cache[b * L:(b + 1) * L], np.full(L, new0[b]), th, layout)
        assert np.abs(got[dst_off[b]:dst_off[b] + L] - shift).max() < 1e-11
    # ABSOLUTE mode: cache of un-rotated keys
    got_abs = oracle.reencode(k_raw, [0, L], dst_off, lens, th, new_pos0=new0, layout=layout,
                              mode=oracle.REENC_ABSOLUTE)
    assert np.abs(got_abs - got).max() < 1e-11
    # non-zero old_pos0 in SHIFT mode: net rotation is new - old
    k_cache5 = oracle.rope_dense(k_raw, local_pos + 5, th, layout)
    got5 = oracle.reencode(k_cache5, [0, L], dst_off, lens, th, old_pos0=[5, 5], new_pos0=new0,
                           layout=layout)
    assert np.abs(got5 - got).max() < 1e-11


def test_p5_norm_preservation_and_zero_shift_identity():
    L, H, D = 11, 2, 32
    th = oracle.theta(500000.0, D)
    k = rnd(11, 3, L, H, D)  # 3 layers
    out = oracle.reencode(k, [0], [0], [L], th, new_pos0=[31000])
    pn_in = k[..., 0::2] ** 2 + k[..., 1::2] ** 2
    pn_out = out[..., 0::2] ** 2 + out[..., 1::2] ** 2
    assert np.abs(pn_in - pn_out).max() < 1e-11
    assert np.abs(out - k).max() > 0.1  # it did rotate
    # ABSOLUTE mode with new_pos0 = -u is not expressible; zero shift in SHIFT mode:
    same = oracle.reencode(k, [0], [0], [L], th, new_pos0=[0])
    assert np.abs(same - k).max() < 1e-15


def test_p5b_half_layout_is_a_permutation_of_interleaved():
    D = 16
    th = oracle.theta(10000.0, D)
    x = rnd(13, D)
    perm = np.empty(D, dtype=int)  # interleaved index -> half index
    perm[0::2] = np.arange(D // 2)
    perm[1::2] = np.arange(D // 2) + D // 2
    y_int = oracle.rope(x, 77.0, th, oracle.LAYOUT_INTERLEAVED)
    x_half = np.empty(D)
    x_half[perm] = x
    y_half = oracle.rope(x_half, 77.0, th, oracle.LAYOUT_HALF)
    assert np.abs(y_half[perm] - y_int).max() < TOL
    # attention is unchanged when q and k are permuted alike
    T, H = 12, 2
    q, k, v = rnd(14, T, H, D), rnd(15, T, H, D), rnd(16, T, H, D)
    qh, kh = np.empty_like(q), np.empty_like(k)
    qh[..., perm], kh[..., perm] = q, k
    o_i, _ = oracle.encode_blocks(q, k, v, [0, 5, T], th, layout=oracle.LAYOUT_INTERLEAVED)
    o_h, _ = oracle.encode_blocks(qh, kh, v, [0, 5, T], th, layout=oracle.LAYOUT_HALF)
    assert np.abs(o_i - o_h).max() < TOL


# ---- P3: relative-position invariance -------------------------------------------------
def test_p3_local_positions_equal_absolute_positions():
    T, H, D = 20, 2, 16
    offs = [0, 7, 20]
    th = oracle.theta(10000.0, D)
    q, k, v = rnd(21, T, H, D), rnd(22, T, H, D), rnd(23, T, H, D)
    o_local, _ = oracle.encode_blocks(q, k, v, offs, th)
    pos = np.arange(T)
    qa, ka = oracle.rope_dense(q, pos, th, 0), oracle.rope_dense(k, pos, th, 0)
    o_abs, _ = oracle.encode_blocks(qa, ka, v, offs, th, rope_mode=oracle.ROPE_NONE)
    assert np.abs(o_local - o_abs).max() < 1e-11


# ---- P4: pipeline == brute force under the explicit mask ----------------------------
def run_pipeline(q, k, v, offs, th, layout, q_to_kv=None):
    """encode passages (local) -> re-encode (shift) -> final block; returns [T, Hq, D]."""
    offs = np.asarray(offs)
    t_ctx = int(offs[-2])
    T = int(offs[-1])
    out = np.empty_like(q)
    if t_ctx > 0:
        o_p, k_local = oracle.encode_blocks(q[:t_ctx], k[:t_ctx], v[:t_ctx], offs[:-1], th,
                                            layout=layout, q_to_kv=q_to_kv)
        out[:t_ctx] = o_p
        lens = np.diff(offs[:-1])
        k_ctx = oracle.reencode(k_local, offs[:-2], offs[:-2], lens, th, layout=layout)
    else:
        k_ctx = np.zeros((0,) + k.shape[1:])
    out[t_ctx:] = oracle.final_block(q[t_ctx:], k_ctx, v[:t_ctx], k[t_ctx:], v[t_ctx:],
                                     [0, T - t_ctx], [0, t_ctx], th, layout=layout, q_to_kv=q_to_kv)
    return out


@pytest.mark.parametrize("offs", [[0, 64], [0, 1, 2, 3], [0, 5, 6, 30, 41], [0, 17, 17, 40, 64],
                                  [0, 20, 21]])
@pytest.mark.parametrize("layout", [oracle.LAYOUT_INTERLEAVED, oracle.LAYOUT_HALF])
def test_p4_pipeline_equals_bruteforce(offs, layout):
    T, Hq, Hkv, D = offs[-1], 4, 2, 8
    th = oracle.theta(10000.0, D)
    q, k, v = rnd(31, T, Hq, D), rnd(32, T, Hkv, D), rnd(33, T, Hkv, D)
    got = run_pipeline(q, k, v, offs, th, layout)
    ref = oracle.masked_attention_bruteforce(q, k, v, offs, th, layout=layout)
    assert np.abs(got - ref).max() < 1e-11


@settings(max_examples=25, deadline=None, derandomize=True)
@given(lens=st.lists(st.integers(min_value=0, max_value=9), min_size=0, max_size=5),
       l_q=st.integers(min_value=1, max_value=9), hkv=st.integers(min_value=1, max_value=2),
       g=st.integers(min_value=1, max_value=3), layout=st.sampled_from([oracle.LAYOUT_INTERLEAVED, oracle.LAYOUT_HALF]),
       seed=st.integers(min_value=0, max_value=10**6))
def test_p4_pipeline_equals_bruteforce_on_drawn_splits(lens, l_q, hkv, g, layout, seed):
    """The same pin on block splits, head groupings and layouts drawn by the test framework: empty
    passages, no passages at all, one-token blocks, one to three query heads per KV head."""
    offs = np.concatenate([[0], np.cumsum(lens + [l_q])]).astype(np.int64)
    T, D = int(offs[-1]), 8
    th = oracle.theta(10000.0, D)
    q, k, v = rnd(seed, T, hkv * g, D), rnd(seed + 1, T, hkv, D), rnd(seed + 2, T, hkv, D)
    got = run_pipeline(q, k, v, offs, th, layout)
    ref = oracle.masked_attention_bruteforce(q, k, v, offs, th, layout=layout)
    assert np.abs(got - ref).max() < 1e-11


def test_block_mask_small_case_by_hand():
    M = oracle.block_mask([0, 2, 3, 5]).astype(int)
    expect = np.array([[1, 0, 0, 0, 0],
                       [1, 1, 0, 0, 0],
                       [0, 0, 1, 0, 0],
                       [1, 1, 1, 1, 0],
                       [1, 1, 1, 1, 1]])
    assert (M == expect).all()


# ---- P6 / P7 / P8: normalisation and the mask's lower edge ----------------------------
def test_p6_p7_p8_rows():
    T, Hq, Hkv, D = 30, 4, 2, 8
    offs = [0, 9, 9, 22, 30]
    th = oracle.theta(10000.0, D)
    q, k, v = rnd(41, T, Hq, D), rnd(42, T, Hkv, D), rnd(43, T, Hkv, D)
    o, _ = oracle.encode_blocks(q, k, v, offs, th)
    for start in (0, 9, 22):  # P7: first token of each block returns its own v
        for h in range(Hq):
            assert np.array_equal(o[start, h], v[start, h // 2])
    for b in range(len(offs) - 1):  # P6: convex combination of visible v rows
        for t in range(offs[b], offs[b + 1]):
            vis = v[offs[b]:t + 1]
            for h in range(Hq):
                lo, hi = vis[:, h // 2].min(axis=0), vis[:, h // 2].max(axis=0)
                assert (o[t, h] >= lo - 1e-12).all() and (o[t, h] <= hi + 1e-12).all()
    # P8: constant v -> output is that constant
    vc = np.broadcast_to(rnd(44, 1, Hkv, D), (T, Hkv, D)).copy()
    oc, _ = oracle.encode_blocks(q, k, vc, offs, th)
    for h in range(Hq):
        assert np.abs(oc[:, h] - vc[:, h // 2]).max() < 1e-13
    # softmax weights sum to one: with v = one-hot over keys the output is the weights
    Tk = 6
    onehot = np.zeros((Tk, 1, Tk))
    onehot[np.arange(Tk), 0, np.arange(Tk)] = 1.0
    qq, kk = rnd(45, Tk, 1, Tk), rnd(46, Tk, 1, Tk)
    w, _ = oracle.encode_blocks(qq, kk, onehot, [0, Tk], oracle.theta(10000.0, Tk))
    assert np.abs(w[:, 0].sum(axis=1) - 1.0).max() < 1e-14
    assert np.abs(np.triu(w[:, 0], 1)).max() == 0.0  # nothing above the diagonal
    # final block, no context: first row returns v
    of = oracle.final_block(q[:5], np.zeros((0, Hkv, D)), np.zeros((0, Hkv, D)), k[:5], v[:5], [0, 5],
                            [0, 0], th)
    assert np.array_equal(of[0, 3], v[0, 1])


def test_softmax_scale_and_weights_closed_form():
    """Two keys, D = 2, no rotation: weights are a logistic of scale * (s1 - s0)."""
    q = np.array([[[2.0, 0.0]], [[2.0, 0.0]]])
    k = np.array([[[1.0, 0.0]], [[3.0, 0.0]]])
    v = np.array([[[10.0, 0.0]], [[20.0, 1.0]]])
    th = oracle.theta(10000.0, 2)
    o, _ = oracle.encode_blocks(q, k, v, [0, 2], th, rope_mode=oracle.ROPE_NONE, scale=0.25)
    w1 = 1.0 / (1.0 + math.exp(-0.25 * (6.0 - 2.0)))
    assert abs(o[1, 0, 0] - (10.0 * (1 - w1) + 20.0 * w1)) < 1e-13
    assert abs(o[1, 0, 1] - w1) < 1e-14
    # default scale is 1/sqrt(D)
    o2, _ = oracle.encode_blocks(q, k, v, [0, 2], th, rope_mode=oracle.ROPE_NONE)
    w2 = 1.0 / (1.0 + math.exp(-(4.0 / math.sqrt(2.0))))
    assert abs(o2[1, 0, 1] - w2) < 1e-14


# ---- P9: permutation invariance and split / merge --------------------------------------
def test_p9_context_permutation_and_split_merge():
    Lq, Tc, Hq, Hkv, D = 6, 40, 4, 2, 8
    th = oracle.theta(10000.0, D)
    qf, kf, vf = rnd(51, Lq, Hq, D), rnd(52, Lq, Hkv, D), rnd(53, Lq, Hkv, D)
    kc, vc = rnd(54, Tc, Hkv, D), rnd(55, Tc, Hkv, D)
    ref = oracle.final_block(qf, kc, vc, kf, vf, [0, Lq], [0, Tc], th)
    perm = np.random.default_rng(56).permutation(Tc)
    got = oracle.final_block(qf, kc[perm], vc[perm], kf, vf, [0, Lq], [0, Tc], th)
    assert np.abs(got - ref).max() < 1e-12
    # split the context into 3 chunks; the last chunk also takes the causal part
    cuts = [0, 13, 29, Tc]
    parts = []
    for i in range(3):
        last = i == 2
        kci, vci = kc[cuts[i]:cuts[i + 1]], vc[cuts[i]:cuts[i + 1]]
        if last:
            o, m, l = oracle.final_block(qf, kci, vci, kf, vf, [0, Lq], [0, len(kci)], th,
                                         q_pos0=[Tc], want_stats=True)
        else:
            # context-only partial: express "no causal part" with brute force on the chunk
            qr = oracle.rope_dense(qf, Tc + np.arange(Lq), th, 0)
            o = np.empty((Lq, Hq, D)); m = np.empty((Lq, Hq)); l = np.empty((Lq, Hq))
            for h in range(Hq):
                S = (qr[:, h] @ kci[:, h // 2].T) / math.sqrt(D)
                m[:, h] = S.max(axis=1)
                P = np.exp(S - m[:, h][:, None])
                l[:, h] = P.sum(axis=1)
                o[:, h] = (P @ vci[:, h // 2]) / l[:, h][:, None]
        parts.append((o, m, l))
    merged = oracle.merge_partials(*zip(*parts))
    assert np.abs(merged - ref).max() < 1e-12


# ---- P10: independence of blocks ---------------------------------------------------------
def test_p10_no_cross_block_visibility():
    T, Hq, Hkv, D = 26, 2, 2, 8
    offs = [0, 8, 15, 26]
    th = oracle.theta(10000.0, D)
    q, k, v = rnd(61, T, Hq, D), rnd(62, T, Hkv, D), rnd(63, T, Hkv, D)
    base = run_pipeline(q, k, v, offs, th, 0)
    k2, v2 = k.copy(), v.copy()
    k2[3] += 1.0
    v2[3] -= 2.0  # token 3 is in block 0
    pert = run_pipeline(q, k2, v2, offs, th, 0)
    assert np.array_equal(pert[8:15], base[8:15])          # block 1 untouched
    assert np.array_equal(pert[:3], base[:3])              # causal: earlier rows of block 0 untouched
    assert np.abs(pert[3:8] - base[3:8]).max() > 1e-3      # later rows of block 0 change
    assert np.abs(pert[15:] - base[15:]).min() > 0.0       # every final-block row changes


# ---- P11: GQA == MHA with replicated KV heads; explicit head map ----------------------
def test_p11_gqa_is_replicated_mha():
    T, Hq, Hkv, D = 19, 6, 2, 8
    offs = [0, 6, 13, 19]
    th = oracle.theta(10000.0, D)
    q, k, v = rnd(71, T, Hq, D), rnd(72, T, Hkv, D), rnd(73, T, Hkv, D)
    got = run_pipeline(q, k, v, offs, th, 0)
    krep, vrep = np.repeat(k, 3, axis=1), np.repeat(v, 3, axis=1)
    ref = run_pipeline(q, krep, vrep, offs, th, 0)
    assert np.abs(got - ref).max() < TOL
    # an explicit q_to_kv map equal to the default changes nothing; a different one does
    same = run_pipeline(q, k, v, offs, th, 0, q_to_kv=[0, 0, 0, 1, 1, 1])
    assert np.array_equal(same, got)
    other = run_pipeline(q, k, v, offs, th, 0, q_to_kv=[1, 0, 0, 1, 1, 0])
    assert np.array_equal(other[:, 1:5], got[:, 1:5]) and np.abs(other[:, 0] - got[:, 0]).max() > 1e-3
    bf = oracle.masked_attention_bruteforce(q, k, v, offs, th, q_to_kv=[1, 0, 0, 1, 1, 0])
    assert np.abs(other - bf).max() < 1e-11


# ---- P12: batched == per prompt; row subsets -------------------------------------------
def test_p12_batched_equals_per_prompt_and_row_subsets():
    Hq, Hkv, D = 4, 2, 8
    th = oracle.theta(10000.0, D)
    lq, tc = [3, 7, 1], [10, 0, 25]
    cu_q, cu_c = np.concatenate([[0], np.cumsum(lq)]), np.concatenate([[0], np.cumsum(tc)])
    qf, kf, vf = rnd(81, cu_q[-1], Hq, D), rnd(82, cu_q[-1], Hkv, D), rnd(83, cu_q[-1], Hkv, D)
    kc, vc = rnd(84, cu_c[-1], Hkv, D), rnd(85, cu_c[-1], Hkv, D)
    got = oracle.final_block(qf, kc, vc, kf, vf, cu_q, cu_c, th)
    for n in range(3):
        a, b = cu_q[n], cu_q[n + 1]
        c, d = cu_c[n], cu_c[n + 1]
        one = oracle.final_block(qf[a:b], kc[c:d], vc[c:d], kf[a:b], vf[a:b], [0, b - a], [0, d - c], th)
        assert np.array_equal(one, got[a:b])
    rows = [10, 0, 4]
    sub = oracle.final_block(qf, kc, vc, kf, vf, cu_q, cu_c, th, rows=rows)
    assert np.array_equal(sub, got[rows])
    # encode: a batch of prompts is just a longer block list; row subsets agree
    T = 24
    q, k, v = rnd(86, T, Hq, D), rnd(87, T, Hkv, D), rnd(88, T, Hkv, D)
    offs = [0, 5, 11, 24]
    full, kl = oracle.encode_blocks(q, k, v, offs, th)
    for b in range(3):
        a, e = offs[b], offs[b + 1]
        one, kl1 = oracle.encode_blocks(q[a:e], k[a:e], v[a:e], [0, e - a], th)
        assert np.array_equal(one, full[a:e]) and np.array_equal(kl1, kl[a:e])
    sub, _ = oracle.encode_blocks(q, k, v, offs, th, rows=[23, 5, 0])
    assert np.array_equal(sub, full[[23, 5, 0]])


def test_q_pos0_override_and_final_positions():
    """Final block sits right after the context unless q_pos0 says otherwise; with an
    override the result equals brute force on a sequence padded to that position."""
    Lq, Tc, H, D = 4, 6, 1, 8
    th = oracle.theta(10000.0, D)
    qf, kf, vf = rnd(91, Lq, H, D), rnd(92, Lq, H, D), rnd(93, Lq, H, D)
    kc_raw, vc = rnd(94, Tc, H, D), rnd(95, Tc, H, D)
    kc = oracle.rope_dense(kc_raw, np.arange(Tc), th, 0)
    default = oracle.final_block(qf, kc, vc, kf, vf, [0, Lq], [0, Tc], th)
    explicit = oracle.final_block(qf, kc, vc, kf, vf, [0, Lq], [0, Tc], th, q_pos0=[Tc])
    assert np.array_equal(default, explicit)
    ref = oracle.masked_attention_bruteforce(np.concatenate([np.zeros((Tc, H, D)), qf]),
                                             np.concatenate([kc_raw, kf]), np.concatenate([vc, vf]),
                                             [0, Tc, Tc + Lq], th)[Tc:]
    assert np.abs(default - ref).max() < 1e-12
    moved = oracle.final_block(qf, kc, vc, kf, vf, [0, Lq], [0, Tc], th, q_pos0=[Tc + 3])
    assert np.abs(moved - default).max() > 1e-4


# ---- the paper's FLOP bookkeeping (Table 3) ---------------------------------------------
def test_table3_flops_are_linear_in_tokens():
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "table3_flops_tft.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    per_token = 7.5e11 / 50.0
    for length, vanilla, block in rows:
        assert float(block) == 7.5e11
        assert abs(float(vanilla) - per_token * int(length)) / float(vanilla) < 0.03


@pytest.mark.parametrize("layout", [oracle.LAYOUT_INTERLEAVED, oracle.LAYOUT_HALF])
def test_shift_of_the_key_equals_opposite_shift_of_the_query(layout):
    """The identity the block-cache entry point rests on (Eq. 2-3 applied to q instead of k): a score
    depends on positions only through their difference, so re-encoding a cached key by a shift
    gives the same score as turning the query back by that shift and leaving the key alone; and a
    final block computed from per-block re-encoded keys does not care where in the cache the
    blocks were stored."""
    D = 16
    th = oracle.theta(10000.0, D)
    rng = np.random.default_rng(31)
    q, k = rng.standard_normal(D), rng.standard_normal(D)
    for p_q, u, old0, new0 in [(900, 3, 0, 512), (40, 0, 17, 5), (12345, 77, 1000, 0)]:
        k_cached = oracle.rope(k, old0 + u, th, layout)                    # as it sits in the cache
        k_moved = oracle.reencode(k_cached[None, None, :], [0], [0], [1], th, old_pos0=[old0 + u], new_pos0=[new0 + u],
                                  layout=layout)[0, 0]
        s_reencoded = oracle.rope(q, p_q, th, layout) @ k_moved
        s_turned_q = oracle.rope(q, p_q - (new0 - old0), th, layout) @ k_cached
        s_direct = oracle.rope(q, p_q, th, layout) @ oracle.rope(k, new0 + u, th, layout)
        assert abs(s_reencoded - s_direct) < 1e-9 and abs(s_turned_q - s_direct) < 1e-9
    # cache placement does not matter
    Hq = Hkv = 1
    lens, slots = [5, 3, 4], [20, 0, 9]
    cache_k, cache_v = rng.standard_normal((30, Hkv, D)), rng.standard_normal((30, Hkv, D))
    qf, kf, vf = rng.standard_normal((2, Hq, D)), rng.standard_normal((2, Hkv, D)), rng.standard_normal((2, Hkv, D))
    new0 = np.concatenate([[0], np.cumsum(lens)[:-1]]).astype(np.int32)
    T = sum(lens)
    k_ctx = oracle.reencode(cache_k, slots, new0, lens, th, new_pos0=new0, layout=layout, out=np.zeros((T, Hkv, D)))
    v_ctx = np.concatenate([cache_v[s:s + n] for s, n in zip(slots, lens)])
    o1 = oracle.final_block(qf, k_ctx, v_ctx, kf, vf, [0, 2], [0, T], th, layout=layout)
    packed_k = np.concatenate([cache_k[s:s + n] for s, n in zip(slots, lens)])
    k_ctx2 = oracle.reencode(packed_k, new0, new0, lens, th, new_pos0=new0, layout=layout)
    o2 = oracle.final_block(qf, k_ctx2, v_ctx, kf, vf, [0, 2], [0, T], th, layout=layout)
    np.testing.assert_allclose(o1, o2, rtol=0, atol=1e-12)


# --------------------------------------------------------------------------------------------
# gradient of the masked attention (what a block fine-tune step runs backward)
# --------------------------------------------------------------------------------------------
def _torch_masked_attention(q, k, v, offs, th, layout):
    """The definition again, in plain torch ops on fp64 tensors (so that autograd can differentiate
    it): rotate at positions 0..T-1, mask, softmax, weighted sum.  Written apart from the oracle."""
    T, hq, d = q.shape
    hkv = k.shape[1]
    pos = torch.arange(T, dtype=torch.float64)
    ang = pos[:, None] * torch.as_tensor(th)[None, :]
    c, s = torch.cos(ang)[:, None, :], torch.sin(ang)[:, None, :]

    def rot(x):
        if layout == oracle.LAYOUT_HALF:
            a, b = x[..., : d // 2], x[..., d // 2:]
            return torch.cat([c * a - s * b, s * a + c * b], dim=-1)
        a, b = x[..., 0::2], x[..., 1::2]
        return torch.stack([c * a - s * b, s * a + c * b], dim=-1).reshape(x.shape)

    qr, kr = rot(q), rot(k)
    blk = torch.zeros(T, dtype=torch.long)
    for b in range(len(offs) - 1):
        blk[offs[b]:offs[b + 1]] = b
    t, s_ = torch.arange(T)[:, None], torch.arange(T)[None, :]
    mask = (s_ <= t) & ((blk[None, :] == blk[:, None]) | (blk[:, None] == len(offs) - 2))
    outs = []
    for h in range(hq):
        g = h // (hq // hkv)
        sc = (qr[:, h] @ kr[:, g].T) / math.sqrt(d)
        sc = sc.masked_fill(~mask, float("-inf"))
        outs.append(torch.softmax(sc, dim=1) @ v[:, g])
    return torch.stack(outs, dim=1)


@pytest.mark.parametrize("layout", [oracle.LAYOUT_INTERLEAVED, oracle.LAYOUT_HALF])
def test_backward_equals_autograd_of_the_definition(layout):
    rng = np.random.default_rng(41 + layout)
    offs = [0, 5, 6, 13, 20]
    T, hq, hkv, d = 20, 4, 2, 8
    th = oracle.theta(10000.0, d)
    q, k, v, do = (rng.standard_normal((T, h, d)) for h in (hq, hkv, hkv, hq))
    dq, dk, dv, lse = oracle.masked_attention_backward_bruteforce(q, k, v, do, offs, th, layout=layout)
    tq, tk, tv = (torch.tensor(x, requires_grad=True) for x in (q, k, v))
    out = _torch_masked_attention(tq, tk, tv, offs, th, layout)
    assert np.allclose(out.detach().numpy(), oracle.masked_attention_bruteforce(q, k, v, offs, th, layout=layout), atol=1e-12)
    (out * torch.tensor(do)).sum().backward()
    assert np.allclose(dq, tq.grad.numpy(), atol=1e-11)
    assert np.allclose(dk, tk.grad.numpy(), atol=1e-11)
    assert np.allclose(dv, tv.grad.numpy(), atol=1e-11)


def test_backward_equals_finite_differences_and_respects_the_mask():
    rng = np.random.default_rng(43)
    offs = [0, 4, 9, 12]
    T, hq, hkv, d = 12, 2, 1, 4
    th = oracle.theta(10000.0, d)
    q, k, v, do = (rng.standard_normal((T, h, d)) for h in (hq, hkv, hkv, hq))
    dq, dk, dv, lse = oracle.masked_attention_backward_bruteforce(q, k, v, do, offs, th)
    loss = lambda q_, k_, v_: float((oracle.masked_attention_bruteforce(q_, k_, v_, offs, th) * do).sum())
    eps = 1e-6
    for arr, grad, which in ((q, dq, 0), (k, dk, 1), (v, dv, 2)):
        for _ in range(6):
            idx = tuple(int(rng.integers(0, n)) for n in arr.shape)
            hi, lo = arr.copy(), arr.copy()
            hi[idx] += eps
            lo[idx] -= eps
            args_hi = [q, k, v]; args_lo = [q, k, v]
            args_hi[which], args_lo[which] = hi, lo
            fd = (loss(*args_hi) - loss(*args_lo)) / (2 * eps)
            assert abs(fd - grad[idx]) < 1e-7 * max(1.0, abs(fd)), (which, idx)
    # a key of passage 0 is seen by passage 0 and by the last block only: with the output gradient
    # zero on those rows its gradient vanishes, whatever the rows of passage 1 carry
    do2 = do.copy()
    do2[0:4] = 0.0
    do2[9:12] = 0.0
    _, dk2, dv2, _ = oracle.masked_attention_backward_bruteforce(q, k, v, do2, offs, th)
    assert np.all(dk2[0:4] == 0.0) and np.all(dv2[0:4] == 0.0)
    assert np.any(dk2[4:9] != 0.0)
    # log-sum-exp: exp(lse) is the sum of exp(scaled scores) over the visible keys
    pos = np.arange(T)
    qr, kr = oracle.rope_dense(q, pos, th, 0), oracle.rope_dense(k, pos, th, 0)
    M = oracle.block_mask(offs)
    S = (qr[:, 1] @ kr[:, 0].T) / math.sqrt(d)
    assert np.allclose(np.exp(lse[:, 1]), (np.exp(S) * M).sum(axis=1), rtol=1e-12)


def test_backward_term_sums_bound_the_gradients_and_are_tight_for_one_sign():
    """masked_attention_backward_term_sums is the scale the GPU gradient tolerance is stated against:
    by the triangle inequality it bounds the gradient's magnitude element by element (for dq and dk,
    pair norm by pair norm: the rotation back is orthogonal), and where every product has one sign
    (dV with a non-negative output gradient) it equals the gradient itself."""
    rng = np.random.default_rng(77)
    T, hq, hkv, d = 37, 4, 2, 16
    offs = [0, 9, 9, 21, 37]
    th = oracle.theta(10000.0, d)
    q, k, v = (rng.standard_normal((T, h, d)) for h in (hq, hkv, hkv))
    for layout in (oracle.LAYOUT_INTERLEAVED, oracle.LAYOUT_HALF):
        do = rng.standard_normal((T, hq, d))
        dq, dk, dv, _ = oracle.masked_attention_backward_bruteforce(q, k, v, do, offs, th, layout=layout)
        aq, ak, av = oracle.masked_attention_backward_term_sums(q, k, v, do, offs, th, layout=layout)

        def pair_norm(x):
            if layout == oracle.LAYOUT_HALF:
                n = np.sqrt(x[..., :d // 2] ** 2 + x[..., d // 2:] ** 2)
                return np.concatenate([n, n], axis=-1)
            return np.repeat(np.sqrt(x[..., 0::2] ** 2 + x[..., 1::2] ** 2), 2, axis=-1)

        assert (np.abs(dv) <= av + 1e-12).all() and (pair_norm(dq) <= aq + 1e-12).all() and (pair_norm(dk) <= ak + 1e-12).all()
        assert (av > 0).all()
        do_pos = np.abs(do)
        _, _, dv_pos, _ = oracle.masked_attention_backward_bruteforce(q, k, v, do_pos, offs, th, layout=layout)
        _, _, av_pos = oracle.masked_attention_backward_term_sums(q, k, v, do_pos, offs, th, layout=layout)
        assert np.allclose(dv_pos, av_pos, rtol=1e-12, atol=1e-12)
    # dq and dk: every product written out in loops, on a case small enough for that (one KV head,
    # two query heads; softmax and output recomputed here from the rotated rows)
    T, hq, d = 5, 2, 4
    offs = [0, 2, 5]
    th = oracle.theta(10000.0, d)
    q, k, v, do = rng.standard_normal((T, hq, d)), rng.standard_normal((T, 1, d)), rng.standard_normal((T, 1, d)), rng.standard_normal((T, hq, d))
    aq, ak, _ = oracle.masked_attention_backward_term_sums(q, k, v, do, offs, th)
    qr, kr = oracle.rope_dense(q, np.arange(T), th, oracle.LAYOUT_INTERLEAVED), oracle.rope_dense(k, np.arange(T), th, oracle.LAYOUT_INTERLEAVED)
    mask, sc = oracle.block_mask(offs), 1.0 / np.sqrt(d)
    want_q, want_k = np.zeros((T, hq, d)), np.zeros((T, 1, d))
    for h in range(hq):
        for i in range(T):
            vis = [j for j in range(T) if mask[i, j]]
            e = np.array([np.exp(sc * float(qr[i, h] @ kr[j, 0])) for j in vis])
            prob = e / e.sum()
            out = sum(pj * v[j, 0] for pj, j in zip(prob, vis))
            for pj, j in zip(prob, vis):
                share = pj * sum(abs(do[i, h, c] * v[j, 0, c]) + abs(do[i, h, c] * out[c]) for c in range(d))
                for c in range(d):
                    want_q[i, h, c] += sc * share * abs(kr[j, 0, c])
                    want_k[j, 0, c] += sc * share * abs(qr[i, h, c])
    pn = lambda x: np.repeat(np.sqrt(x[..., 0::2] ** 2 + x[..., 1::2] ** 2), 2, axis=-1)
    assert np.allclose(aq, pn(want_q), rtol=1e-10) and np.allclose(ak, pn(want_k), rtol=1e-10)
    # a row that sees a single key: its dS is zero, its share of the term sums is not
    assert (aq[0] > 0).all() and (aq[2] > 0).all()
