"""The allocation-free entry point against the one it is a variant of: same inputs, same kernels,
so the outputs must be equal bit for bit.  Two calls in a row share the static array; the second
is smaller, so stale partials of the first lie behind what it writes."""
import numpy as np
import pytest

from paper_2409_15355_amd import workloads as wl
from gpu_util import dev_bf16, host_bits

pytestmark = pytest.mark.gpu


def _case(ba, torch, seed, hq, hkv, d, lq_list, ctx_list):
    cu_q = np.concatenate([[0], np.cumsum(lq_list)]).astype(np.int32)
    cu_ctx = np.concatenate([[0], np.cumsum(ctx_list)]).astype(np.int32)
    Tq, Tc = int(cu_q[-1]), int(cu_ctx[-1])
    heads = ba.Heads(hq, hkv, d, 500000.0)
    qf = dev_bf16(wl.normal_bf16_bits(seed, (Tq, hq, d)))
    kf = dev_bf16(wl.normal_bf16_bits(seed + 1, (Tq, hkv, d)))
    vf = dev_bf16(wl.normal_bf16_bits(seed + 2, (Tq, hkv, d)))
    kc = dev_bf16(wl.normal_bf16_bits(seed + 3, (max(Tc, 1), hkv, d)))
    vc = dev_bf16(wl.normal_bf16_bits(seed + 4, (max(Tc, 1), hkv, d)))
    nbytes = ba.ba_final_block_attention_workspace_bytes(heads, cu_q, cu_ctx, ba.ROPE_APPLY, True)
    assert nbytes <= ba.STATIC_SCRATCH_BYTES
    ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")
    o_ref = torch.full_like(qf, float("nan"))
    kr_ref = torch.full_like(kf, float("nan"))
    ba.ba_final_block_attention(heads, qf, kc, vc, kf, vf, o_ref, kr_ref, cu_q, cu_ctx, None, ba.ROPE_APPLY, ws)
    o = torch.full_like(qf, float("nan"))
    kr = torch.full_like(kf, float("nan"))
    ba.ba_final_block_attention_static(heads, qf, kc, vc, kf, vf, o, kr, cu_q, cu_ctx, None, ba.ROPE_APPLY)
    torch.cuda.synchronize()
    assert not torch.isnan(o_ref.float()).any() and not torch.isnan(o.float()).any()
    assert np.array_equal(host_bits(o), host_bits(o_ref)), "outputs differ"
    assert np.array_equal(host_bits(kr), host_bits(kr_ref)), "rotated final-block keys differ"
    return nbytes


def test_static_scratch_entry_point_equals_the_workspace_one():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2409_15355_amd import binding as ba
    ba.load()
    # first call: several KV splits (partials in the scratch array); second call: smaller, fewer splits
    big = _case(ba, torch, 9100, 32, 8, 128, [96, 40], [6000, 3001])
    small = _case(ba, torch, 9200, 32, 8, 128, [17], [700])
    assert small < big
    # and one that does not fit: rejected before anything is launched
    heads = ba.Heads(32, 8, 128, 500000.0)
    cu_q = np.array([0, 4096], dtype=np.int32)
    cu_ctx = np.array([0, 8192], dtype=np.int32)
    assert ba.ba_final_block_attention_workspace_bytes(heads, cu_q, cu_ctx, ba.ROPE_APPLY, False) > ba.STATIC_SCRATCH_BYTES
    x = torch.zeros(4096, 32, 128, dtype=torch.bfloat16, device="cuda")
    kv = torch.zeros(8192, 8, 128, dtype=torch.bfloat16, device="cuda")
    kvf = torch.zeros(4096, 8, 128, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(ba.BaError) as ei:
        ba.ba_final_block_attention_static(heads, x, kv, kv, kvf, kvf, x, None, cu_q, cu_ctx, None, ba.ROPE_APPLY)
    assert ei.value.status == -4
