"""Helpers shared by the GPU parity tests: host <-> device conversion, tolerances."""
from __future__ import annotations

import numpy as np

import oracle
from paper_2409_15355_amd import workloads as wl

# Tolerances of the parity gate (bf16 outputs of the attention steps).
MAX_ABS_TOL = 2e-2
MEAN_ABS_TOL = 2e-3
# fp32 re-encode: per rotated pair, ||gpu - oracle||_2 <= REL_TOL * ||oracle pair||_2
REENC_F32_REL_TOL = 1e-5


def dev_bf16(bits: np.ndarray):
    """uint16 bf16 bit patterns -> torch.bfloat16 tensor on cuda:0."""
    import torch
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).cuda()


def host_bits(t) -> np.ndarray:
    """torch.bfloat16 tensor -> uint16 bit patterns on the host."""
    import torch
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def host_f64(t) -> np.ndarray:
    import torch
    if t.dtype == torch.bfloat16:
        return oracle.bf16_bits_to_f64(host_bits(t))
    return t.detach().cpu().numpy().astype(np.float64)


def assert_attention_close(got_f64: np.ndarray, ref_f64: np.ndarray, what: str = ""):
    assert got_f64.shape == ref_f64.shape, (got_f64.shape, ref_f64.shape)
    assert np.isfinite(got_f64).all(), f"{what}: non-finite output"
    err = np.abs(got_f64 - ref_f64)
    mx, mean = float(err.max()) if err.size else 0.0, float(err.mean()) if err.size else 0.0
    assert mx <= MAX_ABS_TOL and mean <= MEAN_ABS_TOL, f"{what}: max abs {mx:.3e}, mean abs {mean:.3e}"
    return mx, mean


def pair_norm_rel_err(got: np.ndarray, ref: np.ndarray, layout: int) -> float:
    """max over rotated pairs of ||got - ref|| / ||ref|| (pairs as the layout defines)."""
    D = ref.shape[-1]
    if layout == oracle.LAYOUT_HALF:
        ga, gb, ra, rb = got[..., :D // 2], got[..., D // 2:], ref[..., :D // 2], ref[..., D // 2:]
    else:
        ga, gb, ra, rb = got[..., 0::2], got[..., 1::2], ref[..., 0::2], ref[..., 1::2]
    num = np.sqrt((ga - ra) ** 2 + (gb - rb) ** 2)
    den = np.sqrt(ra ** 2 + rb ** 2)
    return float((num / np.maximum(den, 1e-30)).max())


def assert_reencode_bf16(got_bits: np.ndarray, ref_f64: np.ndarray, layout: int, what: str = "", roundings: int = 1):
    """The kernel rotates in fp32 and rounds once to bf16: each element must be within one
    bf16 step of the oracle value (half a step from rounding plus slack for the fp32
    rotation landing on the other side of a rounding boundary), measured against the
    pair norm because a rotated component can be arbitrarily close to zero; and nearly
    all elements must equal the correctly rounded oracle value.  `roundings` = number of
    bf16 roundings between the oracle's fp64 chain and the device value (2 when the input
    of the rotation was itself a rotated, rounded key)."""
    got = oracle.bf16_bits_to_f64(got_bits)
    D = ref_f64.shape[-1]
    if layout == oracle.LAYOUT_HALF:
        nrm = np.sqrt(ref_f64[..., :D // 2] ** 2 + ref_f64[..., D // 2:] ** 2)
        nrm = np.concatenate([nrm, nrm], axis=-1)
    else:
        nrm = np.repeat(np.sqrt(ref_f64[..., 0::2] ** 2 + ref_f64[..., 1::2] ** 2), 2, axis=-1)
    err = np.abs(got - ref_f64)
    assert (err <= roundings * 2.0 ** -8 * nrm + 1e-30).all(), f"{what}: max err/norm {float((err / np.maximum(nrm, 1e-30)).max()):.3e}"
    if roundings > 1:
        return
    exact = wl.f32_to_bf16_bits(ref_f64.astype(np.float32))
    # (a fraction of few elements is coarse: one element in 128 is already 0.8 %, so small tensors may
    # have two elements on the other side of a rounding boundary)
    wrong = int((exact != got_bits).sum())
    frac = 1.0 - wrong / exact.size
    assert frac > 0.995 or wrong <= 2, f"{what}: only {frac:.4f} of elements equal the rounded oracle value"
