"""Seeded synthetic inputs for the Block-attention hot path.

This module holds NO arithmetic of the method: only random draws, bf16 bit
conversion and the shapes / block structure of the five benchmark workloads.  The
same arrays are handed to the HIP library and to the CPU oracle.

Stand-in note: the paper measures on RAG prompts built from public QA corpora; what
the kernels see of such a prompt is only its shape (passage count, passage lengths,
query length, head geometry).  These generators reproduce those shapes with i.i.d.
N(0,1) values rounded to bf16.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

BASE_SEED = 240915355


def tensor_seed(cfg: int, tensor_index: int) -> int:
    return BASE_SEED + 1000 * cfg + tensor_index


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float32 -> bfloat16 bit patterns (uint16).  Finite inputs."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal_f32(seed: int, shape) -> np.ndarray:
    rng = np.random.Generator(np.random.Philox(seed))
    return rng.standard_normal(size=shape, dtype=np.float32)


def normal_bf16_bits(seed: int, shape) -> np.ndarray:
    return f32_to_bf16_bits(normal_f32(seed, shape))


@dataclass
class Prompt:
    """One prompt: passage lengths and the final (query) block length."""
    passage_lens: List[int]
    final_len: int

    @property
    def t_ctx(self) -> int:
        return int(sum(self.passage_lens))


@dataclass
class Workload:
    name: str
    cfg: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    rope_base: float
    prompts: List[Prompt]
    n_layers: int = 1
    notes: str = ""
    extra: dict = field(default_factory=dict)

    # ---- derived block structure -------------------------------------------------
    def passage_block_offsets(self) -> np.ndarray:
        """Offsets of all passage blocks of all prompts packed back to back
        (the encode call's block list)."""
        lens = [l for p in self.prompts for l in p.passage_lens]
        return np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)

    def cu_ctx(self) -> np.ndarray:
        return np.concatenate([[0], np.cumsum([p.t_ctx for p in self.prompts])]).astype(np.int32)

    def cu_q(self) -> np.ndarray:
        return np.concatenate([[0], np.cumsum([p.final_len for p in self.prompts])]).astype(np.int32)

    def passage_new_pos0(self) -> np.ndarray:
        """Absolute start position of every passage inside its own prompt."""
        out = []
        for p in self.prompts:
            out.extend(np.concatenate([[0], np.cumsum(p.passage_lens)[:-1]]).tolist() if p.passage_lens else [])
        return np.asarray(out, dtype=np.int32)


def config1() -> Workload:
    return Workload("cfg1-tiny-mha-d64", 1, 4, 4, 64, 10000.0, [Prompt([128, 128], 64)])


def config2() -> Workload:
    return Workload("cfg2-llama8b-10x200", 2, 32, 8, 128, 500000.0, [Prompt([200] * 10, 64)])


def config3() -> Workload:
    rng = np.random.Generator(np.random.Philox(tensor_seed(3, 900)))
    prompts = []
    for _ in range(8):
        lens = rng.integers(100, 301, size=20).tolist()
        fin = int(rng.integers(32, 129))
        prompts.append(Prompt([int(x) for x in lens], fin))
    return Workload("cfg3-llama8b-ragged-8x20", 3, 32, 8, 128, 500000.0, prompts)


def config4(n_layers: int = 32, n_passages: int = 32, passage_len: int = 1000) -> Workload:
    rng = np.random.Generator(np.random.Philox(tensor_seed(4, 900)))
    perm = rng.permutation(n_passages).astype(np.int32)
    w = Workload("cfg4-reencode-32x32x1000", 4, 32, 8, 128, 500000.0,
                 [Prompt([passage_len] * n_passages, 0)], n_layers=n_layers)
    w.extra["slot_of_passage"] = perm           # passage b moves to slot perm[b]
    w.extra["new_pos0"] = (perm * passage_len).astype(np.int32)
    return w


def config5(n_layers: int = 32, n_passages: int = 31, passage_len: int = 1024,
            final_len: int = 256) -> Workload:
    return Workload("cfg5-llama8b-32k-final", 5, 32, 8, 128, 500000.0,
                    [Prompt([passage_len] * n_passages, final_len)], n_layers=n_layers)


def small_ragged(seed: int, n_prompts: int, n_passages: int, lo: int, hi: int, qlo: int, qhi: int,
                 hq: int, hkv: int, d: int, base: float = 10000.0) -> Workload:
    """Miniature of config 3 for tests the oracle finishes in seconds."""
    rng = np.random.Generator(np.random.Philox(seed))
    prompts = []
    for _ in range(n_prompts):
        lens = [int(x) for x in rng.integers(lo, hi + 1, size=n_passages)]
        prompts.append(Prompt(lens, int(rng.integers(qlo, qhi + 1))))
    return Workload(f"ragged-{seed}", 0, hq, hkv, d, base, prompts)
