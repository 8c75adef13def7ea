"""Seeded synthetic inputs shaped like the paper's workloads.

This module only *describes* workloads (sizes, which modules a prompt imports,
how many uncached tokens follow) and draws random tensors.  It holds none of
the method's arithmetic: no position layout, no RoPE, no masking, no attention.
Callers get schema entry sizes and union ids and compute start positions with
whichever implementation they are exercising.

The paper evaluates on LongBench documents of 4K-10K tokens (about 5K on
average) used as prompt modules, with a short task directive as uncached text
(Sec. 5.1, 5.2); that suite is not available here, so these configurations
stand in for it by shape only.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np
import torch


@dataclass
class Prompt:
    """One request: imported modules in buffer order and a trailing run of uncached text."""
    module_ids: List[int]
    n_new: int                       # uncached tokens, placed after the imported module that ends last
    # optional extra run of uncached text placed right after `gap_after` (a module id)
    gap_after: Optional[int] = None
    n_gap: int = 0


@dataclass
class Workload:
    name: str
    config_index: int                # 1-based index into the benchmark's config list (0 = extra test case)
    dtype: str                       # "f32" | "bf16"
    n_layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    rope_base: float
    max_pos: int
    sizes: List[int]                 # schema entries in schema order; module id = index
    union_ids: List[int]             # -1 = ordinary module, else union id (children adjacent)
    prompts: List[Prompt] = field(default_factory=list)

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    @property
    def row_bytes(self) -> int:
        return self.n_kv_heads * self.head_dim * self.elem_bytes

    def used_module_ids(self) -> List[int]:
        seen = []
        for p in self.prompts:
            for m in p.module_ids:
                if m not in seen:
                    seen.append(m)
        return sorted(seen)


# ------------------------------------------------------------------ tensors
def _gen(workload: Workload, layer: int, kind: int, ident: int) -> torch.Generator:
    g = torch.Generator(device="cpu")
    seed = (((1000 * workload.config_index + layer) * 65536 + ident) * 8 + kind) % (2 ** 62)
    g.manual_seed(seed)
    return g


def _normal(workload: Workload, gen: torch.Generator, shape: Sequence[int]) -> torch.Tensor:
    """N(0,1) drawn in fp32 on the CPU, rounded to the workload dtype (RNE for bf16)."""
    return torch.randn(*shape, generator=gen, dtype=torch.float32).to(workload.torch_dtype)


def module_raw_kv(workload: Workload, layer: int, module_id: int) -> Tuple[torch.Tensor, torch.Tensor]:
    """(K, V) of one prompt module for one layer, [len, Hkv, d].

    K is 'raw': tests that need position-encoded keys rotate it with the
    implementation under test; benchmarks may store it as is (the pool treats
    module states as opaque bytes).
    """
    n = workload.sizes[module_id]
    shape = (n, workload.n_kv_heads, workload.head_dim)
    return (_normal(workload, _gen(workload, layer, 0, module_id), shape),
            _normal(workload, _gen(workload, layer, 1, module_id), shape))


def new_token_qkv(workload: Workload, layer: int, prompt_index: int, n_tokens: int):
    """(Q, K, V) of a prompt's uncached tokens for one layer: [n, Hq, d], [n, Hkv, d], [n, Hkv, d]."""
    q = _normal(workload, _gen(workload, layer, 2, prompt_index), (n_tokens, workload.n_q_heads, workload.head_dim))
    k = _normal(workload, _gen(workload, layer, 3, prompt_index), (n_tokens, workload.n_kv_heads, workload.head_dim))
    v = _normal(workload, _gen(workload, layer, 4, prompt_index), (n_tokens, workload.n_kv_heads, workload.head_dim))
    return q, k, v


def address_coded(workload: Workload, layer: int, module_id: int, which: int) -> torch.Tensor:
    """Module states whose every 16-bit word encodes (layer, module, K-or-V, row, column).

    Used by placement tests: a row copied to the wrong place, or from the wrong
    module, cannot go unnoticed.  Includes NaN, -0.0 and denormal bit patterns
    by construction (all 16-bit patterns occur), which a bytewise copy must keep.
    """
    n = workload.sizes[module_id]
    cols = workload.n_kv_heads * workload.head_dim * workload.elem_bytes // 2
    r = torch.arange(n, dtype=torch.int64).unsqueeze(1)
    c = torch.arange(cols, dtype=torch.int64).unsqueeze(0)
    word = (r * 40503 + c * 9973 + module_id * 6151 + layer * 389 + which * 127 + 12345) % 65536
    words = (word - 65536 * (word >= 32768)).to(torch.int16)   # reinterpret 0..65535 as int16
    flat = words.contiguous().view(torch.uint8).reshape(n, -1)
    return flat.view(workload.torch_dtype).reshape(n, workload.n_kv_heads, workload.head_dim)


# ------------------------------------------------------------------ configs
def tiny_fp32() -> Workload:
    """Config 1: 1 layer, 8 heads (MHA), d 64; three 128-token modules; 32 uncached tokens."""
    return Workload("tiny_fp32", 1, "f32", 1, 8, 8, 64, 10000.0, 1024,
                    [128, 128, 128], [-1, -1, -1], [Prompt([0, 1, 2], 32)])


def llama7b_doc(n_layers: int = 32) -> Workload:
    """Config 2: Llama-2-7B-shaped attention (32/32 heads, d 128); a 64-token system module, a
    2048-token document module, 128 uncached tokens."""
    return Workload("llama7b_doc", 2, "bf16", n_layers, 32, 32, 128, 10000.0, 4096,
                    [64, 2048], [-1, -1], [Prompt([0, 1], 128)])


def long_doc_8k(n_layers: int = 32) -> Workload:
    """Config 3: GQA 32/8, d 128; four 2048-token modules (8192 assembled), 256 uncached tokens."""
    return Workload("long_doc_8k", 3, "bf16", n_layers, 32, 8, 128, 10000.0, 16384,
                    [2048] * 4, [-1] * 4, [Prompt([0, 1, 2, 3], 256)])


def sparse_selection(n_layers: int = 32, seed: int = 0, n_prompts: int = 1) -> Workload:
    """Config 4: pool of 64 modules, lengths uniform in [64, 512], arranged as 32 unions of two
    siblings so that the schema fits 16384 position IDs; each prompt imports one sibling of 12
    unions chosen from the seed, in shuffled buffer order; 64 uncached tokens."""
    rng = np.random.default_rng(4000 + seed)
    while True:
        sizes = [int(x) for x in rng.integers(64, 513, size=64)]
        span = sum(max(sizes[2 * u], sizes[2 * u + 1]) for u in range(32))
        if span + 64 <= 16384:
            break
    union_ids = [i // 2 for i in range(64)]
    prompts = []
    for _ in range(n_prompts):
        unions = rng.choice(32, size=12, replace=False)
        picks = [int(2 * u + rng.integers(0, 2)) for u in unions]
        prompts.append(Prompt(picks, 64))
    return Workload("sparse_selection", 4, "bf16", n_layers, 32, 8, 128, 10000.0, 16384,
                    sizes, union_ids, prompts)


def batched_serving(n_layers: int = 32, n_prompts: int = 16) -> Workload:
    """Config 5: 16 concurrent prompts share one 4096-token module; each adds two private
    512-token modules and 128 uncached tokens.  The private modules of different prompts are
    alternatives at the same schema location, i.e. two unions of n_prompts children."""
    sizes = [4096] + [512] * n_prompts + [512] * n_prompts
    union_ids = [-1] + [0] * n_prompts + [1] * n_prompts
    prompts = [Prompt([0, 1 + b, 1 + n_prompts + b], 128) for b in range(n_prompts)]
    return Workload("batched_serving", 5, "bf16", n_layers, 32, 8, 128, 10000.0, 8192,
                    sizes, union_ids, prompts)


def by_name(name: str, **kw) -> Workload:
    table = {"tiny_fp32": tiny_fp32, "llama7b_doc": llama7b_doc, "long_doc_8k": long_doc_8k,
             "sparse_selection": sparse_selection, "batched_serving": batched_serving}
    return table[name](**kw)


# ------------------------------------------------- reduced / edge-case workloads for tests
def custom(name: str, dtype: str, n_q_heads: int, n_kv_heads: int, head_dim: int, sizes: Sequence[int],
           union_ids: Optional[Sequence[int]], prompts: Sequence[Prompt], n_layers: int = 1,
           max_pos: int = 16384, config_index: int = 0, rope_base: float = 10000.0) -> Workload:
    return Workload(name, config_index, dtype, n_layers, n_q_heads, n_kv_heads, head_dim, rope_base, max_pos,
                    list(sizes), list(union_ids) if union_ids is not None else [-1] * len(sizes), list(prompts))
