"""Independent yardsticks for pinning the oracle (no oracle or product code here)."""
from __future__ import annotations

import numpy as np
import torch


def rope_complex(x: np.ndarray, pos, base: float = 10000.0) -> np.ndarray:
    """RoPE as a complex multiplication: z_i = x_i + 1j*x_{i+d/2};  z_i * exp(1j*pos*theta_i).

    A different route to the same rotation than the oracle's real-valued cos/sin update.
    """
    x = np.asarray(x, dtype=np.float64)
    n, h, d = x.shape
    half = d // 2
    theta = np.exp(-np.log(base) * (2.0 * np.arange(half) / d))
    ang = np.asarray(pos, dtype=np.float64)[:, None] * theta[None, :]
    z = (x[..., :half] + 1j * x[..., half:]) * np.exp(1j * ang)[:, None, :]
    return np.concatenate([z.real, z.imag], axis=-1)


def sdpa_causal(q_rot: np.ndarray, k_rot: np.ndarray, v: np.ndarray) -> np.ndarray:
    """Textbook causal attention via torch's library routine, fp64.  Inputs [n, H, d]."""
    q = torch.from_numpy(np.ascontiguousarray(q_rot)).permute(1, 0, 2).unsqueeze(0)
    k = torch.from_numpy(np.ascontiguousarray(k_rot)).permute(1, 0, 2).unsqueeze(0)
    vv = torch.from_numpy(np.ascontiguousarray(v)).permute(1, 0, 2).unsqueeze(0)
    o = torch.nn.functional.scaled_dot_product_attention(q, k, vv, is_causal=True)
    return o.squeeze(0).permute(1, 0, 2).contiguous().numpy()


def sdpa_masked(q_rot: np.ndarray, k_rot: np.ndarray, v: np.ndarray, allow: np.ndarray) -> np.ndarray:
    """Library attention with an explicit boolean mask allow[nq, nk]; inputs [n, H, d], same H."""
    q = torch.from_numpy(np.ascontiguousarray(q_rot)).permute(1, 0, 2).unsqueeze(0)
    k = torch.from_numpy(np.ascontiguousarray(k_rot)).permute(1, 0, 2).unsqueeze(0)
    vv = torch.from_numpy(np.ascontiguousarray(v)).permute(1, 0, 2).unsqueeze(0)
    m = torch.from_numpy(np.ascontiguousarray(allow)).unsqueeze(0).unsqueeze(0)
    o = torch.nn.functional.scaled_dot_product_attention(q, k, vv, attn_mask=m)
    return o.squeeze(0).permute(1, 0, 2).contiguous().numpy()


def schema_starts(oracle_or_binding_layout, workload):
    starts, span = oracle_or_binding_layout(workload.sizes, workload.union_ids)
    return starts, span
