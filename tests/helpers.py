"""Shared helpers for the GPU parity tests: host<->device marshalling and set comparison."""
from __future__ import annotations

import numpy as np
import torch

from paper_2511_12201_amd import synth


def to_device(x: np.ndarray, dtype: str) -> torch.Tensor:
    """float32 host array -> device tensor of the layer dtype (bf16 arrays must lie on the bf16 grid)."""
    if dtype == "bf16":
        return torch.from_numpy(synth.bf16_bits(x)).view(torch.bfloat16).cuda()
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda()


def to_host(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.bfloat16:
        return t.detach().float().cpu().numpy()
    return t.detach().cpu().numpy()


def lists_to_padded(lists, n_heads: int, width: int):
    """list[batch][head] of index arrays -> (idx [B,H,width] int32 device, cnt [B,H] int32 device)."""
    B = len(lists)
    idx = np.zeros((B, n_heads, width), dtype=np.int32)
    cnt = np.zeros((B, n_heads), dtype=np.int32)
    for b in range(B):
        for h in range(n_heads):
            a = np.asarray(lists[b][h], dtype=np.int32)
            idx[b, h, : a.size] = a
            cnt[b, h] = a.size
    return torch.from_numpy(idx).cuda(), torch.from_numpy(cnt).cuda()


def padded_to_lists(idx: torch.Tensor, cnt: torch.Tensor):
    idx, cnt = idx.cpu().numpy(), cnt.cpu().numpy()
    return [[idx[b, h, : cnt[b, h]].copy() for h in range(idx.shape[1])] for b in range(idx.shape[0])]


def near_cut_only(got: np.ndarray, want: np.ndarray, values: np.ndarray, cut: float, rel: float) -> bool:
    """True iff every index in the symmetric difference has a value within rel of the cut."""
    diff = np.setxor1d(got, want)
    if diff.size == 0:
        return True
    return bool(np.all(np.abs(values[diff].astype(np.float64) - cut) <= rel * max(abs(cut), 1e-30)))
