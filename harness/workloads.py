"""Primes a PbsaCache with the synthetic state of a named workload (data movement only)."""
from __future__ import annotations

import numpy as np
import torch

from . import synth
from paper_2604_21221_amd.cache import PbsaCache


def bf16_tensor(bits: np.ndarray, device) -> torch.Tensor:
    """uint16 bf16 bit patterns (numpy) -> torch.bfloat16 tensor on `device`, bits unchanged."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(device).view(torch.bfloat16)


def bits_of(t: torch.Tensor) -> np.ndarray:
    """torch.bfloat16 tensor -> uint16 bit patterns on the host."""
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def cache_for_workload(w: synth.Workload, layer: int = 0, device="cuda:0", fold=True, ring_chunks=None):
    """Returns (cache, index of the first chunk to run).  Warm workloads get C seeded persistent slots,
    the pre-filled summary (if any) and their full window (global chunks 0..w-1); cold ones nothing."""
    c = PbsaCache(w.H, w.d, w.B, w.Nq, w.window_chunks, w.C, w.k, np.float32(w.scale), fold=fold, device=device,
                  ring_chunks=ring_chunks)
    if w.cold_start:
        return c, 0
    Kp, Vp = synth.persistent_init(w, layer)
    ids = (-100 - torch.arange(w.C, dtype=torch.int64))[None, :].repeat(w.H, 1)
    c.set_persistent(bf16_tensor(Kp, device), bf16_tensor(Vp, device),
                     torch.full((w.H, w.C), w.B, dtype=torch.int32, device=device), ids)
    if w.summary_prefill:
        S_sum, S_cnt = synth.summary_init(w, layer)
        c.set_summary(torch.from_numpy(S_sum).to(device), torch.from_numpy(S_cnt).to(device))
    for g in range(w.window_chunks):
        _, K, V = synth.chunk_qkv(w, layer, g)
        c.append_chunk(bf16_tensor(K, device), bf16_tensor(V, device), g)
    return c, w.window_chunks
