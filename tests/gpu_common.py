"""Shared helpers of the GPU parity tests (HIP library vs CPU oracle on the same seeded inputs)."""
import numpy as np
import torch

import oracle
from helpers import to_np


def dev_index(ix_np):
    """numpy index dict -> torch tensors on the GPU."""
    return {k: torch.from_numpy(np.ascontiguousarray(v)).cuda() for k, v in ix_np.items() if k != "vectors"}


def oracle_stages(ix, Q, nprobe):
    S = oracle.coarse(Q, ix["centroids"])
    probes = oracle.select(S, nprobe)
    L = oracle.lut_f32(Q, ix["centroids"], ix["codebooks"], probes)
    LUT8, B, delta = oracle.quantise(L)
    return S, probes, L, LUT8, B, delta
