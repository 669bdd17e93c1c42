"""Helpers shared by the GPU parity tests: host <-> device marshalling only."""
import numpy as np


def dev(x, dtype):
    """numpy fp32 (already representable in `dtype`) -> torch device tensor of the stage dtype."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda()
    return t.to(torch.bfloat16) if dtype == "bf16" else t


def host(t):
    """torch device tensor -> numpy float64."""
    return t.detach().float().cpu().numpy().astype(np.float64)


def dev_weights(blocks, dtype):
    return [{k: (None if v is None else dev(v, dtype)) for k, v in b.items()} for b in blocks]


def rel_l2(a, b):
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    return float(np.linalg.norm((a - b).ravel()) / max(np.linalg.norm(b.ravel()), 1e-300))
