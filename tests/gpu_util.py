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


def token_rel_l2(a, b):
    """Per-token relative L2 over the last axis -> flat array of the leading dimensions."""
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    a2, b2 = a.reshape(-1, a.shape[-1]), b.reshape(-1, b.shape[-1])
    return np.linalg.norm(a2 - b2, axis=1) / np.maximum(np.linalg.norm(b2, axis=1), 1e-300)


def assert_close(got, want, tol, tag=""):
    """The comparison every recompute test makes, for activations and gradients alike:
      * relative L2 of the whole tensor <= tol (the stated tolerance: 1e-4 fp32, 2e-2 bf16);
      * relative L2 of every token's row <= tol (2 tol in fp32, where a row of a small test stage has few elements);
      * element by element |got - want| <= 2^-7 |want| + 5 tol RMS(want row): the first term is the output rounding
        (bf16 keeps 8 significant bits), the second bounds what the accumulated error of one element may be next to its
        row -- five times the row's allowed relative L2.  A single wrong lane (an element off by its own magnitude) in
        a row of thousands moves the row's relative L2 by 1/sqrt(D) and would pass the row test; it fails this one.
    Returns (whole, worst token, worst element in units of the bound) for the caller to print."""
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    whole = rel_l2(got, want)
    tok = token_rel_l2(got, want)
    row_rms = np.sqrt(np.mean(want.reshape(-1, want.shape[-1]) ** 2, axis=1)).reshape(want.shape[:-1] + (1,))
    bound = 2.0 ** -7 * np.abs(want) + 5.0 * tol * row_rms
    elem = float(np.max(np.abs(got - want) / np.maximum(bound, 1e-300)))
    assert whole <= tol, (tag, "whole", whole)
    assert tok.max() <= (2 * tol if tol < 1e-3 else tol), (tag, "token", int(tok.argmax()), float(tok.max()))
    assert elem <= 1.0, (tag, "element", elem, np.unravel_index(np.argmax(np.abs(got - want) / np.maximum(bound, 1e-300)), got.shape))
    return whole, float(tok.max()), elem
