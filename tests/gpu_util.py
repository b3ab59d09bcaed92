"""Helpers of the GPU parity tests: move a synthetic workload to the device, slice (b, h) pairs
for the oracle, and the error metric (max |x - ref| / max |ref| per tensor)."""
import numpy as np
import torch


def to_dev(w, device="cuda"):
    dt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    t = {}
    for name, arr in w.arrays.items():
        if arr is None:
            t[name] = None
        elif name in ("q", "k", "v", "dO"):
            t[name] = torch.from_numpy(arr).to(device=device, dtype=dt)   # exact: values are representable
        else:
            t[name] = torch.from_numpy(arr).to(device)
    return t


def host(x):
    return None if x is None else x.detach().float().cpu().numpy().astype(np.float64)


def select_pairs(w, pairs):
    """Oracle inputs for the selected (b, h) pairs, packed as B=1, H=len(pairs)."""
    bs = [p[0] for p in pairs]
    hs = [p[1] for p in pairs]
    out = {}
    for name, arr in w.arrays.items():
        if arr is None:
            out[name] = None
        elif name in ("S0", "M0"):
            out[name] = arr[bs, hs][None].astype(np.float64)                  # [1, P, dk, dv]
        else:
            out[name] = np.moveaxis(arr[bs, :, hs], 0, 1)[None].astype(np.float64)  # [1, T, P, ...]
    return out


def gather_pairs(x, pairs, is_state=False):
    """Same packing for a device result given as numpy [B,T,H,...] or [B,H,dk,dv]."""
    bs = [p[0] for p in pairs]
    hs = [p[1] for p in pairs]
    if is_state:
        return x[bs, hs][None]
    return np.moveaxis(x[bs, :, hs], 0, 1)[None]


def rel_err(x, ref):
    den = np.abs(ref).max()
    return float(np.abs(x - ref).max() / (den if den > 0 else 1.0))
