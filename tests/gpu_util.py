"""Helpers of the GPU parity tests: move a synthetic workload to the device, slice (b, h) pairs
for the oracle, and the two error metrics per tensor: max |x - ref| / max |ref| (the bound the tolerances are
stated for) and the RMS-relative error rms(x - ref) / rms(ref), which a few large entries cannot hide behind."""
import numpy as np

from paper_2605_05838_amd import synth


def to_dev(w, device="cuda"):
    return synth.to_device(w, device)


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


def rms_rel_err(x, ref):
    den = np.sqrt(np.mean(np.square(ref)))
    return float(np.sqrt(np.mean(np.square(x - ref))) / (den if den > 0 else 1.0))


def worst_err(x, ref):
    """The larger of the two metrics: what the tests bound."""
    return max(rel_err(x, ref), rms_rel_err(x, ref))


def fmt_errs(errs):
    """{name: (max-normalised, rms-relative)} as a short string."""
    return "{" + ", ".join(f"{k}: {a:.2e}/{b:.2e}" for k, (a, b) in errs.items()) + "}"
