"""Helpers shared by the GPU parity tests: host arrays -> device tensors, oracle calls, error metric."""
import numpy as np
import torch

from oracle import c_oracle

TOL = {"f32": 1e-4, "bf16": 2e-2}   # max|err| / RMS(oracle), the bar the build is held to


def to_dev(x, dtype):
    """numpy inputs (float32 holding f32 or bf16-representable values) -> GPU tensors."""
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    out = {}
    for key, a in x.items():
        if not isinstance(a, np.ndarray):
            continue
        t = torch.from_numpy(np.ascontiguousarray(a))
        if key in ("Q", "K", "V", "q", "k", "v", "k_cache", "v_cache"):
            t = t.to(tdt)      # exact: the values are representable
        out[key] = t.cuda()
    return out


def rel_err(got, ref):
    """max |got - ref| / RMS(ref), over the whole tensor."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    rms = np.sqrt(np.mean(ref * ref))
    return float(np.max(np.abs(got - ref)) / (rms if rms > 0 else 1.0))


def host(t):
    return t.detach().float().cpu().numpy() if t.is_floating_point() else t.detach().cpu().numpy()


def oracle_fwd(x, **kw):
    return c_oracle.fwd(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], x["mask"], **kw)
