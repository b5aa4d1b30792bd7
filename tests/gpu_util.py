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


def bf16_half_ulp(ref):
    """Half a unit in the last place of bf16 (8 significant bits) at each |ref|: the rounding
    error a correctly rounded bf16 store of the exact value may carry."""
    a = np.abs(np.asarray(ref, dtype=np.float64))
    e = np.floor(np.log2(np.maximum(a, 2.0 ** -126)))
    return np.where(a > 0, 2.0 ** (e - 8), 0.0)


def rel_err(got, ref, stored=None):
    """max |got - ref| / RMS(ref), over the whole tensor.

    stored="bf16": the tensor under test was written in bf16.  The storage rounding of the exact
    result (up to 2^-8 |ref|, which for these workloads alone reaches 3.6e-2 .. 5e-2 of RMS(O) on
    the largest elements) is not a compute error, so half a bf16 ulp of the reference is
    subtracted element-wise before the maximum is taken."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    rms = np.sqrt(np.mean(ref * ref))
    diff = np.abs(got - ref)
    if stored == "bf16":
        diff = np.maximum(diff - bf16_half_ulp(ref), 0.0)
    return float(np.max(diff) / (rms if rms > 0 else 1.0))


def stored(dtype):
    return "bf16" if dtype == "bf16" else None


def host(t):
    return t.detach().float().cpu().numpy() if t.is_floating_point() else t.detach().cpu().numpy()


def oracle_fwd(x, **kw):
    return c_oracle.fwd(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], x["mask"], **kw)
