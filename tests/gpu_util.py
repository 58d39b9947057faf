"""Helpers shared by the GPU parity tests: move synthetic inputs to the device in the storage
type of the configuration, run the HIP path through the ctypes binding, and compare with the
oracle with the tolerance of the benchmark spec: max|gpu - oracle| / max|oracle| per tensor."""
import numpy as np
import torch

TOL = {"f32": 1e-4, "bf16": 2e-2}


def tdtype(dt):
    return torch.bfloat16 if dt == "bf16" else torch.float32


def dev(a, dt=None):
    """numpy -> cuda tensor; dt 'bf16'/'f32' for storage-typed tensors, None for float state, ints stay ints."""
    if a is None:
        return None
    t = torch.from_numpy(np.ascontiguousarray(a))
    if t.dtype in (torch.int32, torch.int64):
        return t.to(torch.int32).cuda()
    t = t.to(torch.float32)
    return t.to(tdtype(dt)).cuda() if dt else t.cuda()


def host(t):
    return None if t is None else t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def rel_err(got, ref):
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.isfinite(got).all(), "non-finite values in GPU result"
    return np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-30)


def check(name, got, ref, tol):
    e = rel_err(host(got) if isinstance(got, torch.Tensor) else got, ref)
    print("    %-6s rel err %.3e (tol %.1e)" % (name, e, tol), flush=True)
    assert e < tol, (name, e)
    return e
