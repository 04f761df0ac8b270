"""Helpers of the GPU parity tests (the HIP path vs the CPU oracle on the same seeded inputs)."""
import numpy as np
import torch

TOL_F32 = 1e-4     # relative L2, fp32 workloads
TOL_BF16 = 2e-2    # relative L2, bf16 workloads
TOL_DISC = 1e-3    # relative, discrepancy scalar on identical branch outputs


def dev(a, dtype=torch.float32):
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return t if dtype == torch.float32 else t.to(dtype)


def host(t):
    torch.cuda.synchronize()
    return t.detach().float().cpu().numpy().astype(np.float64)


def rel_l2(got, ref):
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    den = np.linalg.norm(ref)
    num = np.linalg.norm(got - ref)
    return num / den if den > 0 else num


def tdt(name):
    return torch.bfloat16 if name == "bf16" else torch.float32


def tol(name):
    return TOL_BF16 if name == "bf16" else TOL_F32
