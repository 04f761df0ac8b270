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


ROW_SLACK = 2.0    # a single row may be off by this factor more than the whole tensor


def worst_row(got, ref):
    """Largest relative L2 error of one row (a row = the last axis: one token, one sample; trailing axes are
    merged until a row has at least 64 elements, so a latent [B, H, W, 16] is judged per line of W * 16).
    The error of row r is ||got_r - ref_r|| / max(||ref_r||, rms of the row norms), so that rows which are
    nearly zero in the reference are measured against a typical row instead of against nothing."""
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    if ref.ndim < 2 or ref.size == 0:
        return rel_l2(got, ref)
    shape = list(ref.shape)
    while len(shape) > 2 and shape[-1] < 64:
        shape[-2:] = [shape[-2] * shape[-1]]
    g, r = got.reshape(-1, shape[-1]), ref.reshape(-1, shape[-1])
    rn = np.linalg.norm(r, axis=1)
    floor = np.sqrt(np.mean(rn * rn))
    den = np.maximum(rn, floor)
    den[den == 0] = 1.0
    return float(np.max(np.linalg.norm(g - r, axis=1) / den))


def err(got, ref):
    """The parity figure of the GPU tests: the whole-tensor relative L2 error, or the worst single row's
    divided by ROW_SLACK when that is larger.  `err(got, ref) < tol` therefore demands rel-L2 < tol for the
    tensor AND < ROW_SLACK * tol for every row: one wrong token row among thousands (a ragged tile, a merge of
    split partial results, a gate taken from the neighbouring sample) fails it, which a norm over the whole
    tensor would not notice."""
    return max(rel_l2(got, ref), worst_row(got, ref) / ROW_SLACK)


def tdt(name):
    return torch.bfloat16 if name == "bf16" else torch.float32


def tol(name):
    return TOL_BF16 if name == "bf16" else TOL_F32
