"""Helpers of the GPU parity tests: run the HIP entry points on torch tensors and hand the
same inputs to the CPU oracle."""
import numpy as np
import torch

import fs_inputs
import oracle
import paper_2301_02959_amd as fs

DEV = "cuda:0"


def to_dev(a, dtype=None):
    t = torch.as_tensor(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.to(DEV)


def placement_dev(pl_np):
    """uint32 numpy -> int32 torch on the device (same bits)."""
    return torch.from_numpy(np.ascontiguousarray(pl_np).view(np.int32)).to(DEV)


def hip_route(ids, offsets, T, B, row_base, placement, U, W, self_, n=None, want_tiers=True):
    """All arguments are device tensors.  Returns device outputs + status int."""
    n = int(offsets[-1].item()) if n is None else n
    bo = torch.full((U + 1,), -7, dtype=torch.int64, device=DEV)
    rows = torch.full((max(n, 1),), -7, dtype=torch.int64, device=DEV)
    pos = torch.full((max(n, 1),), -7, dtype=torch.int32, device=DEV)
    tc = torch.full((3,), -7, dtype=torch.int64, device=DEV) if want_tiers else None
    st = torch.zeros(1, dtype=torch.int32, device=DEV)
    rc = fs.fs_route_bucketize(ids, offsets, T, B, row_base, placement, n, U, W, self_, bo, rows, pos, tc, st,
                               raise_on_error=False)
    torch.cuda.synchronize()
    return rc, int(st.item()), bo, rows[:n], pos[:n], tc


def hip_bwd(grad, rows, pos, j0, j1, R, variant=0, cap=None):
    m = j1 - j0
    cap = m if cap is None else cap
    D = grad.shape[1]
    uniq = torch.full((max(cap, 1),), -7, dtype=torch.int64, device=DEV)
    rg = torch.full((max(cap, 1), D), float("nan"), dtype=torch.float32, device=DEV)
    nu = torch.full((1,), -7, dtype=torch.int64, device=DEV)
    st = torch.zeros(1, dtype=torch.int32, device=DEV)
    rc = fs.fs_seq_grad_bwd(grad, rows, pos, j0, j1, R, variant, uniq, rg, cap, nu, st, raise_on_error=False)
    torch.cuda.synchronize()
    k = int(nu.item())
    return rc, int(st.item()), uniq[:min(k, cap)], rg[:min(k, cap)], k


def bits(t: torch.Tensor) -> np.ndarray:
    """Host bytes of a tensor, for bit-exact comparison."""
    return t.detach().cpu().contiguous().view(torch.uint8).numpy().reshape(-1)


def oracle_dtype(cfg_dtype: str) -> int:
    return {"f32": oracle.F32, "f16": oracle.F16, "bf16": oracle.BF16}[cfg_dtype]


def batch_on(cfg, device):
    b = fs_inputs.make_batch(cfg, device)
    pl = fs_inputs.make_placement(cfg, b["perms"], device)
    return b, pl
