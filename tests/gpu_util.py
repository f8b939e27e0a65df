"""Helpers for the GPU parity tests: host<->device conversion of the seeded inputs and error norms."""
import numpy as np
import torch

DEV = "cuda:0"


def dev(a, dtype=None):
    """float32 NumPy array -> device tensor; dtype 'bf16' casts (exact for bf16-representable values)."""
    t = torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    if dtype == "bf16":
        t = t.to(torch.bfloat16)
    return t


def host(t):
    if t.dtype == torch.bfloat16:
        t = t.to(torch.float32)
    return t.detach().cpu().numpy()


def bits(t):
    """Raw bit patterns of a device tensor as a NumPy integer array."""
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy()
    if t.dtype == torch.float32:
        return t.view(torch.int32).cpu().numpy()
    return t.cpu().numpy()


def attn_errors(got, want):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    max_abs = float(np.abs(got - want).max())
    rel_fro = float(np.linalg.norm((got - want).ravel()) / max(np.linalg.norm(want.ravel()), 1e-300))
    return max_abs, rel_fro


ATTN_MAX_ABS = 2e-2
ATTN_REL_FRO = 5e-3
SCORE_MAX_ABS = 1e-3


def attention_workspace(D):
    """Device buffer with which the attention launch may cut its work into equal runs."""
    from paper_2601_21896_amd import binding as B
    return torch.empty(B.pafu_attention_workspace_bytes(1, 1, D), dtype=torch.uint8, device=DEV)


def step_workspace(args):
    """Device buffer of pafu_step_workspace_bytes(args) bytes, attached to the argument struct."""
    from paper_2601_21896_amd import binding as B
    ws = torch.empty(max(B.pafu_step_workspace_bytes(args), 16), dtype=torch.uint8, device=DEV)
    args.workspace = ws.data_ptr()
    args.workspace_bytes = ws.numel()
    args._keep_ws = ws
    return ws
