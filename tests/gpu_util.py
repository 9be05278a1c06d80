"""Helpers of the GPU parity tests: device buffers through torch, oracle-side rounding."""
import numpy as np
import torch

from oracle import model as om

DEV = "cuda:0"
TDT = {0: torch.float32, 1: torch.bfloat16}


def quant(a, dtype):
    """What the device holds after storing `a` (fp32 numpy) in the storage type, as float64."""
    a = np.asarray(a, dtype=np.float32)
    return (om.round_to_bf16(a) if dtype == 1 else a).astype(np.float64)


def dev(a, dtype):
    return torch.tensor(np.asarray(a, dtype=np.float32)).to(TDT[dtype]).to(DEV).contiguous()


def host(t):
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def rel_l2(got, ref):
    return float(np.linalg.norm(np.asarray(got, dtype=np.float64) - ref) / max(np.linalg.norm(ref), 1e-30))


def sync():
    torch.cuda.synchronize()
