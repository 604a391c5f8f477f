"""Helpers shared by the GPU parity tests (marshalling only)."""
import numpy as np
import torch

from paper_2509_06040_amd import binding as br
from paper_2509_06040_amd import synth

DEV = "cuda"


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    return t.to(dtype) if dtype is not None else t


def host(t):
    torch.cuda.synchronize()
    return t.detach().float().cpu().numpy() if t.dtype == torch.bfloat16 else t.detach().cpu().numpy()


def bytes_buffer(n):
    return torch.empty(max(int(n), 256), dtype=torch.uint8, device=DEV)


def rel_l2(a, b):
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def make_model(cfg, W):
    return br.Model(cfg, br.upload_weights(cfg, W))


def cond_dev(cfg, cond):
    return dev(cond, torch.bfloat16 if cfg["dtype"] == synth.BF16 else torch.float32)
