"""Helpers shared by the GPU parity tests (no arithmetic of the method here)."""
import numpy as np
import torch

import lt_workloads as W

TOL_OUT = 2e-3       # max |out_gpu - out_oracle| on fp32-accumulated outputs
TOL_LSE = 2e-3
TOL_RATIO = 1e-4     # max |r_gpu - r_oracle|, also applied to every rho


def say(*a):
    """Name the case before its GPU step, flushed, so a fault can be traced to it."""
    print(*a, flush=True)


def randn_bf16(shape, seed, device="cuda:0", scale=1.0):
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return (torch.randn(tuple(shape), generator=g, device=device, dtype=torch.float32) * scale).to(torch.bfloat16)


def bits(t):
    return W.bf16_bits(t)


def f64(t):
    return t.detach().cpu().numpy().astype(np.float64)
