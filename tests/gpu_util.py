"""Helpers for the GPU parity tests: move seeded numpy inputs to the device and back.
No arithmetic of the method lives here."""
import numpy as np
import torch


def dev():
    return torch.device("cuda:0")


def bf16_to_gpu(bits):
    """uint16 BF16 bit patterns -> torch.bfloat16 tensor on the GPU."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).to(dev())


def to_gpu(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(dev())


def u8(t):
    return t.cpu().numpy().astype(np.uint8, copy=False)


def bf16_out_to_f64(t):
    return t.float().cpu().numpy().astype(np.float64)


def scalar(t):
    return np.float32(t.cpu().numpy().reshape(-1)[0])
