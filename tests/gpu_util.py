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


def assert_same_bits(got, want, tag):
    """Bit-exact comparison with a short report instead of an array dump."""
    got = np.ascontiguousarray(got); want = np.ascontiguousarray(want)
    assert got.shape == want.shape and got.dtype.itemsize == want.dtype.itemsize, (tag, got.shape, want.shape)
    view = {1: np.uint8, 2: np.uint16, 4: np.uint32, 8: np.uint64}[got.dtype.itemsize]
    bad = np.flatnonzero(got.view(view).ravel() != want.view(view).ravel())
    if bad.size:
        i = int(bad[0])
        raise AssertionError(f"{tag}: {bad.size} of {got.size} elements differ; first at flat index {i}: "
                             f"got {got.ravel()[i]!r} want {want.ravel()[i]!r}")
