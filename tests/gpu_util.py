"""Plumbing shared by the GPU tests: numpy storage arrays <-> device tensors."""
import numpy as np

from paper_2207_10741_amd import binding as B, synth


def torch_mod():
    import torch
    return torch


def dev():
    return torch_mod().device("cuda:0")


def to_dev(storage: np.ndarray, dtype: int):
    """Storage array (float32, uint16 bit patterns or E4M3 bytes) -> device tensor of that dtype."""
    torch = torch_mod()
    if dtype == synth.F32:
        return torch.from_numpy(np.ascontiguousarray(storage, dtype=np.float32)).to(dev())
    if dtype == synth.FP8:
        return torch.from_numpy(np.ascontiguousarray(storage, dtype=np.uint8)).to(dev()).view(torch.float8_e4m3fn)
    t = torch.from_numpy(np.ascontiguousarray(storage).view(np.int16)).to(dev())
    return t.view(torch.bfloat16 if dtype == synth.BF16 else torch.float16)


def to_storage_np(t, dtype: int) -> np.ndarray:
    """Device tensor -> the storage array the oracle reads (no value conversion)."""
    torch = torch_mod()
    if dtype == synth.F32:
        return t.detach().cpu().numpy()
    if dtype == synth.FP8:
        return t.detach().view(torch.uint8).cpu().numpy()
    return t.detach().view(torch.int16).cpu().numpy().view(np.uint16)


def to_f64(t) -> np.ndarray:
    return t.detach().to(torch_mod().float64).cpu().numpy()


def mask_dev(mask: np.ndarray):
    return torch_mod().from_numpy(np.ascontiguousarray(mask, dtype=np.uint8)).to(dev())


def rel_err(got: np.ndarray, want: np.ndarray, keep: np.ndarray) -> float:
    """max |gpu - oracle| over the whole tensor, relative to the RMS of the oracle's kept outputs."""
    rms = float(np.sqrt(np.mean(np.square(want[keep])))) if keep.any() else 1.0
    if rms == 0.0:
        rms = 1.0
    return float(np.abs(got - want).max()) / rms
