"""Helpers for the GPU parity tests: moving synthetic inputs to the device and results
back into the oracle's storage types.  No arithmetic of the method lives here."""
from __future__ import annotations

import numpy as np
import torch

import synth

TORCH_DTYPE = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}
RTOL = {"f32": 1e-5, "f16": 2e-2, "bf16": 2e-2}


def storage_to_torch(st: np.ndarray, dtype: str, device="cuda") -> torch.Tensor:
    if dtype == "bf16":
        return torch.from_numpy(st.view(np.int16).copy()).view(torch.bfloat16).to(device)
    return torch.from_numpy(np.ascontiguousarray(st)).to(device)


def values_to_torch(x_f32: np.ndarray, dtype: str, device="cuda") -> torch.Tensor:
    return storage_to_torch(synth.storage_array(x_f32, dtype), dtype, device)


def torch_to_storage(t: torch.Tensor) -> np.ndarray:
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def coo_to_device(row, col, val_f32, dtype, device="cuda"):
    return (torch.from_numpy(np.ascontiguousarray(row, dtype=np.int32)).to(device),
            torch.from_numpy(np.ascontiguousarray(col, dtype=np.int32)).to(device),
            values_to_torch(val_f32, dtype, device))


def bits(a: np.ndarray) -> np.ndarray:
    a = np.ascontiguousarray(a)
    return a.view(np.uint16 if a.dtype.itemsize == 2 else np.uint32)


def assert_format_equal(got_g, got_AM, got_AK, got_AV, want):
    g, AM, AK, AV = want
    assert got_g == g
    assert tuple(got_AM.shape) == AM.shape and tuple(got_AK.shape) == AK.shape
    assert tuple(got_AV.shape) == AV.shape
    assert np.array_equal(got_AM.cpu().numpy(), AM), "AM differs"
    assert np.array_equal(got_AK.cpu().numpy(), AK), "AK differs"
    assert np.array_equal(bits(torch_to_storage(got_AV)), bits(AV)), "AV differs"
