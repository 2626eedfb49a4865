"""Helpers shared by the GPU parity tests: host<->device marshalling and the error metric."""
import numpy as np
import torch

from paper_2203_05705_amd import workloads as WL

TOL = {"f32": 1e-5, "bf16": 2e-2}      # max |gpu - oracle| / max |oracle| per output tensor


def to_dev(a: np.ndarray, dtype: str) -> torch.Tensor:
    """Host array (float32 values, or uint16 bf16 bit patterns) -> device tensor, bytes unchanged."""
    if dtype == "bf16":
        assert a.dtype == np.uint16
        return torch.from_numpy(a.view(np.int16).copy()).cuda().view(torch.bfloat16)
    assert a.dtype == np.float32
    return torch.from_numpy(a.copy()).cuda()


def from_vals(a: np.ndarray, dtype: str) -> torch.Tensor:
    """fp64/fp32 values -> device tensor of the storage dtype (rounded once, on the host)."""
    a32 = np.ascontiguousarray(a, dtype=np.float32)
    return to_dev(WL.f32_to_bf16_bits(a32) if dtype == "bf16" else a32, dtype)


def stored(a: np.ndarray, dtype: str) -> np.ndarray:
    """Exact fp64 values of `a` after rounding to the storage dtype (host side)."""
    a32 = np.ascontiguousarray(a, dtype=np.float32)
    return WL.bf16_to_f64(WL.f32_to_bf16_bits(a32)) if dtype == "bf16" else a32.astype(np.float64)


def to_host(t: torch.Tensor) -> np.ndarray:
    """Device tensor -> fp64 values."""
    return t.detach().float().cpu().numpy().astype(np.float64)


def raw_bits(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.bfloat16:
        return t.detach().view(torch.int16).cpu().numpy().view(np.uint16)
    return t.detach().view(torch.int32).cpu().numpy().view(np.uint32)


def max_rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    den = float(np.max(np.abs(ref)))
    if den == 0.0:
        return float(np.max(np.abs(got)))
    return float(np.max(np.abs(got - ref)) / den)


def assert_parity(got_t: torch.Tensor, ref: np.ndarray, dtype: str, zero_mask=None, what=""):
    """Float parity within TOL[dtype]; positions where zero_mask is True must hold exactly +0.0."""
    got = to_host(got_t)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.all(np.isfinite(got)), what
    err = max_rel_err(got, ref)
    assert err <= TOL[dtype], f"{what}: max rel err {err:.3e} > {TOL[dtype]}"
    if zero_mask is not None:
        bits = raw_bits(got_t)
        assert np.all(bits[np.broadcast_to(zero_mask, bits.shape)] == 0), f"{what}: dropped entries are not +0.0"
    return err
