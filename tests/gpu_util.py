"""Helpers shared by the GPU parity tests: host bits <-> device tensors, error metrics."""
import numpy as np
import torch

from paper_2401_09486_amd import workloads as wl

# tolerances of the parity bar: fp32 data max abs 1e-5; bf16 data max abs 2e-2 and mean abs 2e-3
F32_MAX = 1e-5
BF16_MAX, BF16_MEAN = 2e-2, 2e-3


def to_dev(a: np.ndarray) -> torch.Tensor:
    """float32 array -> float32 tensor; uint16 array (bf16 bits) -> bfloat16 tensor, same bits."""
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(a).cuda()


def to_host_f64(x: torch.Tensor) -> np.ndarray:
    if x.dtype == torch.bfloat16:
        bits = x.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
        return wl.bf16_bits_to_f32(bits).astype(np.float64)
    return x.cpu().numpy().astype(np.float64)


def host_bits(x: torch.Tensor) -> np.ndarray:
    """device tensor -> what the oracle accepts (float32 array or uint16 bf16 bits)."""
    if x.dtype == torch.bfloat16:
        return x.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    return x.cpu().numpy()


def check(got: np.ndarray, want: np.ndarray, dtype: str, what: str = ""):
    assert got.shape == want.shape, (got.shape, want.shape)
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    err = np.abs(got - want)
    mx, mean = float(err.max()), float(err.mean())
    if dtype == "f32":
        assert mx <= F32_MAX, f"{what}: max abs err {mx:.3e} > {F32_MAX}"
    else:
        assert mx <= BF16_MAX, f"{what}: max abs err {mx:.3e} > {BF16_MAX}"
        assert mean <= BF16_MEAN, f"{what}: mean abs err {mean:.3e} > {BF16_MEAN}"
    return mx, mean


def check_grad(got: np.ndarray, want: np.ndarray, dtype: str, what: str = ""):
    """The bar of the outputs, applied to the gradients as it stands: fp32 data max |err| <= 1e-5 max(1, |want|)
    (fp32 rounding is relative); bf16 data max |err| <= 2e-2 and mean |err| <= 2e-3, absolute.  Gradients are sums
    over many rows, returned in the storage dtype (bf16 rounds at 2^-9 |value|), so the absolute bar only holds
    while |value| stays in the single digits: with unit-normal upstream gradients and the configurations' input
    scales it does (max |value| 4.5 at the long-context shape); the magnitudes are printed with the errors."""
    assert got.shape == want.shape, (got.shape, want.shape)
    assert np.isfinite(got).all(), f"{what}: non-finite gradient"
    err = np.abs(got - want)
    mag = np.abs(want)
    mx, mean = float(err.max()), float(err.mean())
    print(f"[grad] {what}: max abs err {mx:.3e} mean abs err {mean:.3e} max|ref| {float(mag.max()):.3e} "
          f"mean|ref| {float(mag.mean()):.3e}", flush=True)
    if dtype == "f32":
        rel = float((err / np.maximum(1.0, mag)).max())
        assert rel <= F32_MAX, f"{what}: max err {rel:.3e} (relative above 1) > {F32_MAX}"
    else:
        assert mx <= BF16_MAX, f"{what}: max abs err {mx:.3e} > {BF16_MAX}"
        assert mean <= BF16_MEAN, f"{what}: mean abs err {mean:.3e} > {BF16_MEAN}"
    return mx
