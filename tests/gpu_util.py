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
    """Gradients are sums over many rows and are not bounded by the value range as the outputs are, so
    the bar scales with the value: fp32 data |err| <= 1e-5 (1 + |want|); bf16 data
    |err| <= 2e-2 (1 + |want|) and mean |err| <= 2e-3 (1 + mean |want|) -- the output bar at magnitude
    <= 1, and a few bf16 roundings (2^-9 each: weights, score gradients, result) above it."""
    assert got.shape == want.shape, (got.shape, want.shape)
    assert np.isfinite(got).all(), f"{what}: non-finite gradient"
    err = np.abs(got - want)
    mag = np.abs(want)
    rel = float((err / (1.0 + mag)).max())
    if dtype == "f32":
        assert rel <= F32_MAX, f"{what}: scaled max err {rel:.3e} > {F32_MAX}"
    else:
        assert rel <= BF16_MAX, f"{what}: scaled max err {rel:.3e} > {BF16_MAX}"
        mean, bar = float(err.mean()), BF16_MEAN * (1.0 + float(mag.mean()))
        assert mean <= bar, f"{what}: mean abs err {mean:.3e} > {bar:.3e}"
    return rel
