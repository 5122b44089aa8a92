"""Helpers shared by the GPU parity tests: device transfer and the comparison rule."""
import numpy as np
import torch

NORMWISE_TOL = 1e-2      # ||C_gpu - C_ref||_F / ||C_ref||_F
ELEMENTWISE_TOL = 2e-2   # max |C_gpu - C_ref| / max |C_ref|


_shared_ws = None


def shared_workspace():
    """Register (again) the one torch-owned split-K scratch area the GPU tests share: 4 KiB of flags
    plus 256 slots of a 256 x 256 fp32 tile, which covers every product."""
    global _shared_ws
    from paper_2502_08145_amd import binding as B
    torch.cuda.synchronize()
    if _shared_ws is None:
        _shared_ws = torch.empty((B.WORKSPACE_ALL,), dtype=torch.uint8, device="cuda")
    B.axonn_linear_set_workspace(_shared_ws)
    return _shared_ws


def to_device(bits: np.ndarray) -> torch.Tensor:
    """numpy uint16 bf16 bit patterns -> bf16 CUDA tensor holding exactly those bits."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def to_host_bits(t: torch.Tensor) -> np.ndarray:
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def bits_to_f64(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def f64_to_bf16_bits_rne(x: np.ndarray) -> np.ndarray:
    """fp64 -> bf16 bits, round to nearest even directly from the fp64 value.

    Only used where x is exactly representable in fp32 (integer-valued sums), so that the
    double rounding fp64 -> fp32 -> bf16 cannot differ from a single rounding.
    """
    f = x.astype(np.float32)
    assert np.array_equal(f.astype(np.float64), x), "value not exact in fp32"
    u = f.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def errors(c_gpu_bits: np.ndarray, c_ref: np.ndarray):
    got = bits_to_f64(c_gpu_bits)
    diff = got - c_ref
    ref_norm = np.linalg.norm(c_ref.ravel())
    ref_max = np.abs(c_ref).max() if c_ref.size else 0.0
    normwise = np.linalg.norm(diff.ravel()) / ref_norm if ref_norm > 0 else np.linalg.norm(diff.ravel())
    elementwise = np.abs(diff).max() / ref_max if ref_max > 0 else np.abs(diff).max()
    return float(normwise), float(elementwise)


def assert_close(c_gpu_bits: np.ndarray, c_ref: np.ndarray, what: str = ""):
    """The acceptance rule: normwise relative error <= 1e-2 and elementwise error
    <= 2e-2 * max|ref| (bf16 output, fp32 accumulation)."""
    assert np.isfinite(bits_to_f64(c_gpu_bits)).all(), f"{what}: non-finite output"
    nw, ew = errors(c_gpu_bits, c_ref)
    assert nw <= NORMWISE_TOL, f"{what}: normwise relative error {nw:.3e} > {NORMWISE_TOL}"
    assert ew <= ELEMENTWISE_TOL, f"{what}: elementwise error {ew:.3e} > {ELEMENTWISE_TOL} * max|ref|"
    return nw, ew
