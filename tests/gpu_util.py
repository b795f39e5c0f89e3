"""Helpers for the GPU parity tests: host <-> device marshalling of the seeded
inputs and error norms.  No arithmetic of the method lives here."""
import numpy as np
import torch

import workloads as wl
import paper_2602_05754_amd as tf


def dev(a_f32: np.ndarray, dtype: str) -> torch.Tensor:
    """float32 host array -> device tensor of storage type dtype ("f32"/"bf16")."""
    if dtype == "bf16":
        bits = wl.f32_to_bf16_bits(a_f32).view(np.int16)
        return torch.from_numpy(bits).cuda().view(torch.bfloat16).reshape(a_f32.shape)
    return torch.from_numpy(np.ascontiguousarray(a_f32, dtype=np.float32)).cuda()


def host64(t: torch.Tensor) -> np.ndarray:
    """device tensor -> float64 host array (exact up-cast)."""
    return t.detach().to(torch.float64).cpu().numpy()


def raw_bytes(t: torch.Tensor) -> bytes:
    return t.detach().contiguous().view(torch.uint8).cpu().numpy().tobytes()


def rel_fro(got: np.ndarray, ref: np.ndarray) -> float:
    ref = np.asarray(ref, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    den = np.linalg.norm(ref.ravel())
    num = np.linalg.norm((got - ref).ravel())
    return float(num / den) if den > 0 else float(num)


def assert_elementwise(got, exact, dtype: str, label: str, scale: float = 1.0) -> None:
    """Every element within the bound that one rounding of an fp32-accumulated sum allows:
    bf16 storage |got - exact| <= 2^-8 |exact| + 1e-3 rms(exact), fp32 storage
    |got - exact| <= 1e-5 (|exact| + rms(exact)); `scale` widens the fp32 bound for sums of
    bf16 products accumulated over several calls."""
    exact = np.asarray(exact, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    assert got.shape == exact.shape, f"{label}: shape {got.shape} against {exact.shape}"
    rms = float(np.sqrt(np.mean(exact ** 2))) if exact.size else 0.0
    if dtype == "bf16":
        bound = 2.0 ** -8 * np.abs(exact) + 1e-3 * rms
    else:
        bound = scale * 1e-5 * (np.abs(exact) + rms)
    bad = ~(np.abs(got - exact) <= bound)          # a NaN in `got` fails
    if bad.any():
        i = np.unravel_index(int(np.argmax(np.where(bad, np.abs(got - exact), 0.0))), exact.shape)
        raise AssertionError(f"{label}: {int(bad.sum())} of {bad.size} elements off, worst at {i}: "
                             f"got {got[i]:.6e} exact {exact[i]:.6e} (rms {rms:.3e})")


def canary(shape, torch_dtype) -> torch.Tensor:
    """Device buffer filled with a recognisable non-trivial bit pattern (NaN payloads)."""
    n = int(np.prod(shape))
    if torch_dtype == torch.float32:
        bits = (np.uint32(0x7FC00000) + (np.arange(n, dtype=np.uint32) % np.uint32(0x3FFFFF))).view(np.int32)
        return torch.from_numpy(bits).cuda().view(torch.float32).reshape(shape)
    bits = (np.uint16(0x7FC0) + (np.arange(n, dtype=np.uint32) % 63).astype(np.uint16)).view(np.int16)
    return torch.from_numpy(bits).cuda().view(torch.bfloat16).reshape(shape)


TDT = {"f32": torch.float32, "bf16": torch.bfloat16}
CODE = {"f32": tf.TF_F32, "bf16": tf.TF_BF16}
TOL = {"f32": 1e-5, "bf16": 1e-2}      # relative Frobenius bounds per output tensor
