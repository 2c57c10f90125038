"""Shared pieces of the GPU parity tests: tolerance checks written out once."""
import numpy as np
import torch

from paper_2605_03644_amd import workloads as wl


def check_reencode_f32(k_gpu: np.ndarray, k_exact: np.ndarray, k_src: np.ndarray, rel: float = 1e-5):
    """Per rotation pair (i, i+d/2): |y_gpu - y_exact|_2 <= rel * |x pair|_2  (rotation keeps pair norms)."""
    d = k_gpu.shape[-1]
    h = d // 2
    err = np.sqrt((k_gpu[..., :h].astype(np.float64) - k_exact[..., :h]) ** 2 +
                  (k_gpu[..., h:].astype(np.float64) - k_exact[..., h:]) ** 2)
    norm = np.sqrt(k_src[..., :h].astype(np.float64) ** 2 + k_src[..., h:].astype(np.float64) ** 2)
    bad = err > rel * norm + 1e-30
    assert not bad.any(), f"{bad.sum()} pairs beyond {rel} relative; worst ratio {np.max(err / (norm + 1e-30)):.3e}"
    return float(np.max(err / (norm + 1e-30)))


def check_reencode_bf16(k_gpu_bits: np.ndarray, k_oracle_bits: np.ndarray, k_exact: np.ndarray,
                        k_src_bits: np.ndarray, min_equal: float = 0.99, rel: float = 1e-5):
    """Stored bf16 keys.  (a) >= 99 % are bit-identical to the oracle's round-to-nearest-even of the
    exact key.  (b) Every element is the rounding of an fp32 value that meets the fp32 bar:
    |y_gpu - y_exact| <= half a bf16 spacing at y (2^-8 |y|) + rel * |x pair|_2.  (A distance in
    representable values would be meaningless where the rotation cancels to ~0.)"""
    frac = float((k_gpu_bits == k_oracle_bits).mean())
    assert frac >= min_equal, f"only {frac:.4f} of bf16 keys bit-equal"
    d = k_exact.shape[-1]
    h = d // 2
    src = storage_to_f64(k_src_bits)
    norm = np.sqrt(src[..., :h] ** 2 + src[..., h:] ** 2)
    norm = np.concatenate([norm, norm], axis=-1)
    err = np.abs(storage_to_f64(k_gpu_bits) - k_exact)
    bound = 2.0 ** -8 * np.abs(k_exact) * (1 + 1e-6) + rel * norm + 1e-38
    bad = err > bound
    assert not bad.any(), f"{bad.sum()} bf16 keys beyond rounding + {rel} relative; worst excess {np.max(err - bound):.3e}"
    return frac


def check_attention(o_gpu: np.ndarray, o_ref: np.ndarray, max_abs: float = 2e-2, rel_fro: float = 1e-2):
    diff = np.abs(o_gpu.astype(np.float64) - o_ref)
    assert np.isfinite(o_gpu).all()
    assert diff.max() <= max_abs, f"attention max-abs error {diff.max():.3e} > {max_abs}"
    fro = np.linalg.norm(o_gpu.astype(np.float64) - o_ref) / max(np.linalg.norm(o_ref), 1e-30)
    assert fro <= rel_fro, f"attention relative Frobenius error {fro:.3e} > {rel_fro}"
    return float(diff.max()), float(fro)


def to_storage(t: torch.Tensor) -> np.ndarray:
    return wl.as_numpy_storage(t)


def storage_to_f64(a: np.ndarray) -> np.ndarray:
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return a.astype(np.float64)
