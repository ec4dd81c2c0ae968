"""Helpers shared by the GPU parity tests: host <-> device plumbing only."""
import numpy as np
import torch

from paper_2503_24358_amd import synth


def to_device(raw: np.ndarray, dtype: str) -> torch.Tensor:
    """raw as produced by synth.store -> device tensor of the matching torch dtype."""
    if dtype == synth.BF16:
        return torch.from_numpy(raw.view(np.int16).copy()).cuda().view(torch.bfloat16)
    return torch.from_numpy(raw.copy()).cuda()


def codes_to_host(codes: torch.Tensor) -> np.ndarray:
    return codes.cpu().numpy().view(np.uint32)


def half_to_host(t: torch.Tensor) -> np.ndarray:
    return t.cpu().numpy().view(np.float16) if t.dtype == torch.float16 else t.cpu().numpy()


def out_to_f64(t: torch.Tensor) -> np.ndarray:
    return t.float().cpu().numpy().astype(np.float64)


def round_to(x64: np.ndarray, torch_dtype) -> np.ndarray:
    """float64 -> value of the nearest representable number of the output dtype."""
    if torch_dtype == torch.float32:
        return x64.astype(np.float32).astype(np.float64)
    if torch_dtype == torch.float16:
        return x64.astype(np.float16).astype(np.float64)
    # bf16: round float64 -> float32 exactly representable first would double-round; go through
    # integer arithmetic on the float64 value instead
    m, e = np.frexp(x64)                       # x = m * 2^e, 0.5 <= |m| < 1
    q = np.rint(m * 256.0) / 256.0             # 8 significant bits, ties to even
    return np.ldexp(q, e)
