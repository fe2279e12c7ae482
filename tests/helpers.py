"""Host<->device plumbing shared by the GPU tests (no method arithmetic)."""
import numpy as np

from paper_2302_06058_amd import synth


def to_dev(a: np.ndarray, dtype: str):
    """Stored host array (uint16 bf16 bits / float32) -> device tensor."""
    import torch
    if dtype == synth.BF16:
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def i32_dev(a: np.ndarray):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


def words(t) -> np.ndarray:
    """Device int32 bit-word tensor -> host uint32 array."""
    return t.cpu().numpy().view(np.uint32)


def from_dev_f64(t, dtype: str) -> np.ndarray:
    """Device tensor -> exact float64 values on the host."""
    import torch
    if dtype == synth.BF16:
        bits = t.view(torch.int16).cpu().numpy().view(np.uint16)
        return synth.to_f64(bits, synth.BF16)
    return t.cpu().numpy().astype(np.float64)


def raw_bits(t, dtype: str) -> np.ndarray:
    """Device tensor -> the stored bit patterns (uint16 / uint32)."""
    import torch
    if dtype == synth.BF16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.view(torch.int32).cpu().numpy().view(np.uint32)


def f64_to_raw(v: np.ndarray, dtype: str) -> np.ndarray:
    """Exactly representable float64 values -> stored bit patterns."""
    v32 = v.astype(np.float32)
    assert (v32.astype(np.float64) == v).all()
    if dtype == synth.BF16:
        u = v32.view(np.uint32)
        assert ((u & 0xFFFF) == 0).all()
        return (u >> 16).astype(np.uint16)
    return v32.view(np.uint32)


def rel_err(got: np.ndarray, want: np.ndarray) -> float:
    """max|got - want| / max|want| (infinity-norm relative error)."""
    denom = float(np.max(np.abs(want)))
    return float(np.max(np.abs(got - want))) / (denom if denom > 0 else 1.0)
