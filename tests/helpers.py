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


def untile24(values: np.ndarray, index: np.ndarray, rows: int, cols: int):
    """Fragment-major 2:4 operand buffers (layout stated in include/bimask.h) -> row-major
    slot values [rows, cols/2] and index words [rows, ceil(cols/32)], plus a flag telling
    whether all padding (rows >= rows, cols >= cols) is zero.  Pure index permutation."""
    Rp, Cp = -(-rows // 32) * 32, -(-cols // 128) * 128
    ks = Cp // 128
    v = values.reshape(Rp // 32, ks, 4, 2, 32, 8)          # [rt][st][s4][h][r%32][e]
    v = v.transpose(0, 4, 1, 3, 2, 5).reshape(Rp, Cp // 2)  # slot = st*64 + h*32 + s4*8 + e
    x = index.reshape(Rp // 32, ks, 2, 32, 2)              # [rt][st][h][r%32][w]
    x = x.transpose(0, 3, 1, 2, 4).reshape(Rp, Cp // 32)    # word = st*4 + h*2 + w
    pad_zero = bool((v[rows:] == 0).all() and (v[:, cols // 2:] == 0).all()
                    and (x[rows:] == 0).all())
    wv = -(-cols // 32)
    tail_bits = cols % 32
    xr = x[:rows, :wv].copy()
    if tail_bits:
        pad_zero = pad_zero and bool(((xr[:, -1] >> np.uint32(tail_bits)) == 0).all())
    pad_zero = pad_zero and bool((x[:rows, wv:] == 0).all())
    return v[:rows, :cols // 2], xr, pad_zero


def untile_dense(values: np.ndarray, rows: int, cols: int):
    """Fragment-major DENSE operand buffer (ratios with N > 2; layout stated in include/bimask.h) -> row-major
    [rows, cols] entries, plus a flag telling whether all padding (rows >= rows, cols >= cols) is zero.
    Pure index permutation."""
    Rp, Cp = -(-rows // 32) * 32, -(-cols // 128) * 128
    ks = Cp // 128
    v = values.reshape(Rp // 32, ks, 4, 2, 2, 32, 8)        # [rt][st][s4][x][hs][r%32][e]
    v = v.transpose(0, 5, 1, 3, 2, 4, 6).reshape(Rp, Cp)     # k = st*128 + x*64 + s4*16 + hs*8 + e
    pad_zero = bool((v[rows:] == 0).all() and (v[:, cols:] == 0).all())
    return v[:rows, :cols], pad_zero


class GemmError:
    """Running comparison of a GEMM output with its float64 reference, fed chunk by chunk.

    rel      max|got - ref| / max|ref| over everything seen (the stated tolerance is on this figure)
    excess   max over the elements of |got - ref| / bound, with the element's own rounding budget
                 bound = 2^-8 |ref| + 8 sqrt(K) 2^-24 S + tiny,   S = sum_k |a_k| |b_k|
             (bf16 keeps 8 significant bits, so rounding to nearest errs by at most half a unit in the
             last place = 2^-8 |value|: the first term has no slack, a truncating conversion would show
             as excess 2; fp32 accumulation of K terms errs by about sqrt(K) 2^-24 S, allowed 8 times
             that).  A single dropped or misplaced product is about S / K and shows as excess > 1 for
             the lengths used here; for fp32 outputs (24 significant bits) the first term is 2^-23 |ref|.
    """

    def __init__(self, K: int, out_bits: int = 8):
        self.K, self.out_bits = K, out_bits
        self.max_err = self.max_ref = self.excess = 0.0
        self.n = 0

    def add(self, got: np.ndarray, ref: np.ndarray, S: np.ndarray):
        err = np.abs(got - ref)
        self.max_err = max(self.max_err, float(err.max()))
        self.max_ref = max(self.max_ref, float(np.abs(ref).max()))
        bound = np.abs(ref) * 2.0 ** -self.out_bits + S * (8.0 * np.sqrt(self.K) * 2.0 ** -24) + 1e-300
        self.excess = max(self.excess, float((err / bound).max()))
        self.n += got.size

    @property
    def rel(self) -> float:
        return self.max_err / (self.max_ref if self.max_ref > 0 else 1.0)

    def __repr__(self):
        return f"rel {self.rel:.2e} excess {self.excess:.2f} over {self.n} outputs"
