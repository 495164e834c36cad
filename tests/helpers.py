"""Shared helpers of the GPU parity tests."""
import numpy as np
import torch

from oracle import deltacnn_oracle as orc

NP_DTYPE = {"f32": np.float32, "f16": np.float16, "f64": np.float64}
# acceptance tolerances on values (max relative error, see rel_err)
TOL = {"f32": 1e-4, "f16": 2e-2}
# denominator floor of rel_err, as a fraction of the reference tensor's largest magnitude
FLOOR = 1e-3
# unit round-off of the fp32 accumulators both element types are summed in
U32 = 2.0 ** -24


def ulp(x, S: str) -> np.ndarray:
    """Spacing of storage type S at |x| (NaN counts as 0), in float64."""
    v = np.abs(np.nan_to_num(np.asarray(x, np.float64), nan=0.0, posinf=0.0, neginf=0.0)).astype(NP_DTYPE[S])
    return np.spacing(v).astype(np.float64)


def rel_err(got, ref, floor: float = FLOOR, slack=None) -> float:
    """max over elements of max(|got - ref| - slack, 0) / max(|ref|, floor * max|ref|).

    The floor (1e-3 of the tensor's largest magnitude) only keeps the quotient finite for
    elements that are zero; it is NOT widened to absorb rounding.  What the arithmetic
    cannot decide is stated per element instead, as `slack` (absolute, same shape as ref):
    * a K-term sum accumulated in fp32 carries an absolute error proportional to the sum
      of the magnitudes of its terms whatever its own value, so an element that cancels has
      no bounded error relative to itself: see sum_slack;
    * when a convolution sum is rounded to the storage type and then enters a second
      operation (activation on accumulated state, residual add, projection add), the two
      sides may round the intermediate to neighbouring values; the result inherits that one
      unit in the last place of the INTERMEDIATE, which can be large relative to a result
      that cancels: see the callers, which pass ulp(intermediate)."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    if ref.size == 0:
        return 0.0
    scale = np.abs(ref).max()
    err = np.abs(got - ref)
    if slack is not None:
        err = np.maximum(err - np.asarray(slack, np.float64), 0.0)
    if scale == 0:
        return float(err.max())
    den = np.maximum(np.abs(ref), floor * scale)
    return float((err / den).max())


def worst(got, ref, floor: float = FLOOR, slack=None) -> str:
    """Where rel_err takes its maximum, for assertion messages."""
    got = np.asarray(got, np.float64).reshape(-1)
    ref = np.asarray(ref, np.float64).reshape(-1)
    if ref.size == 0:
        return "empty"
    sl = np.zeros_like(ref) if slack is None else np.broadcast_to(np.asarray(slack, np.float64), np.shape(slack) if np.ndim(slack) else ref.shape).reshape(-1)
    scale = np.abs(ref).max()
    q = np.maximum(np.abs(got - ref) - sl, 0.0) / np.maximum(np.abs(ref), floor * max(scale, 1e-300))
    i = int(np.argmax(q))
    return f"worst element {i}: got {got[i]!r} ref {ref[i]!r} slack {sl[i]:.3e} scale {scale:.3e}"


def sum_slack(conv: "orc.Conv", x_zero_filled: np.ndarray, bias: bool = False) -> np.ndarray:
    """Absolute error allowance of a convolution sum accumulated in fp32 (any order) against the
    float64 sum: 8 u * sum_k |w_k| |x_k| with u = 2^-24.  The worst case of a K-term recursive sum
    is K u sum|terms| (K = 288 ... 4608 here).  Measured on the CPU against the float64 oracle: a
    stock fp32 library convolution needs up to 7.3 u sum|terms| (3x3x64), an emulation of the matrix
    cores' schedule (16 exact products added per step into an fp32 accumulator) 1.2 u."""
    a = orc.conv_dense(np.abs(np.asarray(x_zero_filled, np.float64)), np.abs(conv.w.astype(np.float64)),
                       conv.stride, conv.pad, conv.dw)
    if bias and conv.b is not None:
        a = a + np.abs(conv.b.astype(np.float64))
    return 8.0 * U32 * a


def to_np(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().numpy()


def poison(shape, dtype, device="cuda"):
    """A device buffer full of NaN: whatever the library reads from unflagged pixels shows up."""
    return torch.full(shape, float("nan"), dtype=dtype, device=device)


def upload_delta(data: np.ndarray, mask: np.ndarray, device="cuda"):
    """A test input as device tensors: data, mask, and the index list / count a producing layer would
    have left with it (the ascending flagged pixel indices) -- built on the host because this
    input has no producing layer."""
    import paper_2203_03996_amd as pkg
    flat = np.flatnonzero(mask.reshape(-1)).astype(np.int32)
    idx = np.zeros(mask.size, np.int32)
    idx[:flat.size] = flat
    return pkg.Delta(torch.from_numpy(np.ascontiguousarray(data)).to(device),
                     torch.from_numpy(np.ascontiguousarray(mask.astype(np.uint8))).to(device),
                     torch.from_numpy(idx).to(device),
                     torch.tensor([flat.size], dtype=torch.int32, device=device))


def check_delta(out, ref, S, what, exact_values=False, allow_mask_diff=None, slack=None, floor=FLOOR):
    """Compare a library Delta (torch views) with an oracle Delta.
    Returns the number of tolerated mask mismatches (threshold ties)."""
    g_mask = to_np(out.mask)
    r_mask = ref.mask
    diff = g_mask != r_mask
    n_diff = int(diff.sum())
    if n_diff:
        assert allow_mask_diff is not None, f"{what}: {n_diff} mask mismatches"
        assert np.all(allow_mask_diff[diff]), f"{what}: mask mismatch away from a threshold tie"
    if out.count is not None and out.idx is not None:
        cnt = int(to_np(out.count)[0])
        idx = to_np(out.idx)[:cnt]
        assert cnt == int(g_mask.sum()), f"{what}: count {cnt} vs mask {int(g_mask.sum())}"
        assert np.array_equal(idx, np.flatnonzero(g_mask.reshape(-1))), f"{what}: index list is not the ordered compaction"
        if n_diff == 0:
            assert np.array_equal(idx, ref.idx), f"{what}: index list differs from the oracle"
    both = (g_mask == 1) & (r_mask == 1)
    g = to_np(out.data)[both]
    r = ref.data[both]
    assert not np.isnan(g.astype(np.float64)).any(), f"{what}: NaN in a flagged output (an unflagged value was read)"
    if exact_values:
        assert np.array_equal(g, r), f"{what}: values differ (max abs {np.abs(g.astype(np.float64) - r).max()})"
    else:
        e = rel_err(g, r, floor, None if slack is None else np.broadcast_to(slack, ref.data.shape)[both])
        assert e <= TOL[S], f"{what}: max relative error {e:.3e} > {TOL[S]}"
    return n_diff
