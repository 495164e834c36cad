"""The entry point that allocates nothing (dcnn_mask_compact_static) against dcnn_mask_compact: same masks,
lists and counts, bit for bit, on two calls in a row of which the second is smaller (the library's static
scratch keeps the first call's contents), through the C ABI."""
import numpy as np
import pytest
import torch

import paper_2203_03996_amd as pkg
from oracle import deltacnn_oracle as orc
from tests.helpers import to_np

pytestmark = pytest.mark.gpu


def _both(ctx, plain, m, k, stride, pad, mb=None, want_mask=True):
    n, h, w = m.shape
    oh, ow = (h + 2 * pad - k) // stride + 1, (w + 2 * pad - k) // stride + 1
    md = torch.from_numpy(m).cuda()
    mbd = None if mb is None else torch.from_numpy(mb).cuda()
    ref_mask, ref_idx, ref_cnt = plain.mask_compact(md, k, stride, pad, mask_b=mbd)
    plain.sync()
    # the caller's buffers, poisoned so that stale contents would show
    mask_out = torch.full((n, oh, ow), 7, dtype=torch.uint8, device="cuda") if want_mask else None
    idx = torch.full((n * oh * ow,), -5, dtype=torch.int32, device="cuda")
    cnt = torch.full((1,), -9, dtype=torch.int32, device="cuda")
    ctx.mask_compact_static(md, mask_out, idx, cnt, k, stride, pad, mask_b=mbd)
    ctx.sync()
    c = int(to_np(cnt)[0])
    assert c == int(to_np(ref_cnt)[0])
    assert np.array_equal(to_np(idx)[:c], to_np(ref_idx)[:c])
    if want_mask:
        assert np.array_equal(to_np(mask_out), to_np(ref_mask))
    # and both are the oracle's window dilation + ordered compaction
    want = orc.window_mask(m, k, stride, pad)
    if mb is not None:
        want = want | mb
    assert np.array_equal(to_np(ref_mask), want) and np.array_equal(to_np(idx)[:c], orc.compact(want)[0])
    return c


def test_static_scratch_variant_matches_the_workspace_variant_on_two_calls_in_a_row():
    rng = np.random.default_rng(12)
    ctx = pkg.Context(0)                                   # no workspace at all
    plain = pkg.Context(64 * 128 * 128)
    big = (rng.random((64, 128, 128)) < 0.1).astype(np.uint8)      # 1 Mi pixels, 512 chunks
    c1 = _both(ctx, plain, big, 3, 1, 1)
    small = (rng.random((3, 37, 53)) < 0.3).astype(np.uint8)       # three chunks, ragged tail, after the big call
    c2 = _both(ctx, plain, small, 3, 1, 1)
    assert c1 > c2 > 0
    # list only (the output mask goes to the static scratch), a union with a second mask, strided windows, one chunk
    _both(ctx, plain, big[:5], 3, 2, 1, want_mask=False)
    mb = (rng.random((3, 37, 53)) < 0.05).astype(np.uint8)
    _both(ctx, plain, small, 1, 1, 0, mb=mb)
    _both(ctx, plain, small[:1, :7, :5], 3, 1, 1)
    _both(ctx, plain, np.zeros((2, 40, 40), np.uint8), 3, 1, 1)
    _both(ctx, plain, big, 7, 2, 3)


def test_static_scratch_variant_rejects_maps_beyond_its_limit_without_launching():
    ctx = pkg.Context(0)
    n, h, w = 65, 256, 256                                 # 65 * 65536 > 4 Mi output pixels
    m = torch.zeros((n, h, w), dtype=torch.uint8, device="cuda")
    idx = torch.full((16,), -5, dtype=torch.int32, device="cuda")   # far too small: nothing may be written
    cnt = torch.full((1,), -9, dtype=torch.int32, device="cuda")
    with pytest.raises(pkg.DcnnError) as e:
        ctx.mask_compact_static(m, None, idx, cnt, 1, 1, 0)
    assert e.value.status == 5 and "static scratch" in str(e.value)
    ctx.sync()
    assert int(to_np(cnt)[0]) == -9 and np.all(to_np(idx) == -5)
    with pytest.raises(pkg.DcnnError):                     # the workspace variant refuses a context without workspace
        ctx.mask_compact(m[:1], 1, 1, 0)
    with pytest.raises(pkg.DcnnError):
        ctx.mask_compact_static(m[:1], None, None, cnt, 1, 1, 0)
