"""The replay entry point that allocates nothing (for callers that cannot allocate or bring a workspace): its
output against replay_reduction's, bit for bit, on two calls in a row, the second with a smaller input; sizes
beyond the library's fixed scratch array are refused."""
from __future__ import annotations

import numpy as np
import pytest

import oracle as O
import prs_inputs

pytestmark = pytest.mark.gpu


def _case(prs, p, sizes, per, dtype):
    import torch
    q = len(sizes)
    s = O.uni_greedy(p, sizes, 3, 1, 1)
    seg_off = np.arange(q + 1, dtype=np.int64) * per
    seg_off[-1] -= per // 3                                             # ragged last segment
    n = int(seg_off[-1])
    buf = torch.from_numpy(prs_inputs.replay_buffers(p, n, dtype)).cuda()
    src, dst, seg = (torch.from_numpy(a).cuda() for a in (s.src, s.dst, s.seg))
    want, st0 = prs.replay_reduction(p, q, seg_off, src, dst, seg, buf)
    out = torch.full((n,), 7, dtype=buf.dtype, device="cuda")
    status = torch.full((1,), -5, dtype=torch.int32, device="cuda")
    prs.replay_reduction_static(p, q, seg_off, src, dst, seg, buf, out, status)
    torch.cuda.synchronize()
    assert int(st0.item()) == 0 and int(status.item()) == 0
    assert out.cpu().numpy().tobytes() == want.cpu().numpy().tobytes(), (p, q, dtype)
    assert out.cpu().numpy().tobytes() == O.replay(p, seg_off, s.src, s.dst, s.seg, buf.cpu().numpy()).tobytes()


def test_replay_without_allocation_matches_replay_with_a_workspace():
    import torch
    import paper_1310_4645_amd as prs
    assert torch.cuda.is_available()
    prs.load_library()
    _case(prs, 200, [5] * 12, 4096, "f32")          # first call on this GPU takes hold of the scratch array
    _case(prs, 37, [4] * 3, 1000, "f32")            # smaller: the array still holds the larger call's programs
    _case(prs, 37, [4] * 3, 1000, "i32")
    _case(prs, 2000, [2] * 5, 512, "f64")           # more than 1536 processors: the builder's arrays come from the scratch too
    # too many processors x segments for the fixed array: refused, nothing enqueued
    p, q = 4096, 600
    one = torch.zeros(8, dtype=torch.int32, device="cuda")
    off = np.zeros(q + 1, np.int64)
    rc = prs.load_library().replay_reduction_static(p, q, off.ctypes.data, one.data_ptr(), one.data_ptr(), one.data_ptr(),
                                                    (p - 1) * q, one.data_ptr(), 0, 0, prs.PRS_I32, one.data_ptr(),
                                                    one.data_ptr(), None)
    assert rc == 2                                   # PRS_ENOSPC
