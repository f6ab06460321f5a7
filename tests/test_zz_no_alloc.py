"""The scan entry point that allocates nothing (its status words live in an array of the
library's code object) against the entry point that takes a workspace: same kernels, so the
results must be bit-identical; two calls in a row share the array, the second one smaller."""
import numpy as np
import pytest
import torch

import paper_2511_11939_amd as P
from oracle import inclusive_scan_u32_ref
from workloads import scan_input_u32

pytestmark = pytest.mark.gpu
TILE = 16384


def _with_workspace(x_dev, n):
    s, nbytes = P.prism_scan_workspace_size(n)
    assert s == 0
    ws = torch.empty(max(nbytes, 8), dtype=torch.uint8, device="cuda")
    out = torch.full((n,), -1, dtype=torch.int32, device="cuda")
    P.scan_u32(x_dev, out, n, ws)
    assert P.prism_scan_check(ws, torch.cuda.current_stream().cuda_stream) == 0
    return out


def _static(x_dev, n, flag):
    out = torch.full((n,), -1, dtype=torch.int32, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    assert P.prism_scan_u32_static(x_dev, out, n, flag, stream) == 0
    return out


def test_static_scratch_matches_the_workspace_entry_point_twice_in_a_row():
    flag = torch.full((1,), 7, dtype=torch.int32, device="cuda")
    sizes = [37 * TILE + 4321, 5 * TILE + 17]          # the second call is the smaller one
    outs = []
    xs = []
    for i, n in enumerate(sizes):
        x = scan_input_u32(900 + i, n)
        x_dev = torch.from_numpy(x.view(np.int32)).cuda()
        xs.append((x, x_dev))
    # both static calls back to back on one stream, nothing in between
    for (x, x_dev), n in zip(xs, sizes):
        outs.append(_static(x_dev, n, flag))
    torch.cuda.synchronize()
    assert int(flag.item()) == 0                        # cleared by the call, never set
    for (x, x_dev), n, got in zip(xs, sizes, outs):
        want = _with_workspace(x_dev, n)
        assert torch.equal(got, want)
        assert (got.cpu().numpy().view(np.uint32) == inclusive_scan_u32_ref(x)).all()


def test_static_scratch_limits_and_arguments():
    S = P.Status
    x = torch.zeros(16, dtype=torch.int32, device="cuda")
    assert P.prism_scan_u32_static(x, x, (1 << 30) + 1, None, None) == S.WORKSPACE   # beyond the built-in scratch
    assert P.prism_scan_u32_static(x, x, -1, None, None) == S.INVALID_ARG
    assert P.prism_scan_u32_static(None, x, 4, None, None) == S.INVALID_ARG
    assert P.prism_scan_u32_static(x, x, 0, None, None) == S.OK
    assert P.prism_scan_u32_static(x.data_ptr(), x.data_ptr() + 8, 8, None, None) == S.INVALID_ARG  # partial overlap
    # in place, no flag
    y = torch.ones(1000, dtype=torch.int32, device="cuda")
    assert P.prism_scan_u32_static(y, y, 1000, None, torch.cuda.current_stream().cuda_stream) == S.OK
    torch.cuda.synchronize()
    assert (y.cpu().numpy() == np.arange(1, 1001)).all()
