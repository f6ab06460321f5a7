"""The lane layouts the kernels are built on, shown on the device through the library's own
device functions (prism_layout_probe): the accumulator layout of the 16x16x32 matrix
instruction (lane::acc_row / lane::acc_col) and the transposing LDS read that serves operands
kept as k-rows.  One-hot inputs locate single entries; integer matrices check all at once."""
import numpy as np
import pytest
import torch

import paper_2511_11939_amd as P
from workloads import to_bf16_bits, to_f16_bits

pytestmark = pytest.mark.gpu


def _dev16(x, enc):
    return torch.from_numpy(enc(np.asarray(x, dtype=np.float32).ravel()).view(np.int16)).cuda()


def _product(r, c, what, enc):
    out = torch.full((16 * 16,), -1.0, dtype=torch.float32, device="cuda")
    assert P.prism_layout_probe(what, _dev16(r, enc), _dev16(c, enc), out, torch.cuda.current_stream().cuda_stream) == 0
    torch.cuda.synchronize()
    return out.cpu().numpy().reshape(16, 16)


@pytest.mark.parametrize("what,enc", [(P.LAYOUT_ACCUMULATOR_BF16, to_bf16_bits), (P.LAYOUT_ACCUMULATOR_F16, to_f16_bits)])
def test_accumulator_layout_one_hot_and_integers(what, enc):
    # one-hot: R has a single 1 at (i, k), C a single 1 at (j, k): the product has a single 1 at (i, j)
    for (i, j, k) in [(0, 0, 0), (3, 9, 5), (15, 0, 31), (7, 7, 16), (12, 5, 8), (1, 14, 23)]:
        r = np.zeros((16, 32), np.float32); c = np.zeros((16, 32), np.float32)
        r[i, k] = 1.0; c[j, k] = 1.0
        d = _product(r, c, what, enc)
        want = np.zeros((16, 16), np.float32); want[i, j] = 1.0
        assert (d == want).all(), (i, j, k)
        c[j, k] = 0.0; c[j, (k + 1) % 32] = 1.0            # different k in the two operands: nothing meets
        assert (_product(r, c, what, enc) == 0.0).all()
    rng = np.random.default_rng(11)
    r = rng.integers(-8, 9, size=(16, 32)).astype(np.float32)
    c = rng.integers(-8, 9, size=(16, 32)).astype(np.float32)
    assert (_product(r, c, what, enc) == r @ c.T).all()


def test_transposing_read_of_k_rows():
    x = np.arange(32 * 128, dtype=np.uint16).reshape(32, 128)      # value names its (k, element)
    for m in (x, (x * 7 + 3).astype(np.uint16)):
        src = torch.from_numpy(m.view(np.int16).copy()).cuda()
        out = torch.full((128 * 32,), -1, dtype=torch.int16, device="cuda")
        assert P.prism_layout_probe(P.LAYOUT_K_ROWS_READ, src, None, out, torch.cuda.current_stream().cuda_stream) == 0
        torch.cuda.synchronize()
        got = out.cpu().numpy().view(np.uint16).reshape(128, 32)
        assert (got == m.T).all()


def test_layout_probe_arguments():
    S = P.Status
    buf = torch.zeros(4096, dtype=torch.int16, device="cuda")
    assert P.prism_layout_probe(99, buf, buf, buf, None) == S.UNSUPPORTED
    assert P.prism_layout_probe(P.LAYOUT_ACCUMULATOR_BF16, None, buf, buf, None) == S.INVALID_ARG
    assert P.prism_layout_probe(P.LAYOUT_ACCUMULATOR_BF16, buf, None, buf, None) == S.INVALID_ARG
    assert P.prism_layout_probe(P.LAYOUT_K_ROWS_READ, buf.data_ptr() + 2, None, buf, None) == S.INVALID_ARG
