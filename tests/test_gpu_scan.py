"""GPU parity of the single-pass prefix scan (through the C ABI) against the CPU oracle:
bit-exact, every element."""
import numpy as np
import pytest
import torch

import paper_2511_11939_amd as P
from oracle import inclusive_scan_u32_ref
from workloads import scan_input_u32

pytestmark = pytest.mark.gpu
TILE = 16384


def _ws(n):
    s, nbytes = P.prism_scan_workspace_size(n)
    assert s == 0
    return torch.empty(max(nbytes, 8), dtype=torch.uint8, device="cuda")


def _run(x: np.ndarray, *, in_place=False, offset=0, ws=None):
    """x: uint32 host array.  offset: leading elements skipped on the device buffers, which
    makes the pointers 4- but not 16-byte aligned."""
    n = x.size
    buf = torch.zeros(n + offset + 8, dtype=torch.int32, device="cuda")
    buf[offset:offset + n] = torch.from_numpy(x.view(np.int32)).cuda()
    out = buf if in_place else torch.full((n + offset + 8,), -1, dtype=torch.int32, device="cuda")
    ws = _ws(n) if ws is None else ws
    P.scan_u32(buf.data_ptr() + 4 * offset, out.data_ptr() + 4 * offset, n, ws)
    assert P.prism_scan_check(ws, torch.cuda.current_stream().cuda_stream) == 0
    got = out.cpu().numpy().view(np.uint32)
    if not in_place:
        assert (got[:offset] == 0xFFFFFFFF).all() and (got[offset + n:] == 0xFFFFFFFF).all()   # nothing else written
    return got[offset:offset + n]


@pytest.mark.parametrize("n", [1, 2, 63, 64, 65, 255, 1023, 1024, 1025, TILE - 1, TILE, TILE + 1,
                               3 * TILE + 777, 64 * TILE, 65 * TILE + 5, 1_000_003])
def test_sizes_around_lane_wave_chunk_and_tile_edges(n):
    x = scan_input_u32(n, n)
    assert (_run(x) == inclusive_scan_u32_ref(x)).all()


@pytest.mark.parametrize("offset,in_place", [(0, True), (1, False), (3, True), (2, False)])
def test_in_place_and_unaligned_pointers(offset, in_place):
    n = 9 * TILE + 123
    x = scan_input_u32(77, n)
    assert (_run(x, in_place=in_place, offset=offset) == inclusive_scan_u32_ref(x)).all()


def test_closed_forms_and_wraparound():
    n = 300 * TILE + 1
    assert (_run(np.ones(n, np.uint32)) == np.arange(1, n + 1, dtype=np.uint32)).all()
    got = _run(np.full(n, 0xFFFFFFFF, np.uint32))
    assert (got == (0 - np.arange(1, n + 1, dtype=np.uint64)).astype(np.uint32)).all()


def test_many_tiles_long_look_back_chain_and_workspace_reuse():
    """2^24 elements = 1024 tiles (windows of 64 predecessors are walked many times); the same
    workspace serves three calls in a row, with a shorter problem in between."""
    n = 1 << 24
    ws = _ws(n)
    x = scan_input_u32(5, n)
    want = inclusive_scan_u32_ref(x)
    assert (_run(x, ws=ws) == want).all()
    small = scan_input_u32(6, 10 * TILE + 9)
    assert (_run(small, ws=ws) == inclusive_scan_u32_ref(small)).all()
    assert (_run(x, ws=ws, in_place=True) == want).all()


def test_benchmark_size_every_element():
    n = 1 << 28
    x = scan_input_u32(0x5EED0007, n)
    d_in = torch.from_numpy(x.view(np.int32)).cuda()
    d_out = torch.empty_like(d_in)
    ws = _ws(n)
    P.scan_u32(d_in, d_out, n, ws)
    assert P.prism_scan_check(ws, torch.cuda.current_stream().cuda_stream) == 0
    got = d_out.cpu().numpy().view(np.uint32)
    assert (got == inclusive_scan_u32_ref(x)).all()


def test_empty_input_and_error_codes():
    P.scan_u32(None, None, 0, None)
    x = torch.zeros(100, dtype=torch.int32, device="cuda")
    with pytest.raises(P.PrismError):
        P.scan_u32(x, x, 100, None)                       # no workspace


def test_bounded_wait_gives_up_cleanly(set_hook):
    """With a poll budget of zero a look-back that meets an unpublished tile gives up: the
    kernel still terminates, and either the result is right (nobody had to wait) or the
    error word says so."""
    set_hook("PRISM_SCAN_SPIN_LIMIT", "0")
    n = 1500 * TILE
    x = scan_input_u32(11, n)
    d = torch.from_numpy(x.view(np.int32)).cuda()
    out = torch.empty_like(d)
    ws = _ws(n)
    P.scan_u32(d, out, n, ws)
    status = P.prism_scan_check(ws, torch.cuda.current_stream().cuda_stream)
    ok = bool((out.cpu().numpy().view(np.uint32) == inclusive_scan_u32_ref(x)).all())
    assert status in (0, int(P.Status.LAUNCH))
    assert ok or status == int(P.Status.LAUNCH)


def test_seeded_sweep_of_sizes_offsets_and_modes():
    rng = np.random.default_rng(99)
    for i in range(25):
        n = int(rng.integers(1, 6 * TILE))
        offset = int(rng.integers(0, 4))
        x = scan_input_u32(1000 + i, n)
        got = _run(x, in_place=bool(rng.integers(0, 2)), offset=offset)
        assert (got == inclusive_scan_u32_ref(x)).all(), (n, offset)
