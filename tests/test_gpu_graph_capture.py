"""The library allocates nothing, never synchronises and clears its scratch with kernels, so
its calls can be recorded into a HIP graph.  Each graph is replayed several times with eager
work and synchronisations in between, and every replay is compared with the eager result."""
import numpy as np
import pytest
import torch

import paper_2511_11939_amd as P
from oracle import inclusive_scan_u32_ref
from workloads import scan_input_u32, to_bf16_bits

pytestmark = pytest.mark.gpu


def test_gemm_with_split_k_and_scan_replay_from_a_graph():
    rng = np.random.default_rng(0)
    M, N, K = 256, 512, 2048
    a = to_bf16_bits(rng.standard_normal(M * K).astype(np.float32))
    b = to_bf16_bits(rng.standard_normal(N * K).astype(np.float32))
    A = torch.from_numpy(a.view(np.int16)).cuda()
    B = torch.from_numpy(b.view(np.int16)).cuda()
    C = torch.zeros(M * N, dtype=torch.float32, device="cuda")
    desc = P.make_desc(c_dtype="f32", split_k=4)
    _, ws_bytes = P.prism_gemm_workspace_size(desc, M, N, K, 1)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    desc.workspace, desc.workspace_bytes = ws.data_ptr(), ws_bytes

    n = 40 * 16384 + 77
    x = scan_input_u32(21, n)
    d_in = torch.from_numpy(x.view(np.int32)).cuda()
    d_out = torch.zeros_like(d_in)
    _, sws_bytes = P.prism_scan_workspace_size(n)
    sws = torch.empty(sws_bytes, dtype=torch.uint8, device="cuda")

    # eager results first
    P.gemm(A, B, C, M=M, N=N, K=K, desc=desc)
    P.scan_u32(d_in, d_out, n, sws)
    torch.cuda.synchronize()
    c_eager = C.clone()
    assert (d_out.cpu().numpy().view(np.uint32) == inclusive_scan_u32_ref(x)).all()

    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            P.gemm(A, B, C, M=M, N=N, K=K, desc=desc, stream=side)
            P.scan_u32(d_in, d_out, n, sws, stream=side)
    for replay in range(4):
        C.fill_(-1.0)                      # eager work between the replays
        d_out.zero_()
        ws.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(C, c_eager), f"replay {replay}: gemm differs from the eager run"
        assert (d_out.cpu().numpy().view(np.uint32) == inclusive_scan_u32_ref(x)).all(), f"replay {replay}: scan"
        assert P.prism_scan_check(sws, torch.cuda.current_stream().cuda_stream) == 0
