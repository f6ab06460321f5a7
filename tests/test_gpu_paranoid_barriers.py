"""Race check: the library built with a workgroup barrier after every LDS phase of its main
loops (PRISM_PARANOID_BARRIERS) must give the same bits as the normal build, whose hand-placed
waits and single barrier per K step are meant to be sufficient."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2511_11939_amd as P
from paper_2511_11939_amd import build as _build
from workloads import to_bf16_bits, to_f16_bits

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def paranoid():
    lib = ctypes.CDLL(_build.PARANOID_LIB_PATH)
    i64, vp = ctypes.c_int64, ctypes.c_void_p
    lib.prism_gemm_batched.argtypes = [ctypes.POINTER(P.GemmDesc), i64, i64, i64, vp, i64, i64, vp, i64, i64, vp, i64, i64, i64, vp]
    lib.prism_gemm_batched.restype = ctypes.c_int
    lib.prism_reread_environment.argtypes = []
    lib.prism_reread_environment.restype = None
    return lib


CASES = [
    # M, N, K, batch, layout_b, ab, hooks
    (512, 512, 192, 1, "col", "bf16", {"PRISM_GEMM_CONFIG": "0"}),      # 256x256 tiles, odd number of K steps
    (768, 512, 64, 1, "col", "bf16", {"PRISM_GEMM_CONFIG": "0"}),       # one K step
    (4096, 4096, 512, 1, "col", "bf16", {}),                            # a full round of 256 tiles
    (384, 640, 320, 3, "col", "f16", {"PRISM_GEMM_CONFIG": "1"}),       # 128x128 tiles, two workgroups per compute unit
    (256, 384, 256, 1, "row", "bf16", {}),                              # row-major B: transposing LDS reads
    (512, 512, 512, 24, "col", "bf16", {"PRISM_PERSISTENT": "1", "PRISM_GEMM_CONFIG": "0"}),   # persistent pipe
    (300, 200, 100, 1, "col", "bf16", {}),                              # staged kernel
]


@pytest.mark.parametrize("M,N,K,batch,layout_b,ab,hooks", CASES)
def test_paranoid_build_gives_the_same_bits(paranoid, set_hook, M, N, K, batch, layout_b, ab, hooks):
    for name, value in hooks.items():
        set_hook(name, value)
    paranoid.prism_reread_environment()
    rng = np.random.default_rng(M + N + K)
    enc = to_bf16_bits if ab == "bf16" else to_f16_bits
    a = torch.from_numpy(enc(rng.standard_normal(batch * M * K).astype(np.float32)).view(np.int16)).cuda()
    b = torch.from_numpy(enc(rng.standard_normal(batch * K * N).astype(np.float32)).view(np.int16)).cuda()
    outs = []
    stream = torch.cuda.current_stream().cuda_stream
    for lib in (P.load_library(), paranoid):
        c = torch.full((batch * M * N,), float("nan"), dtype=torch.float32, device="cuda")
        d = P.make_desc(ab_dtype=ab, c_dtype="f32", layout_b=layout_b, split_k=1)
        ldb = N if layout_b == "row" else K
        s = lib.prism_gemm_batched(ctypes.byref(d), M, N, K, a.data_ptr(), K, M * K, b.data_ptr(), ldb, K * N,
                                   c.data_ptr(), N, M * N, batch, stream)
        assert s == 0
        torch.cuda.synchronize()
        outs.append(c.cpu().numpy())
    assert not np.isnan(outs[0]).any()
    assert (outs[0].view(np.uint32) == outs[1].view(np.uint32)).all()
    import os
    for name in hooks:                      # the paranoid library keeps its own copy of the hooks
        os.environ.pop(name, None)
    paranoid.prism_reread_environment()
