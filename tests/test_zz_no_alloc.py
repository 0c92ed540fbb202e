"""The entry point that allocates nothing (w2_matmul_a8_fused_noalloc: the scratch memory is an array built
into the library) against w2_matmul_a8_fused with a caller's workspace of the same size, through the C ABI:
bit-equal outputs on calls in a row, the later ones with smaller inputs, and the size limit."""
import ctypes

import numpy as np
import pytest

from paper_2508_06753_amd import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def w2():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2508_06753_amd import binding
    return binding


def dev(a):
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def test_no_alloc_entry_matches_workspace_entry(w2):
    lib = w2.raw()
    p = lambda t: ctypes.c_void_p(t.data_ptr())
    s = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    K, N, G = 2048, 528, 128
    codes, scales = synth.make_weights(K, N, G, 0, seed=5)
    packed = w2.prepack(dev(codes), dev(scales), G, 0)
    ws = torch.empty(w2.NOALLOC_SCRATCH_BYTES, dtype=torch.uint8, device="cuda")
    assert lib.w2_init() == 0
    # large first (quantise launch + tiled kernel with K split across workgroups out of the scratch), then
    # smaller ones that reuse the buffer's head (mid-M and small-M kernels), then one row (no scratch used)
    for M, dt in ((200, torch.float32), (40, torch.bfloat16), (5, torch.float32), (1, torch.float32), (130, torch.bfloat16)):
        X = dev(synth.make_activations(M, K, seed=100 + M)).to(dt)
        y_ref = torch.full((M, N), 0x7FC1, dtype=torch.int16, device="cuda")      # a NaN pattern no result has
        y_new = torch.full((M, N), 0x7FC2, dtype=torch.int16, device="cuda")
        x_dt = w2.DT_F32 if dt == torch.float32 else w2.DT_BF16
        rc = lib.w2_matmul_a8_fused(p(packed), K, N, G, p(X), x_dt, K, M, p(y_ref), N, p(ws), ws.numel(), s)
        assert rc == 0, lib.w2_last_error()
        rc = lib.w2_matmul_a8_fused_noalloc(p(packed), K, N, G, p(X), x_dt, K, M, p(y_new), N, s)
        assert rc == 0, lib.w2_last_error()
        torch.cuda.synchronize()
        assert torch.equal(y_ref, y_new), f"M={M}: outputs differ"
        assert not torch.any(y_new == 0x7FC2), f"M={M}: outputs left unwritten"


def test_no_alloc_entry_rejects_what_does_not_fit(w2):
    lib = w2.raw()
    p = lambda t: ctypes.c_void_p(t.data_ptr())
    s = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    K, N, G = 8192, 64, 128
    codes, scales = synth.make_weights(K, N, G, 0, seed=6)
    packed = w2.prepack(dev(codes), dev(scales), G, 0)
    M = w2.NOALLOC_SCRATCH_BYTES // K                       # M*K fills the buffer: no room for the scales
    X = torch.zeros((M, K), dtype=torch.bfloat16, device="cuda")
    Y = torch.full((M, N), 7.0, dtype=torch.bfloat16, device="cuda")
    rc = lib.w2_matmul_a8_fused_noalloc(p(packed), K, N, G, p(X), w2.DT_BF16, K, M, p(Y), N, s)
    assert rc == w2.ERR_BUFFER_TOO_SMALL
    assert b"scratch" in lib.w2_last_error()
    torch.cuda.synchronize()
    assert torch.all(Y == 7.0)
    # two rows fewer leave room for the scales (4 bytes a row)
    rc = lib.w2_matmul_a8_fused_noalloc(p(packed), K, N, G, p(X), w2.DT_BF16, K, M - 2, p(Y), N, s)
    assert rc == 0, lib.w2_last_error()
    torch.cuda.synchronize()
    assert torch.all(Y[: M - 2] == 0.0) and torch.all(Y[M - 2:] == 7.0)
