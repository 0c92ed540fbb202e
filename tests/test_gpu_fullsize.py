"""GPU parity at the full benchmark sizes, in the launch configuration the
benchmark times (AUTO dispatch).  The oracle evaluates every row on a seeded
sample of output columns plus the first and last 64 columns (tile edges);
columns are independent, so a column subset of the oracle's inputs gives the
same values as the full problem."""
import numpy as np
import pytest

import oracle
from paper_2508_06753_amd import synth
from test_gpu_parity import bf16_bits, check_y, dev

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def w2():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2508_06753_amd import binding
    return binding


def sample_cols(N, n, seed):
    rng = np.random.default_rng(seed)
    mid = rng.choice(np.arange(64, N - 64), size=n, replace=False)
    return np.unique(np.concatenate([np.arange(64), mid, np.arange(N - 64, N)]))


_weights = {}


def weights(w2, K, N, G, codec, seed):
    """Weights are the expensive part to draw; cache per shape inside the module."""
    key = (K, N, G, codec, seed)
    if key not in _weights:
        _weights.clear()                      # keep at most one large problem alive
        codes, scales = synth.make_weights(K, N, G, codec, seed=seed)
        packed = w2.prepack(dev(codes), dev(scales), G, codec)
        _weights[key] = (codes, scales, packed)
    return _weights[key]


def workspace(w2, M, K, N, G, a16=False):
    n = w2.workspace_size(M, K, N, G, a16=a16)
    return torch.empty(n, dtype=torch.uint8, device="cuda") if n else None


def check_a8(w2, M, K, N, G, codec, seed, ncols=256, acc_check=True, use_ws=False):
    codes, scales, packed = weights(w2, K, N, G, codec, seed)
    X = synth.make_activations(M, K, seed=seed + 1000 + M)
    xq, sx, _ = w2.quantize_rows(dev(X), G)
    oq, osx, _ = oracle.quantize_rows(X, G, want_gsum=False)
    assert np.array_equal(xq.cpu().numpy(), oq)
    assert np.array_equal(sx.cpu().numpy().view(np.uint32), osx.view(np.uint32))
    cols = sample_cols(N, ncols, seed)
    cs, ss = np.ascontiguousarray(codes[:, cols]), np.ascontiguousarray(scales[:, cols])
    Y = w2.matmul_a8(packed, K, N, G, xq, sx, workspace=workspace(w2, M, K, N, G) if use_ws else None)
    Yo, y64 = oracle.matmul_a8(cs, ss, G, codec, oq, osx)
    mag = oracle.a8_term_magnitude(cs, ss, G, codec, oq, osx)
    check_y(bf16_bits(Y)[:, cols], Yo, y64, mag, f"a8 full M={M} K={K} N={N} G={G}")
    if acc_check:
        # int32 group accumulators, bit-exact, on a slice of rows to bound the output size
        mr = min(M, 16)
        acc = w2.debug_group_acc_a8(packed, K, N, G, xq[:mr].contiguous())
        oacc = oracle.group_acc(cs, G, codec, oq[:mr])
        assert np.array_equal(acc.cpu().numpy()[:, :, cols], oacc)


def check_a16(w2, M, K, N, G, codec, seed, ncols=128, use_ws=False):
    codes, scales, packed = weights(w2, K, N, G, codec, seed)
    Xb = synth.f32_to_bf16_bits(synth.make_activations(M, K, seed=seed + 2000 + M))
    cols = sample_cols(N, ncols, seed)
    cs, ss = np.ascontiguousarray(codes[:, cols]), np.ascontiguousarray(scales[:, cols])
    Y = w2.matmul_a16(packed, K, N, G, dev(Xb).view(torch.bfloat16),
                      workspace=workspace(w2, M, K, N, G, a16=True) if use_ws else None)
    Yo, y64, mag = oracle.matmul_a16(cs, ss, G, codec, Xb)
    check_y(bf16_bits(Y)[:, cols], Yo, y64, mag, f"a16 full M={M} K={K} N={N} G={G}")


@pytest.mark.parametrize("name", list(synth.SHAPES_8B))
def test_8b_decode_layer(w2, name):
    """8B-class decode layer, M = 1 and 4, w2a8 and w2a16, G = 128, seed 1."""
    K, N = synth.SHAPES_8B[name]
    for M in (1, 4):
        check_a8(w2, M, K, N, 128, 0, seed=1)
        check_a16(w2, M, K, N, 128, 0, seed=1)


@pytest.mark.parametrize("name", list(synth.SHAPES_8B))
def test_8b_small_batch_a16(w2, name):
    """w2a16 at M = 5 .. 16 on the 8B-class projections: AUTO takes the decode kernel's wide form where a
    workgroup can hold the rows (K = 4096), the small-M and mid-M kernels on the down projection."""
    K, N = synth.SHAPES_8B[name]
    for M in (5, 8, 11, 16):
        check_a16(w2, M, K, N, 128, 0, seed=1, ncols=64)


@pytest.mark.parametrize("name", list(synth.SHAPES_8B))
def test_8b_decode_layer_fused_quantise(w2, name):
    """The benchmark's step at M=1: fp32 row in, one fused launch, against the oracle."""
    K, N = synth.SHAPES_8B[name]
    codes, scales, packed = weights(w2, K, N, 128, 0, 1)
    X = synth.make_activations(1, K, seed=77)
    Y = w2.matmul_a8_fused(packed, K, N, 128, dev(X))
    oq, osx, _ = oracle.quantize_rows(X, 128, want_gsum=False)
    cols = sample_cols(N, 512, 5)
    cs, ss = np.ascontiguousarray(codes[:, cols]), np.ascontiguousarray(scales[:, cols])
    Yo, y64 = oracle.matmul_a8(cs, ss, 128, 0, oq, osx)
    mag = oracle.a8_term_magnitude(cs, ss, 128, 0, oq, osx)
    check_y(bf16_bits(Y)[:, cols], Yo, y64, mag, f"a8 fused full {name}")


@pytest.mark.parametrize("G", [64, 128])
def test_small_batch_sweep_gate_up(w2, G):
    """gate+up 4096 x 28672, M in {1,2,4,8,16}, w2a8, both group sizes, seed 2."""
    K, N = synth.SHAPES_8B["gate_up"]
    for M in (1, 2, 4, 8, 16):
        check_a8(w2, M, K, N, G, 0, seed=2, ncols=128, acc_check=(M in (1, 16)))


@pytest.mark.parametrize("name", list(synth.SHAPES_27B))
def test_27b_decode_ternary(w2, name):
    """27B-class decode shapes, ternary codes (about one third zeros), M = 1 and 8, seed 3."""
    K, N = synth.SHAPES_27B[name]
    for M in (1, 8):
        check_a8(w2, M, K, N, 128, 1, seed=3, ncols=128)


def test_70b_prefill_gate_up(w2):
    """70B-class gate+up 8192 x 57344, M = 2048 (the benchmark's prefill launch) and M = 512."""
    K, N = synth.SHAPES_70B["gate_up"]
    check_a8(w2, 2048, K, N, 128, 0, seed=4, ncols=256)
    check_a8(w2, 512, K, N, 128, 0, seed=4, ncols=64, acc_check=False)


def test_70b_prefill_down(w2):
    """70B-class down 28672 x 8192 at M = 2048 and M = 512 (w2a8), and w2a16."""
    K, N = synth.SHAPES_70B["down"]
    check_a8(w2, 2048, K, N, 128, 0, seed=4, ncols=64, acc_check=False)
    check_a8(w2, 512, K, N, 128, 0, seed=4, ncols=128)
    check_a16(w2, 256, K, N, 128, 0, seed=4, ncols=64)


@pytest.mark.parametrize("name", ["gate_up", "down"])
def test_70b_prefill_tiled_kernel_accumulators(w2, name):
    """The int32 group accumulators of the PREFILL kernel at the full K of the 70B-class shapes (8192 and
    28672: 64 and 224 groups, the long pipelines and every periodic bias settlement), bit for bit, on a
    band of rows that spans two row tiles with a ragged second one.  The kernel family is forced: AUTO
    would send so few rows to the mid-M kernel."""
    K, N = synth.SHAPES_70B[name]
    G, rows = 128, 80
    codes, scales, packed = weights(w2, K, N, G, 0, 4)
    X = synth.make_activations(rows, K, seed=4321)
    xq, _, _ = w2.quantize_rows(dev(X), G)
    oq, _, _ = oracle.quantize_rows(X, G, want_gsum=False)
    assert np.array_equal(xq.cpu().numpy(), oq)
    cols = sample_cols(N, 192, 17)
    acc = w2.debug_group_acc_a8(packed, K, N, G, xq, variant=w2.VARIANT_TILED)        # [rows][K/G][N] on the device
    got = acc[:, :, torch.from_numpy(cols).cuda()].cpu().numpy()
    del acc
    oacc = oracle.group_acc(np.ascontiguousarray(codes[:, cols]), G, 0, oq)
    assert np.array_equal(got, oacc)


def test_70b_prefill_gate_up_a16(w2):
    """The benchmark's w2a16 prefill launch: 8192 x 57344 at M = 2048 (128-row scale-folded tiles)."""
    K, N = synth.SHAPES_70B["gate_up"]
    check_a16(w2, 2048, K, N, 128, 0, seed=4, ncols=64)


@pytest.mark.parametrize("name", list(synth.SHAPES_8B))
def test_8b_between_decode_and_prefill(w2, name):
    """8B-class projections at M = 32 (mid-M kernels) and M = 128 (tiled kernels; with the workspace
    w2_workspace_size asks for, so K is split across workgroups where the planner wants it), both paths."""
    K, N = synth.SHAPES_8B[name]
    for M in (32, 128):
        check_a8(w2, M, K, N, 128, 0, seed=1, ncols=64, acc_check=False, use_ws=True)
        check_a16(w2, M, K, N, 128, 0, seed=1, ncols=64, use_ws=True)


def test_8b_gate_up_gated_epilogue_m1(w2):
    """The chained layer's gate+up call: bf16 row in, quantised in the kernel, silu(gate) * up out."""
    K, N = synth.SHAPES_8B["gate_up"]
    codes, scales, packed = weights(w2, K, N, 128, 0, 1)
    Xb = synth.f32_to_bf16_bits(synth.make_activations(1, K, seed=78))
    Y = w2.matmul_a8_fused_epi(packed, K, N, 128, dev(Xb).view(torch.bfloat16), act=w2.ACT_SILU_MUL)
    oq, osx, _ = oracle.quantize_rows(Xb, 128, x_is_bf16=True, want_gsum=False)
    blocks = np.unique(np.concatenate([np.arange(4), np.random.default_rng(9).choice(N // 32, 12), [N // 32 - 1]]))
    cols = (blocks[:, None] * 32 + np.arange(32)[None, :]).reshape(-1)          # whole gate/up block pairs
    cs, ss = np.ascontiguousarray(codes[:, cols]), np.ascontiguousarray(scales[:, cols])
    _, y64 = oracle.matmul_a8(cs, ss, 128, 0, oq, osx)
    mag = oracle.a8_term_magnitude(cs, ss, 128, 0, oq, osx)
    _, out = oracle.epilogue(y64, act=2)
    ocols = (blocks[:, None] * 16 + np.arange(16)[None, :]).reshape(-1)
    yg = synth.bf16_bits_to_f32(bf16_bits(Y)[:, ocols]).astype(np.float64)
    d = (1e-2 * np.abs(y64) + 2.0 ** -10 * mag).reshape(1, -1, 2, 16)
    z = y64.reshape(1, -1, 2, 16)
    tol = (1.1 * d[:, :, 0] * (np.abs(z[:, :, 1]) + d[:, :, 1]) + np.abs(z[:, :, 0]) * d[:, :, 1]).reshape(1, -1)
    assert np.all(np.abs(yg - out) <= tol + 2.0 ** -8 * np.abs(out))
