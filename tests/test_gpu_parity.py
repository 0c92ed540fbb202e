"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle
on the same seeded inputs.  Integer work (packed round trip, int8 codes,
int32 group accumulators) must match bit for bit; bf16 outputs must satisfy
|Y - Yor| <= 1e-2*|Yor| + 2^-10 * sum|terms| (the second term is the floor for
outputs that are a cancelling sum; fp32 vs fp64 association alone moves
those)."""
import numpy as np
import pytest

import oracle
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


def bf16_bits(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def bits_to_f64(b):
    return synth.bf16_bits_to_f32(b).astype(np.float64)


def check_y(Y_gpu_bits, Y_or_bits, y64, mag, what):
    yg = bits_to_f64(Y_gpu_bits)
    yo = bits_to_f64(Y_or_bits)
    tol = 1e-2 * np.abs(yo) + 2.0 ** -10 * mag
    bad = np.abs(yg - yo) > tol
    assert not bad.any(), (f"{what}: {bad.sum()} of {bad.size} outputs off; worst "
                           f"{np.abs(yg - yo)[bad].max()} vs tol {tol[bad].min()}")
    # typical-size outputs: must be within a bf16 ulp or so, without the floor
    big = np.abs(yo) > 0.05 * np.sqrt(np.mean(yo ** 2) + 1e-300)
    if big.any():
        rel = np.abs(yg - yo)[big] / np.abs(yo)[big]
        assert rel.max() <= 1e-2, f"{what}: max relative error {rel.max()}"


# ------------------------------------------------------------------ prepack
@pytest.mark.parametrize("codec", [0, 1])
@pytest.mark.parametrize("K,N,G", [(256, 16, 128), (512, 40, 64), (1024, 272, 128), (768, 8, 64)])
def test_prepack_roundtrip(w2, codec, K, N, G):
    codes, scales = synth.make_weights(K, N, G, codec, seed=K + N)
    packed = w2.prepack(dev(codes), dev(scales), G, codec)
    assert packed.numel() == w2.packed_size(K, N, G)
    c2, s2 = w2.debug_unpack(packed, K, N, G, codec)
    assert np.array_equal(c2.cpu().numpy(), codes)
    assert np.array_equal(s2.cpu().numpy().view(np.uint16), scales)


def test_prepack_counts_bad_codes(w2):
    codes, scales = synth.make_weights(256, 32, 128, 1, seed=3)
    codes[5, 7] = 3
    codes[200, 31] = 3
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    w2.prepack(dev(codes), dev(scales), 128, 1, bad_codes=flag)
    assert int(flag.item()) == 2
    flag.zero_()
    w2.prepack(dev(codes), dev(scales), 128, 0, bad_codes=flag)     # 3 is legal under int2
    assert int(flag.item()) == 0
    assert oracle.check_codes(codes, 1) == oracle.ERR_BAD_CODE


# ------------------------------------------------------------------ quantise
@pytest.mark.parametrize("M,K", [(1, 256), (3, 1024), (5, 4096), (2, 14336), (70, 512)])
@pytest.mark.parametrize("G", [64, 128])
def test_quantize_bit_exact_fp32(w2, M, K, G):
    X = synth.make_activations(M, K, seed=M * 1000 + K)
    if M > 2:
        X[1] = 0.0                                   # all-zero row
        X[2] *= np.float32(1e-20)                    # tiny values
    xq, sx, gs = w2.quantize_rows(dev(X), G, want_gsum=True)
    oq, os_, og = oracle.quantize_rows(X, G)
    assert np.array_equal(xq.cpu().numpy(), oq)
    assert np.array_equal(sx.cpu().numpy().view(np.uint32), os_.view(np.uint32))
    assert np.array_equal(gs.cpu().numpy(), og)


def test_quantize_ties_and_bf16_and_stride(w2):
    X = np.zeros((2, 256), np.float32)
    X[0, :8] = [127.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 126.5]
    X[1] = synth.make_activations(1, 256, seed=9)[0]
    xq, sx, _ = w2.quantize_rows(dev(X))
    oq, os_, _ = oracle.quantize_rows(X, 128)
    assert xq.cpu().numpy()[0, :8].tolist() == [127, 0, 2, 2, 0, -2, -2, 126]
    assert np.array_equal(xq.cpu().numpy(), oq)
    # bf16 input
    Xb = synth.f32_to_bf16_bits(synth.make_activations(4, 1024, seed=10))
    xq, sx, gs = w2.quantize_rows(dev(Xb).view(torch.bfloat16), 64, want_gsum=True)
    oq, os_, og = oracle.quantize_rows(Xb, 64, x_is_bf16=True)
    assert np.array_equal(xq.cpu().numpy(), oq)
    assert np.array_equal(sx.cpu().numpy().view(np.uint32), os_.view(np.uint32))
    assert np.array_equal(gs.cpu().numpy(), og)
    # strided rows
    Xw = synth.make_activations(3, 1024, seed=11)
    t = dev(Xw)[:, :512]
    xq, sx, _ = w2.quantize_rows(t)
    oq, os_, _ = oracle.quantize_rows(np.ascontiguousarray(Xw[:, :512]), 128)
    assert np.array_equal(xq.cpu().numpy(), oq)


@pytest.mark.parametrize("G", [64, 128])
@pytest.mark.parametrize("M", [1, 3])
def test_quantize_bf16_single_tile_row_with_group_sums(w2, M, G):
    # K = 256 in bf16 is half of what one wave covers at eight elements per lane: the lanes past the
    # end of the row must contribute neither to the abs-max nor to the group sums
    Xb = synth.f32_to_bf16_bits(synth.make_activations(M, 256, seed=40 + M))
    xq, sx, gs = w2.quantize_rows(dev(Xb).view(torch.bfloat16), G, want_gsum=True)
    oq, os_, og = oracle.quantize_rows(Xb, G, x_is_bf16=True)
    assert np.array_equal(xq.cpu().numpy(), oq)
    assert np.array_equal(sx.cpu().numpy().view(np.uint32), os_.view(np.uint32))
    assert np.array_equal(gs.cpu().numpy(), og)


# ------------------------------------------------------------------ w2a8
def run_a8_case(w2, M, K, N, G, codec, variant, seed, tune=None):
    """`tune`: overrides (w2_tuning_t fields) passed with every call, so that the case runs the
    workgroup shape it names whatever the library would pick by itself."""
    codes, scales, X = synth.make_problem(M, K, N, G, codec, seed)
    packed = w2.prepack(dev(codes), dev(scales), G, codec)
    xq, sx, _ = w2.quantize_rows(dev(X), G)
    oq, osx, _ = oracle.quantize_rows(X, G)
    assert np.array_equal(xq.cpu().numpy(), oq)
    acc = w2.debug_group_acc_a8(packed, K, N, G, xq, variant, tune=tune)
    oacc = oracle.group_acc(codes, G, codec, oq)
    assert np.array_equal(acc.cpu().numpy(), oacc), "int32 group accumulators differ"
    Y = w2.matmul_a8(packed, K, N, G, xq, sx, variant=variant, tune=tune)
    Y2 = w2.matmul_a8(packed, K, N, G, xq, sx, variant=variant, tune=tune)
    assert torch.equal(Y.view(torch.int16), Y2.view(torch.int16)), "not deterministic"
    Yo, y64 = oracle.matmul_a8(codes, scales, G, codec, oq, osx)
    mag = oracle.a8_term_magnitude(codes, scales, G, codec, oq, osx)
    check_y(bf16_bits(Y), Yo, y64, mag, f"a8 M={M} K={K} N={N} G={G} codec={codec} variant={variant}")


# shapes span several 16x256 tiles, ragged N (not a multiple of 16 / 64 / 256), one-tile K
SMALL_SHAPES = [(256, 16), (512, 40), (1024, 272), (2048, 1032), (768, 8)]


@pytest.mark.parametrize("G", [64, 128])
@pytest.mark.parametrize("K,N", SMALL_SHAPES)
@pytest.mark.parametrize("M", [1, 2, 3, 4])
def test_a8_dot4(w2, M, K, N, G):
    run_a8_case(w2, M, K, N, G, (M + K) % 2, w2.VARIANT_DOT4, seed=M + K + N + G)


@pytest.mark.parametrize("G", [64, 128])
@pytest.mark.parametrize("K,N", SMALL_SHAPES)
@pytest.mark.parametrize("M", [1, 4, 7, 16])
def test_a8_smallm(w2, M, K, N, G):
    run_a8_case(w2, M, K, N, G, (M + K) % 2, w2.VARIANT_SMALLM, seed=M + K + N + G)


@pytest.mark.parametrize("shape", [None, (4, 1, 2), (8, 8, 4), (16, 2, 8), (8, 1, 8), (2, 2, 2), (16, 16, 2)])
@pytest.mark.parametrize("G", [64, 128])
@pytest.mark.parametrize("K,N", SMALL_SHAPES + [(5120, 48)])
@pytest.mark.parametrize("M", [1, 2, 3, 4, 5, 8, 9, 13, 16, 17, 24, 32])
def test_a8_gemv(w2, M, K, N, G, shape):
    # the decode kernel: the library's own workgroup shape and forced ones (waves, column blocks, window):
    # runs of one tile, runs shorter and longer than the window, uneven runs (20 tiles over 8 ranges); from
    # five rows on the wide form (every accumulator row in use, at most eight waves), from seventeen on with
    # two row tiles
    if M * (K + 32) > 140 * 1024:
        pytest.skip("the rows do not fit a workgroup's local memory")
    tune = None if shape is None else {"small_waves": shape[0], "small_cbw": shape[1], "gemv_window": shape[2]}
    run_a8_case(w2, M, K, N, G, (M + K) % 2, w2.VARIANT_GEMV, seed=M + K + N + G, tune=tune)


@pytest.mark.parametrize("cbw,ks", [(3, 1), (3, 4), (5, 2), (7, 2), (6, 2), (1, 3), (2, 5), (9, 1), (15, 1)])
@pytest.mark.parametrize("K,N,G", [(1024, 272, 128), (2048, 1032, 64), (5120, 48, 128), (768, 8, 64)])
@pytest.mark.parametrize("M", [1, 2, 3, 4])
def test_a8_gemv_any_workgroup_width(w2, M, K, N, G, cbw, ks):
    # up to four rows a workgroup of the decode kernel holds any number of column blocks (not only powers of
    # two) times any number of K ranges: int32 accumulators, Y, the fused entry (same bits as quantise + matmul
    # in the same shape) and, for even widths, the gated epilogue; a last workgroup with missing column blocks
    if -(-(K // 256) // min(ks, K // 256)) > 16:
        pytest.skip("a wave's run is limited to 16 tiles")
    tune = {"gemv_cbw": cbw, "gemv_ks": ks}
    run_a8_case(w2, M, K, N, G, (M + K) % 2, w2.VARIANT_GEMV, seed=M + K + N + G + cbw, tune=tune)
    codes, scales, X = synth.make_problem(M, K, N, G, 0, M + K + cbw)
    packed = w2.prepack(dev(codes), dev(scales), G, 0)
    xq, sx, _ = w2.quantize_rows(dev(X), G)
    Y2 = w2.matmul_a8(packed, K, N, G, xq, sx, variant=w2.VARIANT_GEMV, tune=tune)
    if cbw * min(ks, K // 256) * 64 * 32 >= K * (1 if M == 1 else 2 if M == 2 else 4):      # the threads can hold the fp32 rows
        Yf = w2.matmul_a8_fused_epi(packed, K, N, G, dev(X), tune=tune)
        assert torch.equal(Yf.view(torch.int16), Y2.view(torch.int16))
    if cbw % 2 == 0 and N % 32 == 0:
        oq, osx, _ = oracle.quantize_rows(X, G)
        _, y64 = oracle.matmul_a8(codes, scales, G, 0, oq, osx)
        mag = oracle.a8_term_magnitude(codes, scales, G, 0, oq, osx)
        Yg = w2.matmul_a8_epi(packed, K, N, G, xq, sx, act=2, variant=w2.VARIANT_GEMV, tune=tune)
        check_epilogue(bf16_bits(Yg), y64, mag, None, 2, f"gated, cbw={cbw} ks={ks} M={M}")


@pytest.mark.parametrize("cbw,ks", [(3, 2), (5, 1), (7, 1), (6, 1), (1, 5), (3, 1)])
@pytest.mark.parametrize("K,N,G", [(1024, 272, 128), (2048, 1032, 64), (768, 40, 128)])
@pytest.mark.parametrize("M", [5, 8, 13, 16, 17, 32])
def test_a8_gemv_wide_form_any_workgroup_width(w2, M, K, N, G, cbw, ks):
    # from five rows on (every accumulator row in use; two row tiles from seventeen): the same freedom of width,
    # the epilogue's (row, column) split by an exact fp32 quotient; plain and, for even widths, gated
    tune = {"gemv_cbw": cbw, "gemv_ks": ks}
    run_a8_case(w2, M, K, N, G, (M + K) % 2, w2.VARIANT_GEMV, seed=M + K + N + G + cbw, tune=tune)
    if cbw % 2 == 0 and N % 32 == 0:
        codes, scales, X = synth.make_problem(M, K, N, G, 0, M + K + cbw)
        packed = w2.prepack(dev(codes), dev(scales), G, 0)
        xq, sx, _ = w2.quantize_rows(dev(X), G)
        oq, osx, _ = oracle.quantize_rows(X, G)
        _, y64 = oracle.matmul_a8(codes, scales, G, 0, oq, osx)
        mag = oracle.a8_term_magnitude(codes, scales, G, 0, oq, osx)
        Yg = w2.matmul_a8_epi(packed, K, N, G, xq, sx, act=2, variant=w2.VARIANT_GEMV, tune=tune)
        check_epilogue(bf16_bits(Yg), y64, mag, None, 2, f"wide, gated, cbw={cbw} ks={ks} M={M}")


def test_a8_gemv_workgroup_shape_limits(w2):
    # shapes the kernel cannot run are refused before anything is launched
    codes, scales, X = synth.make_problem(8, 512, 64, 128, 0, 3)
    packed = w2.prepack(dev(codes), dev(scales), 128, 0)
    xq, sx, _ = w2.quantize_rows(dev(X), 128)
    for M, tune, act in ((1, {"gemv_cbw": 9, "gemv_ks": 2}, 0),        # more than 16 waves
                         (8, {"gemv_cbw": 8, "gemv_ks": 2}, 0),        # the wide form: at most 8 waves
                         (1, {"gemv_cbw": 3, "gemv_ks": 2}, 2)):       # the gated epilogue pairs column blocks
        Y = torch.full((M, 64), 7.0, dtype=torch.bfloat16, device="cuda")
        with pytest.raises(w2.W2Error):
            w2.matmul_a8_epi(packed, 512, 64, 128, xq[:M], sx[:M], act=act, out=Y, variant=w2.VARIANT_GEMV, tune=tune)
        assert torch.all(Y == 7.0)


@pytest.mark.parametrize("bf16_in", [False, True])
@pytest.mark.parametrize("M", [1, 2, 4, 8])
def test_production_kernels_hold_exact_group_sums(w2, M, bf16_in):
    """The int32 group accumulators of the kernels the benchmark times, read through Y itself (no debug
    instantiation): activations in {-1, 0, 1} plus one 127 per row on a k whose weights are all zero, so that
    the quantisation is the identity (inv = 1, sx = 1); scales 1.0 in ONE group and 0 elsewhere, so that
    Y[m][n] = acc[m][g][n], a small integer that bf16 holds exactly.  Every group in turn, K = 4096, through the
    fused entry point (one launch for M <= 2) and through quantise + matmul."""
    K, N, G = 4096, 80, 128
    rng = np.random.default_rng(77 + M)
    codes = rng.integers(0, 4, size=(K, N), dtype=np.uint8)
    codes[5, :] = 2                                          # q = 0 under the int2 codec
    X = rng.integers(-1, 2, size=(M, K)).astype(np.float32)
    X[:, 5] = 127.0
    oq, osx, _ = oracle.quantize_rows(X, G)
    assert np.array_equal(oq, X.astype(np.int8)) and np.all(osx == 1.0)
    oacc = oracle.group_acc(codes, G, 0, oq)                 # [M][K/G][N]
    assert np.abs(oacc).max() <= 256
    Xd = dev(X).to(torch.bfloat16) if bf16_in else dev(X)
    ws = torch.empty(max(w2.workspace_size(M, K, N, G), 16), dtype=torch.uint8, device="cuda")
    xq, sx, _ = w2.quantize_rows(Xd, G)
    assert np.array_equal(xq.cpu().numpy(), oq)
    for g in range(K // G):
        scales = np.zeros((K // G, N), np.uint16)
        scales[g, :] = 0x3F80
        packed = w2.prepack(dev(codes), dev(scales), G, 0)
        want = oacc[:, g, :].astype(np.float64)
        Yf = w2.matmul_a8_fused(packed, K, N, G, Xd, workspace=ws)
        assert np.array_equal(bits_to_f64(bf16_bits(Yf)), want), f"fused entry, group {g}"
        Y2 = w2.matmul_a8(packed, K, N, G, xq, sx)
        assert np.array_equal(bits_to_f64(bf16_bits(Y2)), want), f"quantise + matmul, group {g}"


@pytest.mark.parametrize("cbw", [0, 2, 4, 8])
@pytest.mark.parametrize("G", [64, 128])
@pytest.mark.parametrize("K,N", [(256, 16), (1024, 272), (2304, 1032), (768, 8)])
@pytest.mark.parametrize("M", [9, 16, 17, 31, 32, 33, 50, 64])
def test_a8_midm(w2, M, K, N, G, cbw):
    # one / two / four 16-row tiles per streamed weight tile; every split of the eight waves
    # into column blocks x k-splits; K of one chunk, of a ragged last chunk (2304 = 2 x 1024 + 256)
    run_a8_case(w2, M, K, N, G, (M + K) % 2, w2.VARIANT_MIDM, seed=M + K + N + G, tune={"midm_cbw": cbw})


@pytest.mark.parametrize("M", [65, 100, 128, 130, 256])
@pytest.mark.parametrize("K,N,G", [(1024, 272, 128), (768, 48, 64)])
def test_midm_row_bands(w2, M, K, N, G):
    # more than 64 rows: bands of 64 rows on grid.y (ragged last band), both activation types, and the
    # integer accumulators of every band bit for bit
    run_a8_case(w2, M, K, N, G, M % 2, w2.VARIANT_MIDM, seed=M + K)
    run_a16_case(w2, M, K, N, G, M % 2, w2.VARIANT_MIDM, seed=M + K)


def test_a8_midm_long_k_and_limits(w2):
    run_a8_case(w2, 64, 8192, 48, 128, 0, w2.VARIANT_MIDM, seed=7)
    run_a8_case(w2, 40, 14336, 32, 64, 1, w2.VARIANT_MIDM, seed=8)
    run_a8_case(w2, 3, 512, 40, 128, 0, w2.VARIANT_MIDM, seed=9)       # small M is allowed, just not chosen
    codes, scales, X = synth.make_problem(257, 256, 16, 128, 0, 9)      # more than four bands of 64 rows
    packed = w2.prepack(dev(codes), dev(scales), 128, 0)
    xq, sx, _ = w2.quantize_rows(dev(X), 128)
    with pytest.raises(w2.W2Error):
        w2.matmul_a8(packed, 256, 16, 128, xq, sx, variant=w2.VARIANT_MIDM)


@pytest.mark.parametrize("bn", [64, 128, 256])
@pytest.mark.parametrize("G", [64, 128])
@pytest.mark.parametrize("K,N", [(256, 16), (1024, 272), (512, 1032)])
@pytest.mark.parametrize("M", [1, 17, 127, 128, 200])
def test_a8_tiled(w2, M, K, N, G, bn):
    # the three workgroup widths (two, four and eight waves); ragged M, N; one to four stages of K
    run_a8_case(w2, M, K, N, G, (M + K) % 2, w2.VARIANT_TILED, seed=M + K + N + G, tune={"tiled_bn": bn})


@pytest.mark.parametrize("bn", [64, 128])
@pytest.mark.parametrize("kw", [2, 4])
@pytest.mark.parametrize("G", [64, 128])
@pytest.mark.parametrize("K,N", [(1024, 272), (2048, 1032), (4096, 48), (512, 16)])
@pytest.mark.parametrize("M", [1, 33, 64, 100])
def test_a8_tiled_k_split_inside_workgroup(w2, M, K, N, G, kw, bn):
    # 64-row tiles, 128- and 64-column workgroups whose 2 or 4 groups of waves take K ranges of their own and
    # add up in LDS (K = 512 with four groups: the ranges cannot be equal, the plain kernel runs); with and
    # without the split across workgroups on top
    tune = {"tiled_bm": 64, "tiled_bn": bn, "tiled_kw": kw}
    run_a8_case(w2, M, K, N, G, (M + K) % 2, w2.VARIANT_TILED, seed=M + K + N + G + kw, tune=tune)
    if K >= 2048:
        codes, scales, X = synth.make_problem(M, K, N, G, 0, M + K + N)
        packed = w2.prepack(dev(codes), dev(scales), G, 0)
        xq, sx, _ = w2.quantize_rows(dev(X), G)
        ws = torch.empty(4 * M * N * 4, dtype=torch.uint8, device="cuda")
        Y = w2.matmul_a8(packed, K, N, G, xq, sx, variant=w2.VARIANT_TILED, workspace=ws, tune=dict(tune, splitk=2))
        oq, osx, _ = oracle.quantize_rows(X, G)
        Yo, y64 = oracle.matmul_a8(codes, scales, G, 0, oq, osx)
        mag = oracle.a8_term_magnitude(codes, scales, G, 0, oq, osx)
        check_y(bf16_bits(Y), Yo, y64, mag, f"a8 tiled kw={kw} split-K 2 M={M} K={K} N={N} G={G}")


@pytest.mark.parametrize("G", [64, 128])
@pytest.mark.parametrize("M,K,N", [(40, 14336, 272), (100, 7168, 1032), (64, 4352, 48), (128, 3072, 528), (33, 2048, 2064)])
def test_a8_tiled_planned_k_split(w2, M, K, N, G):
    # one or two row tiles with a workspace for 16 parts: the library's own choice of K ranges across and
    # inside workgroups (tile counts with many divisors, a prime one, few and many column tiles); a second
    # call with room for fewer parts must still be correct (another plan), and so must one without a workspace
    codes, scales, X = synth.make_problem(M, K, N, G, 0, M + K + N + G)
    packed = w2.prepack(dev(codes), dev(scales), G, 0)
    xq, sx, _ = w2.quantize_rows(dev(X), G)
    oq, osx, _ = oracle.quantize_rows(X, G)
    Yo, y64 = oracle.matmul_a8(codes, scales, G, 0, oq, osx)
    mag = oracle.a8_term_magnitude(codes, scales, G, 0, oq, osx)
    for parts in (16, 3, 0):
        ws = torch.empty(parts * M * N * 4, dtype=torch.uint8, device="cuda") if parts else None
        Y = w2.matmul_a8(packed, K, N, G, xq, sx, variant=w2.VARIANT_TILED, workspace=ws, tune={"tiled_bm": 64})
        Y2 = w2.matmul_a8(packed, K, N, G, xq, sx, variant=w2.VARIANT_TILED, workspace=ws, tune={"tiled_bm": 64})
        assert torch.equal(Y.view(torch.int16), Y2.view(torch.int16)), "not deterministic"
        check_y(bf16_bits(Y), Yo, y64, mag, f"a8 tiled planned split, room for {parts} parts, M={M} K={K} N={N} G={G}")


@pytest.mark.parametrize("bn,kw", [(128, 1), (128, 2), (256, 1)])
@pytest.mark.parametrize("G", [64, 128])
@pytest.mark.parametrize("K,N", [(256, 16), (1024, 272), (2560, 1032), (4608, 48)])
@pytest.mark.parametrize("M", [1, 33, 64, 100])
def test_a8_tiled_deep_weight_window(w2, M, K, N, G, bn, kw):
    # 64-row tiles with eight weight stages (and as many activation register sets) in flight per wave: fewer
    # stages than the window (K = 256), exactly one window (1024), a last window cut short (2560: 20 stages,
    # 4608: 36), with the K split across workgroups on top
    tune = {"tiled_bm": 64, "tiled_bn": bn, "tiled_kw": kw, "tiled_wd": 8}
    run_a8_case(w2, M, K, N, G, (M + K) % 2, w2.VARIANT_TILED, seed=M + K + N + G + kw, tune=tune)
    if K >= 2048:
        codes, scales, X = synth.make_problem(M, K, N, G, 0, M + K + N)
        packed = w2.prepack(dev(codes), dev(scales), G, 0)
        xq, sx, _ = w2.quantize_rows(dev(X), G)
        ws = torch.empty(4 * M * N * 4, dtype=torch.uint8, device="cuda")
        Y = w2.matmul_a8(packed, K, N, G, xq, sx, variant=w2.VARIANT_TILED, workspace=ws, tune=dict(tune, splitk=3))
        oq, osx, _ = oracle.quantize_rows(X, G)
        Yo, y64 = oracle.matmul_a8(codes, scales, G, 0, oq, osx)
        mag = oracle.a8_term_magnitude(codes, scales, G, 0, oq, osx)
        check_y(bf16_bits(Y), Yo, y64, mag, f"a8 tiled wd=8 bn={bn} kw={kw} split-K 3 M={M} K={K} N={N} G={G}")


@pytest.mark.parametrize("bn", [128, 256])
@pytest.mark.parametrize("K,N", [(256, 16), (1024, 272), (512, 1032), (4608, 48)])
@pytest.mark.parametrize("M", [1, 17, 127, 128, 129, 300])
def test_a8_tiled_128_row_tiles(w2, M, K, N, bn):
    # the prefill kernel with 128-row tiles: both workgroup widths; ragged M and N; one stage pair up to 36
    # stages (K = 4608: two periodic bias settlements); accumulators bit for bit, outputs to tolerance
    run_a8_case(w2, M, K, N, 128, (M + K) % 2, w2.VARIANT_TILED, seed=M + K + N, tune={"tiled_bm": 128, "tiled_bn": bn})


@pytest.mark.parametrize("act", [0, 2])
@pytest.mark.parametrize("bn", [128, 256])
@pytest.mark.parametrize("splitk", [0, 2, 3, 8])
@pytest.mark.parametrize("M,K,N", [(129, 4608, 288), (300, 2048, 544), (128, 7168, 64), (256, 1024, 1056)])
def test_a8_tiled_128_row_tiles_split_k(w2, M, K, N, splitk, bn, act):
    # the 128-row kernel with K cut into ranges across workgroups (its own rule, or forced part counts: uneven
    # ranges, more parts than the workspace holds), partial results summed by the second launch; both widths;
    # plain and gated epilogue; against the oracle and, for the plain epilogue, bit for bit against ... the
    # unsplit kernel is NOT expected to match bit for bit (another order of additions)
    codes, scales, X = synth.make_problem(M, K, N, 128, 0, M + K + N + splitk)
    packed = w2.prepack(dev(codes), dev(scales), 128, 0)
    xq, sx, _ = w2.quantize_rows(dev(X), 128)
    ws = torch.empty(5 * M * N * 4, dtype=torch.uint8, device="cuda")
    tune = {"tiled_bm": 128, "tiled_bn": bn, "splitk": splitk}
    Y = w2.matmul_a8_epi(packed, K, N, 128, xq, sx, act=act, variant=w2.VARIANT_TILED, workspace=ws, tune=tune)
    Y2 = w2.matmul_a8_epi(packed, K, N, 128, xq, sx, act=act, variant=w2.VARIANT_TILED, workspace=ws, tune=tune)
    assert torch.equal(Y.view(torch.int16), Y2.view(torch.int16)), "not deterministic"
    oq, osx, _ = oracle.quantize_rows(X, 128)
    Yo, y64 = oracle.matmul_a8(codes, scales, 128, 0, oq, osx)
    mag = oracle.a8_term_magnitude(codes, scales, 128, 0, oq, osx)
    if act == 0:
        check_y(bf16_bits(Y), Yo, y64, mag, f"a8 128-row tiles split-K {splitk} bn={bn} M={M} K={K} N={N}")
    else:
        check_epilogue(bf16_bits(Y), y64, mag, None, act, f"a8 128-row tiles split-K {splitk} gated bn={bn} M={M} K={K} N={N}")


@pytest.mark.parametrize("M", [20, 100, 300])
def test_a8_one_fma_dequant_keeps_denormals(w2, M):
    # the mid-M and prefill kernels read BIAS + 64*sum as an fp32 denormal and multiply by sw * 2^64: a build
    # that flushed denormals would return zeros here.  Unit scales, xq = small integers, sx = 1: exact results.
    K, N, G = 512, 48, 128
    rng = np.random.default_rng(M)
    codes = rng.integers(0, 4, size=(K, N), dtype=np.uint8)
    scales = np.full((K // G, N), 0x3F80, np.uint16)
    xq = rng.integers(-2, 3, size=(M, K)).astype(np.int8)
    packed = w2.prepack(dev(codes), dev(scales), G, 0)
    want = (xq.astype(np.int64) @ (codes.astype(np.int64) - 2)).astype(np.float64)
    assert np.abs(want).max() <= 256 and np.abs(want).max() > 8
    for variant, tune in ((w2.VARIANT_MIDM, None), (w2.VARIANT_TILED, {"tiled_bm": 64}), (w2.VARIANT_TILED, {"tiled_bm": 128})):
        if variant == w2.VARIANT_MIDM and M > 256:
            continue
        Y = w2.matmul_a8(packed, K, N, G, torch.from_numpy(xq).cuda(), torch.ones(M, device="cuda"), variant=variant, tune=tune)
        assert np.array_equal(bits_to_f64(bf16_bits(Y)), want), (variant, tune)


@pytest.mark.parametrize("M", [1, 4, 8, 9, 16, 17, 64, 65, 130])
def test_a8_auto_dispatch(w2, M):
    run_a8_case(w2, M, 1024, 528, 128, 0, w2.VARIANT_AUTO, seed=M)


def _auto_cases():
    # seeded draws over the shape space AUTO decides on: M on both sides of every switch between kernel families,
    # shallow and deep K, narrow and wide N (multiples of 8, mostly not of 64), both group sizes
    rng = np.random.default_rng(20250811)
    ms = [1, 3, 5, 8, 9, 12, 16, 17, 24, 32, 33, 40, 64, 65, 96, 128, 129, 192, 256, 300]
    cases = []
    for i in range(48):
        M = int(ms[i % len(ms)])
        K = int(rng.choice([256, 512, 1024, 2048, 3072, 4096, 7168, 14336]))
        n_max = max(16, min(4096, (3 << 20) // K))
        N = int(rng.integers(2, n_max // 8 + 1)) * 8
        cases.append((M, K, N, int(rng.choice([64, 128])), i))
    return cases


@pytest.mark.parametrize("M,K,N,G,seed", _auto_cases())
def test_auto_dispatch_over_random_shapes(w2, M, K, N, G, seed):
    # the library's own choice of kernel, launch shape and K split, with the workspace w2_workspace_size asks
    # for and without one, w2a8 and w2a16, against the oracle
    codes, scales, X = synth.make_problem(M, K, N, G, seed % 2, 1000 + seed)
    packed = w2.prepack(dev(codes), dev(scales), G, seed % 2)
    xq, sx, _ = w2.quantize_rows(dev(X), G)
    oq, osx, _ = oracle.quantize_rows(X, G)
    assert np.array_equal(xq.cpu().numpy(), oq)
    Yo, y64 = oracle.matmul_a8(codes, scales, G, seed % 2, oq, osx)
    mag = oracle.a8_term_magnitude(codes, scales, G, seed % 2, oq, osx)
    Xb = synth.f32_to_bf16_bits(X)
    Yo16, y64_16, mag16 = oracle.matmul_a16(codes, scales, G, seed % 2, Xb)
    for with_ws in (True, False):
        n8, n16 = w2.workspace_size(M, K, N, G), w2.workspace_size(M, K, N, G, a16=True)
        ws8 = torch.empty(n8, dtype=torch.uint8, device="cuda") if with_ws and n8 else None
        ws16 = torch.empty(n16, dtype=torch.uint8, device="cuda") if with_ws and n16 else None
        Y = w2.matmul_a8(packed, K, N, G, xq, sx, workspace=ws8)
        check_y(bf16_bits(Y), Yo, y64, mag, f"a8 auto M={M} K={K} N={N} G={G} workspace={with_ws}")
        Y16 = w2.matmul_a16(packed, K, N, G, dev(Xb).view(torch.bfloat16), workspace=ws16)
        check_y(bf16_bits(Y16), Yo16, y64_16, mag16, f"a16 auto M={M} K={K} N={N} G={G} workspace={with_ws}")


@pytest.mark.parametrize("codec", [0, 1])
def test_config0_gemv_2048(w2, codec):
    """The single-GEMV configuration: M=1, K=N=2048, G=128, seed 0."""
    run_a8_case(w2, 1, 2048, 2048, 128, codec, w2.VARIANT_AUTO, seed=0)


def test_a8_lds_chunking_long_k(w2):
    # K large enough that 16 rows do not fit one LDS chunk: exercises the chunk loop
    run_a8_case(w2, 16, 14336, 64, 128, 0, w2.VARIANT_SMALLM, seed=5)
    run_a8_case(w2, 2, 14336, 64, 128, 1, w2.VARIANT_DOT4, seed=6)


def test_a8_rows_independent_across_variants(w2):
    M, K, N, G = 4, 1024, 272, 128
    codes, scales, X = synth.make_problem(M, K, N, G, 0, 77)
    packed = w2.prepack(dev(codes), dev(scales), G, 0)
    xq, sx, _ = w2.quantize_rows(dev(X), G)
    accs = [w2.debug_group_acc_a8(packed, K, N, G, xq, v).cpu().numpy()
            for v in (w2.VARIANT_DOT4, w2.VARIANT_SMALLM, w2.VARIANT_TILED)]
    assert np.array_equal(accs[0], accs[1]) and np.array_equal(accs[0], accs[2])
    one = w2.debug_group_acc_a8(packed, K, N, G, xq[2:3].contiguous(), w2.VARIANT_DOT4).cpu().numpy()
    assert np.array_equal(one[0], accs[0][2])


def test_a8_closed_forms(w2):
    K, N, G = 512, 48, 128
    # all weights at the zero-point value -> Y == 0
    codes = np.full((K, N), 2, np.uint8)
    _, scales, X = synth.make_problem(2, K, N, G, 0, 1)
    packed = w2.prepack(dev(codes), dev(scales), G, 0)
    xq, sx, _ = w2.quantize_rows(dev(X), G)
    for v in (w2.VARIANT_DOT4, w2.VARIANT_SMALLM, w2.VARIANT_TILED):
        Y = w2.matmul_a8(packed, K, N, G, xq, sx, variant=v)
        assert torch.all(Y.view(torch.int16) == 0)
    # unit scales, xq = 1, sx = 1 -> column sums of q, exact in bf16 when |sum| < 256
    codes, _, _ = synth.make_problem(1, K, N, G, 1, 2)         # ternary: values average to 0
    ones = np.full((K // G, N), 0x3F80, np.uint16)
    packed = w2.prepack(dev(codes), dev(ones), G, 1)
    xq1 = torch.ones((1, K), dtype=torch.int8, device="cuda")
    sx1 = torch.ones(1, dtype=torch.float32, device="cuda")
    colsum = (codes.astype(np.int64) - 1).sum(0)
    assert np.abs(colsum).max() < 256
    for v in (w2.VARIANT_DOT4, w2.VARIANT_SMALLM, w2.VARIANT_TILED):
        Y = w2.matmul_a8(packed, K, N, G, xq1, sx1, variant=v)
        assert np.array_equal(bits_to_f64(bf16_bits(Y))[0], colsum.astype(np.float64))


# ------------------------------------------------------------------ fused quantise + matmul
@pytest.mark.parametrize("bf16_in", [False, True])
@pytest.mark.parametrize("G", [64, 128])
@pytest.mark.parametrize("K,N", [(256, 16), (1024, 272), (2048, 1032), (4096, 512), (14336, 64)])
@pytest.mark.parametrize("M", [1, 2, 3, 4])
def test_a8_fused_equals_two_call_path(w2, M, K, N, G, bf16_in):
    codes, scales, X = synth.make_problem(M, K, N, G, M % 2, seed=M + K + N)
    if M > 1:
        X[1] = 0.0                                            # all-zero row
    packed = w2.prepack(dev(codes), dev(scales), G, M % 2)
    if bf16_in:
        Xb = synth.f32_to_bf16_bits(X)
        Xd = dev(Xb).view(torch.bfloat16)
        oq, osx, _ = oracle.quantize_rows(Xb, G, x_is_bf16=True)
    else:
        Xd = dev(X)
        oq, osx, _ = oracle.quantize_rows(X, G)
    try:
        Yf = w2.matmul_a8_fused(packed, K, N, G, Xd)
    except w2.W2Error as e:                                   # shape beyond the fused budget
        assert e.status == w2.ERR_UNSUPPORTED_SHAPE
        return
    xq, sx, _ = w2.quantize_rows(Xd, G)
    Y2 = w2.matmul_a8(packed, K, N, G, xq, sx)
    assert torch.equal(Yf.view(torch.int16), Y2.view(torch.int16)), "fused and two-call results differ"
    Yo, y64 = oracle.matmul_a8(codes, scales, G, M % 2, oq, osx)
    mag = oracle.a8_term_magnitude(codes, scales, G, M % 2, oq, osx)
    check_y(bf16_bits(Yf), Yo, y64, mag, f"a8 fused M={M} K={K} N={N} G={G} bf16_in={bf16_in}")


@pytest.mark.parametrize("bf16_in", [False, True])
@pytest.mark.parametrize("G", [64, 128])
@pytest.mark.parametrize("K,N", [(256, 16), (1024, 272), (4096, 512), (5120, 48), (14336, 40)])
@pytest.mark.parametrize("M", [5, 6, 8])
def test_a8_fused_wide_one_launch(w2, M, K, N, G, bf16_in):
    # five to eight rows quantised inside the decode kernel's wide form (tuning field fused_rows), against the
    # oracle and, with the same workgroup shape forced on both, bit for bit against quantise + matmul; rows too
    # long for a workgroup's registers take the two launches after all
    codes, scales, X = synth.make_problem(M, K, N, G, M % 2, seed=M + K + N)
    X[1] = 0.0                                                # all-zero row
    packed = w2.prepack(dev(codes), dev(scales), G, M % 2)
    if bf16_in:
        Xb = synth.f32_to_bf16_bits(X)
        Xd = dev(Xb).view(torch.bfloat16)
        oq, osx, _ = oracle.quantize_rows(Xb, G, x_is_bf16=True)
    else:
        Xd = dev(X)
        oq, osx, _ = oracle.quantize_rows(X, G)
    ks = min(4, K // 256)
    shape = {"gemv_cbw": 2, "gemv_ks": ks}
    ws = torch.empty(w2.workspace_size(M, K, N, G), dtype=torch.uint8, device="cuda")
    Yf = w2.matmul_a8_fused_epi(packed, K, N, G, Xd, workspace=ws, tune=dict(shape, fused_rows=8))
    Yo, y64 = oracle.matmul_a8(codes, scales, G, M % 2, oq, osx)
    mag = oracle.a8_term_magnitude(codes, scales, G, M % 2, oq, osx)
    check_y(bf16_bits(Yf), Yo, y64, mag, f"a8 fused wide M={M} K={K} N={N} G={G} bf16_in={bf16_in}")
    pieces = K * (2 if bf16_in else 4) // 16
    if -(-pieces // (2 if bf16_in else 4)) <= 512:   # one launch: the same sums in the same order
        xq, sx, _ = w2.quantize_rows(Xd, G)
        Y2 = w2.matmul_a8(packed, K, N, G, xq, sx, variant=w2.VARIANT_GEMV, tune=shape)
        assert torch.equal(Yf.view(torch.int16), Y2.view(torch.int16)), "fused and two-call results differ"


def test_a8_fused_rejects_large_m(w2):
    codes, scales, X = synth.make_problem(5, 256, 16, 128, 0, 1)
    packed = w2.prepack(dev(codes), dev(scales), 128, 0)
    with pytest.raises(w2.W2Error) as e:
        w2.matmul_a8_fused(packed, 256, 16, 128, dev(X))                       # M > 4 without a workspace
    assert e.value.status == w2.ERR_UNSUPPORTED_SHAPE
    small = torch.empty(64, dtype=torch.uint8, device="cuda")
    with pytest.raises(w2.W2Error) as e:
        w2.matmul_a8_fused(packed, 256, 16, 128, dev(X), workspace=small)      # workspace too small
    assert e.value.status == w2.ERR_BUFFER_TOO_SMALL


@pytest.mark.parametrize("bf16_in", [False, True])
@pytest.mark.parametrize("M,K,N,G", [(3, 1024, 272, 128), (4, 4096, 512, 64), (7, 512, 40, 128), (40, 1024, 272, 128),
                                     (130, 512, 1032, 64), (2, 28672, 64, 128)])
def test_a8_fused_with_workspace_equals_two_call_path(w2, M, K, N, G, bf16_in):
    # with a workspace the call covers every M (quantise + the kernel family picked for M); the
    # result is the two-call result bit for bit; (2, 28672) is two rows too long for one launch
    codes, scales, X = synth.make_problem(M, K, N, G, 0, seed=M + K + N)
    packed = w2.prepack(dev(codes), dev(scales), G, 0)
    Xd = dev(synth.f32_to_bf16_bits(X)).view(torch.bfloat16) if bf16_in else dev(X)
    nbytes = w2.workspace_size(M, K, N, G)
    assert nbytes >= M * K + 4 * M
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    Y = w2.matmul_a8_fused(packed, K, N, G, Xd, workspace=ws)
    xq, sx, _ = w2.quantize_rows(Xd, G)
    Y2 = w2.matmul_a8(packed, K, N, G, xq, sx)
    assert torch.equal(Y.view(torch.int16), Y2.view(torch.int16))


def test_workspace_size_rule(w2):
    assert w2.workspace_size(1, 4096, 4096, 128) == 0            # one launch covers it
    assert w2.workspace_size(2, 4096, 4096, 128) == 0
    assert w2.workspace_size(2, 28672, 4096, 128) > 0            # two rows of 112 KiB as fp32
    assert w2.workspace_size(3, 4096, 4096, 128) >= 3 * 4096 + 12
    assert w2.workspace_size(2048, 8192, 57344, 128, a16=True) == 0   # enough output tiles: no split-K
    quant = lambda M, K: (M * K + 4 * M + 255) // 256 * 256      # int8 rows + one scale per row
    assert w2.workspace_size(2048, 8192, 57344, 128) == quant(2048, 8192)
    # few output tiles and a deep K: room for the split-K partial results, whole fp32 copies of the output
    for a16 in (False, True):
        extra = w2.workspace_size(128, 14336, 4096, 128, a16=a16) - (0 if a16 else quant(128, 14336))
        assert extra > 0 and extra % (128 * 4096 * 4) == 0 and 2 <= extra // (128 * 4096 * 4) <= 16
    # the mid-M kernel splits a deep K too (14 chunks of 1024 k and more), not a shallow one
    extra = w2.workspace_size(16, 28672, 8192, 128) - quant(16, 28672)
    assert extra > 0 and extra % (16 * 8192 * 4) == 0 and 2 <= extra // (16 * 8192 * 4) <= 16
    assert w2.workspace_size(16, 4096, 28672, 128) == quant(16, 4096)


@pytest.mark.parametrize("splitk", [0, 2, 3, 5])
@pytest.mark.parametrize("G", [64, 128])
@pytest.mark.parametrize("M,K,N", [(65, 1024, 272), (130, 2304, 48), (200, 512, 1032)])
def test_tiled_split_k(w2, M, K, N, G, splitk):
    # K cut into ranges computed by different workgroups, fp32 partial results summed by a second launch:
    # forced numbers of parts (uneven ranges included) and the planner's own choice (0), both kernels
    tune = {"splitk": splitk}
    codes, scales, X = synth.make_problem(M, K, N, G, 0, M + K + N + G)
    packed = w2.prepack(dev(codes), dev(scales), G, 0)
    ws = torch.empty(16 * M * N * 4, dtype=torch.uint8, device="cuda")
    xq, sx, _ = w2.quantize_rows(dev(X), G)
    Y = w2.matmul_a8(packed, K, N, G, xq, sx, variant=w2.VARIANT_TILED, workspace=ws, tune=tune)
    oq, osx, _ = oracle.quantize_rows(X, G)
    assert np.array_equal(xq.cpu().numpy(), oq)
    Yo, y64 = oracle.matmul_a8(codes, scales, G, 0, oq, osx)
    mag = oracle.a8_term_magnitude(codes, scales, G, 0, oq, osx)
    check_y(bf16_bits(Y), Yo, y64, mag, f"a8 split-K {splitk} M={M} K={K} N={N} G={G}")
    Xb = synth.f32_to_bf16_bits(X)
    Y16 = w2.matmul_a16(packed, K, N, G, dev(Xb).view(torch.bfloat16), workspace=ws, tune=tune)
    Yo, y64, mag = oracle.matmul_a16(codes, scales, G, 0, Xb)
    check_y(bf16_bits(Y16), Yo, y64, mag, f"a16 split-K {splitk} M={M} K={K} N={N} G={G}")
    if splitk >= 2:
        # a workspace too small for two parts: no split, same contract
        small = torch.empty(M * N * 4, dtype=torch.uint8, device="cuda")
        Y1 = w2.matmul_a8(packed, K, N, G, xq, sx, variant=w2.VARIANT_TILED, workspace=small)
        Y0 = w2.matmul_a8(packed, K, N, G, xq, sx, variant=w2.VARIANT_TILED)
        assert torch.equal(Y1.view(torch.int16), Y0.view(torch.int16))


@pytest.mark.parametrize("cbw,splitk", [(2, 2), (4, 3), (8, 2), (2, 5), (0, 0)])
@pytest.mark.parametrize("G", [64, 128])
@pytest.mark.parametrize("M,K,N", [(9, 2304, 272), (33, 5376, 48), (64, 3072, 1032), (100, 2048, 272), (16, 14336, 64)])
def test_midm_split_k(w2, M, K, N, G, cbw, splitk):
    # the mid-M kernel with K cut into ranges of whole 1024-k chunks across workgroups: every workgroup
    # width, forced part counts (uneven ranges, more parts than chunks: clamped), a ragged last chunk that
    # overlaps its predecessor (2304, 5376), two bands of rows, and the planner's own choice (deep K: splits)
    tune = {"midm_cbw": cbw, "splitk": splitk}
    codes, scales, X = synth.make_problem(M, K, N, G, 0, M + K + N + G + cbw)
    packed = w2.prepack(dev(codes), dev(scales), G, 0)
    ws = torch.empty(16 * M * N * 4, dtype=torch.uint8, device="cuda")
    xq, sx, _ = w2.quantize_rows(dev(X), G)
    Y = w2.matmul_a8(packed, K, N, G, xq, sx, variant=w2.VARIANT_MIDM, workspace=ws, tune=tune)
    Y2 = w2.matmul_a8(packed, K, N, G, xq, sx, variant=w2.VARIANT_MIDM, workspace=ws, tune=tune)
    assert torch.equal(Y.view(torch.int16), Y2.view(torch.int16)), "not deterministic"
    oq, osx, _ = oracle.quantize_rows(X, G)
    assert np.array_equal(xq.cpu().numpy(), oq)
    Yo, y64 = oracle.matmul_a8(codes, scales, G, 0, oq, osx)
    mag = oracle.a8_term_magnitude(codes, scales, G, 0, oq, osx)
    check_y(bf16_bits(Y), Yo, y64, mag, f"a8 mid-M split-K {splitk} cbw={cbw} M={M} K={K} N={N} G={G}")
    Xb = synth.f32_to_bf16_bits(X)
    Y16 = w2.matmul_a16(packed, K, N, G, dev(Xb).view(torch.bfloat16), variant=w2.VARIANT_MIDM, workspace=ws, tune=tune)
    Yo, y64, mag = oracle.matmul_a16(codes, scales, G, 0, Xb)
    check_y(bf16_bits(Y16), Yo, y64, mag, f"a16 mid-M split-K {splitk} cbw={cbw} M={M} K={K} N={N} G={G}")
    if splitk >= 2:
        # a workspace too small for two parts: no split, the unsplit kernel's bits
        small = torch.empty(M * N * 4, dtype=torch.uint8, device="cuda")
        Y1 = w2.matmul_a8(packed, K, N, G, xq, sx, variant=w2.VARIANT_MIDM, workspace=small, tune=tune)
        Y0 = w2.matmul_a8(packed, K, N, G, xq, sx, variant=w2.VARIANT_MIDM, tune={"midm_cbw": cbw})
        assert torch.equal(Y1.view(torch.int16), Y0.view(torch.int16))


# ------------------------------------------------------------------ fused epilogues
def check_epilogue(Yg_bits, y64, mag, bias, act, what):
    """Tolerance: the matmul's own (1e-2 relative + 2^-10 of the summed term magnitudes) carried through
    the epilogue: silu has slope <= 1.1, the gated product is bilinear in (silu(gate), up)."""
    Yo, out = oracle.epilogue(y64, bias=bias, act=act)
    yg = bits_to_f64(Yg_bits)
    b = 0.0 if bias is None else synth.bf16_bits_to_f32(bias).astype(np.float64)[None, :]
    z = y64 + b
    dz = 1e-2 * np.abs(y64) + 2.0 ** -10 * mag                      # what the matmul itself may be off by
    if act == 2:
        M, N = z.shape
        zb = z.reshape(M, N // 32, 2, 16)
        db = dz.reshape(M, N // 32, 2, 16)
        g, u = zb[:, :, 0, :].reshape(M, -1), zb[:, :, 1, :].reshape(M, -1)
        dg, du = db[:, :, 0, :].reshape(M, -1), db[:, :, 1, :].reshape(M, -1)
        sg = g / (1.0 + np.exp(-g))
        tol = 1.1 * dg * (np.abs(u) + du) + np.abs(sg) * du + 2.0 ** -8 * np.abs(out)
    else:
        tol = (1.1 if act == 1 else 1.0) * dz + 2.0 ** -8 * np.abs(out)
    bad = np.abs(yg - out) > tol
    assert yg.shape == out.shape and not bad.any(), f"{what}: {bad.sum()} of {bad.size} outputs off"
    # and on the whole it is bf16-accurate: the median error is a fraction of an ulp of the result
    nz = np.abs(out) > 1e-3 * np.abs(out).max()
    assert np.median(np.abs(yg - out)[nz] / np.abs(out)[nz]) < 2.0 ** -8, what


EPI_VARIANTS = [("SMALLM", 2, [1, 3, 16]), ("DOT4", 1, [2]), ("MIDM", 4, [5, 33, 64]), ("TILED", 3, [7, 130])]


@pytest.mark.parametrize("with_bias,act", [(True, 0), (False, 1), (True, 1), (False, 2), (True, 2)])
@pytest.mark.parametrize("G", [64, 128])
@pytest.mark.parametrize("K,N", [(256, 32), (1024, 288), (512, 1056)])
def test_a8_fused_epilogues(w2, K, N, G, with_bias, act):
    # bias and activation applied in the kernels' stores, every kernel family; N = 288, 1056: ragged last workgroup
    rng = np.random.default_rng(K + N + G + act)
    bias = synth.f32_to_bf16_bits(rng.standard_normal(N).astype(np.float32)) if with_bias else None
    bias_d = dev(bias) if with_bias else None
    for name, variant, Ms in EPI_VARIANTS:
        for M in Ms:
            codes, scales, X = synth.make_problem(M, K, N, G, 0, M + K + N)
            packed = w2.prepack(dev(codes), dev(scales), G, 0)
            xq, sx, _ = w2.quantize_rows(dev(X), G)
            oq, osx, _ = oracle.quantize_rows(X, G)
            _, y64 = oracle.matmul_a8(codes, scales, G, 0, oq, osx)
            mag = oracle.a8_term_magnitude(codes, scales, G, 0, oq, osx)
            Y = w2.matmul_a8_epi(packed, K, N, G, xq, sx, bias=bias_d, act=act, variant=variant)
            check_epilogue(bf16_bits(Y), y64, mag, bias, act, f"epilogue {name} M={M} K={K} N={N} G={G} act={act}")


@pytest.mark.parametrize("act", [1, 2])
@pytest.mark.parametrize("M", [1, 2, 4, 5, 8, 40, 130])
def test_a8_fused_entry_with_epilogue_and_split_k(w2, M, act):
    # the one-call entry point (quantisation fused or through the workspace) with bias + activation; for the large M
    # the tiled kernel splits K and the epilogue runs in the reduce launch
    K, N, G = 1024, 320, 128
    tune = {"splitk": 3} if M > 64 else None
    codes, scales, X = synth.make_problem(M, K, N, G, 0, M + act)
    bias = synth.f32_to_bf16_bits(np.random.default_rng(M).standard_normal(N).astype(np.float32))
    packed = w2.prepack(dev(codes), dev(scales), G, 0)
    ws = torch.empty(w2.workspace_size(M, K, N, G) + 4 * M * N * 4, dtype=torch.uint8, device="cuda")
    Y = w2.matmul_a8_fused_epi(packed, K, N, G, dev(X), bias=dev(bias), act=act, workspace=ws, tune=tune)
    oq, osx, _ = oracle.quantize_rows(X, G)
    _, y64 = oracle.matmul_a8(codes, scales, G, 0, oq, osx)
    mag = oracle.a8_term_magnitude(codes, scales, G, 0, oq, osx)
    check_epilogue(bf16_bits(Y), y64, mag, bias, act, f"fused entry + epilogue M={M} act={act}")


A16_EPI_VARIANTS = [("GEMV", 6, [1, 2, 3, 6, 13]), ("SMALLM", 2, [1, 5, 16]), ("SCALED16 small", 5, [3]), ("MIDM", 4, [9, 40, 100]),
                    ("SCALED16 tiled", 5, [130]), ("TILED", 3, [70])]


@pytest.mark.parametrize("with_bias,act", [(True, 0), (False, 1), (True, 2), (False, 2)])
@pytest.mark.parametrize("G", [64, 128])
@pytest.mark.parametrize("K,N", [(256, 32), (1024, 288)])
def test_a16_fused_epilogues(w2, K, N, G, with_bias, act):
    # the same epilogues on the unquantised-activation path, every kernel family, split-K reduce included
    rng = np.random.default_rng(K + N + G + act)
    bias = synth.f32_to_bf16_bits(rng.standard_normal(N).astype(np.float32)) if with_bias else None
    bias_d = dev(bias) if with_bias else None
    for name, variant, Ms in A16_EPI_VARIANTS:
        for M in Ms:
            codes, scales, X = synth.make_problem(M, K, N, G, 0, M + K + N)
            Xb = synth.f32_to_bf16_bits(X)
            packed = w2.prepack(dev(codes), dev(scales), G, 0)
            ws = torch.empty(4 * M * N * 4, dtype=torch.uint8, device="cuda")
            Y = w2.matmul_a16_epi(packed, K, N, G, dev(Xb).view(torch.bfloat16), bias=bias_d, act=act, variant=variant,
                                  workspace=ws, tune={"splitk": 2})
            _, y64, mag = oracle.matmul_a16(codes, scales, G, 0, Xb)
            check_epilogue(bf16_bits(Y), y64, mag, bias, act, f"a16 epilogue {name} M={M} K={K} N={N} G={G} act={act}")


def test_epilogue_argument_errors(w2):
    K, N, G = 256, 48, 128                                   # N % 32 != 0
    codes, scales, X = synth.make_problem(1, K, N, G, 0, 0)
    packed = w2.prepack(dev(codes), dev(scales), G, 0)
    xq, sx, _ = w2.quantize_rows(dev(X), G)
    with pytest.raises(w2.W2Error):
        w2.matmul_a8_epi(packed, K, N, G, xq, sx, act=w2.ACT_SILU_MUL)
    with pytest.raises(w2.W2Error):
        w2.matmul_a8_epi(packed, K, N, G, xq, sx, act=7)
    # no epilogue through the new entry point = the plain call, bit for bit
    Y0 = w2.matmul_a8(packed, K, N, G, xq, sx)
    Y1 = w2.matmul_a8_epi(packed, K, N, G, xq, sx)
    assert torch.equal(Y0.view(torch.int16), Y1.view(torch.int16))


# ------------------------------------------------------------------ w2a16
def run_a16_case(w2, M, K, N, G, codec, variant, seed, tune=None):
    codes, scales, X = synth.make_problem(M, K, N, G, codec, seed)
    Xb = synth.f32_to_bf16_bits(X)
    packed = w2.prepack(dev(codes), dev(scales), G, codec)
    Xd = dev(Xb).view(torch.bfloat16)
    Y = w2.matmul_a16(packed, K, N, G, Xd, variant=variant, tune=tune)
    Y2 = w2.matmul_a16(packed, K, N, G, Xd, variant=variant, tune=tune)
    assert torch.equal(Y.view(torch.int16), Y2.view(torch.int16)), "not deterministic"
    Yo, y64, mag = oracle.matmul_a16(codes, scales, G, codec, Xb)
    check_y(bf16_bits(Y), Yo, y64, mag, f"a16 M={M} K={K} N={N} G={G} codec={codec} variant={variant}")


@pytest.mark.parametrize("G", [64, 128])
@pytest.mark.parametrize("K,N", SMALL_SHAPES)
@pytest.mark.parametrize("M", [1, 4, 7, 16])
def test_a16_smallm(w2, M, K, N, G):
    run_a16_case(w2, M, K, N, G, (M + K) % 2, w2.VARIANT_SMALLM, seed=M + K + N + G)


@pytest.mark.parametrize("shape", [None, (1, 1, 2), (3, 2, 2), (8, 1, 4), (2, 4, 8), (5, 1, 2), (1, 8, 2)])
@pytest.mark.parametrize("G", [64, 128])
@pytest.mark.parametrize("K,N", SMALL_SHAPES + [(5120, 48), (14336, 40)])
@pytest.mark.parametrize("M", [1, 2, 3, 4, 5, 8, 11, 16])
def test_a16_gemv(w2, M, K, N, G, shape):
    # w2a16 through the decode kernel (bf16 rows as they are, bf16 matrix instruction, the group's accumulator
    # started from -130 x the group's row sum): the library's workgroup shape and forced ones (column blocks,
    # K ranges, window), runs of one tile and runs longer than the window, long rows, ragged N; five rows and
    # more: the wide form (every accumulator row in use)
    tune = None
    rl = 1 if M == 1 else 2 if M == 2 else 4 if M <= 4 else 8 if M <= 8 else 16
    slots = 32 if rl > 4 else 16
    lds = 512 + M * (2 * K + 32) + 16 + 8 * rl * 64 + 8 * 16 * (16 * (256 // G) * 2) + (K // G) * (64 if rl > 4 else 16)
    if lds > 160 * 1024 or 512 * (slots // rl) < K // 8:
        pytest.skip("the rows do not fit a workgroup (local memory, registers)")
    if shape is not None:
        cbw, ks, win = shape
        ks = min(ks, K // 256)
        if -(-(K // 256) // ks) > 16 or cbw * ks * 64 * (slots // rl) < K // 8:
            pytest.skip("a run is limited to 16 tiles / the threads must hold the rows")
        tune = {"gemv_cbw": cbw, "gemv_ks": ks, "gemv_window": win}
    run_a16_case(w2, M, K, N, G, (M + K) % 2, w2.VARIANT_GEMV, seed=M + K + N + G, tune=tune)


def test_a16_gemv_exact_integers_and_limits(w2):
    # unit scales, small-integer activations: every product and sum is exact whatever the order
    K, N, G = 4096, 80, 128
    codes, _, _ = synth.make_problem(1, K, N, G, 0, 5)
    ones = np.full((K // G, N), 0x3F80, np.uint16)
    packed = w2.prepack(dev(codes), dev(ones), G, 0)
    rng = np.random.default_rng(1)
    Xi = (rng.integers(-1, 2, size=(16, K)) * (rng.random((16, K)) < 0.05)).astype(np.float32)
    ref = Xi.astype(np.int64) @ (codes.astype(np.int64) - 2)
    assert np.abs(ref).max() < 256
    for M in (1, 2, 4, 6, 8, 13, 16):
        Y = w2.matmul_a16(packed, K, N, G, dev(synth.f32_to_bf16_bits(Xi[:M])).view(torch.bfloat16), variant=w2.VARIANT_GEMV)
        assert np.array_equal(bits_to_f64(bf16_bits(Y)), ref[:M].astype(np.float64))
    # seventeen rows, or rows that do not fit a workgroup: refused when forced (AUTO takes another kernel)
    X5 = torch.zeros((17, K), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(w2.W2Error):
        w2.matmul_a16(packed, K, N, G, X5, variant=w2.VARIANT_GEMV)
    Kb = 28672
    codes, scales, X = synth.make_problem(4, Kb, 16, 128, 0, 6)
    pk = w2.prepack(dev(codes), dev(scales), 128, 0)
    Xd = dev(synth.f32_to_bf16_bits(X)).view(torch.bfloat16)
    with pytest.raises(w2.W2Error):
        w2.matmul_a16(pk, Kb, 16, 128, Xd, variant=w2.VARIANT_GEMV)
    run_a16_case(w2, 4, Kb, 16, 128, 0, w2.VARIANT_AUTO, seed=6)       # ... and AUTO still answers
    run_a16_case(w2, 1, Kb, 16, 128, 0, w2.VARIANT_GEMV, seed=7)       # one such row fits
    run_a16_case(w2, 2, Kb, 24, 64, 1, w2.VARIANT_GEMV, seed=8)        # two rows, G = 64: local memory nearly full
    run_a16_case(w2, 2, 32768, 16, 64, 0, w2.VARIANT_AUTO, seed=9)     # ... and the longest K whose runs fit


@pytest.mark.parametrize("G", [64, 128])
@pytest.mark.parametrize("K,N", [(256, 16), (1024, 272), (512, 1032)])
@pytest.mark.parametrize("M", [1, 17, 127, 128, 200])
def test_a16_tiled(w2, M, K, N, G):
    run_a16_case(w2, M, K, N, G, (M + K) % 2, w2.VARIANT_TILED, seed=M + K + N + G)


@pytest.mark.parametrize("cbw", [0, 2, 4, 8])
@pytest.mark.parametrize("G", [64, 128])
@pytest.mark.parametrize("K,N", [(256, 16), (1024, 272), (768, 1032), (2304, 48)])
@pytest.mark.parametrize("M", [1, 9, 16, 17, 31, 32, 33, 50, 64])
def test_a16_midm(w2, M, K, N, G, cbw):
    # weight stream read once, scale-folded weights; every workgroup shape; K = 768, 2304: chunks that overlap
    run_a16_case(w2, M, K, N, G, (M + K) % 2, w2.VARIANT_MIDM, seed=M + K + N + G, tune={"midm_cbw": cbw})


def test_a16_midm_long_k_and_limits(w2):
    run_a16_case(w2, 40, 14336, 64, 128, 0, w2.VARIANT_MIDM, seed=3)
    K, N, G = 256, 16, 128
    codes, scales, X = synth.make_problem(257, K, N, G, 0, 0)          # more than four bands of 64 rows
    packed = w2.prepack(dev(codes), dev(scales), G, 0)
    with pytest.raises(w2.W2Error):
        w2.matmul_a16(packed, K, N, G, dev(synth.f32_to_bf16_bits(X)).view(torch.bfloat16), variant=w2.VARIANT_MIDM)


@pytest.mark.parametrize("M", [1, 16, 17, 64, 65, 130])
def test_a16_auto_dispatch(w2, M):
    run_a16_case(w2, M, 1024, 528, 128, 0, w2.VARIANT_AUTO, seed=M)


@pytest.mark.parametrize("G", [64, 128])
@pytest.mark.parametrize("K,N", SMALL_SHAPES)
@pytest.mark.parametrize("M", [1, 4, 7, 16])
def test_a16_scale_folded_weights(w2, M, K, N, G):
    # the alternative construction: weights built as sw*q by a byte permute, no dequant step
    run_a16_case(w2, M, K, N, G, (M + K) % 2, w2.VARIANT_SCALED16, seed=M + K + N + G)


@pytest.mark.parametrize("bn", [128, 256])
@pytest.mark.parametrize("G", [64, 128])
@pytest.mark.parametrize("K,N", [(256, 16), (1024, 272), (768, 1032)])
@pytest.mark.parametrize("M", [17, 127, 128, 129, 300])
def test_a16_scale_folded_weights_large_m(w2, M, K, N, G, bn):
    # the same construction in the tiled kernel; both workgroup widths; K = 768 is an odd number of tiles
    run_a16_case(w2, M, K, N, G, (M + K) % 2, w2.VARIANT_SCALED16, seed=M + K + N + G, tune={"tiled_bn": bn})


def test_a16_scale_folded_zero_scales_and_exact_integers(w2):
    # a group with scale 0 contributes exactly nothing (-2 * 0 must not become a denormal), and with
    # unit scales and small-integer activations every product and sum is exact
    K, N, G = 512, 48, 128
    codes, scales, _ = synth.make_problem(1, K, N, G, 0, 3)
    sc = np.full((K // G, N), 0x3F80, np.uint16)
    sc[1, :] = 0                                             # one all-zero group row
    sc[2, ::3] = 0x8000                                      # negative zero as well
    packed = w2.prepack(dev(codes), dev(sc), G, 0)
    rng = np.random.default_rng(1)
    Xi = rng.integers(-2, 3, size=(5, K)).astype(np.float32)
    Y = w2.matmul_a16(packed, K, N, G, dev(synth.f32_to_bf16_bits(Xi)).view(torch.bfloat16), variant=w2.VARIANT_SCALED16)
    sw = synth.bf16_bits_to_f32(sc).astype(np.float64)
    W = (codes.astype(np.int64) - 2) * np.repeat(sw, G, axis=0)
    ref = Xi.astype(np.float64) @ W
    assert np.abs(ref).max() < 256
    assert np.array_equal(bits_to_f64(bf16_bits(Y)), ref)
    # the same through the large-M kernel of this construction (M > 16)
    Xi = rng.integers(-2, 3, size=(150, K)).astype(np.float32)
    Y = w2.matmul_a16(packed, K, N, G, dev(synth.f32_to_bf16_bits(Xi)).view(torch.bfloat16), variant=w2.VARIANT_SCALED16)
    ref = Xi.astype(np.float64) @ W
    assert np.abs(ref).max() < 256
    assert np.array_equal(bits_to_f64(bf16_bits(Y)), ref)


def test_a16_lds_chunking_and_outliers(w2):
    run_a16_case(w2, 16, 14336, 64, 128, 0, w2.VARIANT_SMALLM, seed=5)
    # activation outliers: the 130*X_g cancellation must stay inside the tolerance
    M, K, N, G = 4, 2048, 64, 128
    codes, scales, X = synth.make_problem(M, K, N, G, 0, 21)
    X[:, ::97] *= np.float32(60.0)
    X[2] += np.float32(3.0)                                  # a row with a large mean
    Xb = synth.f32_to_bf16_bits(X)
    packed = w2.prepack(dev(codes), dev(scales), G, 0)
    Y = w2.matmul_a16(packed, K, N, G, dev(Xb).view(torch.bfloat16))
    Yo, y64, mag = oracle.matmul_a16(codes, scales, G, 0, Xb)
    check_y(bf16_bits(Y), Yo, y64, mag, "a16 outliers")


def test_a16_exact_small_integers(w2):
    # unit scales and small-integer activations: every product and sum is exact
    K, N, G = 512, 48, 128
    codes, _, _ = synth.make_problem(1, K, N, G, 1, 2)
    ones = np.full((K // G, N), 0x3F80, np.uint16)
    packed = w2.prepack(dev(codes), dev(ones), G, 1)
    rng = np.random.default_rng(0)
    Xi = rng.integers(-2, 3, size=(3, K)).astype(np.float32)
    Y = w2.matmul_a16(packed, K, N, G, dev(synth.f32_to_bf16_bits(Xi)).view(torch.bfloat16))
    ref = Xi.astype(np.int64) @ (codes.astype(np.int64) - 1)
    assert np.abs(ref).max() < 256
    assert np.array_equal(bits_to_f64(bf16_bits(Y)), ref.astype(np.float64))


@pytest.mark.parametrize("K,N", [(256, 16), (4096, 50), (14336, 129), (1040, 7)])
def test_int8_gemv_comparator_is_exact(w2, K, N):
    # the benchmark's int8-weight GEMV: integer dot products, compared bit for bit
    rng = np.random.default_rng(K + N)
    W8 = rng.integers(-128, 128, size=(N, K), dtype=np.int8)
    xq = rng.integers(-127, 128, size=K, dtype=np.int8)
    out = w2.debug_int8_gemv(dev(W8), dev(xq))
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), (W8.astype(np.int64) @ xq.astype(np.int64)).astype(np.int32))
    with pytest.raises(w2.W2Error):
        w2.debug_int8_gemv(dev(W8[:, :K - 8].copy()), dev(xq[:K - 8].copy()))    # K % 16 != 0


# ------------------------------------------------------------------ argument errors
def test_argument_errors_write_nothing(w2):
    import ctypes
    lib = w2.raw()
    out = ctypes.c_size_t(0)
    assert lib.w2_packed_size(100, 64, 128, ctypes.byref(out)) == w2.ERR_UNSUPPORTED_SHAPE
    assert lib.w2_packed_size(256, 64, 32, ctypes.byref(out)) == w2.ERR_UNSUPPORTED_SHAPE
    assert lib.w2_packed_size(256, 64, 128, None) == w2.ERR_INVALID_ARG
    assert b"multiple of 256" in lib.w2_last_error() or b"NULL" in lib.w2_last_error()
    codes, scales, X = synth.make_problem(1, 256, 64, 128, 0, 0)
    packed = w2.prepack(dev(codes), dev(scales), 128, 0)
    xq, sx, _ = w2.quantize_rows(dev(X))
    Y = torch.full((1, 64), 7.0, dtype=torch.bfloat16, device="cuda")
    s = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    p = lambda t: ctypes.c_void_p(t.data_ptr())
    # misaligned Y, short ldy, forced variant that does not cover M
    assert lib.w2_matmul_a8(p(packed), 256, 64, 128, p(xq), p(sx), 1,
                            ctypes.c_void_p(Y.data_ptr() + 2), 64, None, 0, s) == w2.ERR_MISALIGNED
    assert lib.w2_matmul_a8(p(packed), 256, 64, 128, p(xq), p(sx), 1, p(Y), 32, None, 0, s) == w2.ERR_MISALIGNED
    assert lib.w2_matmul_a8(p(packed), 256, 64, 128, None, p(sx), 1, p(Y), 64, None, 0, s) == w2.ERR_INVALID_ARG
    # overrides outside what the header allows are refused, field by field, before anything is launched
    for field, value in (("variant", 9), ("variant", w2.VARIANT_SCALED16), ("small_waves", 17), ("small_cbw", 3),
                         ("gemv_cbw", 17), ("gemv_ks", -1), ("fused_rows", 9),
                         ("small_kc", 100), ("midm_cbw", 3), ("tiled_bn", 32), ("splitk", 17), ("stream_unroll", 1),
                         ("tiled_group_m", -1)):
        t = w2.Tuning()
        setattr(t, field, value)
        assert lib.w2_matmul_a8_ex(p(packed), 256, 64, 128, p(xq), p(sx), 1, p(Y), 64, None, 0, ctypes.byref(t),
                                   s) == w2.ERR_INVALID_ARG, field
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    t = w2.Tuning()
    t.stream_blocks = 70000
    assert lib.w2_debug_stream_read(p(packed), 1024, p(sink), ctypes.byref(t), s) == w2.ERR_INVALID_ARG
    # M == 0 is a no-op
    assert lib.w2_matmul_a8(p(packed), 256, 64, 128, p(xq), p(sx), 0, p(Y), 64, None, 0, s) == 0
    torch.cuda.synchronize()
    assert torch.all(Y == 7.0)
    with pytest.raises(w2.W2Error):
        w2.matmul_a8(packed, 256, 64, 128, xq.repeat(5, 1), sx.repeat(5), variant=w2.VARIANT_DOT4)


# ------------------------------------------------------------------ HIP graph replays
def test_graph_replays_match_eager(w2):
    """The benchmark replays its steps from HIP graphs: a captured chain (fused call -> gated epilogue call ->
    fused call with bf16 input, a split-K tiled call and a w2a16 call beside it) is replayed several times with
    eager launches and synchronisations in between; every replay must reproduce the eager results bit for bit,
    also after the inputs changed."""
    K, N, G = 1024, 512, 128
    codes, scales, X = synth.make_problem(1, K, N, G, 0, 11)
    packed = w2.prepack(dev(codes), dev(scales), G, 0)
    codes2, scales2, _ = synth.make_problem(1, N // 2, 256, G, 0, 12)
    packed2 = w2.prepack(dev(codes2), dev(scales2), G, 0)
    Mt = 130
    _, _, Xt = synth.make_problem(Mt, K, N, G, 0, 13)
    x_in = dev(X)
    xt = dev(Xt)
    xtb = xt.to(torch.bfloat16)
    ws = torch.empty(w2.workspace_size(Mt, K, N, G) + 4 * Mt * N * 4, dtype=torch.uint8, device="cuda")
    ws16 = torch.empty(4 * Mt * N * 4, dtype=torch.uint8, device="cuda")
    h = torch.empty((1, N // 2), dtype=torch.bfloat16, device="cuda")
    y = torch.empty((1, 256), dtype=torch.bfloat16, device="cuda")
    yt = torch.empty((Mt, N), dtype=torch.bfloat16, device="cuda")
    y16 = torch.empty((Mt, N), dtype=torch.bfloat16, device="cuda")
    if True:
        def step():
            w2.matmul_a8_fused_epi(packed, K, N, G, x_in, act=w2.ACT_SILU_MUL, out=h)
            w2.matmul_a8_fused(packed2, N // 2, 256, G, h, out=y)
            # quantise + tiled split-K + reduce
            w2.matmul_a8_fused_epi(packed, K, N, G, xt, out=yt, workspace=ws, tune={"splitk": 3})
            w2.matmul_a16(packed, K, N, G, xtb, out=y16, workspace=ws16, tune={"splitk": 3})

        def eager():
            step()
            torch.cuda.synchronize()
            return [t.clone() for t in (h, y, yt, y16)]

        ref = eager()
        s = torch.cuda.Stream()
        s.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(s):
            step()                                           # warm-up on the capture stream
        torch.cuda.current_stream().wait_stream(s)
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            step()
        for rep in range(4):
            for t in (h, y, yt, y16):
                t.zero_()                                    # eager work between the replays
            if rep == 2:                                     # new inputs in the same buffers
                x_in.mul_(-0.5)
                xt.add_(0.25)
                xtb.copy_(xt.to(torch.bfloat16))
                ref = eager()
                for t in (h, y, yt, y16):
                    t.zero_()
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            for got, want, name in zip((h, y, yt, y16), ref, ("gated", "chained", "split-K a8", "a16")):
                assert torch.equal(got.view(torch.int16), want.view(torch.int16)), f"replay {rep}: {name} differs from eager"


# ------------------------------------------------------------------ row strides
@pytest.mark.parametrize("M", [1, 3, 5, 40, 100, 130, 300])
def test_row_strides_of_inputs_and_outputs(w2, M):
    """Y with a row stride above N (both paths, every kernel family AUTO reaches, split-K and the gated epilogue
    included) and bf16 X with a row stride above K: the padding columns of Y must stay untouched."""
    K, N, G = 1024, 272, 128
    codes, scales, X = synth.make_problem(M, K, N, G, 0, 100 + M)
    packed = w2.prepack(dev(codes), dev(scales), G, 0)
    xq, sx, _ = w2.quantize_rows(dev(X), G)
    oq, osx, _ = oracle.quantize_rows(X, G)
    Yo, y64 = oracle.matmul_a8(codes, scales, G, 0, oq, osx)
    mag = oracle.a8_term_magnitude(codes, scales, G, 0, oq, osx)
    ws = torch.empty(w2.workspace_size(M, K, N, G) + 3 * M * N * 4, dtype=torch.uint8, device="cuda")
    ldy = N + 40
    big = torch.full((M, ldy), 7.0, dtype=torch.bfloat16, device="cuda")
    w2.matmul_a8(packed, K, N, G, xq, sx, out=big[:, :N], workspace=ws)
    check_y(bf16_bits(big[:, :N].contiguous()), Yo, y64, mag, f"a8 strided Y M={M}")
    assert torch.all(big[:, N:] == 7.0), "a8: columns past N were written"
    # w2a16: strided X and strided Y
    Xb = synth.f32_to_bf16_bits(X)
    xw = torch.zeros((M, K + 64), dtype=torch.bfloat16, device="cuda")
    xw[:, :K] = dev(Xb).view(torch.bfloat16)
    big.fill_(7.0)
    w2.matmul_a16(packed, K, N, G, xw[:, :K], out=big[:, :N], workspace=ws)
    Yo16, y64_16, mag16 = oracle.matmul_a16(codes, scales, G, 0, Xb)
    check_y(bf16_bits(big[:, :N].contiguous()), Yo16, y64_16, mag16, f"a16 strided X and Y M={M}")
    assert torch.all(big[:, N:] == 7.0), "a16: columns past N were written"
    # gated epilogue into a strided output of N/2 columns (N = 288 here: a multiple of 32)
    N2 = 288
    codes2, scales2, _ = synth.make_problem(1, K, N2, G, 0, 200 + M)
    packed2 = w2.prepack(dev(codes2), dev(scales2), G, 0)
    _, y64g = oracle.matmul_a8(codes2, scales2, G, 0, oq, osx)
    magg = oracle.a8_term_magnitude(codes2, scales2, G, 0, oq, osx)
    out = torch.full((M, N2 // 2 + 24), 7.0, dtype=torch.bfloat16, device="cuda")
    w2.matmul_a8_epi(packed2, K, N2, G, xq, sx, act=w2.ACT_SILU_MUL, out=out[:, :N2 // 2], workspace=ws)
    check_epilogue(bf16_bits(out[:, :N2 // 2].contiguous()), y64g, magg, None, 2, f"gated, strided Y M={M}")
    assert torch.all(out[:, N2 // 2:] == 7.0), "gated epilogue: columns past N/2 were written"


@pytest.mark.parametrize("M,K,N", [(1000, 512, 136), (2049, 256, 8), (515, 768, 520)])
def test_large_ragged_m_both_paths(w2, M, K, N):
    # many row tiles with a ragged last one, narrow and ragged N, both tiled kernels (AUTO), G = 64
    G = 64
    run_a8_case(w2, M, K, N, G, 1, w2.VARIANT_AUTO, seed=M + N)
    run_a16_case(w2, M, K, N, G, 1, w2.VARIANT_AUTO, seed=M + N)
