"""Pins for the CPU oracle (no GPU): the oracle is checked against things that
are not itself -- a hand-worked example, numpy int64/fp64 matmuls of the
dequantised operands, closed forms, invariants and exact special cases --
chosen so that a dropped term, a wrong sign/index/zero-point or a transposed
operand fails at least one test."""
import math

import numpy as np
import pytest

import oracle
from paper_2508_06753_amd import synth


def _ints(rows):
    return np.array([[int(v) for v in r] for r in rows])


def _floats(rows):
    return np.array([[float(v) for v in r] for r in rows], dtype=np.float64)


def _hex16(rows):
    return np.array([[int(v, 16) for v in r] for r in rows], dtype=np.uint16)


def _exact_bf16_bits(a):
    """bf16 bits of values that are exactly representable (test data only)."""
    f = np.asarray(a, np.float32)
    bits = (f.view(np.uint32) >> 16).astype(np.uint16)
    assert np.array_equal((bits.astype(np.uint32) << 16).view(np.float32), f)
    return bits


def _q(codes, codec):
    return codes.astype(np.int64) - (2 if codec == 0 else 1)


# ---------------------------------------------------------------- worked example
@pytest.mark.parametrize("codec,name", [(0, "int2"), (1, "ternary")])
def test_worked_example(worked_example, codec, name):
    w = worked_example
    G = int(w["G"][0][0])
    codes = _ints(w[f"codes_{name}"]).astype(np.uint8)
    scales = _exact_bf16_bits(_floats(w["scales"]))
    X = _floats(w["X"]).astype(np.float32)
    xq, sx, gs = oracle.quantize_rows(X, G)
    assert np.array_equal(xq, _ints(w["xq"]))
    assert [float(s).hex() for s in sx] == [float.fromhex(h).hex() for h in w["sx_hex"][0]]
    assert np.array_equal(gs, _ints(w["gsum"]))
    acc = oracle.group_acc(codes, G, codec, xq)
    assert np.array_equal(acc[0], _ints(w[f"acc_{name}_m0"]))
    assert np.array_equal(acc[1], _ints(w[f"acc_{name}_m1"]))
    Y, y64 = oracle.matmul_a8(codes, scales, G, codec, xq, sx)
    np.testing.assert_allclose(y64, _floats(w[f"y_a8_{name}"]), rtol=0, atol=6e-7)
    if name == "int2":
        assert np.array_equal(Y, _hex16(w["Y_a8_int2_bf16"]))
    # the tolerance floor: hand-worked values (numerators over 127; sx is 4/127, 1/127 rounded to fp32)
    tm = oracle.a8_term_magnitude(codes, scales, G, codec, xq, sx)
    np.testing.assert_allclose(tm, _floats(w[f"mag_a8_{name}_times127"]) / 127.0, rtol=1e-7, atol=0)
    Y16, y16, _ = oracle.matmul_a16(codes, scales, G, codec, _exact_bf16_bits(X))
    assert np.array_equal(y16, _floats(w[f"y_a16_{name}"]))        # exact dyadics
    if name == "int2":
        assert np.array_equal(Y16, _hex16(w["Y_a16_int2_bf16"]))


# ---------------------------------------------------------------- bf16 rounding
def test_bf16_rounding_closed_forms():
    f = oracle.f64_to_bf16
    # exactly representable values keep their bits
    assert f(np.array([1.0, -2.0, 0.5, 0.0, 384.0])).tolist() == [0x3F80, 0xC000, 0x3F00, 0, 0x43C0]
    # 1 + 2^-8 is a tie between 1.0 (even) and 1+2^-7 -> even; 1 + 3*2^-8 ties up to even 1+2^-6
    assert f(np.array([1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8])).tolist() == [0x3F80, 0x3F82]
    # just above / below a tie
    assert f(np.array([1 + 2.0 ** -8 + 2.0 ** -40, 1 + 3 * 2.0 ** -8 - 2.0 ** -40])).tolist() == [0x3F81, 0x3F81]
    # a value that double-rounds wrongly via fp32: 1 + 2^-8 + 2^-30 -> fp32 tie-> 1+2^-8 -> bf16 1.0 (wrong);
    # one rounding gives 1+2^-7
    assert f(np.array([1 + 2.0 ** -8 + 2.0 ** -30])).tolist() == [0x3F81]
    # overflow, subnormals, sign of zero, mantissa carry into the exponent
    assert f(np.array([3.4e38 * 1.01, -1e39])).tolist() == [0x7F80, 0xFF80]
    assert f(np.array([2.0 ** -133, 2.0 ** -134, 3 * 2.0 ** -134, -0.0])).tolist() == [1, 0, 2, 0x8000]
    assert f(np.array([1.99999999])).tolist() == [0x4000]
    # round trip of every finite bf16 pattern
    bits = np.arange(0, 0x7F80, dtype=np.uint16)
    vals = (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    assert np.array_equal(f(vals), bits)
    assert np.array_equal(oracle.bf16_to_f32(bits[::37]), vals[::37].astype(np.float32))


def test_synth_bf16_matches_oracle_rounding():
    rng = np.random.default_rng(5)
    a = rng.standard_normal(5000).astype(np.float32) * np.float32(10.0) ** rng.integers(-5, 5, 5000)
    assert np.array_equal(synth.f32_to_bf16_bits(a), oracle.f64_to_bf16(a.astype(np.float64)))


# ---------------------------------------------------------------- quantisation
def test_quantize_properties():
    rng = np.random.default_rng(1)
    X = rng.standard_normal((5, 256)).astype(np.float32)
    X[2] = 0.0                                   # all-zero row
    X[3] *= 1e-3
    xq, sx, gs = oracle.quantize_rows(X, 64)
    assert np.all(xq[2] == 0) and sx[2] == 0.0
    amax = np.abs(X).max(axis=1)
    for m in (0, 1, 3, 4):
        assert np.abs(xq[m]).max() == 127          # the abs-max entry maps to +-127
        assert sx[m] == np.float32(amax[m]) / np.float32(127)
        # within half a step of the real-valued quotient (plus fp32 rounding slack)
        err = np.abs(xq[m].astype(np.float64) - X[m].astype(np.float64) * 127.0 / float(amax[m]))
        assert err.max() <= 0.5 + 1e-4
        assert np.all(np.sign(xq[m]) * np.sign(X[m]) >= 0)
    assert np.array_equal(gs, xq.reshape(5, 4, 64).astype(np.int64).sum(-1))
    # power-of-two scaling of a row changes sx by that factor and leaves xq alone
    xq2, sx2, _ = oracle.quantize_rows(X * np.float32(8.0), 64)
    assert np.array_equal(xq2, xq) and np.array_equal(sx2, sx * np.float32(8.0))
    # negation is antisymmetric (symmetric clamp, half-to-even is odd-symmetric)
    xq3, sx3, _ = oracle.quantize_rows(-X, 64)
    assert np.array_equal(xq3, -xq) and np.array_equal(sx3, sx)


def test_quantize_ties_half_to_even():
    # amax = 127 -> inv = 1 exactly, so t = x and ties are visible
    X = np.array([[127.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 126.5] + [0.0] * 56], np.float32)
    xq, sx, _ = oracle.quantize_rows(X, 64)
    assert xq[0, :8].tolist() == [127, 0, 2, 2, 0, -2, -2, 126]
    assert sx[0] == np.float32(1.0)


def test_quantize_bf16_input_equals_widened_fp32():
    rng = np.random.default_rng(2)
    Xb = synth.f32_to_bf16_bits(rng.standard_normal((3, 128)).astype(np.float32))
    a = oracle.quantize_rows(Xb, 64, x_is_bf16=True)
    b = oracle.quantize_rows(synth.bf16_bits_to_f32(Xb), 64)
    for u, v in zip(a, b):
        assert np.array_equal(u, v)


# ---------------------------------------------------------------- integer part
@pytest.mark.parametrize("codec", [0, 1])
@pytest.mark.parametrize("K,N,G", [(64, 8, 64), (128, 24, 64), (256, 64, 128)])
def test_group_acc_equals_numpy_int64_matmul(codec, K, N, G):
    for seed in range(20):
        codes, scales, X = synth.make_problem(3, K, N, G, codec, seed)
        xq, sx, _ = oracle.quantize_rows(X, G)
        acc = oracle.group_acc(codes, G, codec, xq)
        q = _q(codes, codec)
        ref = np.einsum("mgk,gkn->mgn", xq.astype(np.int64).reshape(3, K // G, G),
                        q.reshape(K // G, G, N))
        assert np.array_equal(acc, ref)


def test_group_acc_operand_order_and_zero_point():
    # one-hot activations pick out single rows of q: catches transposes and a wrong zero-point
    K, N, G = 64, 5, 64
    codes = (np.arange(K * N).reshape(K, N) % 4).astype(np.uint8)
    for k in (0, 7, 63):
        xq = np.zeros((1, K), np.int8)
        xq[0, k] = 3
        assert np.array_equal(oracle.group_acc(codes, G, 0, xq)[0, 0], 3 * (codes[k].astype(int) - 2))
    codes_t = np.minimum(codes, 2)
    xq = np.ones((1, K), np.int8)
    assert np.array_equal(oracle.group_acc(codes_t, G, 1, xq)[0, 0], (codes_t.astype(int) - 1).sum(0))


def test_codec_identity_and_bad_code():
    codes, scales, X = synth.make_problem(2, 128, 16, 64, 1, 3)
    xq, sx, gs = oracle.quantize_rows(X, 64)
    a_t = oracle.group_acc(codes, 64, 1, xq)
    a_i = oracle.group_acc(codes, 64, 0, xq)
    assert np.array_equal(a_t, a_i + gs[:, :, None])        # (c-1) = (c-2) + 1
    codes[5, 3] = 3
    with pytest.raises(oracle.OracleError) as e:
        oracle.group_acc(codes, 64, 1, xq)
    assert e.value.rc == oracle.ERR_BAD_CODE
    assert oracle.check_codes(codes, 0) == 0


def test_all_zero_point_codes_give_zero():
    for codec, z in ((0, 2), (1, 1)):
        codes = np.full((128, 8), z, np.uint8)
        _, scales, X = synth.make_problem(2, 128, 8, 64, codec, 0)
        xq, sx, _ = oracle.quantize_rows(X, 64)
        Y, y64 = oracle.matmul_a8(codes, scales, 64, codec, xq, sx)
        assert np.all(y64 == 0) and np.all(Y == 0)
        Y16, y16, _ = oracle.matmul_a16(codes, scales, 64, codec, synth.f32_to_bf16_bits(X))
        assert np.all(y16 == 0)


# ---------------------------------------------------------------- floating part
@pytest.mark.parametrize("codec", [0, 1])
def test_a8_against_numpy_fp64_dequantised_matmul(codec):
    for seed in range(25):
        rng = np.random.default_rng(seed)
        M = int(rng.integers(1, 5))
        K = int(rng.choice([64, 128, 256]))
        N = int(rng.integers(1, 65))
        G = 64 if K == 64 else int(rng.choice([64, 128]))
        codes, scales, X = synth.make_problem(M, K, N, G, codec, seed)
        xq, sx, _ = oracle.quantize_rows(X, G)
        Y, y64 = oracle.matmul_a8(codes, scales, G, codec, xq, sx)
        sw = synth.bf16_bits_to_f32(scales).astype(np.float64)
        Wd = np.repeat(sw, G, axis=0) * _q(codes, codec)
        Xd = sx.astype(np.float64)[:, None] * xq.astype(np.float64)
        ref = Xd @ Wd                                        # numpy fp64 matmul
        mag = np.abs(Xd) @ np.abs(Wd)
        assert np.all(np.abs(y64 - ref) <= 1e-13 * mag + 1e-300)
        bf = oracle.bruteforce_a8(codes, scales, G, codec, xq, sx)
        assert np.all(np.abs(bf - ref) <= 1e-13 * mag + 1e-300)
        assert np.array_equal(Y, oracle.f64_to_bf16(y64))
        tm = oracle.a8_term_magnitude(codes, scales, G, codec, xq, sx)
        assert np.all(tm <= mag * (1 + 1e-12)) and np.all(tm >= np.abs(y64) * (1 - 1e-12))
        # ... and it IS |sx| * sum_g |sw_g * acc_g|, recomputed with numpy from the integer group sums
        # (checked above against numpy int64); every product sw*acc is exact in fp64 (8 x 17 bits), so only
        # the order of the fp64 additions could differ: g ascending on both sides -> equal to the last bit
        acc = oracle.group_acc(codes, G, codec, xq).astype(np.float64)            # [M][K/G][N]
        terms = np.abs(sw[None, :, :] * acc)
        ref_tm = np.zeros((M, N))
        for g in range(K // G):
            ref_tm += terms[:, g, :]
        ref_tm *= np.abs(sx.astype(np.float64))[:, None]
        assert np.array_equal(tm, ref_tm)
        # the two plausible mistakes do not pass: |.| of the whole sum, |.| per k
        if K // G > 1 and N > 8:
            assert np.any(tm > np.abs(y64) * 1.01) and np.any(tm < mag * 0.99)


@pytest.mark.parametrize("codec", [0, 1])
def test_a16_against_numpy_fp64_matmul(codec):
    for seed in range(25):
        rng = np.random.default_rng(100 + seed)
        M = int(rng.integers(1, 5))
        K = int(rng.choice([64, 128, 256]))
        N = int(rng.integers(1, 65))
        G = 64 if K == 64 else int(rng.choice([64, 128]))
        codes, scales, X = synth.make_problem(M, K, N, G, codec, seed)
        Xb = synth.f32_to_bf16_bits(X)
        Y, y64, mag = oracle.matmul_a16(codes, scales, G, codec, Xb)
        Wd = np.repeat(synth.bf16_bits_to_f32(scales).astype(np.float64), G, axis=0) * _q(codes, codec)
        Xd = synth.bf16_bits_to_f32(Xb).astype(np.float64)
        ref = Xd @ Wd
        refmag = np.abs(Xd) @ np.abs(Wd)
        assert np.all(np.abs(y64 - ref) <= 1e-13 * refmag + 1e-300)
        assert np.all(np.abs(mag - refmag) <= 1e-12 * refmag)
        assert np.array_equal(Y, oracle.f64_to_bf16(y64))


def test_unit_scales_reduce_to_column_sums_and_int_gemm():
    K, N, G = 256, 32, 128
    codes, _, X = synth.make_problem(3, K, N, G, 0, 9)
    ones = np.full((K // G, N), 0x3F80, np.uint16)
    # xq = 1, sx = 1  ->  y = column sums of q (exact small integers)
    xq1 = np.ones((1, K), np.int8)
    Y, y64 = oracle.matmul_a8(codes, ones, G, 0, xq1, np.ones(1, np.float32))
    assert np.array_equal(y64[0], _q(codes, 0).sum(0).astype(np.float64))
    # general xq with unit scales: an ordinary int8 GEMM (numpy int64)
    xq, sx, _ = oracle.quantize_rows(X, G)
    _, y64 = oracle.matmul_a8(codes, ones, G, 0, xq, np.ones(3, np.float32))
    assert np.array_equal(y64, (xq.astype(np.int64) @ _q(codes, 0)).astype(np.float64))


def test_linearity_in_scales_and_row_independence():
    codes, scales, X = synth.make_problem(4, 256, 16, 128, 0, 11)
    xq, sx, _ = oracle.quantize_rows(X, 128)
    Y, y64 = oracle.matmul_a8(codes, scales, 128, 0, xq, sx)
    s2 = scales.copy()
    s2[:, 3] += 0x0080                                  # bf16 exponent + 1: column 3 scales doubled
    Y2, y2 = oracle.matmul_a8(codes, s2, 128, 0, xq, sx)
    assert np.array_equal(y2[:, 3], 2 * y64[:, 3]) and np.array_equal(np.delete(y2, 3, 1), np.delete(y64, 3, 1))
    for m in range(4):
        Ym, _ = oracle.matmul_a8(codes, scales, 128, 0, xq[m:m + 1], sx[m:m + 1])
        assert np.array_equal(Ym[0], Y[m])
    # permuting k inside a group (codes and activations together) leaves acc unchanged
    perm = np.arange(256)
    rng = np.random.default_rng(0)
    perm[:128] = rng.permutation(128)
    perm[128:] = 128 + rng.permutation(128)
    assert np.array_equal(oracle.group_acc(codes[perm], 128, 0, xq[:, perm]),
                          oracle.group_acc(codes, 128, 0, xq))


def test_a8_close_to_unquantised_product_sanity_band():
    # not a pin from the paper (it prints no error bound): int8 absmax noise is about 1 %
    codes, scales, X = synth.make_problem(4, 2048, 64, 128, 0, 4)
    xq, sx, _ = oracle.quantize_rows(X, 128)
    _, y8 = oracle.matmul_a8(codes, scales, 128, 0, xq, sx)
    _, y16, _ = oracle.matmul_a16(codes, scales, 128, 0, synth.f32_to_bf16_bits(X))
    rel_rms = np.sqrt(np.mean((y8 - y16) ** 2) / np.mean(y16 ** 2))
    assert rel_rms < 0.03


# ------------------------------------------------------------------ fused epilogue (Sec. II-D)
def test_epilogue_silu_closed_forms_and_identities():
    z = np.array([[0.0, 1.0, -1.0, 30.0, -30.0, 0.5, -0.5, 2.0]], np.float64)
    _, out = oracle.epilogue(z, act=1)
    assert out[0, 0] == 0.0                                        # silu(0) = 0
    assert abs(out[0, 1] - 1.0 / (1.0 + math.e ** -1.0)) < 1e-15   # silu(1) = 1 / (1 + 1/e)
    assert abs(out[0, 3] - 30.0) < 1e-11 and abs(out[0, 4]) < 1e-11   # x for large x, 0 for very negative x
    # silu(x) - silu(-x) = x, and silu(x) + silu(-x) = x tanh(x/2)
    assert np.allclose(out[0, 1] - out[0, 2], 1.0, atol=1e-15) and np.allclose(out[0, 5] - out[0, 6], 0.5, atol=1e-15)
    assert np.allclose(out[0, 1] + out[0, 2], np.tanh(0.5), atol=1e-15)
    # slope 1/2 at the origin (a dropped factor or a sign error in the exponent changes it)
    h = 1e-6
    _, d = oracle.epilogue(np.array([[h, -h]], np.float64), act=1)
    assert abs((d[0, 0] - d[0, 1]) / (2 * h) - 0.5) < 1e-9
    # no activation: identity, one rounding to bf16
    Y, same = oracle.epilogue(z, act=0)
    assert np.array_equal(same, z) and np.array_equal(Y, oracle.f64_to_bf16(z))


def test_epilogue_bias_and_gated_layout_by_brute_force():
    rng = np.random.default_rng(5)
    M, N = 3, 64
    y = rng.standard_normal((M, N))
    bias_f = rng.standard_normal(N).astype(np.float32)
    bias = synth.f32_to_bf16_bits(bias_f)
    b64 = synth.bf16_bits_to_f32(bias).astype(np.float64)
    _, out = oracle.epilogue(y, bias=bias, act=0)
    assert np.array_equal(out, y + b64[None, :])                   # bias is per column, added before anything else
    Y, out = oracle.epilogue(y, bias=bias, act=2)
    assert out.shape == (M, N // 2)
    for m in range(M):
        for no in range(N // 2):
            b, l = divmod(no, 16)
            g = y[m, 32 * b + l] + b64[32 * b + l]                 # gate: even 16-column block
            u = y[m, 32 * b + 16 + l] + b64[32 * b + 16 + l]       # up: the odd block after it
            ref = g / (1.0 + math.exp(-g)) * u
            assert abs(out[m, no] - ref) <= 1e-15 * max(1.0, abs(ref))
    assert np.array_equal(Y, oracle.f64_to_bf16(out))
    # gate = 0 gives 0 whatever up is; swapping the two blocks changes the result (not symmetric)
    y0 = y.copy(); y0[:, 0:16] = 0.0
    _, o0 = oracle.epilogue(y0, act=2)
    assert np.all(o0[:, 0:16] == 0.0)
    ys = y.copy(); ys[:, 0:16], ys[:, 16:32] = y[:, 16:32].copy(), y[:, 0:16].copy()
    _, o1 = oracle.epilogue(ys, act=2)
    _, o2 = oracle.epilogue(y, act=2)
    assert not np.allclose(o1[:, 0:16], o2[:, 0:16])
    with pytest.raises(oracle.OracleError):
        oracle.epilogue(np.zeros((1, 48)), act=2)                  # N must be a multiple of 32
