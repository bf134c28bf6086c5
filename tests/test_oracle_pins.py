"""Pins for the CPU oracle: it is checked against things other than itself.

Hand-worked instances of Eq. 2, closed forms, invariants stated in the paper,
numpy's int64 matmul as a library special case, and an fp64 group-wise
("segmented GEMM", Fig. 2(b)) reference that must agree with the dual-grained
result because S = s1 * S2 (Eq. 5).  No GPU needed.
"""
import json
import os

import numpy as np
import pytest

import oracle
import workloads

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _tiny():
    with open(os.path.join(GOLDEN, "tiny_case.json")) as f:
        return json.load(f)


# ----------------------------------------------------------------------------
# P1: hand-worked instance of Eq. 2
# ----------------------------------------------------------------------------
def test_tiny_case_expand_gemm_epilogue():
    t = _tiny()
    g = t["group"]
    xq = np.array(t["xq"], np.int8)
    w4 = np.array(t["w4"], np.int8)
    s2 = np.array(t["s2"], np.uint8)
    ws8, bad = oracle.expand(w4, s2, g)
    assert bad == 0
    assert ws8.tolist() == t["ws8"]
    acc, wrapped = oracle.gemm_i32(xq, ws8)
    assert wrapped == 0
    assert acc.tolist() == t["acc"]
    out = oracle.epilogue(acc, np.array(t["sx"], np.float32), np.array(t["s1"], np.float32))
    assert out.dtype == np.float16
    # -1079.5 is a tie between fp16 neighbours 1079 and 1080 -> even (1080)
    assert out.astype(np.float64).tolist() == t["out_fp16"]
    out2, acc2 = oracle.linear_a8w4(xq, np.array(t["sx"], np.float32), w4, s2,
                                    np.array(t["s1"], np.float32), g)
    assert np.array_equal(out2, out) and np.array_equal(acc2, acc)


def test_expand_table_properties():
    """All 16 x 15 (nibble, scale) pairs: zero at the zero point, step s2 per nibble step,
    extreme values -120 and 105, everything inside INT8 (range constraint beside Eq. 4)."""
    # row k holds nibble value k - 8, column n holds scale n + 1; test-only group size 1
    w4 = np.repeat(np.arange(-8, 8, dtype=np.int8)[:, None], 15, axis=1)   # [16, 15]
    s2 = np.repeat(np.arange(1, 16, dtype=np.uint8)[None, :], 16, axis=0)  # [16, 15]
    ws8, bad = oracle.expand(w4, s2, 1)
    assert bad == 0
    t = ws8.astype(np.int64)
    assert (t[8] == 0).all()                      # w4 = 0 row
    assert (np.diff(t, axis=0) == np.arange(1, 16)[None, :]).all()
    assert t[0, 14] == -120 and t[15, 14] == 105 and t[0, 0] == -8 and t[15, 0] == 7
    assert t.min() >= -128 and t.max() <= 127


def test_expand_flags_values_outside_int8():
    # relaxed scales (Appendix B allows S2 > 15): 20 * -8 = -160 does not fit
    w4 = np.array([[-8], [6], [7], [0]], np.int8)
    s2 = np.array([[20]], np.uint8)
    ws8, bad = oracle.expand(w4, s2, 4)
    assert bad == 2  # -160 and 140; 120 fits
    assert ws8[:, 0].tolist() == [-128, 120, 127, 0]


# ----------------------------------------------------------------------------
# P3: GEMM against numpy's int64 matmul and a differently ordered loop
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("M,K,N", [(1, 8, 1), (3, 64, 5), (17, 256, 33), (8, 1024, 48)])
def test_gemm_matches_numpy_int64(M, K, N):
    rng = np.random.default_rng(M * 1000 + N)
    xq = rng.integers(-127, 128, size=(M, K), dtype=np.int8)
    ws8 = rng.integers(-128, 128, size=(K, N), dtype=np.int8)
    acc, wrapped = oracle.gemm_i32(xq, ws8)
    assert wrapped == 0
    ref = xq.astype(np.int64) @ ws8.astype(np.int64)
    assert np.array_equal(acc.astype(np.int64), ref)
    # transposed-operand pin: (A B)^T = B^T A^T catches a transposed operand or swapped index
    acc_t, _ = oracle.gemm_i32(np.ascontiguousarray(ws8.T), np.ascontiguousarray(xq.T))
    assert np.array_equal(acc_t, acc.T)


def test_gemm_python_loops_k_outer():
    rng = np.random.default_rng(5)
    M, K, N = 3, 12, 4
    xq = rng.integers(-127, 128, size=(M, K), dtype=np.int8)
    ws8 = rng.integers(-128, 128, size=(K, N), dtype=np.int8)
    ref = [[0] * N for _ in range(M)]
    for k in range(K):            # different loop order from the oracle's m-n-k
        for n in range(N):
            for m in range(M):
                ref[m][n] += int(xq[m, k]) * int(ws8[k, n])
    acc, _ = oracle.gemm_i32(xq, ws8)
    assert acc.tolist() == ref


def test_gemm_extreme_magnitude_no_wrap_at_max_K():
    # |acc| <= 127*128*K; K = 22016 (largest LLaMA-65B K) stays far inside INT32
    K = 22016
    xq = np.full((1, K), -127, np.int8)
    ws8 = np.full((K, 1), -128, np.int8)
    acc, wrapped = oracle.gemm_i32(xq, ws8)
    assert wrapped == 0 and int(acc[0, 0]) == 127 * 128 * K


def test_gemm_reports_int32_wrap():
    K = 140000  # 127*127*140000 > 2^31
    xq = np.full((1, K), 127, np.int8)
    ws8 = np.full((K, 1), 127, np.int8)
    _, wrapped = oracle.gemm_i32(xq, ws8)
    assert wrapped == 1


# ----------------------------------------------------------------------------
# P4: closed forms
# ----------------------------------------------------------------------------
def test_closed_forms():
    g, K, N, M = 8, 32, 6, 4
    w4, s2, s1 = workloads.integer_weights(K, N, g, 3)
    ones_x = np.ones((M, K), np.int8)
    sx = np.ones(M, np.float32)
    # (i) xq = 1, w4 = 1  =>  acc = g * sum_j s2[j, n]
    _, acc = oracle.linear_a8w4(ones_x, sx, np.ones((K, N), np.int8), s2, s1, g)
    assert np.array_equal(acc, np.broadcast_to(g * s2.astype(np.int64).sum(0), (M, N)))
    # (ii) s2 = 1  =>  plain INT8 GEMM of the nibble matrix
    xq, _ = workloads.integer_activations(M, K, 4)
    _, acc = oracle.linear_a8w4(xq, sx, w4, np.ones_like(s2), s1, g)
    assert np.array_equal(acc.astype(np.int64), xq.astype(np.int64) @ w4.astype(np.int64))
    # (iii) one-hot activations read out rows of W_s8
    eye = np.eye(K, dtype=np.int8)
    _, acc = oracle.linear_a8w4(eye, np.ones(K, np.float32), w4, s2, s1, g)
    ws8 = np.repeat(s2.astype(np.int64), g, axis=0) * w4.astype(np.int64)
    assert np.array_equal(acc.astype(np.int64), ws8)


# ----------------------------------------------------------------------------
# P5: dual-grained == group-wise quantization with S = s1 * S2 (Eq. 5, Fig. 2(b)/(c))
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("g", [64, 128])
def test_matches_fp64_segmented_groupwise_reference(g):
    M, K, N = 5, 512, 24
    x = workloads.activations(M, K, 11)
    W = workloads.weights(K, N, 11)
    w4, s2, s1 = oracle.quantize_weights_rtn(W, g)
    out, acc, xq, sx = oracle.forward(x, w4, s2, s1, g)
    # segmented GEMM: one integer product per group, combined in floating point
    xhat = sx.astype(np.float64)[:, None] * xq.astype(np.float64)
    ref = np.zeros((M, N))
    for j in range(K // g):
        S = s1.astype(np.float64) * s2[j].astype(np.float64)             # fp group-wise scale
        part = xhat[:, j * g:(j + 1) * g] @ w4[j * g:(j + 1) * g].astype(np.float64)
        ref += part * S[None, :]
    dgq = (sx.astype(np.float64)[:, None] * s1.astype(np.float64)[None, :]) * acc.astype(np.float64)
    assert np.allclose(dgq, ref, rtol=1e-12, atol=1e-12)
    # and the fp16 output is that value up to one fp32 product rounding pair and one fp16 rounding
    assert np.allclose(out.astype(np.float64), ref, rtol=2 ** -10, atol=2 ** -24)


def test_epilogue_order_and_rounding():
    # scale product first, then times acc (Eq. 2 line 1, then line 3), in fp32, one fp16 rounding
    acc = np.array([[3, -7], [2 ** 24 + 1, 100]], np.int32)   # 2^24+1 is not an fp32 number
    sx = np.array([0.1, 3.0], np.float32)
    s1 = np.array([3e-5, 2.0 ** -20], np.float32)
    out = oracle.epilogue(acc, sx, s1)
    exp = np.empty((2, 2), np.float16)
    for m in range(2):
        for n in range(2):
            s = np.float32(sx[m]) * np.float32(s1[n])
            exp[m, n] = np.float16(np.float32(s) * np.float32(acc[m, n]))
    assert np.array_equal(out.view(np.uint16), exp.view(np.uint16))
    # overflow goes to inf (IEEE), not saturation
    big = oracle.epilogue(np.array([[2 ** 30]], np.int32), np.ones(1, np.float32), np.ones(1, np.float32))
    assert np.isinf(big[0, 0])


# ----------------------------------------------------------------------------
# P6: per-token activation quantizer (Section 3.1 symmetric case)
# ----------------------------------------------------------------------------
def test_quant_act_hand_example_ties_to_even():
    # a = 127 -> inv = 1 exactly, so the rounding rule is visible on the halves
    row = np.array([[127, 0.5, 1.5, 2.5, -0.5, -2.5, 3.5, -126.5]], np.float16)
    xq, sx = oracle.quant_act(row)
    assert xq[0].tolist() == [127, 0, 2, 2, 0, -2, 4, -126]
    assert sx[0] == np.float32(1.0)
    row = np.array([[0.5, -1.0, 0.25, 2.0]], np.float16)   # inv = 63.5
    xq, sx = oracle.quant_act(row)
    assert xq[0].tolist() == [32, -64, 16, 127]
    assert sx[0] == np.float32(2.0) / np.float32(127.0)


def test_quant_act_invariants():
    M, K = 9, 640
    x = workloads.activations(M, K, 2)
    xq, sx = oracle.quant_act(x)
    xf = x.astype(np.float64)
    amax = np.abs(xf).max(1)
    # the largest element maps to +-127 and the scale is absmax/127
    am = np.abs(xf).argmax(1)
    assert (np.abs(xq[np.arange(M), am].astype(int)) == 127).all()
    assert np.allclose(sx, amax / 127.0, rtol=1e-6)
    assert xq.min() >= -127 and xq.max() <= 127
    # reconstruction error at most half a step
    err = np.abs(xf - sx.astype(np.float64)[:, None] * xq.astype(np.float64))
    assert (err <= 0.5 * sx.astype(np.float64)[:, None] * (1 + 1e-5)).all()
    # sign symmetry and exact power-of-two scaling
    xq_n, sx_n = oracle.quant_act(-x)
    assert np.array_equal(xq_n, -xq) and np.array_equal(sx_n, sx)
    xq2, sx2 = oracle.quant_act((x.astype(np.float32) * 4).astype(np.float16))
    ok = np.abs(xf).max(1) * 4 < 65504
    assert np.array_equal(xq2[ok], xq[ok]) and np.array_equal(sx2[ok], sx[ok] * 4)
    # rows are independent: permuting rows permutes results
    xq_p, sx_p = oracle.quant_act(x[::-1].copy())
    assert np.array_equal(xq_p, xq[::-1]) and np.array_equal(sx_p, sx[::-1])


def test_quant_act_zero_row_and_single_token():
    x = np.zeros((2, 64), np.float16)
    x[1, 5] = -3.0
    xq, sx = oracle.quant_act(x)
    assert (xq[0] == 0).all() and sx[0] == 0.0
    assert xq[1, 5] == -127 and np.count_nonzero(xq[1]) == 1


# ----------------------------------------------------------------------------
# P7: RTN dual-grained weight quantizer
# ----------------------------------------------------------------------------
def test_weight_quantizer_hand_example():
    # column 0: group 0 absmax 7 -> S' = 1, group 1 absmax 1.4 -> S' = 0.2; s1 = 1/15;
    # s2 = [15, 3]; S = [1.0, 0.2]
    W = np.array([[7.0], [-3.4], [1.2], [0.0], [1.4], [-0.6], [0.32], [0.12]], np.float32)
    w4, s2, s1 = oracle.quantize_weights_rtn(W, 4)
    assert s2[:, 0].tolist() == [15, 3]
    assert w4[:, 0].tolist() == [7, -3, 1, 0, 7, -3, 2, 1]
    assert abs(float(s1[0]) - 1.0 / 15.0) < 1e-8


def test_weight_quantizer_negative_clip_and_zero_column():
    # S' = 0.8/7, 1.0/7 -> s1 = 1/105, s2 = round(12) = 12, 15.  A value of -0.8 in a group
    # whose positive max is also 0.8 maps to -7; the nibble range is [-8, 7]
    W = np.zeros((8, 2), np.float32)
    W[:, 0] = [0.8, -0.8, 0.1, 0.0, 1.0, -1.0, 0.55, 0.0]
    w4, s2, s1 = oracle.quantize_weights_rtn(W, 4)
    assert s2[:, 0].tolist() == [12, 15]
    assert w4[:, 0].tolist() == [7, -7, 1, 0, 7, -7, 4, 0]   # 0.55/(1/7) = 3.85 -> 4
    assert s1[1] == 1.0 and (s2[:, 1] == 1).all() and (w4[:, 1] == 0).all()


@pytest.mark.parametrize("g", [64, 128])
def test_weight_quantizer_invariants(g):
    K, N = 1024, 96
    W = workloads.weights(K, N, 7)
    w4, s2, s1 = oracle.quantize_weights_rtn(W, g)
    assert w4.min() >= -8 and w4.max() <= 7 and s2.min() >= 1 and s2.max() <= 15
    Wf = W.astype(np.float64)
    absmax = np.abs(Wf).reshape(K // g, g, N).max(1)          # [ng, N]
    # the group with the largest S' of each column gets scale 15
    assert (s2[absmax.argmax(0), np.arange(N)] == 15).all()
    assert np.allclose(s1, absmax.max(0) / 7.0 / 15.0, rtol=1e-6)
    S = np.repeat(s1.astype(np.float64)[None, :] * s2.astype(np.float64), g, axis=0)
    deq = S * w4
    clipped = (w4 == -8) | (w4 == 7)
    assert (np.abs(Wf - deq)[~clipped] <= 0.5 * S[~clipped] * (1 + 1e-5)).all()
    # expanded weights satisfy the INT8 constraint (beside Eq. 4) with room: |W_s8| <= 120
    ws8, bad = oracle.expand(w4, s2, g)
    assert bad == 0 and np.abs(ws8.astype(int)).max() <= 120
    # s2 is the rounded ratio of the group-wise scale to s1 (Eq. 5)
    ratio = (absmax / 7.0) / s1.astype(np.float64)[None, :]
    assert (np.abs(s2 - np.clip(ratio, 1, 15)) <= 0.5 + 1e-4).all()


# ----------------------------------------------------------------------------
# P8: packed device format
# ----------------------------------------------------------------------------
def test_pack_hand_offsets():
    with open(os.path.join(GOLDEN, "layout_offsets.json")) as f:
        lay = json.load(f)
    K, N, g = lay["K"], lay["N"], lay["group"]
    qb, sb = oracle.packed_sizes(K, N, g)
    assert qb == K * N // 2 and sb == lay["scales_bytes"]
    for e in lay["qweight"]:
        w4 = np.full((K, N), -8, np.int8)           # stored nibble 0 everywhere
        w4[e["k"], e["n"]] = 5                       # stored nibble 13 at one spot
        qw, sc, bad = oracle.pack(w4, np.ones((K // g, N), np.uint8), g)
        assert bad == 0
        nz = np.flatnonzero(qw)
        assert nz.tolist() == [e["byte"]]
        assert qw[e["byte"]] == (13 << 4 if e["high_nibble"] else 13)
    for e in lay["scales"]:
        s2 = np.ones((K // g, N), np.uint8)
        s2[e["gi"], e["n"]] = 9
        qw, sc, bad = oracle.pack(np.zeros((K, N), np.int8), s2, g)
        assert np.flatnonzero(sc == 9).tolist() == [e["byte"]]
        assert (qw == 0x88).all()                    # w4 = 0 -> nibble 8 in both halves


@pytest.mark.parametrize("K,N,g", [(128, 16, 128), (256, 48, 64), (768, 32, 128), (640, 16, 64)])
def test_pack_roundtrip_and_padding(K, N, g):
    w4, s2, _ = workloads.integer_weights(K, N, g, K + N)
    qw, sc, bad = oracle.pack(w4, s2, g)
    assert bad == 0
    w4b, s2b = oracle.unpack(qw, sc, K, N, g)
    assert np.array_equal(w4b, w4) and np.array_equal(s2b, s2)
    # every (group, column) byte is used once; the rest is zero padding
    assert np.count_nonzero(sc) == s2.size
    # a permutation of nibbles: multiset of stored nibbles == multiset of w4 + 8
    nib = np.concatenate([qw & 15, qw >> 4])
    assert np.array_equal(np.bincount(nib, minlength=16), np.bincount((w4 + 8).ravel(), minlength=16))


def test_pack_counts_out_of_range_inputs():
    K, N, g = 128, 16, 128
    w4 = np.zeros((K, N), np.int8)
    s2 = np.ones((1, N), np.uint8)
    w4[3, 3] = 8
    w4[4, 4] = -9
    s2[0, 5] = 0
    s2[0, 6] = 16
    qw, sc, bad = oracle.pack(w4, s2, g)
    assert bad == 4
    w4b, s2b = oracle.unpack(qw, sc, K, N, g)
    assert w4b[3, 3] == 0 and w4b[4, 4] == 0 and s2b[0, 5] == 1 and s2b[0, 6] == 1


# ----------------------------------------------------------------------------
# config 0 of the benchmark definition end to end (oracle finishes in seconds)
# ----------------------------------------------------------------------------
def test_config0_end_to_end_properties():
    M, K, N, g = 8, 1024, 1024, 128
    x = workloads.activations(M, K, 0)
    W = workloads.weights(K, N, 0)
    w4, s2, s1 = oracle.quantize_weights_rtn(W, g)
    out, acc, xq, sx = oracle.forward(x, w4, s2, s1, g)
    assert out.shape == (M, N) and out.dtype == np.float16 and np.isfinite(out).all()
    ws8, _ = oracle.expand(w4, s2, g)
    assert np.array_equal(acc.astype(np.int64), xq.astype(np.int64) @ ws8.astype(np.int64))
    # the quantized layer approximates the fp product of the same operands: the error is
    # dominated by the INT8 activation step (outlier channels set a coarse per-token scale)
    ref = x.astype(np.float64) @ W.astype(np.float64)
    rel = np.linalg.norm(out.astype(np.float64) - ref) / np.linalg.norm(ref)
    assert rel < 0.35
    # without outliers the same layer is accurate to a few percent
    x0 = workloads.activations(M, K, 0, outlier_frac=0.0)
    out0, *_ = oracle.forward(x0, w4, s2, s1, g)
    ref0 = x0.astype(np.float64) @ W.astype(np.float64)
    assert np.linalg.norm(out0.astype(np.float64) - ref0) / np.linalg.norm(ref0) < 0.12


# ---------------------------------------------------------------- static activation scale
def test_quant_act_static_hand_values():
    # scale 0.5: 0.74/0.5 = 1.48 -> 1; 0.76 -> 1.52 -> 2; ties to even: 1.25 -> 2.5 -> 2, 1.75 -> 3.5 -> 4;
    # saturation: 100 -> 200 -> 127, -64 -> -128 -> -127; signs are symmetric
    x = np.array([[0.74, 0.76, 1.25, 1.75, 100.0, -64.0, -0.76, 0.0]], np.float32)
    xq, sx = oracle.quant_act_static(x, 0.5)
    assert xq.tolist() == [[1, 2, 2, 4, 127, -127, -2, 0]] and sx.tolist() == [0.5]


def test_quant_act_static_equals_dynamic_when_the_scale_is_exact():
    # a row whose absmax is 127 * 2^-5 has the dynamic scale 2^-5 exactly, and both x * (127/a) and
    # x / s are then exact scalings by 32: the two quantizers must agree
    rng = np.random.default_rng(8)
    x = rng.normal(0, 1, (6, 512)).astype(np.float16).astype(np.float32)
    x = np.clip(x, -3.9, 3.9)
    x[:, 17] = 127 * 2.0 ** -5
    xd, sd = oracle.quant_act(x)
    xs, ss = oracle.quant_act_static(x, 2.0 ** -5)
    assert (sd == np.float32(2.0 ** -5)).all() and np.array_equal(xd, xs) and np.array_equal(sd, ss)


def test_quant_act_static_error_bound_and_saturation():
    rng = np.random.default_rng(9)
    x = rng.normal(0, 1, (4, 2048)).astype(np.float16).astype(np.float32)
    s = np.float32(0.02)
    xq, _ = oracle.quant_act_static(x, float(s))
    inside = np.abs(x) <= 127 * s
    assert (np.abs(x - s * xq)[inside] <= 0.5 * s * (1 + 1e-6)).all()
    assert (np.abs(xq[~inside]) == 127).all() and (np.sign(xq[~inside]) == np.sign(x[~inside])).all()


# ---------------------------------------------------------------- gated-MLP producer
def test_silu_mul_hand_values_and_fp16_rounding():
    # silu(0) = 0; silu(g) -> g for large g, -> 0 for very negative g; silu(1) = 0.7310585786...
    GU = np.array([[0.0, 1.0, 20.0, -20.0, 2.0,   3.0, 2.0, 0.5, 4.0, -1.5]], np.float32)
    h = oracle.silu_mul(GU)
    assert h[0, 0] == 0
    assert h[0, 1] == np.float16(0.7310585786300049 * 2.0)
    assert h[0, 2] == np.float16(10.0)                      # 20 * (1 - 2e-9) * 0.5
    assert abs(float(h[0, 3])) < 1e-6                       # -20 * e^-20 * 4: a subnormal fp16 or zero
    assert h[0, 4] == np.float16(-1.5 * 2.0 / (1.0 + np.exp(-2.0)))


def test_silu_mul_equals_numpy_fp64_then_two_roundings():
    rng = np.random.default_rng(14)
    GU = (rng.normal(0, 2, (5, 512)) * rng.choice([1e-3, 1, 8], (5, 512))).astype(np.float16)
    g, u = GU[:, :256].astype(np.float64), GU[:, 256:].astype(np.float64)
    ref = ((g / (1.0 + np.exp(-g))) * u).astype(np.float32).astype(np.float16)
    assert np.array_equal(oracle.silu_mul(GU).view(np.uint16), ref.view(np.uint16))


def test_rmsnorm_hand_values_and_numpy_fp64():
    # a row of +-3 has mean square 9: y = x / 3 * gamma exactly (eps = 0)
    x = np.array([[3, -3, 3, -3]], np.float16)
    y = oracle.rmsnorm(x, np.array([1, 2, 0.5, 4], np.float16), 0.0)
    assert y.tolist() == [[1.0, -2.0, 0.5, -4.0]]
    rng = np.random.default_rng(15)
    x = (rng.normal(0, 1, (6, 384)) * rng.choice([0.05, 1, 30], (6, 1))).astype(np.float16)
    gamma = rng.normal(1, 0.2, 384).astype(np.float16)
    x64, g64 = x.astype(np.float64), gamma.astype(np.float64)
    eps = 1e-5
    ref = (x64 / np.sqrt((x64 ** 2).mean(axis=1, keepdims=True) + np.float64(np.float32(eps))) * g64)
    ref = ref.astype(np.float32).astype(np.float16)
    got = oracle.rmsnorm(x, gamma, eps)
    # numpy's pairwise mean and x/sqrt differ from 1/sqrt and a running sum in the last fp64 bits only:
    # after two roundings at most a handful of ties can differ, and on this data none does
    assert np.array_equal(got.view(np.uint16), ref.view(np.uint16))


# ---------------------------------------------------------------- batched INT8 product for attention (Section 4.1)
def test_bmm_hand_worked_case():
    """Two batches of a 2 x 3 by 2 x 3 product, sums written out by hand: batch 0 row 0 = (1, -2, 3) against
    (4, 5, -6) -> 4 - 10 - 18 = -24 and against (-1, 0, 2) -> -1 + 0 + 6 = 5; a swapped operand, a product along
    the wrong axis or batches mixed up change at least one of the eight numbers."""
    a = np.array([[[1, -2, 3], [0, 7, -1]], [[127, -127, 1], [2, 2, 2]]], np.int8)
    b = np.array([[[4, 5, -6], [-1, 0, 2]], [[127, 127, -128], [-3, 4, 5]]], np.int8)
    acc, wrapped = oracle.bmm_s8_acc(a, b)
    assert wrapped == 0
    assert acc.tolist() == [[[-24, 5], [41, -2]], [[-128, -884], [252, 12]]]
    # scale epilogue: (sa[m] * sb[n]) * acc with power-of-two scales is exact
    sa = np.array([[0.5, 2.0], [1.0, 0.25]], np.float32)
    sb = np.array([[1.0, 4.0], [0.125, 2.0]], np.float32)
    out, _ = oracle.bmm_s8(a, b, sa, sb)
    assert out.dtype == np.float16
    assert out.tolist() == [[[-12.0, 10.0], [82.0, -16.0]], [[-16.0, -1768.0], [7.875, 6.0]]]


def test_bmm_against_numpy_int64_one_hot_and_the_pinned_gemm():
    rng = np.random.default_rng(5)
    B, M, N, K = 3, 17, 29, 200
    a = rng.integers(-128, 128, (B, M, K), dtype=np.int8)
    b = rng.integers(-128, 128, (B, N, K), dtype=np.int8)
    acc, wrapped = oracle.bmm_s8_acc(a, b)
    assert wrapped == 0
    assert np.array_equal(acc.astype(np.int64), np.einsum("bmk,bnk->bmn", a.astype(np.int64), b.astype(np.int64)))
    # each batch is the (separately pinned) GEMM of Eq. 2 on the transposed second operand
    for i in range(B):
        g, _ = oracle.gemm_i32(a[i], np.ascontiguousarray(b[i].T))
        assert np.array_equal(acc[i], g)
    # swapping the operands transposes the result; permuting the batches permutes it
    acc_t, _ = oracle.bmm_s8_acc(b, a)
    assert np.array_equal(acc_t, acc.transpose(0, 2, 1))
    perm = [2, 0, 1]
    assert np.array_equal(oracle.bmm_s8_acc(a[perm], b[perm])[0], acc[perm])
    # one-hot rows of the second operand read out columns of the first
    e = np.zeros((B, 4, K), np.int8)
    ks = [3, 77, 199, 0]
    for j, k in enumerate(ks):
        e[:, j, k] = 1
    assert np.array_equal(oracle.bmm_s8_acc(a, e)[0], a[:, :, ks].astype(np.int32))


def test_bmm_reports_int32_wrap():
    K = 140000                                         # 128 * 128 * K > 2^31
    a = np.full((1, 1, K), -128, np.int8)
    acc, wrapped = oracle.bmm_s8_acc(a, a)
    assert wrapped == 1
    with pytest.raises(OverflowError):
        oracle.bmm_s8(a, a, np.ones((1, 1), np.float32), np.ones((1, 1), np.float32))
