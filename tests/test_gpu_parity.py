"""Parity of the HIP path with the CPU oracle, element by element, through the C ABI.

Integers (packed bytes, quantized weights and activations, INT32 sums) must be bit-exact.
The fp16 output must be within max(1e-3 relative, 1 fp16 ulp) of the oracle's.
"""
import numpy as np
import pytest

import oracle
import workloads

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dgq():
    import paper_2310_04836_amd as m
    return m


@pytest.fixture(scope="module")
def torch():
    import torch as t
    return t


def dev(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    return t.cpu().numpy()


def assert_fp16_close(got, ref):
    """|got - ref| <= max(1e-3 |ref|, 1 ulp of ref in fp16)."""
    assert got.dtype == np.float16 and ref.dtype == np.float16
    g = got.astype(np.float64)
    r = ref.astype(np.float64)
    ulp = np.spacing(np.abs(ref)).astype(np.float64)
    bad = ~(np.abs(g - r) <= np.maximum(1e-3 * np.abs(r), ulp))
    assert not bad.any(), "%d of %d outputs outside tolerance, first at %s" % (
        bad.sum(), bad.size, np.argwhere(bad)[0])


# ----------------------------------------------------------------------------
# a1: per-token activation quantizer
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("M,K", [(8, 1024), (1, 4096), (16, 11008), (5, 22016), (3, 128),
                                 (33, 5120), (2, 32768), (4, 24576 + 128)])
def test_quant_act_bit_exact(dgq, torch, M, K):
    x = workloads.activations(M, K, seed=M + K)
    if M > 2:
        x[1] = 0                      # a zero token
        x[2, : K // 2] = 0
    xq, sx = dgq.quant_act(dev(torch, x))
    oxq, osx = oracle.quant_act(x)
    assert np.array_equal(host(xq), oxq)
    assert np.array_equal(host(sx).view(np.uint32), osx.view(np.uint32))


def test_quant_act_ties_and_extremes(dgq, torch):
    K = 128
    x = np.zeros((3, K), np.float16)
    x[0, :8] = [127, 0.5, 1.5, 2.5, -0.5, -2.5, 3.5, -126.5]     # inv = 1: halves round to even
    x[1, :3] = [65504, -65504, 1.0]                               # fp16 max
    x[2, :3] = [6e-8, -6e-8, 0]                                   # fp16 subnormals
    xq, sx = dgq.quant_act(dev(torch, x))
    oxq, osx = oracle.quant_act(x)
    assert host(xq)[0, :8].tolist() == [127, 0, 2, 2, 0, -2, 4, -126]
    assert np.array_equal(host(xq), oxq) and np.array_equal(host(sx), osx)


# ----------------------------------------------------------------------------
# weight side: RTN quantizer, pack, unpack
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("K,N,g", [(1024, 1024, 128), (512, 96, 64), (1408, 80, 128)])
def test_rtn_quantizer_bit_exact(dgq, torch, K, N, g):
    W = workloads.weights(K, N, seed=K + N)
    W[:, 3] = 0                       # an all-zero output channel
    W[: g, 5] = 0                     # an all-zero group
    w4, s2, s1 = dgq.quantize_weights_rtn(dev(torch, W), g)
    ow4, os2, os1 = oracle.quantize_weights_rtn(W, g)
    assert np.array_equal(host(w4), ow4)
    assert np.array_equal(host(s2), os2)
    assert np.array_equal(host(s1).view(np.uint32), os1.view(np.uint32))


@pytest.mark.parametrize("K,N,g", [(128, 16, 128), (256, 48, 64), (1408, 272, 128), (640, 4096 + 16, 64)])
def test_pack_bytes_and_unpack(dgq, torch, K, N, g):
    w4, s2, s1 = workloads.integer_weights(K, N, g, seed=K * 3 + N)
    pw, bad = dgq.pack_weights(dev(torch, w4), dev(torch, s2), dev(torch, s1), g, return_bad=True)
    oq, osc, obad = oracle.pack(w4, s2, g)
    assert bad == 0 and obad == 0
    assert np.array_equal(host(pw.qweight), oq)
    assert np.array_equal(host(pw.scales), osc)
    ws8, nbad = oracle.expand(w4, s2, g)
    assert nbad == 0
    assert np.array_equal(host(dgq.unpack_weights(pw)), ws8)


def test_pack_counts_out_of_range(dgq, torch):
    K, N, g = 128, 32, 64
    w4 = np.zeros((K, N), np.int8)
    s2 = np.ones((K // g, N), np.uint8)
    w4[3, 3], w4[4, 4], s2[0, 5], s2[1, 6] = 8, -9, 0, 16
    pw, bad = dgq.pack_weights(dev(torch, w4), dev(torch, s2), dev(torch, np.ones(N, np.float32)), g,
                               return_bad=True)
    oq, osc, obad = oracle.pack(w4, s2, g)
    assert bad == obad == 4
    assert np.array_equal(host(pw.qweight), oq) and np.array_equal(host(pw.scales), osc)


# ----------------------------------------------------------------------------
# a2 + a3: expansion and INT8 GEMM, raw INT32 sums
# ----------------------------------------------------------------------------
def _acc_case(dgq, torch, M, K, N, g, seed, path=0, onehot=False):
    w4, s2, s1 = workloads.integer_weights(K, N, g, seed)
    if onehot:
        xq = np.zeros((M, K), np.int8)
        ks = (np.arange(M) * 37 + 5) % K
        xq[np.arange(M), ks] = 1
    else:
        xq, _ = workloads.integer_activations(M, K, seed)
    pw = dgq.pack_weights(dev(torch, w4), dev(torch, s2), dev(torch, s1), g)
    acc = host(dgq.linear_a8w4_acc(dev(torch, xq), pw, path=path))
    ws8, _ = oracle.expand(w4, s2, g)
    if onehot:
        # closed form: a one-hot token reads out one row of W_s8
        assert np.array_equal(acc, ws8[ks].astype(np.int32))
    oacc, wrapped = oracle.gemm_i32(xq, ws8)
    assert wrapped == 0
    assert np.array_equal(acc, oacc), "mismatch at %s" % (np.argwhere(acc != oacc)[:4].tolist(),)


@pytest.mark.parametrize("g", [128, 64])
@pytest.mark.parametrize("M", [1, 16, 40])
def test_onehot_probe_stream_path(dgq, torch, M, g):
    """Reads single rows of W_s8 through the GEMM: pins nibble order, k pairing and lane maps."""
    _acc_case(dgq, torch, M, 512, 64, g, seed=M, path=1, onehot=True)


@pytest.mark.parametrize("g", [128, 64])
@pytest.mark.parametrize("M", [1, 130])
def test_onehot_probe_tiled_path(dgq, torch, M, g):
    _acc_case(dgq, torch, M, 512, 320, g, seed=M, path=2, onehot=True)     # 64-token tiles


@pytest.mark.parametrize("g", [128, 64])
def test_onehot_probe_tiled_path_128_token_tiles(dgq, torch, g):
    _acc_case(dgq, torch, 2048, 256, 4096, g, seed=9, path=2, onehot=True)  # 16 x 16 tiles of 128 x 256


@pytest.mark.parametrize("M,K,N,g", [
    (1, 128, 16, 128), (1, 128, 16, 64), (8, 1024, 1024, 128), (4, 4096, 256, 64), (16, 1408, 80, 128),
    (17, 2048, 48, 128), (32, 640, 112, 64), (33, 1152, 64, 128), (64, 3072, 32, 64), (3, 11008, 64, 128),
])
def test_acc_bit_exact_stream_path(dgq, torch, M, K, N, g):
    _acc_case(dgq, torch, M, K, N, g, seed=M * 7 + N, path=1)
    _acc_case(dgq, torch, M, K, N, g, seed=M * 7 + N, path=3)


# Decode kernel (M <= 16): every steps-per-wavefront variant, short last slices, idle
# wavefronts, several column tiles per workgroup with a ragged count, K split over
# workgroups through the workspace (K/128 > 96), and more tiles than one workgroup buffers.
@pytest.mark.parametrize("M,K,N,g", [
    (1, 1024, 48, 128),        # 8 steps: 8 active wavefronts of 1 step
    (16, 2176, 8240, 64),      # 17 steps: 2 per wavefront, last one short; 515 tiles on 256 workgroups
    (5, 5120, 4112, 128),      # 40 steps: 3 per wavefront, 14 active
    (16, 8192, 272, 64),       # 64 steps: 4 per wavefront
    (7, 10240, 64, 128),       # 80 steps: 5 per wavefront
    (16, 11008, 4096, 128),    # 86 steps: 6 per wavefront, 15 active, last one short
    (9, 13824, 528, 128),      # 108 steps: split in 2 parts of 54 -> 4 per wavefront
    (16, 22016, 1040, 64),     # 172 steps: split in 2 parts of 86
    (2, 128, 131200, 128),     # 8200 tiles: more than 32 per workgroup on 256 CUs
])
def test_acc_bit_exact_decode_kernel(dgq, torch, M, K, N, g):
    _acc_case(dgq, torch, M, K, N, g, seed=M + K, path=1)


def test_decode_workspace_contract(dgq, torch):
    M, K, N, g = 4, 22016, 64, 128
    need = dgq.linear_workspace_bytes(M, N, K, g)
    assert need == 65536 + 4 * 2 * 2 * 256 * 4             # counters; four workgroup columns x two parts x room for two 16 x 16 tiles
    w4, s2, s1 = workloads.integer_weights(K, N, g, 1)
    xq, sx = workloads.integer_activations(M, K, 1)
    pw = dgq.pack_weights(dev(torch, w4), dev(torch, s2), dev(torch, s1), g)
    small = torch.empty(need - 16, dtype=torch.uint8, device="cuda")
    with pytest.raises(dgq.DGQError) as e:
        dgq.linear_a8w4(dev(torch, xq), dev(torch, sx), pw, workspace=small)
    assert e.value.status == -5
    # zero-filled once; every call leaves the arrival counters zero, so the buffer is reused as it is
    ws = torch.zeros(need, dtype=torch.uint8, device="cuda")
    oout, _ = oracle.linear_a8w4(xq, sx, w4, s2, s1, g)
    for _ in range(3):
        out = host(dgq.linear_a8w4(dev(torch, xq), dev(torch, sx), pw, workspace=ws))
        assert_fp16_close(out, oout)
        ws[65536:] = 0xAB                              # only the counters (the first 64 KiB) must stay zero


@pytest.mark.parametrize("M,K,N,g", [
    (1, 128, 16, 128), (65, 256, 256, 64), (128, 1024, 256, 128), (129, 512, 272, 128), (200, 1408, 528, 64),
    (300, 640, 1040, 128), (512, 1024, 512, 64), (16, 384, 4096 + 48, 128),
    (4000, 256, 4096 + 16, 64),      # 32 x 17 narrow tiles, ragged M and N
    (4000, 256, 4096 - 48, 64),      # 32 x 8 = 256 wide tiles: the eight-wavefront 128 x 512 variant, ragged M and N
    (2000, 384, 8192 - 64, 128),     # 16 x 16 wide tiles
    # two whole rounds of 128 x 512 tiles and more, plus a remainder: two launches, the second on a column range
    (4000, 256, 2 * 4096 + 16, 64),          # 32 token tiles: a round is 8 column tiles; a remainder of 16 channels
    (1024, 384, 2 * 16384 + 272, 128),       # 8 token tiles: a round is 32 column tiles
    (2048, 256, 3 * 8192 + 4096 - 48, 128),  # 16 token tiles, three rounds, ragged remainder with wide tiles of its own
])
def test_acc_bit_exact_tiled_path(dgq, torch, M, K, N, g):
    _acc_case(dgq, torch, M, K, N, g, seed=M * 5 + N, path=2)


# 16 < M <= 64 takes the tiled kernel with a 64-token tile and K split over several
# workgroups whose INT32 partial sums meet in the workspace.
@pytest.mark.parametrize("M,K,N,g", [
    (17, 128, 16, 128),          # one stage, no split
    (64, 4096, 512, 128),        # 2 tiles x 8 parts of 4 stages
    (40, 2048, 272, 64),         # 4 parts, ragged M and N
    (33, 8192, 1040, 128),       # 8 parts
    (64, 11008, 528, 64),        # 86 stages in 8 parts of 10 or 11
    (128, 11008, 528, 128), (200, 4096, 272, 64),   # 64 < M <= 256 with few tiles: split as well
    (48, 1408, 4096 + 64, 128),  # 11 stages, one part: tail of every length mod 6 is in this list
    (64, 896, 64, 64), (64, 1024, 64, 128), (20, 1152, 64, 128), (20, 1280, 64, 64), (20, 1536, 64, 128),
])
def test_acc_bit_exact_mid_m(dgq, torch, M, K, N, g):
    _acc_case(dgq, torch, M, K, N, g, seed=M + K + N, path=0)


def test_tiled_split_workspace_contract(dgq, torch):
    M, K, N, g = 64, 4096, 512, 128
    need = dgq.linear_workspace_bytes(M, N, K, g)
    assert need == 65536 + 2 * 4 * 64 * 256 * 4            # counters; two tiles of 64 x 256 in four parts
    w4, s2, s1 = workloads.integer_weights(K, N, g, 2)
    xq, sx = workloads.integer_activations(M, K, 2)
    pw = dgq.pack_weights(dev(torch, w4), dev(torch, s2), dev(torch, s1), g)
    small = torch.empty(need - 16, dtype=torch.uint8, device="cuda")
    with pytest.raises(dgq.DGQError) as e:
        dgq.linear_a8w4(dev(torch, xq), dev(torch, sx), pw, workspace=small)
    assert e.value.status == -5
    # zero-filled once; every call leaves the arrival counters zero, so the buffer is reused as it is
    ws = torch.zeros(need, dtype=torch.uint8, device="cuda")
    oout, _ = oracle.linear_a8w4(xq, sx, w4, s2, s1, g)
    for _ in range(3):
        out = host(dgq.linear_a8w4(dev(torch, xq), dev(torch, sx), pw, workspace=ws))
        assert_fp16_close(out, oout)
        ws[65536:] = 0xAB                              # only the counters (the first 64 KiB) must stay zero


def test_both_paths_and_split_factors_agree(dgq, torch):
    """Integer sums do not depend on how K is split between wavefronts or on the path."""
    N, g = 128, 128
    for M, K in ((48, 256), (48, 1152), (48, 4096), (12, 1152), (16, 4096)):   # 2, 9, 32 steps
        w4, s2, s1 = workloads.integer_weights(K, N, g, K)
        xq, _ = workloads.integer_activations(M, K, K)
        pw = dgq.pack_weights(dev(torch, w4), dev(torch, s2), dev(torch, s1), g)
        res = []
        for path in (1, 2, 3):
            res.append(host(dgq.linear_a8w4_acc(dev(torch, xq), pw, path=path)))
        assert np.array_equal(res[0], res[1]) and np.array_equal(res[0], res[2])
        assert np.array_equal(res[0].astype(np.int64), xq.astype(np.int64) @ (
            np.repeat(s2.astype(np.int64), g, axis=0) * w4))


def test_extreme_values_no_overflow(dgq, torch):
    # largest magnitudes everywhere: xq = -127, w4 = -8, s2 = 15 -> acc = 127*120*K
    M, K, N, g = 2, 22016, 16, 128
    w4 = np.full((K, N), -8, np.int8)
    s2 = np.full((K // g, N), 15, np.uint8)
    xq = np.full((M, K), -127, np.int8)
    pw = dgq.pack_weights(dev(torch, w4), dev(torch, s2), dev(torch, np.ones(N, np.float32)), g)
    acc = host(dgq.linear_a8w4_acc(dev(torch, xq), pw))
    assert (acc == 127 * 120 * K).all()


# ----------------------------------------------------------------------------
# a4 and the whole path: fp16 output
# ----------------------------------------------------------------------------
def _forward_case(dgq, torch, M, K, N, g, seed, frac=0.01, mult=20.0, cols=None):
    x = workloads.activations(M, K, seed, frac, mult)
    W = workloads.weights(K, N, seed)
    w4, s2, s1 = dgq.quantize_weights_rtn(dev(torch, W), g)
    pw = dgq.pack_weights(w4, s2, s1, g)
    xq, sx = dgq.quant_act(dev(torch, x))
    out = host(dgq.linear_a8w4(xq, sx, pw))
    acc = host(dgq.linear_a8w4_acc(xq, pw))
    # the same path as ONE call (what bench.py times by default): the same bits
    one = host(dgq.quant_linear_a8w4(dev(torch, x), pw))
    assert np.array_equal(one.view(np.uint16), out.view(np.uint16))
    if cols is not None:           # oracle on a sample of output channels
        W = np.ascontiguousarray(W[:, cols])
        out, acc = out[:, cols], acc[:, cols]
        w4, s2, s1 = w4[:, cols], s2[:, cols], s1[cols]
    ow4, os2, os1 = oracle.quantize_weights_rtn(W, g)
    assert np.array_equal(host(w4), ow4) and np.array_equal(host(s2), os2) and np.array_equal(host(s1), os1)
    oout, oacc, oxq, osx = oracle.forward(x, ow4, os2, os1, g)
    assert np.array_equal(host(xq), oxq) and np.array_equal(host(sx), osx)
    assert np.array_equal(acc, oacc)
    assert_fp16_close(out, oout)
    return out, oout


def test_config0_whole_path(dgq, torch):
    out, oout = _forward_case(dgq, torch, 8, 1024, 1024, 128, seed=0)
    assert np.isfinite(out).all()


@pytest.mark.parametrize("M,K,N,g", [(1, 1024, 256, 64), (16, 2048, 512, 128), (50, 1408, 272, 128),
                                     (129, 1024, 528, 64), (384, 512, 256, 128)])
def test_whole_path_small(dgq, torch, M, K, N, g):
    _forward_case(dgq, torch, M, K, N, g, seed=M + N)


def test_epilogue_scales_fp16_rounding(dgq, torch):
    """Known sums times awkward scales: checks (sx*s1)*acc order, int->float and fp16 rounding."""
    M, K, N, g = 4, 128, 16, 128
    w4, s2, s1 = workloads.integer_weights(K, N, g, 9)
    xq, sx = workloads.integer_activations(M, K, 9)
    s1 = (s1 * np.float32(3.3)).astype(np.float32)
    sx[0] = 0.0                                   # zero token scale -> exact zeros
    pw = dgq.pack_weights(dev(torch, w4), dev(torch, s2), dev(torch, s1), g)
    out = host(dgq.linear_a8w4(dev(torch, xq), dev(torch, sx), pw))
    oout, _ = oracle.linear_a8w4(xq, sx, w4, s2, s1, g)
    assert (out[0] == 0).all()
    assert_fp16_close(out, oout)


def _cols(N, n=48, seed=0):
    rng = np.random.default_rng(seed)
    c = np.unique(np.concatenate([[0, 15, 16, N - 1], rng.choice(N, n, replace=False)]))
    return c


# (the full-size LLaMA shapes of the benchmark configurations are in test_gpu_configs.py)


def test_tiled_path_activation_tensor_larger_than_4_gib(dgq, torch):
    """M * K > 2^32 with the longest K the ABI accepts: addresses inside the kernels must not be
    computed in 32 bits.  The INT32 sums of sampled tokens (first tile, the token at byte offset
    2^32 exactly, its neighbours, the last one) are compared with an int64 product."""
    M, K, N, g = 33000, 131072, 16, 128
    rng = np.random.default_rng(11)
    base = rng.integers(-127, 128, size=(1000, K), dtype=np.int8)
    xq = torch.empty((M, K), dtype=torch.int8, device="cuda")
    for b in range(0, M, 1000):                      # token m = base[m % 1000] rotated by m // 1000 + 1
        rows = min(1000, M - b)
        xq[b:b + rows] = torch.from_numpy(np.roll(base[:rows], b // 1000 + 1, axis=1)).cuda()
    w4, s2, s1 = workloads.integer_weights(K, N, g, 11)
    pw = dgq.pack_weights(dev(torch, w4), dev(torch, s2), dev(torch, s1), g)
    acc = dgq.linear_a8w4_acc(xq, pw)
    ws8 = (np.repeat(s2.astype(np.int64), g, axis=0) * w4.astype(np.int64))
    for m in (0, 1, 127, 128, 999, 1000, 32767, 32768, 32769, M - 1):
        row = np.roll(base[m % 1000], m // 1000 + 1).astype(np.int64)
        assert np.array_equal(host(acc[m]).astype(np.int64), row @ ws8), "token %d" % m


# ----------------------------------------------------------------------------
# General operands of Eq. 2: unsigned nibbles, per-group zero points, S2 up to 127
# ----------------------------------------------------------------------------
def _zp_operands(K, N, g, seed):
    """Random (u4, s2, zp, s1) that satisfy the INT8 constraint of Eq. 4: small scales with any
    nibble, large scales with nibbles close to the zero point; every value of the ranges occurs."""
    rng = np.random.default_rng([seed, 77])
    ng = K // g
    s2 = np.where(rng.random((ng, N)) < 0.5, rng.integers(1, 9, (ng, N)), rng.integers(9, 128, (ng, N))).astype(np.uint8)
    zp = rng.integers(0, 16, (ng, N)).astype(np.uint8)
    room = 127 // s2.astype(int)
    lo = np.maximum(0, zp.astype(int) - room)
    hi = np.minimum(15, zp.astype(int) + room)
    r = rng.random((K, N))
    u4 = (np.repeat(lo, g, axis=0) + np.floor(r * np.repeat(hi - lo + 1, g, axis=0))).astype(np.uint8)
    s1 = rng.uniform(1e-4, 4e-4, N).astype(np.float32)
    return u4, s2, zp, s1


@pytest.mark.parametrize("K,N,g", [(128, 16, 128), (384, 48, 128), (384, 272, 64), (1024, 4096 + 16, 64)])
def test_pack_zp_bytes_and_unpack(dgq, torch, K, N, g):
    u4, s2, zp, s1 = _zp_operands(K, N, g, K + N)
    pw, bad = dgq.pack_weights_zp(dev(torch, u4), dev(torch, s2), dev(torch, zp), dev(torch, s1), g, return_bad=True)
    oq, osc, obad = oracle.pack_zp(u4, s2, zp, g)
    assert bad == obad == 0
    assert np.array_equal(host(pw.qweight), oq) and np.array_equal(host(pw.scales), osc)
    ws8, obad = oracle.expand_zp(u4, s2, zp, g)
    assert obad == 0 and np.array_equal(host(dgq.unpack_weights(pw)), ws8)


def test_pack_zp_counts_rule_breakers(dgq, torch):
    K, N, g = 128, 16, 64
    u4 = np.zeros((K, N), np.uint8)
    s2 = np.ones((2, N), np.uint8)
    zp = np.zeros((2, N), np.uint8)
    s2[0, 0], s2[1, 1], zp[0, 2], u4[5, 3] = 0, 128, 16, 16
    s2[1, 4], u4[70, 4] = 20, 7                                     # 140 leaves INT8
    pw, bad = dgq.pack_weights_zp(dev(torch, u4), dev(torch, s2), dev(torch, zp),
                                  dev(torch, np.ones(N, np.float32)), g, return_bad=True)
    oq, osc, obad = oracle.pack_zp(u4, s2, zp, g)
    assert bad == obad == 5
    assert np.array_equal(host(pw.qweight), oq) and np.array_equal(host(pw.scales), osc)


def _acc_case_zp(dgq, torch, M, K, N, g, seed, path=0):
    u4, s2, zp, s1 = _zp_operands(K, N, g, seed)
    xq, _ = workloads.integer_activations(M, K, seed)
    pw = dgq.pack_weights_zp(dev(torch, u4), dev(torch, s2), dev(torch, zp), dev(torch, s1), g)
    acc = host(dgq.linear_a8w4_acc(dev(torch, xq), pw, path=path))
    ws8, bad = oracle.expand_zp(u4, s2, zp, g)
    assert bad == 0
    oacc, wrapped = oracle.gemm_i32(xq, ws8)
    assert wrapped == 0
    assert np.array_equal(acc, oacc), "mismatch at %s" % (np.argwhere(acc != oacc)[:4].tolist(),)


@pytest.mark.parametrize("M,K,N,g", [
    (1, 128, 16, 128), (16, 384, 48, 128), (7, 2176, 272, 64), (16, 11008, 528, 128), (3, 22016, 64, 64),
    (5, 640, 131200 // 8, 128),
])
def test_acc_bit_exact_zp_decode_kernel(dgq, torch, M, K, N, g):
    _acc_case_zp(dgq, torch, M, K, N, g, seed=M + K, path=1)


@pytest.mark.parametrize("M,K,N,g", [
    (17, 128, 16, 128), (64, 4096, 512, 128), (40, 2048, 272, 64), (33, 384, 1040, 128),     # 64-token tiles, split K
    (130, 384, 320, 64), (300, 640, 1040, 128),                                              # 64-token tiles
    (4000, 256, 4096 + 16, 64), (2000, 384, 8192 - 64, 128),                                 # 128-token tiles, both widths
    (4000, 256, 2 * 4096 + 16, 64), (2048, 128, 2 * 8192 + 528, 128),                        # whole rounds + remainder: two launches
])
def test_acc_bit_exact_zp_tiled_kernel(dgq, torch, M, K, N, g):
    _acc_case_zp(dgq, torch, M, K, N, g, seed=M + N, path=0 if M > 16 else 2)


def test_zp_form_with_zero_point_8_equals_signed_nibble_form(dgq, torch):
    M, K, N, g = 48, 1152, 272, 128
    w4, s2, s1 = workloads.integer_weights(K, N, g, 3)
    xq, _ = workloads.integer_activations(M, K, 3)
    a = dgq.pack_weights(dev(torch, w4), dev(torch, s2), dev(torch, s1), g)
    b = dgq.pack_weights_zp(dev(torch, (w4 + 8).astype(np.uint8)), dev(torch, s2),
                            dev(torch, np.full_like(s2, 8)), dev(torch, s1), g)
    assert np.array_equal(host(a.qweight), host(b.qweight))
    for path in (1, 2):
        if path == 1:
            xs = xq[:16]
        else:
            xs = xq
        assert np.array_equal(host(dgq.linear_a8w4_acc(dev(torch, xs), a, path=path)),
                              host(dgq.linear_a8w4_acc(dev(torch, xs), b, path=path)))


def test_zp_form_is_refused_by_the_forced_streaming_kernel(dgq, torch):
    u4, s2, zp, s1 = _zp_operands(128, 16, 128, 1)
    pw = dgq.pack_weights_zp(dev(torch, u4), dev(torch, s2), dev(torch, zp), dev(torch, s1), 128)
    xq, _ = workloads.integer_activations(20, 128, 1)
    with pytest.raises(dgq.DGQError) as e:
        dgq.linear_a8w4_acc(dev(torch, xq), pw, path=3)
    assert e.value.status == -2


@pytest.mark.parametrize("M,K,N,g", [(8, 1024, 256, 128), (64, 1024, 512, 64), (200, 512, 272, 128)])
def test_whole_path_with_grid_searched_weights(dgq, torch, M, K, N, g):
    """fp16 activations -> dgq_quant_act -> dgq_linear_a8w4_zp on weights quantized by the two-phase grid
    search of Section 3.3 (here by the oracle), against the oracle's Eq. 2."""
    x = workloads.activations(M, K, M + N)
    W = workloads.weights(K, N, M + N)
    u4, zp, s2, s1 = oracle.quantize_weights_grid(W, g, n_alpha=21, step=0.025)
    pw, bad = dgq.pack_weights_zp(dev(torch, u4), dev(torch, s2), dev(torch, zp), dev(torch, s1), g, return_bad=True)
    assert bad == 0
    xq, sx = dgq.quant_act(dev(torch, x))
    out = host(dgq.linear_a8w4(xq, sx, pw))
    oxq, osx = oracle.quant_act(x)
    assert np.array_equal(host(xq), oxq) and np.array_equal(host(sx), osx)
    oout, oacc = oracle.linear_a8w4_zp(oxq, osx, u4, s2, zp, s1, g)
    assert np.array_equal(host(dgq.linear_a8w4_acc(xq, pw)), oacc)
    assert_fp16_close(out, oout)


@pytest.mark.parametrize("K,N,g,n_alpha,step", [(256, 64, 128, 51, 0.01), (512, 272, 64, 21, 0.025), (1024, 48, 128, 1, 0.0),
                                                (384, 1040, 128, 11, 0.05)])
def test_grid_search_quantizer_bit_exact(dgq, torch, K, N, g, n_alpha, step):
    W = workloads.weights(K, N, K + N)
    W[:, 3] = 0                                    # an all-zero column
    W[g:2 * g, 5] = 0                              # an all-zero group
    W[:, 7] = np.abs(W[:, 7])                      # one-sided groups
    W[::37, 9] *= 8                                # outliers: clipping pays
    u4, zp, s2, s1 = dgq.quantize_weights_grid(dev(torch, W), g, n_alpha, step)
    ou, oz, os2, os1 = oracle.quantize_weights_grid(W, g, n_alpha, step)
    assert np.array_equal(host(zp), oz)
    assert np.array_equal(host(s1), os1)
    assert np.array_equal(host(s2), os2)
    assert np.array_equal(host(u4), ou)
    pw, bad = dgq.pack_weights_zp(u4, s2, zp, s1, g, return_bad=True)
    assert bad == 0                                # the clip of Eq. 4 keeps every product inside INT8


@pytest.mark.parametrize("M,K,N,g,n_alpha,step", [(8, 256, 64, 128, 51, 0.01), (33, 512, 80, 64, 21, 0.025),
                                                  (70, 384, 272, 128, 11, 0.05), (1, 128, 16, 128, 1, 0.0)])
def test_activation_weighted_grid_search_bit_exact(dgq, torch, M, K, N, g, n_alpha, step):
    """The two-phase search under the output-error objectives of Section 3.3 (Eq. 3, objective of Eq. 5) on
    calibration activations with outlier channels; token counts off the 32-token register block."""
    W = workloads.weights(K, N, K + N + M)
    W[:, 3] = 0
    W[g:2 * g, 5] = 0
    W[:, 7] = np.abs(W[:, 7])
    W[::37, 9] *= 8
    X = workloads.activations(M, K, 3 * M + K)
    u4, zp, s2, s1 = dgq.quantize_weights_grid_act(dev(torch, W), dev(torch, X), g, n_alpha, step)
    ou, oz, os2, os1 = oracle.quantize_weights_grid_act(W, X, g, n_alpha, step)
    assert np.array_equal(host(zp), oz)
    assert np.array_equal(host(s1), os1)
    assert np.array_equal(host(s2), os2)
    assert np.array_equal(host(u4), ou)
    pw, bad = dgq.pack_weights_zp(u4, s2, zp, s1, g, return_bad=True)
    assert bad == 0


@pytest.mark.parametrize("M,K", [(1, 128), (7, 1024), (300, 4096), (64, 11008)])
def test_quant_act_static_bit_exact(dgq, torch, M, K):
    x = workloads.activations(M, K, M + K)
    scale = float(np.float32(np.abs(x.astype(np.float32)).max() / 127 / 3))     # a third of the range: saturates
    xq, sx = dgq.quant_act_static(dev(torch, x), scale)
    oxq, osx = oracle.quant_act_static(x, scale)
    assert np.array_equal(host(xq), oxq) and np.array_equal(host(sx), osx)
    assert (np.abs(oxq) == 127).any()


def test_static_activation_scale_through_the_linear(dgq, torch):
    M, K, N, g = 40, 1024, 272, 128
    x = workloads.activations(M, K, 5)
    w4, s2, s1 = workloads.integer_weights(K, N, g, 5)
    scale = float(np.float32(np.abs(x.astype(np.float32)).max() / 127))
    xq, sx = dgq.quant_act_static(dev(torch, x), scale)
    pw = dgq.pack_weights(dev(torch, w4), dev(torch, s2), dev(torch, s1), g)
    out = host(dgq.linear_a8w4(xq, sx, pw))
    oxq, osx = oracle.quant_act_static(x, scale)
    oout, _ = oracle.linear_a8w4(oxq, osx, w4, s2, s1, g)
    assert_fp16_close(out, oout)


@pytest.mark.parametrize("M,K,N,pct", [(64, 4096, 64, 0.005), (7, 11008, 16, 0.005), (300, 1024, 48, 0.02), (2, 128, 16, 1.0),
                                       (3, 66048, 16, 0.005)])      # more input channels than a grid has rows of blocks
def test_smoothing_bit_exact(dgq, torch, M, K, N, pct):
    x = workloads.activations(M, K, M + K)                       # 1 % of the channels are outliers
    W = workloads.weights(K, N, M + K)
    k = dgq.smooth_scales(dev(torch, x), pct)
    ok = oracle.smooth_scales(x, pct)
    assert np.array_equal(host(k), ok)
    Wo, Xo = dgq.smooth_apply(dev(torch, W), dev(torch, x), k)
    oW, oX = oracle.smooth_apply(W, x, ok)
    assert np.array_equal(host(Wo).view(np.uint16), oW.view(np.uint16))
    assert np.array_equal(host(Xo).view(np.uint16), oX.view(np.uint16))


def test_smooth_apply_with_more_tokens_than_a_grid_has_rows(dgq, torch):
    M, K = 70000, 128
    x = workloads.activations(M, K, 5)
    k = (1.0 + np.arange(K, dtype=np.float32) / 16).astype(np.float32)
    _, Xo = dgq.smooth_apply(None, dev(torch, x), dev(torch, k))
    _, oX = oracle.smooth_apply(np.zeros((K, 16), np.float16), x, k)
    assert np.array_equal(host(Xo).view(np.uint16), oX.view(np.uint16))


def test_smoothing_of_all_zero_activations_is_the_identity(dgq, torch):
    x = np.zeros((3, 256), np.float16)
    assert (host(dgq.smooth_scales(dev(torch, x))) == 1).all()


def test_offline_pipeline_lowers_the_output_error(dgq, torch):
    """Directions the paper reports (Table 1, Table 5), on synthetic data and against the fp64 product of the
    unquantized operands: the grid search beats direct rounding, and smoothing does not undo it."""
    M, K, N, g = 256, 4096, 512, 128
    x = workloads.activations(M, K, 21)
    W = workloads.weights(K, N, 21)
    ref = x.astype(np.float64) @ W.astype(np.float64)

    def err(o):
        return float(np.linalg.norm(host(o).astype(np.float64) - ref) / np.linalg.norm(ref))
    X, Wd = dev(torch, x), dev(torch, W)
    xq, sx = dgq.quant_act(X)
    w4, s2, s1 = dgq.quantize_weights_rtn(Wd, g)
    e_rtn = err(dgq.linear_a8w4(xq, sx, dgq.pack_weights(w4, s2, s1, g)))
    u4, zp, s2, s1 = dgq.quantize_weights_grid(Wd, g)
    e_grid = err(dgq.linear_a8w4(xq, sx, dgq.pack_weights_zp(u4, s2, zp, s1, g)))
    k = dgq.smooth_scales(X)
    Ws, Xs = dgq.smooth_apply(Wd, X, k)
    u4, zp, s2, s1 = dgq.quantize_weights_grid(Ws, g)
    xq2, sx2 = dgq.quant_act(Xs)
    e_smooth = err(dgq.linear_a8w4(xq2, sx2, dgq.pack_weights_zp(u4, s2, zp, s1, g)))
    assert e_grid < 0.95 * e_rtn and e_smooth < 0.95 * e_rtn and e_smooth < 1.05 * e_grid
    # the search that weighs the error by calibration activations (the first 64 tokens: the same outlier channels)
    # does better on the tokens it has not seen than the weight-only search, which cannot see those channels
    def err_held_out(o):
        return float(np.linalg.norm(host(o).astype(np.float64)[64:] - ref[64:]) / np.linalg.norm(ref[64:]))
    u4, zp, s2, s1 = dgq.quantize_weights_grid(Wd, g)
    e_grid_h = err_held_out(dgq.linear_a8w4(xq, sx, dgq.pack_weights_zp(u4, s2, zp, s1, g)))
    u4, zp, s2, s1 = dgq.quantize_weights_grid_act(Wd, X[:64].contiguous(), g)
    e_act_h = err_held_out(dgq.linear_a8w4(xq, sx, dgq.pack_weights_zp(u4, s2, zp, s1, g)))
    print("relative output error: rtn %.4f grid %.4f smooth+grid %.4f; held-out tokens: grid %.4f activation-weighted grid %.4f"
          % (e_rtn, e_grid, e_smooth, e_grid_h, e_act_h))
    assert e_act_h < e_grid_h
    assert e_rtn < 0.2                                  # and all of them are sane


def test_random_shapes_all_plans(dgq, torch):
    """Forty seeded random problems across every plan boundary (M around 16, 64, 256; few and many tiles;
    both group sizes; both operand forms): INT32 sums against an int64 product."""
    rng = np.random.default_rng(2024)
    seen = set()
    for case in range(40):
        M = int(rng.choice([1, 3, 15, 16, 17, 31, 63, 64, 65, 100, 129, 255, 256, 257, 400, 700]))
        K = 128 * int(rng.integers(1, 24))
        N = 16 * int(rng.integers(1, 90)) if case % 4 else 16 * int(rng.integers(200, 600))
        g = int(rng.choice([64, 128]))
        xq, _ = workloads.integer_activations(M, K, case)
        if case % 2:
            u4, s2, zp, s1 = _zp_operands(K, N, g, case)
            pw = dgq.pack_weights_zp(dev(torch, u4), dev(torch, s2), dev(torch, zp), dev(torch, s1), g)
            ws8 = np.repeat(s2.astype(np.int64), g, axis=0) * (u4.astype(np.int64) - np.repeat(zp.astype(np.int64), g, axis=0))
        else:
            w4, s2, s1 = workloads.integer_weights(K, N, g, case)
            pw = dgq.pack_weights(dev(torch, w4), dev(torch, s2), dev(torch, s1), g)
            ws8 = np.repeat(s2.astype(np.int64), g, axis=0) * w4.astype(np.int64)
        seen.add(dgq.linear_plan(M, N, K, g))
        acc = host(dgq.linear_a8w4_acc(dev(torch, xq), pw))
        assert np.array_equal(acc.astype(np.int64), xq.astype(np.int64) @ ws8), (case, M, K, N, g)
    assert len(seen) >= 8, seen                          # decode variants, tiled with and without a K split, ...


@pytest.mark.parametrize("M,I", [(1, 128), (16, 11008), (5, 13824), (3, 22016), (300, 1024)])
def test_silu_mul_quant_act_bit_exact(dgq, torch, M, I):
    rng = np.random.default_rng([M, I])
    GU = (rng.normal(0, 1.5, (M, 2 * I)) * rng.choice([0.01, 1.0, 6.0], (M, 2 * I))).astype(np.float16)
    GU[0, :8] = 0
    xq, sx = dgq.silu_mul_quant_act(dev(torch, GU))
    oxq, osx, _ = oracle.silu_mul_quant_act(GU)
    assert np.array_equal(host(sx), osx)
    assert np.array_equal(host(xq), oxq)


def test_mlp_block_against_the_oracle(dgq, torch):
    """x -> quant -> gate+up linear -> silu*mul fused with quant -> down linear, all through the C ABI,
    against the same chain in the oracle (every integer tensor bit-exact, the fp16 outputs to tolerance)."""
    M, H, I, g = 24, 512, 1408, 128
    x = workloads.activations(M, H, 31)
    w_gu, s2_gu, s1_gu = workloads.integer_weights(H, 2 * I, g, 31)
    w_d, s2_d, s1_d = workloads.integer_weights(I, H, g, 32)
    s1_gu = (s1_gu * np.float32(4)).astype(np.float32)          # pre-activations of order one
    p_gu = dgq.pack_weights(dev(torch, w_gu), dev(torch, s2_gu), dev(torch, s1_gu), g)
    p_d = dgq.pack_weights(dev(torch, w_d), dev(torch, s2_d), dev(torch, s1_d), g)
    xq, sx = dgq.quant_act(dev(torch, x))
    gu = dgq.linear_a8w4(xq, sx, p_gu)
    hq, hs = dgq.silu_mul_quant_act(gu)
    out = host(dgq.linear_a8w4(hq, hs, p_d))
    ogu, _, oxq, osx = oracle.forward(x, w_gu, s2_gu, s1_gu, g)
    assert np.array_equal(host(xq), oxq)
    assert np.isfinite(ogu).all() and 0.2 < np.abs(ogu.astype(np.float32)).mean() < 20
    assert_fp16_close(host(gu), ogu)
    if np.array_equal(host(gu).view(np.uint16), ogu.view(np.uint16)):      # then everything downstream is exact
        ohq, ohs, _ = oracle.silu_mul_quant_act(ogu)
        assert np.array_equal(host(hq), ohq) and np.array_equal(host(hs), ohs)
        oout, _ = oracle.linear_a8w4(ohq, ohs, w_d, s2_d, s1_d, g)
        assert_fp16_close(out, oout)
    else:
        pytest.fail("gate+up outputs differ in bits; the chain cannot be compared exactly")


@pytest.mark.parametrize("M,K", [(1, 128), (16, 4096), (5, 5120), (3, 8192), (300, 1024), (2, 22016)])
def test_rmsnorm_quant_act_bit_exact(dgq, torch, M, K):
    x = workloads.activations(M, K, M + K)
    gamma = np.random.default_rng(K).normal(1, 0.3, K).astype(np.float16)
    xq, sx = dgq.rmsnorm_quant_act(dev(torch, x), dev(torch, gamma), 1e-5)
    oxq, osx, _ = oracle.rmsnorm_quant_act(x, gamma, 1e-5)
    assert np.array_equal(host(sx), osx)
    assert np.array_equal(host(xq), oxq)


# ----------------------------------------------------------------------------
# quantizer + linear as one call (one kernel while M * (K + 16) <= 48 KiB and K is not split)
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("M,K,N,g", [
    (1, 128, 16, 128), (3, 1024, 272, 64), (16, 2048, 512, 128),      # one step per wavefront, idle wavefronts
    (1, 4096, 12288, 128), (7, 4096, 1040, 128), (16, 2944, 272, 128),  # two steps; 23 steps: a short wavefront
    (5, 5120, 528, 64), (8, 6016, 256, 64),                           # three steps (40 and 47 steps)
    (2, 8192, 1024, 128), (5, 8192, 8192, 64),                        # four steps
    (7, 6400, 304, 128),                                              # 50 steps: last wavefront short
    (4, 11008, 4096, 128), (1, 12288, 64, 128),                       # six steps
    (16, 4096, 12288, 128), (6, 8192, 512, 64),                       # rows do not fit the staging area: two launches
    (12, 22016, 512, 128),                                            # K split over workgroups: two launches
    (40, 1408, 272, 128), (130, 1024, 528, 64),                       # M > 16: two launches, tiled GEMM
])
def test_quant_linear_one_call(dgq, torch, M, K, N, g):
    """Same bits as dgq_quant_act + dgq_linear_a8w4, and the oracle's integers behind them."""
    x = workloads.activations(M, K, seed=M + K)
    if M > 2:
        x[1, :] = 0                                                   # a zero token: scale 0, zeros out
    W = workloads.weights(K, N, seed=N)
    w4, s2, s1 = dgq.quantize_weights_rtn(dev(torch, W), g)
    pw = dgq.pack_weights(w4, s2, s1, g)
    xd = dev(torch, x)
    xq, sx = dgq.quant_act(xd)
    two = host(dgq.linear_a8w4(xq, sx, pw))
    sx_out = torch.full((M,), -1.0, dtype=torch.float32, device="cuda")
    one = host(dgq.quant_linear_a8w4(xd, pw, sx_out=sx_out))
    assert np.array_equal(one.view(np.uint16), two.view(np.uint16))
    assert np.array_equal(host(sx_out), host(sx))
    cols = _cols(N, 24, seed=M) if N > 64 else np.arange(N)
    oout, _, _, osx = oracle.forward(x, host(w4)[:, cols], host(s2)[:, cols], host(s1)[cols], g)
    assert np.array_equal(host(sx_out), osx)
    assert_fp16_close(one[:, cols], oout)
    # without the optional output
    again = host(dgq.quant_linear_a8w4(xd, pw))
    assert np.array_equal(again.view(np.uint16), one.view(np.uint16))


def test_quant_linear_one_call_zero_point_form(dgq, torch):
    M, K, N, g = 11, 4096, 528, 64
    x = workloads.activations(M, K, seed=3)
    W = workloads.weights(K, N, seed=4)
    u4, zp, s2, s1 = dgq.quantize_weights_grid(dev(torch, W), g, 21, 0.025)
    pw = dgq.pack_weights_zp(u4, s2, zp, s1, g)
    xd = dev(torch, x)
    xq, sx = dgq.quant_act(xd)
    two = host(dgq.linear_a8w4(xq, sx, pw))
    one = host(dgq.quant_linear_a8w4(xd, pw))
    assert np.array_equal(one.view(np.uint16), two.view(np.uint16))
    oout = oracle.linear_a8w4_zp(host(xq), host(sx), host(u4), host(s2), host(zp), host(s1), g)[0]
    assert_fp16_close(one, oout)


def test_quant_linear_one_call_extreme_rows(dgq, torch):
    """Ties, the largest fp16, denormal rows and a lone nonzero: the in-kernel quantizer takes
    the same decisions as the stand-alone one (and as the oracle's)."""
    M, K, N, g = 6, 1024, 64, 128
    rng = np.random.default_rng(21)
    x = np.zeros((M, K), dtype=np.float16)
    x[0] = rng.integers(-127, 128, K).astype(np.float16) * np.float16(0.5)      # products on .5 ties
    x[0, 0] = 63.5
    x[1] = rng.standard_normal(K).astype(np.float16)
    x[1, 5] = 65504.0
    x[2] = (rng.integers(-40, 41, K) * 5.96e-8).astype(np.float16)               # fp16 denormals only
    x[3, 777] = -3.0                                                             # one nonzero element
    x[4] = rng.standard_normal(K).astype(np.float16) * np.float16(1e-3)
    w4, s2, s1 = workloads.integer_weights(K, N, g, 5)
    pw = dgq.pack_weights(dev(torch, w4), dev(torch, s2), dev(torch, s1), g)
    xd = dev(torch, x)
    xq, sx = dgq.quant_act(xd)
    oxq, osx = oracle.quant_act(x)
    assert np.array_equal(host(xq), oxq) and np.array_equal(host(sx), osx)
    sx_out = torch.empty(M, dtype=torch.float32, device="cuda")
    one = host(dgq.quant_linear_a8w4(xd, pw, sx_out=sx_out))
    two = host(dgq.linear_a8w4(xq, sx, pw))
    assert np.array_equal(host(sx_out), osx)
    assert np.array_equal(one.view(np.uint16), two.view(np.uint16))
    oout, _ = oracle.linear_a8w4(oxq, osx, w4, s2, s1, g)
    assert_fp16_close(one, oout)


@pytest.mark.parametrize("M,K,N,g", [
    (1, 128, 16, 128), (3, 1024, 272, 64),                            # one step per wavefront
    (1, 4096, 22016, 128), (4, 4096, 12288, 128), (11, 4096, 528, 64),  # LLaMA-7B hidden size
    (2, 5120, 1040, 128), (9, 5120, 256, 64),                         # 13B
    (1, 8192, 1024, 128), (5, 8192, 512, 64),                         # 65B
    (4, 11008, 256, 128),                                             # more than four steps per wavefront: two launches
    (16, 4096, 512, 128), (40, 1408, 272, 128),                       # rows too many: two launches
])
def test_rmsnorm_quant_linear_one_call(dgq, torch, M, K, N, g):
    """RMSNorm + quantizer + linear as one call: the token scales are the oracle's, the output has the
    bits of the three-step path (dgq_rmsnorm_quant_act, dgq_linear_a8w4) and meets the oracle's."""
    x = workloads.activations(M, K, seed=2 * M + K)
    if M > 2:
        x[1, :] = 0                                                   # mean square 0: y = 0, scale 0
    gamma = np.random.default_rng(K + 1).normal(1, 0.3, K).astype(np.float16)
    W = workloads.weights(K, N, seed=N + 1)
    w4, s2, s1 = dgq.quantize_weights_rtn(dev(torch, W), g)
    pw = dgq.pack_weights(w4, s2, s1, g)
    xd, gd = dev(torch, x), dev(torch, gamma)
    xq, sx = dgq.rmsnorm_quant_act(xd, gd, 1e-5)
    two = host(dgq.linear_a8w4(xq, sx, pw))
    sx_out = torch.full((M,), -1.0, dtype=torch.float32, device="cuda")
    one = host(dgq.rmsnorm_quant_linear_a8w4(xd, gd, 1e-5, pw, sx_out=sx_out))
    oxq, osx, _ = oracle.rmsnorm_quant_act(x, gamma, 1e-5)
    assert np.array_equal(host(sx_out), osx) and np.array_equal(host(sx), osx)
    assert np.array_equal(host(xq), oxq)
    assert np.array_equal(one.view(np.uint16), two.view(np.uint16))
    cols = _cols(N, 24, seed=M) if N > 64 else np.arange(N)
    oout, _ = oracle.linear_a8w4(oxq, osx, host(w4)[:, cols], host(s2)[:, cols], host(s1)[cols], g)
    assert_fp16_close(one[:, cols], oout)


def test_rmsnorm_quant_linear_one_call_zero_point_form(dgq, torch):
    M, K, N, g = 3, 4096, 272, 128
    x = workloads.activations(M, K, seed=8)
    gamma = np.random.default_rng(2).normal(1, 0.3, K).astype(np.float16)
    W = workloads.weights(K, N, seed=9)
    u4, zp, s2, s1 = dgq.quantize_weights_grid(dev(torch, W), g, 21, 0.025)
    pw = dgq.pack_weights_zp(u4, s2, zp, s1, g)
    xd, gd = dev(torch, x), dev(torch, gamma)
    xq, sx = dgq.rmsnorm_quant_act(xd, gd, 1e-6)
    two = host(dgq.linear_a8w4(xq, sx, pw))
    one = host(dgq.rmsnorm_quant_linear_a8w4(xd, gd, 1e-6, pw))
    assert np.array_equal(one.view(np.uint16), two.view(np.uint16))


# ----------------------------------------------------------------------------
# the launch form bench.py times: calls recorded in a HIP graph and replayed
# ----------------------------------------------------------------------------
def test_graph_replays_equal_eager_results(dgq, torch):
    """Every kind of launch the library makes (decode kernel with and without its K split, the kernels that
    quantize for themselves, tiled kernel with and without K split, stand-alone quantizers) recorded once and replayed three times on changing inputs, with eager
    work and synchronisation between the replays; every replay must reproduce the eager result."""
    g = 128
    cases = [(4, 4096, 272), (3, 22016, 256), (16, 4096, 528), (64, 8192, 512), (130, 1024, 528)]
    packed, xs, outs, outs1, outsr, wss, gammas = [], [], [], [], [], [], []
    for i, (M, K, N) in enumerate(cases):
        W = workloads.weights(K, N, seed=40 + i)
        w4, s2, s1 = dgq.quantize_weights_rtn(dev(torch, W), g)
        packed.append(dgq.pack_weights(w4, s2, s1, g))
        xs.append(torch.empty((M, K), dtype=torch.float16, device="cuda"))
        gammas.append(dev(torch, np.random.default_rng(i).normal(1, 0.2, K).astype(np.float16)))
        outs.append(torch.empty((M, N), dtype=torch.float16, device="cuda"))
        outs1.append(torch.empty((M, N), dtype=torch.float16, device="cuda"))
        outsr.append(torch.empty((M, N), dtype=torch.float16, device="cuda"))
        nb = max(dgq.linear_workspace_bytes(M, N, K, g), dgq.quant_linear_workspace_bytes(M, N, K, g),
                 dgq.rmsnorm_quant_linear_workspace_bytes(M, N, K, g), 16)
        wss.append(torch.zeros(nb, dtype=torch.uint8, device="cuda"))
    bufs = [(torch.empty((M, K), dtype=torch.int8, device="cuda"), torch.empty(M, dtype=torch.float32, device="cuda"))
            for M, K, N in cases]

    def step():
        for i in range(len(cases)):
            xq, sx = bufs[i]
            dgq.quant_act(xs[i], xq, sx)
            dgq.linear_a8w4(xq, sx, packed[i], outs[i], wss[i])
            dgq.quant_linear_a8w4(xs[i], packed[i], outs1[i], None, wss[i])
            dgq.rmsnorm_quant_linear_a8w4(xs[i], gammas[i], 1e-5, packed[i], outsr[i], None, wss[i])

    def fill(seed):
        for i, (M, K, N) in enumerate(cases):
            xs[i].copy_(dev(torch, workloads.activations(M, K, seed=seed + i)))

    fill(100)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                    # warm-up outside capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(3):
        fill(200 + 10 * rep)
        step()                                    # eager, on the new inputs
        torch.cuda.synchronize()
        want = [(o.clone(), o1.clone(), orr.clone()) for o, o1, orr in zip(outs, outs1, outsr)]
        for o, o1, orr in zip(outs, outs1, outsr):
            o.zero_(); o1.zero_(); orr.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for i in range(len(cases)):
            assert torch.equal(outs[i].view(torch.int16), want[i][0].view(torch.int16)), (rep, cases[i], "two calls")
            assert torch.equal(outs1[i].view(torch.int16), want[i][1].view(torch.int16)), (rep, cases[i], "one call")
            assert torch.equal(outsr[i].view(torch.int16), want[i][2].view(torch.int16)), (rep, cases[i], "rmsnorm")
            assert torch.equal(outs[i].view(torch.int16), outs1[i].view(torch.int16))


def test_random_shapes_one_call_forms(dgq, torch):
    """Thirty seeded random decode-size problems (every steps-per-wavefront variant, both group sizes,
    both operand forms, staging area from nearly empty to just too small): the one-call forms give the
    bits of the separate calls, with and without RMSNorm in front."""
    rng = np.random.default_rng(77)
    fused = 0
    for case in range(30):
        M = int(rng.integers(1, 17)) if case % 5 else int(rng.choice([17, 40]))
        K = 128 * int(rng.integers(1, 97)) if case % 3 else 128 * int(rng.integers(1, 33))
        N = 16 * int(rng.integers(1, 70))
        g = int(rng.choice([64, 128]))
        x = workloads.activations(M, K, seed=1000 + case)
        gamma = rng.normal(1, 0.3, K).astype(np.float16)
        if case % 2:
            u4, s2, zp, s1 = _zp_operands(K, N, g, case)
            pw = dgq.pack_weights_zp(dev(torch, u4), dev(torch, s2), dev(torch, zp), dev(torch, s1), g)
        else:
            w4, s2, s1 = workloads.integer_weights(K, N, g, case)
            pw = dgq.pack_weights(dev(torch, w4), dev(torch, s2), dev(torch, s1), g)
        s1d = pw.s1
        s1d.mul_(1e-3)                                   # keep the fp16 outputs finite
        xd, gd = dev(torch, x), dev(torch, gamma)
        fused += dgq.quant_linear_plan(M, N, K, g).startswith("quant_linear")
        xq, sx = dgq.quant_act(xd)
        two = host(dgq.linear_a8w4(xq, sx, pw))
        one = host(dgq.quant_linear_a8w4(xd, pw))
        assert np.array_equal(one.view(np.uint16), two.view(np.uint16)), (case, M, K, N, g)
        assert np.isfinite(one).all()
        yq, sy = dgq.rmsnorm_quant_act(xd, gd, 1e-5)
        two = host(dgq.linear_a8w4(yq, sy, pw))
        one = host(dgq.rmsnorm_quant_linear_a8w4(xd, gd, 1e-5, pw))
        assert np.array_equal(one.view(np.uint16), two.view(np.uint16)), (case, M, K, N, g, "rmsnorm")
    assert 8 <= fused <= 26, fused                       # both the one-kernel and the two-kernel form occur
