"""Parity at the benchmark configurations themselves: every (M, layer shape, group size) that the LLaMA-7B,
13B and 65B workloads of bench.py time, in the launch configuration it times, through the C ABI.

  - M <= 64: every output channel is compared with the oracle (quantized weights, packed bytes, INT8
    activations and token scales, INT32 sums bit for bit; fp16 output to the tolerance below).
  - M > 64: the oracle computes contiguous column slices for ALL tokens: the first and the last 256-column
    tile (first and last band of the tile order, the ragged last band included), and the columns on both
    sides of the first band boundary and at the start of the last band.  On top of that every one of the
    M x N INT32 sums is compared with an fp64 matrix product of the same integers (exact: the sums stay far
    below 2^53) and every fp16 output with the epilogue formula evaluated on those sums; these two use
    library routines on the GPU and say nothing by themselves, but they extend the oracle-checked slices to
    the whole output.

Tolerance of the fp16 output: |got - ref| <= max(1e-3 |ref|, 1 ulp of ref in fp16).
"""
import sys

import numpy as np
import pytest

import oracle
import workloads

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]

# model size -> (token counts of the decode, prefill and sweep configurations, group sizes, seed of bench.py)
MODELS = {
    "7b": ((1, 4, 16, 512, 1024, 2048), (128,), 1),
    "13b": ((1, 16, 1024), (128,), 3),
    "65b": ((1, 8, 64, 512, 2048), (64, 128), 4),
}
CASES = [(size, shape, g) for size, (_, groups, _) in MODELS.items()
         for shape in ("qkv", "o", "gate_up", "down") for g in groups]


@pytest.fixture(scope="module")
def dgq():
    import paper_2310_04836_amd as m
    return m


@pytest.fixture(scope="module")
def torch():
    import torch as t
    return t


_weights_cache = {}


def _weights(size, shape):
    """fp16 weights of one layer; the last one stays cached (the two group sizes of a shape follow each other)."""
    if (size, shape) not in _weights_cache:
        _weights_cache.clear()
        K, N = workloads.LLAMA_SHAPES[size][shape]
        _weights_cache[(size, shape)] = workloads.weights(K, N, MODELS[size][2])
    return _weights_cache[(size, shape)]


def _slices(N):
    """Columns the oracle computes for M > 64 (sorted, unique)."""
    tiles = (N + 255) // 256
    parts = [np.arange(0, 256), np.arange(N - 256, N)]
    if tiles > 8:
        parts.append(np.arange(8 * 256 - 32, 8 * 256 + 32))       # both sides of the first band boundary
        last_band = (tiles - 1) // 8 * 8
        parts.append(np.arange(last_band * 256, last_band * 256 + 32))
    return np.unique(np.concatenate(parts))


def _fp16_close(got, ref):
    g, r = got.astype(np.float64), ref.astype(np.float64)
    ulp = np.spacing(np.abs(ref)).astype(np.float64)
    bad = ~(np.abs(g - r) <= np.maximum(1e-3 * np.abs(r), ulp))
    assert not bad.any(), "%d of %d outputs outside tolerance, first at %s" % (bad.sum(), bad.size, np.argwhere(bad)[0])


def _say(msg):
    print(msg, file=sys.stderr, flush=True)


@pytest.mark.parametrize("size,shape,g", CASES, ids=["llama%s-%s-g%d" % c for c in CASES])
def test_benchmark_configuration(dgq, torch, size, shape, g):
    Ms, _, seed = MODELS[size]
    K, N = workloads.LLAMA_SHAPES[size][shape]
    frac, mult = workloads.OUTLIERS[size]
    W = _weights(size, shape)
    Wd = torch.from_numpy(W).cuda()
    w4, s2, s1 = dgq.quantize_weights_rtn(Wd, g)
    pw, nbad = dgq.pack_weights(w4, s2, s1, g, return_bad=True)
    assert nbad == 0
    del Wd
    hw4, hs2, hs1 = w4.cpu().numpy(), s2.cpu().numpy(), s1.cpu().numpy()

    # weight side, every output channel: the quantizer's integers and the packed bytes
    ow4, os2, os1 = oracle.quantize_weights_rtn(W, g)
    assert np.array_equal(hw4, ow4) and np.array_equal(hs2, os2)
    assert np.array_equal(hs1.view(np.uint32), os1.view(np.uint32))
    oq, osc, obad = oracle.pack(ow4, os2, g)
    assert obad == 0
    assert np.array_equal(pw.qweight.cpu().numpy(), oq) and np.array_equal(pw.scales.cpu().numpy(), osc)
    del oq, osc
    _say("  %s %s g=%d: weights and packed bytes equal the oracle's" % (size, shape, g))

    cols = _slices(N)
    sl = (np.ascontiguousarray(ow4[:, cols]), np.ascontiguousarray(os2[:, cols]), np.ascontiguousarray(os1[cols]))
    ws8_f64 = None
    plans = set()
    for M in Ms:
        x = workloads.activations(M, K, seed + M, frac, mult)       # the arrays bench.py times
        xd = torch.from_numpy(x).cuda()
        xq, sx = dgq.quant_act(xd)
        out = dgq.linear_a8w4(xq, sx, pw)
        acc = dgq.linear_a8w4_acc(xq, pw)
        one = dgq.quant_linear_a8w4(xd, pw)                          # the call bench.py makes
        assert torch.equal(one.view(torch.int16), out.view(torch.int16))
        plans.add(dgq.linear_plan(M, N, K, g))
        oxq, osx = oracle.quant_act(x)
        assert np.array_equal(xq.cpu().numpy(), oxq)
        assert np.array_equal(sx.cpu().numpy().view(np.uint32), osx.view(np.uint32))
        if M <= 64:
            oout, oacc = oracle.linear_a8w4(oxq, osx, ow4, os2, os1, g)
            assert np.array_equal(acc.cpu().numpy(), oacc)
            _fp16_close(out.cpu().numpy(), oout)
            _say("  %s %s g=%d M=%d: all %d output channels equal the oracle's (%s)" %
                 (size, shape, g, M, N, dgq.linear_plan(M, N, K, g)))
            continue
        oout, oacc = oracle.linear_a8w4(oxq, osx, sl[0], sl[1], sl[2], g)
        cd = torch.from_numpy(cols).cuda()
        assert np.array_equal(acc[:, cd].cpu().numpy(), oacc)
        _fp16_close(out[:, cd].cpu().numpy(), oout)
        # every element: exact fp64 product of the same integers, and the epilogue formula on the sums
        if ws8_f64 is None:
            ws8_f64 = w4.double() * s2.double().repeat_interleave(g, 0)
        ref = xq.double() @ ws8_f64
        assert torch.equal(acc.double(), ref)
        del ref
        want = ((sx[:, None] * s1[None, :]) * acc.float()).half()
        diff = (out.float() - want.float()).abs()
        mag = want.float().abs()
        ulp = torch.exp2(torch.floor(torch.log2(mag.clamp_min(2.0 ** -14))) - 10)
        assert bool((diff <= torch.maximum(1e-3 * mag, ulp)).all())
        del mag, ulp
        del want, diff
        _say("  %s %s g=%d M=%d: %d columns equal the oracle's, all %d x %d sums equal the fp64 product (%s)" %
             (size, shape, g, M, cols.size, M, N, dgq.linear_plan(M, N, K, g)))
    # both kernel families ran wherever the configuration spans both regimes
    if min(Ms) <= 16:
        assert any("decode" in p for p in plans), plans
    if max(Ms) > 16:
        assert any("tiled" in p for p in plans), plans
