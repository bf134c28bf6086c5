"""Parity of the batched INT8 product for attention (dgq_bmm_s8) with the CPU oracle, through the C ABI:
INT32 sums bit for bit, fp16 output within max(1e-3 relative, 1 fp16 ulp)."""
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


def _fp16_close(got, ref):
    g, r = got.astype(np.float64), ref.astype(np.float64)
    fin = np.isfinite(r)
    with np.errstate(invalid="ignore", over="ignore"):
        ulp = np.spacing(np.abs(ref)).astype(np.float64)
        bad = np.where(fin, ~(np.abs(g - r) <= np.maximum(1e-3 * np.abs(r), ulp)), g != r)   # overflow: the same infinity
    assert not bad.any(), "%d of %d outputs outside tolerance, first at %s" % (bad.sum(), bad.size, np.argwhere(bad)[0])


def _operands(B, M, N, K, seed):
    rng = np.random.default_rng([seed, 0xE])
    a = rng.integers(-128, 128, (B, M, K), dtype=np.int8)
    b = rng.integers(-128, 128, (B, N, K), dtype=np.int8)
    sa = (0.01 * (1 + rng.random((B, M), dtype=np.float32))).astype(np.float32)
    sb = (0.002 * (1 + rng.random((B, N), dtype=np.float32))).astype(np.float32)
    return a, b, sa, sb


# several tiles with ragged tails in M, N and K (K a multiple of 16 only), one row, one column, N not a multiple
# of 8 (scalar stores), a K of one unit, several batches
@pytest.mark.parametrize("B,M,N,K", [
    (1, 1, 1, 16), (2, 8, 8, 128), (3, 130, 257, 144), (1, 300, 100, 1040), (2, 128, 128, 128), (1, 129, 127, 2064),
    (4, 1, 2048, 128), (2, 77, 128, 4096), (1, 5, 1003, 48), (5, 256, 384, 256),
    # at most 16 rows of A: the dot-product kernel (1, 2-4 and 5-16 rows; K / 16 a power of two and not; one lane
    # group per row of B up to a whole wavefront with several pieces per lane; ragged N)
    (32, 1, 128, 2048), (3, 1, 7, 16), (2, 2, 300, 32), (2, 4, 65, 80), (1, 16, 1000, 1024), (2, 9, 33, 4112),
    (1, 16, 5, 65536), (40, 3, 16, 128), (2, 17, 40, 128),
])
def test_bmm_bit_exact_and_epilogue(dgq, torch, B, M, N, K):
    a, b, sa, sb = _operands(B, M, N, K, seed=M + N + K)
    ad, bd = torch.from_numpy(a).cuda(), torch.from_numpy(b).cuda()
    acc = dgq.bmm_s8_acc(ad, bd).cpu().numpy()
    oout, oacc = oracle.bmm_s8(a, b, sa, sb)
    assert np.array_equal(acc, oacc), "mismatch at %s" % (np.argwhere(acc != oacc)[:4].tolist(),)
    out = dgq.bmm_s8(ad, bd, torch.from_numpy(sa).cuda(), torch.from_numpy(sb).cuda()).cpu().numpy()
    _fp16_close(out, oout)
    # scales left out = all ones
    ones = dgq.bmm_s8(ad, bd).cpu().numpy()
    oones, _ = oracle.bmm_s8(a, b, np.ones((B, M), np.float32), np.ones((B, N), np.float32))
    _fp16_close(ones, oones)                            # sums beyond 65504 overflow to the same infinities


def test_bmm_one_hot_rows_read_out_columns(dgq, torch):
    """Pins the lane maps of both operands: one-hot rows of b read single k of a, and the other way round."""
    B, M, N, K = 2, 96, 70, 272
    rng = np.random.default_rng(3)
    a = rng.integers(-128, 128, (B, M, K), dtype=np.int8)
    e = np.zeros((B, N, K), np.int8)
    ks = (np.arange(N) * 37 + 5) % K
    e[:, np.arange(N), ks] = 1
    acc = dgq.bmm_s8_acc(torch.from_numpy(a).cuda(), torch.from_numpy(e).cuda()).cpu().numpy()
    assert np.array_equal(acc, a[:, :, ks].astype(np.int32))
    acc_t = dgq.bmm_s8_acc(torch.from_numpy(e).cuda(), torch.from_numpy(a).cuda()).cpu().numpy()
    assert np.array_equal(acc_t, a[:, :, ks].astype(np.int32).transpose(0, 2, 1))


def test_bmm_extreme_values(dgq, torch):
    B, M, N, K = 1, 3, 5, 65536                         # the longest K: 128 * 128 * 65536 = 2^30
    a = np.full((B, M, K), -128, np.int8)
    acc = dgq.bmm_s8_acc(torch.from_numpy(a).cuda(), torch.from_numpy(np.full((B, N, K), -128, np.int8)).cuda()).cpu().numpy()
    assert (acc == 1 << 30).all()


def test_attention_products_at_llama7b_shapes(dgq, torch):
    """Scores Q K^T and context P V for 32 heads of 128 channels, as a LLaMA-7B layer has them: per-token INT8
    operands made by dgq_quant_act, every product against the oracle on sampled heads (all elements of those
    heads), and every INT32 sum of every head against an exact fp64 product."""
    H, T, D = 32, 512, 128
    rng = np.random.default_rng(9)
    q = rng.standard_normal((H * T, D)).astype(np.float16)
    k = rng.standard_normal((H * T, D)).astype(np.float16)
    qq, sq = dgq.quant_act(torch.from_numpy(q).cuda())
    kq, sk = dgq.quant_act(torch.from_numpy(k).cuda())
    qq, kq, sq, sk = qq.view(H, T, D), kq.view(H, T, D), sq.view(H, T), sk.view(H, T)
    scores = dgq.bmm_s8(qq, kq, sq, sk)
    sacc = dgq.bmm_s8_acc(qq, kq)
    assert torch.equal(sacc.double(), qq.double() @ kq.double().transpose(1, 2))
    heads = [0, 13, 31]
    oout, oacc = oracle.bmm_s8(qq[heads].cpu().numpy(), kq[heads].cpu().numpy(), sq[heads].cpu().numpy(), sk[heads].cpu().numpy())
    assert np.array_equal(sacc[heads].cpu().numpy(), oacc)
    _fp16_close(scores[heads].cpu().numpy(), oout)
    # the quantized scores approximate the fp64 product of the fp16 operands (quantization error only)
    ref = q.reshape(H, T, D)[heads].astype(np.float64) @ k.reshape(H, T, D)[heads].astype(np.float64).transpose(0, 2, 1)
    assert np.linalg.norm(scores[heads].cpu().numpy().astype(np.float64) - ref) / np.linalg.norm(ref) < 0.03
    # context: probabilities in [0, 1] quantized with the static scale 1/127, V transposed [H][D][T] per-channel... per row
    p = torch.softmax(scores.float() / D ** 0.5, dim=-1)
    pq = torch.round(p * 127).to(torch.int8)
    sp = torch.full((H, T), 1.0 / 127, dtype=torch.float32, device="cuda")
    vt = rng.standard_normal((H * D, T)).astype(np.float16)
    vq, sv = dgq.quant_act(torch.from_numpy(vt).cuda()) if T % 128 == 0 else (None, None)
    vq, sv = vq.view(H, D, T), sv.view(H, D)
    ctx = dgq.bmm_s8(pq, vq, sp, sv)
    cacc = dgq.bmm_s8_acc(pq, vq)
    assert torch.equal(cacc.double(), pq.double() @ vq.double().transpose(1, 2))
    oout, oacc = oracle.bmm_s8(pq[heads].cpu().numpy(), vq[heads].cpu().numpy(), sp[heads].cpu().numpy(), sv[heads].cpu().numpy())
    assert np.array_equal(cacc[heads].cpu().numpy(), oacc)
    _fp16_close(ctx[heads].cpu().numpy(), oout)
