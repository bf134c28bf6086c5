"""The C-ABI library loads without a GPU, exports what include/dgq.h declares, and rejects
bad arguments on the host before anything could be launched."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def dgq():
    import paper_2310_04836_amd as m
    return m


def _declared():
    src = open(os.path.join(ROOT, "include", "dgq.h")).read()
    return re.findall(r"DGQ_API\s+[\w\s\*]+?\b(dgq_\w+)\s*\(", src)


def test_header_symbols_are_exported(dgq):
    names = _declared()
    assert len(names) == 38 and len(set(names)) == 38
    for n in names:
        assert hasattr(dgq.lib, n), n


def test_no_internal_symbols_leak(dgq):
    import subprocess
    out = subprocess.run(["nm", "-D", "--defined-only", dgq._build.LIB], capture_output=True, text=True).stdout
    exported = {l.split()[-1] for l in out.splitlines() if " T " in l}
    assert exported == set(_declared())


def test_status_strings_and_versions(dgq):
    assert dgq.lib.dgq_status_string(0) == b"ok"
    for st in range(-6, 0):
        assert len(dgq.lib.dgq_status_string(st)) > 3
    assert dgq.layout_version() == 1
    assert dgq.lib.dgq_last_hip_error() == 0


def test_packed_sizes(dgq):
    assert dgq.packed_sizes(4096, 12288, 128) == (4096 * 12288 // 2, 12288 // 16 * 8 * 64)
    assert dgq.packed_sizes(11008, 4096, 128) == (11008 * 4096 // 2, 256 * 22 * 64)  # 86 groups -> 22 words
    assert dgq.packed_sizes(256, 32, 64) == (4096, 2 * 1 * 64)
    assert dgq.linear_workspace_bytes(16, 4096, 4096, 128) == 0


@pytest.mark.parametrize("K,N,g", [(100, 16, 128), (0, 16, 128), (128, 8, 128), (128, 24, 128),
                                   (128, 16, 32), (128, 16, 0), (131072 + 128, 16, 128), (64, 16, 64)])
def test_shape_rules(dgq, K, N, g):
    with pytest.raises(dgq.DGQError) as e:
        dgq.packed_sizes(K, N, g)
    assert e.value.status == -2


def test_argument_checks_come_before_any_launch(dgq):
    L = dgq.lib
    good = 0x10000        # never dereferenced: every call below must fail validation first
    odd = 0x10008
    # NULL pointers
    assert L.dgq_quant_act(None, 1, 128, good, good, None) == -1
    assert L.dgq_quant_act(good, 1, 128, None, good, None) == -1
    assert L.dgq_linear_a8w4(good, good, good, good, None, good, 1, 16, 128, 128, None, 0, None) == -1
    assert L.dgq_linear_a8w4_acc(good, good, good, None, 1, 16, 128, 128, 0, None, 0, None) == -1
    assert L.dgq_pack_weights(good, None, 128, 16, 128, good, good, None, None) == -1
    assert L.dgq_unpack_weights(good, good, 128, 16, 128, None, None) == -1
    assert L.dgq_quantize_weights_rtn(good, 128, 16, 128, good, good, None, None) == -1
    # shapes
    assert L.dgq_quant_act(good, 0, 128, good, good, None) == -2
    assert L.dgq_quant_act(good, 1, 100, good, good, None) == -2
    assert L.dgq_linear_a8w4(good, good, good, good, good, good, 0, 16, 128, 128, None, 0, None) == -2
    assert L.dgq_linear_a8w4(good, good, good, good, good, good, 1, 16, 128, 96, None, 0, None) == -2
    assert L.dgq_linear_a8w4(good, good, good, good, good, good, 1, 20, 128, 128, None, 0, None) == -2
    assert L.dgq_linear_a8w4_acc(good, good, good, good, 1, 16, 192, 64, 0, None, 0, None) == -2
    assert L.dgq_pack_weights(good, good, 128, 16, 100, good, good, None, None) == -2
    # alignment
    assert L.dgq_quant_act(odd, 1, 128, good, good, None) == -3
    assert L.dgq_linear_a8w4(good, good, odd, good, good, good, 1, 16, 128, 128, None, 0, None) == -3
    assert L.dgq_pack_weights(good, good, 128, 16, 128, odd, good, None, None) == -3
    assert L.dgq_pack_weights(good, good, 128, 16, 128, good, good, 0x10002, None) == -3
    # general operands
    assert L.dgq_pack_weights_zp(good, good, None, 128, 16, 128, good, good, None, None) == -1
    assert L.dgq_pack_weights_zp(good, good, good, 128, 24, 128, good, good, None, None) == -2
    assert L.dgq_pack_weights_zp(good, odd, good, 128, 16, 128, good, good, None, None) == -3
    assert L.dgq_linear_a8w4_zp(good, good, good, None, good, good, 1, 16, 128, 128, None, 0, None) == -1
    assert L.dgq_linear_a8w4_zp_acc(good, good, good, good, 0, 16, 128, 128, 0, None, 0, None) == -2
    assert L.dgq_unpack_weights_zp(good, good, 128, 16, 32, good, None) == -2
    # grid-search quantizer: alpha grid and workspace are checked on the host
    import ctypes
    f = ctypes.c_float
    assert L.dgq_quantize_weights_grid(good, 128, 16, 128, 0, f(0.01), good, good, good, good, good, 1 << 20, None) == -4
    assert L.dgq_quantize_weights_grid(good, 128, 16, 128, 51, f(0.02), good, good, good, good, good, 1 << 20, None) == -4
    assert L.dgq_quantize_weights_grid(good, 128, 16, 128, 51, f(0.01), good, good, good, good, good, 63, None) == -5
    assert L.dgq_quantize_weights_grid(good, 128, 16, 128, 51, f(0.01), good, good, good, good, None, 64, None) == -1
    assert L.dgq_quantize_weights_grid_act(good, good, good, good, 8, 128, 16, 128, 51, f(0.01), good, good, good, good, good, 100, None) == -5
    assert L.dgq_quantize_weights_grid_act(good, None, good, good, 8, 128, 16, 128, 51, f(0.01), good, good, good, good, good, 1 << 20, None) == -1
    assert L.dgq_quantize_weights_grid_act(good, good, good, good, 0, 128, 16, 128, 51, f(0.01), good, good, good, good, good, 1 << 20, None) == -2
    assert L.dgq_quantize_weights_grid_act(good, good, good, good, 8, 128, 16, 128, 0, f(0.01), good, good, good, good, good, 1 << 20, None) == -4
    assert L.dgq_quant_act_static(good, 1, 128, f(0.0), good, good, None) == -4
    assert L.dgq_quant_act_static(good, 1, 128, f(-1.0), good, good, None) == -4
    assert L.dgq_quant_act_static(good, 1, 100, f(0.1), good, good, None) == -2
    assert L.dgq_quant_act_static(None, 1, 128, f(0.1), good, good, None) == -1
    assert L.dgq_smooth_scales(good, 4, 128, f(0.0), good, good, 512, None) == -4
    assert L.dgq_smooth_scales(good, 4, 128, f(0.005), good, good, 511, None) == -5
    assert L.dgq_smooth_scales(good, 4, 100, f(0.005), good, good, 512, None) == -2
    assert L.dgq_smooth_apply(None, None, good, 1, 128, 16, good, good, None) == -1
    assert L.dgq_smooth_apply(good, None, good, 1, 128, 16, None, None, None) == -1
    assert L.dgq_silu_mul_quant_act(good, 1, 100, good, good, None) == -2
    assert L.dgq_silu_mul_quant_act(good, 1, 24704, good, good, None) == -2
    assert L.dgq_silu_mul_quant_act(odd, 1, 128, good, good, None) == -3
    assert L.dgq_rmsnorm_quant_act(good, good, 1, 128, f(-1e-5), good, good, None) == -4
    assert L.dgq_rmsnorm_quant_act(good, None, 1, 128, f(1e-5), good, good, None) == -1
    assert L.dgq_rmsnorm_quant_act(good, good, 1, 24704, f(1e-5), good, good, None) == -2
    # the entry point that allocates nothing: same checks, and problems beyond its static scratch are refused
    assert L.dgq_linear_a8w4_noalloc(good, good, good, good, None, good, 1, 16, 128, 128, None) == -1
    assert L.dgq_linear_a8w4_noalloc(good, good, good, good, good, good, 1, 20, 128, 128, None) == -2
    assert L.dgq_linear_a8w4_noalloc(good, good, odd, good, good, good, 1, 16, 128, 128, None) == -3
    assert dgq.linear_workspace_bytes(1, 1048576, 16384, 128) > (40 << 20)     # K split of the decode kernel over 2048 workgroup columns
    assert L.dgq_linear_a8w4_noalloc(good, good, good, good, good, good, 1, 1048576, 16384, 128, None) == -5
    # batched INT8 product
    assert L.dgq_bmm_s8(good, None, None, None, good, 1, 8, 8, 128, None) == -1
    assert L.dgq_bmm_s8(good, good, None, None, good, 1, 8, 8, 120, None) == -2       # K % 16
    assert L.dgq_bmm_s8(good, good, None, None, good, 0, 8, 8, 128, None) == -2
    assert L.dgq_bmm_s8(good, good, None, None, good, 70000, 8, 8, 128, None) == -2
    assert L.dgq_bmm_s8(good, good, None, None, good, 1, 8, 8, 65536 + 16, None) == -2
    assert L.dgq_bmm_s8(good, odd, None, None, good, 1, 8, 8, 128, None) == -3
    assert L.dgq_bmm_s8(good, good, 0x10002, None, good, 1, 8, 8, 128, None) == -3
    assert L.dgq_bmm_s8_acc(good, good, None, 1, 8, 8, 128, None) == -1
    # quantizer + linear as one call
    n = ctypes.c_size_t(7)
    assert L.dgq_quant_linear_workspace_bytes(4, 4096, 11008, 128, ctypes.byref(n)) == 0 and n.value == 0
    assert L.dgq_quant_linear_workspace_bytes(16, 4096, 2944, 128, ctypes.byref(n)) == 0 and n.value == 0
    assert L.dgq_quant_linear_workspace_bytes(16, 4096, 4096, 128, ctypes.byref(n)) == 0
    assert n.value == 16 * 4096 + 256                       # two kernels: xq and sx in the workspace
    assert L.dgq_quant_linear_workspace_bytes(64, 8192, 8192, 128, ctypes.byref(n)) == 0
    assert n.value == 64 * 8192 + 256 + 65536 + 32 * 4 * 64 * 256 * 4   # plus counters and K-split partial sums (32 tiles x 4 parts)
    assert L.dgq_quant_linear_workspace_bytes(0, 4096, 4096, 128, ctypes.byref(n)) == -2
    assert L.dgq_quant_linear_a8w4(None, good, good, good, good, None, 1, 16, 128, 128, None, 0, None) == -1
    assert L.dgq_quant_linear_a8w4(good, good, good, good, good, None, 1, 16, 100, 128, None, 0, None) == -2
    assert L.dgq_quant_linear_a8w4(odd, good, good, good, good, None, 1, 16, 128, 128, None, 0, None) == -3
    assert L.dgq_quant_linear_a8w4(good, good, good, good, good, None, 32, 16, 128, 128, None, 0, None) == -5
    assert L.dgq_quant_linear_a8w4_zp(good, good, good, good, good, None, 32, 16, 128, 128, good, 100, None) == -5
    # RMSNorm + quantizer + linear as one call
    assert L.dgq_rmsnorm_quant_linear_workspace_bytes(4, 4096, 4096, 128, ctypes.byref(n)) == 0 and n.value == 0
    assert L.dgq_rmsnorm_quant_linear_workspace_bytes(4, 4096, 11008, 128, ctypes.byref(n)) == 0
    assert n.value == 4 * 11008 + 256                      # more than four steps per wavefront: two kernels
    assert L.dgq_rmsnorm_quant_linear_a8w4(good, None, f(1e-5), good, good, good, good, None, 1, 16, 128, 128, None, 0, None) == -1
    assert L.dgq_rmsnorm_quant_linear_a8w4(good, good, f(-1.0), good, good, good, good, None, 1, 16, 128, 128, None, 0, None) == -4
    assert L.dgq_rmsnorm_quant_linear_a8w4(good, odd, f(1e-5), good, good, good, good, None, 1, 16, 128, 128, None, 0, None) == -3
    assert L.dgq_rmsnorm_quant_linear_a8w4_zp(good, good, f(1e-5), good, good, good, good, None, 32, 16, 128, 128, None, 0, None) == -5
    # measurement aids
    assert L.dgq_probe_mfma(None, 4096, 1, good, 1, None) == -1
    assert L.dgq_probe_mfma(good, 64, 1, good, 1, None) == -2
    assert L.dgq_probe_mfma(good, 4096, 0, good, 1, None) == -2
    assert L.dgq_probe_mfma(odd, 4096, 1, good, 1, None) == -3


def test_quant_linear_plan_names(dgq):
    # one kernel while a workgroup covers K with at most four steps per wavefront
    assert dgq.quant_linear_plan(1, 12288, 4096, 128) == "quant_linear_decode_kernel<2, 2, 128>"
    assert dgq.quant_linear_plan(4, 4096, 11008, 128) == "quant_linear_decode_kernel<6, 1, 128>"
    assert dgq.quant_linear_plan(5, 8192, 8192, 64) == "quant_linear_decode_kernel<4, 1, 64>"
    assert dgq.quant_linear_plan(6, 8192, 8192, 64) == "linear_decode_kernel<4, 1, 64, false, false>"   # 6 * 8208 bytes
    assert dgq.quant_linear_plan(16, 4096, 4096, 128) == "linear_decode_kernel<2, 2, 128, false, false>"
    assert dgq.quant_linear_plan(2, 8192, 22016, 128) == "linear_decode_nt_kernel<6, 1, 128, true>"  # K split; 90 MB of weights: streaming loads
    assert dgq.quant_linear_plan(1, 24576, 8192, 128) == "quant_linear_decode_nt_kernel<4, 1, 128>"
    assert dgq.quant_linear_plan(17, 4096, 4096, 128) == dgq.linear_plan(17, 4096, 4096, 128)
    assert dgq.quant_linear_workspace_bytes(4, 12288, 4096, 128) == 0


def test_linear_plan_names(dgq):
    assert dgq.linear_plan(16, 22016, 4096, 128) == "linear_decode_kernel<2, 2, 128, false, false>"
    assert dgq.linear_plan(1, 4096, 11008, 128) == "linear_decode_kernel<6, 1, 128, false, false>"
    assert dgq.linear_plan(8, 8192, 22016, 64) == "linear_decode_nt_kernel<6, 1, 64, true>"      # 64 MB of weights and more: streaming loads
    assert dgq.linear_plan(8, 512, 22016, 64) == "linear_decode_kernel<6, 1, 64, false, true>"
    # 16 < M <= 64: 64-token tiles; K split over several workgroups per tile where the tiles alone leave CUs idle
    assert dgq.linear_plan(64, 8192, 8192, 128) == "linear_tiled_splitk_kernel<128, 4, 2, 3, false>"
    assert dgq.linear_workspace_bytes(64, 8192, 8192, 128) == 65536 + 32 * 4 * 64 * 256 * 4      # counters + 32 tiles x 4 parts
    assert dgq.linear_plan(17, 44032, 256, 64) == "linear_tiled_kernel<64, 4, 2, 3, false>"      # two stages: nothing to split
    assert dgq.linear_workspace_bytes(17, 44032, 256, 64) == 0
    assert dgq.linear_plan(64, 44032, 8192, 128) == "linear_tiled_kernel<128, 4, 2, 3, false>"    # 172 tiles: no split
    # larger M with few tiles and a long K splits as well, 128-token tiles while every part has a CU to itself
    assert dgq.linear_plan(128, 4096, 11008, 128) == "linear_tiled_splitk_kernel<128, 4, 2, 3, false>"
    assert dgq.linear_plan(512, 4096, 11008, 128) == "linear_tiled_splitk_kernel<128, 4, 2, 3, false>"
    assert dgq.linear_workspace_bytes(512, 4096, 11008, 128) == 65536 + 128 * 2 * 64 * 256 * 4
    assert dgq.linear_plan(512, 8192, 22016, 128) == "linear_tiled_splitk_kernel<128, 4, 4, 3, false>"
    assert dgq.linear_workspace_bytes(512, 8192, 22016, 128) == 65536 + 128 * 2 * 128 * 256 * 4
    assert dgq.linear_plan(1024, 5120, 13824, 128) == "linear_tiled_kernel<128, 4, 4, 3, false>"  # 160 tiles x 2 would not fit the CUs
    # fewer 64-token tiles than CUs: 64-token tiles
    assert dgq.linear_plan(512, 4096, 4096, 64) == "linear_tiled_kernel<64, 4, 2, 3, false>"     # 8 x 16 tiles
    assert dgq.linear_plan(512, 12288, 4096, 64) == "linear_tiled_kernel<64, 4, 4, 3, false>"    # 4 x 48 tiles
    assert dgq.linear_plan(2048, 4096, 4096, 64) == "linear_tiled_kernel<64, 4, 4, 3, false>"
    assert dgq.linear_plan(1024, 22016, 4096, 128) == "linear_tiled_kernel<128, 4, 4, 3, false>"
    # 128 x 512 tiles where their grid fills the CUs in whole rounds, or most of them in one round
    assert dgq.linear_plan(2048, 8192, 22016, 128) == "linear_tiled_kernel<128, 8, 4, 3, false>"   # 16 x 16 wide tiles
    assert dgq.linear_plan(1024, 12288, 4096, 128) == "linear_tiled_kernel<128, 8, 4, 3, false>"   # 8 x 24 wide tiles
    # two or more whole rounds of 128 x 512 tiles plus a remainder: the whole rounds and the rest as two launches
    # (256 CUs, 16 token tiles: a round covers 16 column tiles = 8192 channels)
    assert dgq.linear_plan(2048, 44032, 8192, 128) == ("linear_tiled_cols_kernel<128, 8, 4, 3, false> + "
                                                       "linear_tiled_cols_kernel<128, 4, 4, 3, false>")   # 40960 + 3072
    assert dgq.linear_plan(2048, 22016, 4096, 64) == ("linear_tiled_cols_kernel<64, 8, 4, 3, false> + "
                                                      "linear_tiled_cols_kernel<64, 8, 4, 3, false>")     # 16384 + 5632
    assert dgq.linear_workspace_bytes(2048, 44032, 8192, 128) == 0
    assert dgq.linear_plan(2048, 24576, 8192, 128) == "linear_tiled_kernel<128, 8, 4, 3, false>"   # three whole rounds
    assert dgq.linear_plan(512, 44032, 8192, 128) == "linear_tiled_kernel<128, 4, 4, 3, false>"    # one round and a third: left alone


def test_packed_sizes_zp(dgq):
    assert dgq.packed_sizes_zp(4096, 4096, 128) == (4096 * 4096 // 2, 256 * 16 * 64)
    assert dgq.packed_sizes_zp(384, 48, 128) == (384 * 48 // 2, 3 * 2 * 64)     # 3 groups padded to 4


def test_path_argument_of_the_test_hooks(dgq):
    good = 0x10000
    # an unknown path is a range error, the streaming paths refuse M > 64, both on the host
    assert dgq.lib.dgq_linear_a8w4_acc(good, good, good, good, 8, 16, 128, 128, 7, None, 0, None) == -4
    assert dgq.lib.dgq_linear_a8w4_acc(good, good, good, good, 65, 16, 128, 128, 1, None, 0, None) == -2
    assert dgq.lib.dgq_linear_a8w4_zp_acc(good, good, good, good, 65, 16, 128, 128, 3, None, 0, None) == -2
    # the workspace of a forced path is the one that path needs
    assert dgq.linear_acc_workspace_bytes(64, 8192, 8192, 128, 0) == dgq.linear_workspace_bytes(64, 8192, 8192, 128)
    assert dgq.linear_acc_workspace_bytes(8, 8192, 22016, 128, 1) == 65536 + 128 * 2 * 5 * 256 * 4   # 128 workgroup columns x 2 parts
    assert dgq.linear_acc_workspace_bytes(64, 8192, 8192, 128, 3) == 0
    with pytest.raises(dgq.DGQError):
        dgq.linear_acc_workspace_bytes(65, 8192, 8192, 128, 1)


def test_token_index_without_division_matches_integer_division():
    """The decode kernel that quantizes its own activations finds the token of 8-value vector idx as
    int((idx + 0.5) * (1 / vpr)) in fp32 (vpr = K / 8 vectors per row).  Exhaustive over every K the
    kernel accepts and every index its staging area can hold."""
    import numpy as np
    for K in range(128, 12288 + 1, 128):
        vpr = K // 8
        inv = np.float32(1.0) / np.float32(vpr)
        idx = np.arange(0, 49152 // 8, dtype=np.int32)
        tok = ((idx.astype(np.float32) + np.float32(0.5)) * inv).astype(np.int32)
        assert np.array_equal(tok, idx // vpr), K


def test_fast_rounding_of_the_in_kernel_quantizer_equals_rint_and_clamp():
    """That kernel rounds with fl32(fl32(x * inv) + 1.5 * 2^23) and takes the low byte instead of
    clamp(rint(fl32(x * inv)), -127, 127).  Checked in numpy fp32 for every finite fp16 x with
    |x| <= a, for several hundred row maxima a spread over the whole fp16 range (denormals and
    65504 included)."""
    import numpy as np
    allh = np.arange(0, 0x7C00, dtype=np.uint16).view(np.float16)         # every non-negative finite fp16
    rng = np.random.default_rng(5)
    picks = np.unique(np.concatenate([[1, 2, 3, 0x03FF, 0x0400, 0x3C00, 0x7BFF],
                                      rng.integers(1, 0x7C00, 400)])).astype(np.uint16)
    magic = np.float32(12582912.0)
    for abits in picks:
        a = np.float32(np.uint16(abits).view(np.float16))
        inv = np.float32(127.0) / a
        x = allh[:int(abits) + 1].astype(np.float32)
        x = np.concatenate([x, -x])
        t = x * inv                                                       # fp32 product, rounded once
        ref = np.clip(np.rint(t), -127, 127).astype(np.int32)
        fast = ((t + magic).view(np.uint32) & 0xFF).astype(np.uint8).view(np.int8).astype(np.int32)
        assert np.array_equal(ref, fast), hex(int(abits))
        assert np.abs(ref).max() == 127
