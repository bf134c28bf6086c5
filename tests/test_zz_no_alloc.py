"""dgq_linear_a8w4_noalloc (the entry point for callers that cannot allocate): through the C ABI, its output
equals dgq_linear_a8w4's bit for bit on calls in a row that reuse the library's static scratch, the later
ones with smaller inputs, and both meet the oracle to the fp16 tolerance."""
import numpy as np
import pytest

import oracle
import workloads

pytestmark = pytest.mark.gpu


def _fp16_close(got, ref):
    g, r = got.astype(np.float64), ref.astype(np.float64)
    ulp = np.spacing(np.abs(ref)).astype(np.float64)
    assert (np.abs(g - r) <= np.maximum(1e-3 * np.abs(r), ulp)).all()


def test_noalloc_entry_point_equals_the_workspace_one():
    import torch

    import paper_2310_04836_amd as dgq
    g = 128
    # (M, K, N): the tiled kernel with an eight-way K split (1 MiB of partial sums), then smaller inputs: the
    # decode kernel with its K split over two workgroups, the same with fewer tokens and columns, and a
    # problem that needs no scratch at all.
    cases = [(64, 4096, 512), (16, 22016, 1040), (3, 13824, 272), (4, 1024, 256)]
    needs = [dgq.linear_workspace_bytes(M, N, K, g) for M, K, N in cases]
    assert needs[0] > needs[1] > needs[2] > needs[3] == 0
    for rep in range(2):                                   # the whole sequence twice: the scratch keeps old contents
        for (M, K, N), need in zip(cases, needs):
            w4, s2, s1 = workloads.integer_weights(K, N, g, seed=K + N)
            xq, sx = workloads.integer_activations(M, K, seed=M + rep)
            pw = dgq.pack_weights(torch.from_numpy(w4).cuda(), torch.from_numpy(s2).cuda(), torch.from_numpy(s1).cuda(), g)
            xd, sd = torch.from_numpy(xq).cuda(), torch.from_numpy(sx).cuda()
            ws = torch.zeros(max(need, 16), dtype=torch.uint8, device="cuda")
            want = dgq.linear_a8w4(xd, sd, pw, workspace=ws)
            out = torch.zeros((M, N), dtype=torch.float16, device="cuda")
            torch.cuda.synchronize()
            before = torch.cuda.memory_allocated()
            dgq.linear_a8w4_noalloc(xd, sd, pw, out)
            assert torch.cuda.memory_allocated() == before  # (the binding allocates nothing either)
            torch.cuda.synchronize()
            assert torch.equal(out.view(torch.int16), want.view(torch.int16)), (rep, M, K, N)
            oout, _ = oracle.linear_a8w4(xq, sx, w4, s2, s1, g)
            _fp16_close(out.cpu().numpy(), oout)


def test_noalloc_entry_point_refuses_what_its_scratch_cannot_hold():
    import torch

    import paper_2310_04836_amd as dgq
    M, K, N, g = 1, 16384, 1048576, 128
    assert dgq.linear_workspace_bytes(M, N, K, g) > (40 << 20)
    a = torch.zeros(4096, dtype=torch.uint8, device="cuda")   # never touched: the call fails on the host
    p = a.data_ptr()
    assert dgq.lib.dgq_linear_a8w4_noalloc(p, p, p, p, p, p, M, N, K, g, None) == -5
