"""GPU check of lq_matmul_few_rows_static, the few-row forward product whose scratch is a fixed array inside the
library (for callers that cannot allocate): through the C ABI, against lq_matmul (same kernels, caller's workspace), which
the other tests hold to the oracle; results must be bit-identical.  Two calls in a row, the second with a smaller input,
so that what the first call left in the shared array would show."""
import ctypes as C

import numpy as np
import pytest

from paper_2311_12023_amd import gen

pytestmark = pytest.mark.gpu


def test_few_rows_static_matches_workspace_entry_point(oracle):
    import torch
    assert torch.cuda.is_available()
    from paper_2311_12023_amd import lq

    lib = lq._lib
    limit = lib.lq_matmul_few_rows_static_scratch_bytes()
    assert limit == 4 << 20
    cfg_t = (4, 64, 256, 8, "bf16")
    cfg = lq.config(*cfg_t)
    stream = torch.cuda.current_stream().cuda_stream
    for (m, d, k, rank, seed) in [(8, 1024, 2048, 64, 5), (3, 512, 768, 16, 6)]:      # the second call is the smaller one
        w = gen.weight_matrix(d, k, seed, 8)
        codes, sidx, v = lq.nf_quantize(torch.from_numpy(w).cuda().reshape(-1), cfg)
        l1, l2 = (torch.from_numpy(a).cuda() for a in gen.low_rank_factors(d, k, rank, seed + 100))
        x = torch.from_numpy(gen.activations(m, d, seed + 200)).cuda()
        want = lq.matmul(x, codes, sidx, v, cfg, k, l1, l2)
        got = torch.full((m, k), float("nan"), dtype=torch.float32, device="cuda")
        rc = lib.lq_matmul_few_rows_static(x.data_ptr(), m, d, k, codes.data_ptr(), sidx.data_ptr(), v.data_ptr(), cfg,
                                           l1.data_ptr(), l2.data_ptr(), rank, got.data_ptr(), stream)
        assert rc == 0
        torch.cuda.synchronize()
        assert torch.equal(got, want), (m, d, k)
        # and against the oracle's definition, at the forward product's tolerance
        yref, scale = oracle.matmul(x.cpu().numpy(), oracle.unpack(codes.cpu().numpy(), d * k, 4), sidx.cpu().numpy(),
                                    v.cpu().numpy(), oracle.config(*cfg_t), k, l1.cpu().numpy(), l2.cpu().numpy(),
                                    want_abs=True)
        assert np.max(np.abs(got.cpu().numpy() - yref) - 4e-5 * scale) <= 0
    # sizes beyond the fixed array are refused before anything is launched, as are more than 8 rows
    y = torch.zeros((8, 28672), dtype=torch.float32, device="cuda")
    dummy = torch.zeros(64, dtype=torch.uint8, device="cuda")
    big = lib.lq_matmul_few_rows_static(y.data_ptr(), 8, 8192, 28672, dummy.data_ptr(), dummy.data_ptr(), y.data_ptr(), cfg,
                                        y.data_ptr(), y.data_ptr(), 64, y.data_ptr(), stream)
    assert big == -6                                                                  # LQ_ERR_WORKSPACE
    assert lib.lq_matmul_few_rows_static(y.data_ptr(), 9, 1024, 2048, dummy.data_ptr(), dummy.data_ptr(), y.data_ptr(), cfg,
                                         y.data_ptr(), y.data_ptr(), 64, y.data_ptr(), stream) == -2   # LQ_ERR_SHAPE
