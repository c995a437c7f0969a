"""rvq_encode_static (the entry point that allocates nothing: its scratch is a device array inside
the library image) against rvq_encode, through the C ABI: same codes, std and residuals bit for
bit, on two calls in a row, the second with fewer rows, so that what the first call left in the
shared scratch array is still there when the second runs."""
import numpy as np
import pytest

from paper_2410_15704_amd import synth

pytestmark = pytest.mark.gpu


def test_encode_static_matches_encode_on_two_calls(gpu_device):
    import torch

    from paper_2410_15704_amd import binding as b

    d, depth, K = 1024, 8, 2048
    Xb, _ = synth.llama_key(6000, d)
    dX = torch.from_numpy(Xb.view(np.int16)).cuda().view(torch.bfloat16)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(5)
    C = torch.randn((depth, K, 32), device="cuda", generator=gen) * \
        (0.7 ** torch.arange(depth, device="cuda"))[:, None, None]
    q = b.Quantizer(d=d, dhat=32, depth=depth, K=K, grouping=b.STRIDED, in_dtype=b.BF16, std_dtype=b.F16)
    q.set_codebooks(C.contiguous())
    s = torch.cuda.current_stream().cuda_stream
    for n, row0 in ((6000, 0), (1531, 2000)):  # the second call: fewer rows, and other rows
        x = dX[row0:row0 + n]
        want_c = torch.zeros((n, 32, depth), dtype=torch.int16, device="cuda")
        want_s = torch.zeros(n, dtype=torch.float16, device="cuda")
        want_r = torch.zeros((n, 32, 32), dtype=torch.float32, device="cuda")
        got_c, got_s, got_r = torch.zeros_like(want_c), torch.zeros_like(want_s), torch.zeros_like(want_r)
        assert b.lib.rvq_encode(q.ctx, x.data_ptr(), n, d, 0, depth, want_c.data_ptr(), want_s.data_ptr(),
                                want_r.data_ptr(), s) == 0
        assert b.lib.rvq_encode_static(q.ctx, x.data_ptr(), n, d, 0, depth, got_c.data_ptr(),
                                       got_s.data_ptr(), got_r.data_ptr(), s) == 0
        torch.cuda.synchronize()
        assert torch.equal(got_c, want_c)
        assert torch.equal(got_s, want_s)
        assert torch.equal(got_r, want_r)
        assert int(want_c.max()) > 0  # the reference call did write codes
    # rows already scaled need no scratch; the limit on rows is reported, nothing is enqueued
    big = b.STATIC_MAX_ROWS + 1
    assert b.lib.rvq_encode_static(q.ctx, dX.data_ptr(), big, d, 0, depth, got_c.data_ptr(),
                                   got_s.data_ptr(), None, s) == b.RVQ_EWORKSPACE
    assert b.lib.rvq_encode_static(q.ctx, None, 4, d, 0, depth, got_c.data_ptr(), got_s.data_ptr(),
                                   None, s) == b.RVQ_EINVAL
    assert b.rvq_check_kernels(q.ctx) == 0
    q.close()
