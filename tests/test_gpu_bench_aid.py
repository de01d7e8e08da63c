"""The benchmark's measurement aid (libtpo_bench.so, tpo_stream_scale): the plain streaming
kernel v = u .* D.  One rounding per word, so the result is the exactly rounded product: the
comparison is bit for bit against numpy's product of the same host arrays."""
import numpy as np
import pytest
import torch

from paper_2604_19906_amd import tpo

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype,code", [(np.float64, tpo.TPO_F64), (np.float32, tpo.TPO_F32)])
@pytest.mark.parametrize("count", [0, 1, 3, 64, 257, 4099, 1 << 20, (1 << 20) + 3])
def test_stream_scale_is_the_exact_product(count, dtype, code):
    assert torch.cuda.is_available(), "GPU tests need a device"
    rng = np.random.default_rng(7000 + count % 1000)
    u = rng.standard_normal(count + 4).astype(dtype)
    d = rng.uniform(0.03, 3.0, count + 4).astype(dtype)
    tu, td = torch.from_numpy(u).cuda(), torch.from_numpy(d).cuda()
    tv = torch.full_like(tu, -7.0)
    st = torch.cuda.current_stream().cuda_stream
    rc = tpo.tpo_stream_scale(tu.data_ptr(), td.data_ptr(), tv.data_ptr(), count, code, st)
    assert rc == tpo.TPO_OK
    torch.cuda.synchronize()
    got = tv.cpu().numpy()
    assert np.array_equal(got[:count].view(np.uint8), (u * d)[:count].view(np.uint8))
    assert np.all(got[count:] == -7.0), "words past `count` were written"
    # in place (v == u) is allowed
    rc = tpo.tpo_stream_scale(tu.data_ptr(), td.data_ptr(), tu.data_ptr(), count, code, st)
    assert rc == tpo.TPO_OK
    torch.cuda.synchronize()
    assert np.array_equal(tu.cpu().numpy()[:count].view(np.uint8), (u * d)[:count].view(np.uint8))


def test_stream_scale_rejects_bad_arguments():
    t = torch.zeros(64, dtype=torch.float64, device="cuda")
    p = t.data_ptr()
    st = torch.cuda.current_stream().cuda_stream
    assert tpo.tpo_stream_scale(p + 8, p, p, 4, tpo.TPO_F64, st) == tpo.TPO_ERR_INVALID_ARG
    assert tpo.tpo_stream_scale(p, p, p, -1, tpo.TPO_F64, st) == tpo.TPO_ERR_INVALID_ARG
    assert tpo.tpo_stream_scale(p, p, p, 4, 7, st) == tpo.TPO_ERR_INVALID_ARG
    assert tpo.tpo_stream_scale(0, p, p, 4, tpo.TPO_F64, st) == tpo.TPO_ERR_INVALID_ARG
    torch.cuda.synchronize()
    assert float(t.abs().sum()) == 0.0
