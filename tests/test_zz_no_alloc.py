"""The entry point that allocates nothing (library-owned scratch) against qsync_absmax_scale, through the C ABI."""
import numpy as np
import pytest
import torch

from paper_2407_02327_amd import qsync as Q
from tests.gpu_util import assert_bits_equal, dev, empty, host, say, ws

pytestmark = pytest.mark.gpu


def _both(x, with_sums, with_sq):
    rows, cols = x.shape
    xd = dev(x)
    out = []
    for static in (False, True):
        sc, iv, am = (torch.full((1,), -3.0, dtype=torch.float32, device="cuda") for _ in range(3))
        sq = torch.full((1,), -3.0, dtype=torch.float32, device="cuda") if with_sq else None
        cs = torch.full((cols,), -3.0, dtype=torch.float32, device="cuda") if with_sums else None
        if static:
            Q.qsync_absmax_scale_static(xd, rows, cols, cols, 8, sc, iv, am, cs, sq)
        else:
            w = ws(Q.qsync_absmax_workspace_bytes(rows, cols, Q.PER_TENSOR))
            Q.qsync_absmax_scale(xd, rows, cols, cols, Q.PER_TENSOR, 8, sc, iv, am, cs, w, sumsq_opt=sq)
        torch.cuda.synchronize()
        out.append((sc, iv, am, cs, sq))
    for name, a, b in zip(("scale", "inverse scale", "amax", "column sums", "squared norm"), out[0], out[1]):
        if a is not None:
            assert_bits_equal(host(b), host(a), name)
    assert float(host(out[1][2])[0]) == float(np.abs(x.astype(np.float64)).max())


@pytest.mark.parametrize("dtype", [np.float16, np.float32])
def test_static_scratch_entry_point_equals_the_workspace_one(dtype):
    rng = np.random.default_rng(5)
    # two calls in a row on the shared scratch, the second on a smaller input; then more shapes, with and without
    # the fused column sums and the squared norm
    for rows, cols in [(4096, 1024), (130, 72), (16384, 4096), (3, 5), (1000, 4096), (257, 1000)]:
        for with_sums, with_sq in [(True, True), (False, False), (True, False)]:
            say("absmax static", dtype.__name__, rows, cols, with_sums, with_sq)
            x = (rng.standard_normal((rows, cols)) * 0.7).astype(dtype)
            x[rows // 2, cols // 3] = dtype(-9.25)
            _both(x, with_sums, with_sq)


def test_static_scratch_limit_and_validation():
    x = empty((8, 4112), torch.float32)
    s = empty(1, torch.float32)
    cs = empty(4112, torch.float32)
    with pytest.raises(Q.QsyncError) as e:
        Q.qsync_absmax_scale_static(x, 8, 4112, 4112, 8, s, s, None, cs, None)
    assert e.value.status == Q.ERR_WORKSPACE
    with pytest.raises(Q.QsyncError) as e:
        Q.qsync_absmax_scale_static(x, 8, 4112, 4112, 9, s, s, None, None, None)
    assert e.value.status == Q.ERR_UNSUPPORTED
    Q.qsync_absmax_scale_static(x, 0, 4112, 4112, 8, s, s, None, None, None)        # empty: no-op
    x.fill_(0.5)
    a = empty(1, torch.float32)
    Q.qsync_absmax_scale_static(x, 8, 4112, 4112, 8, s, empty(1, torch.float32), a, None, None)   # wide, no column sums
    assert float(host(a)[0]) == 0.5
