"""GPU parity beyond 2^31 elements: tensors whose flat indices need 64 bits.

The oracle cannot sweep 2.3e9 elements in seconds, so it is evaluated on sampled rows (first rows, rows whose flat
offsets straddle 2^31 and 2^32 bytes, last rows); the scale comes from a planted maximum whose position lies
beyond 2^31 elements, which the maximum pass must find.
"""
import numpy as np
import pytest
import torch

from oracle import qsync_oracle as orc
from paper_2407_02327_amd import qsync as Q
from tests.gpu_util import assert_bits_equal, assert_close, empty, host, say, ws

pytestmark = pytest.mark.gpu


def _sample_rows(rows, cols, nrows=3):
    edge = (1 << 31) // cols
    picks = set(range(nrows)) | set(range(rows - nrows, rows)) | set(range(edge - 1, edge + 2))
    edge2 = (1 << 32) // cols
    if edge2 + 1 < rows:
        picks |= set(range(edge2 - 1, edge2 + 2))
    return sorted(r for r in picks if 0 <= r < rows)


def test_quantize_and_maximum_over_more_than_2_to_31_elements():
    rows, cols = 71680, 32768                                   # 2.35e9 elements, 4.7 GB of binary16
    say("large index: quantize", rows, cols)
    g = torch.Generator(device="cuda")
    g.manual_seed(7)
    x = torch.empty(rows, cols, dtype=torch.float16, device="cuda")
    for r0 in range(0, rows, 8192):                              # uniform in (-1, 1), generated in slabs
        n = min(8192, rows - r0)
        x[r0:r0 + n] = (torch.rand(n, cols, device="cuda", generator=g) * 2 - 1).half()
    prow, pcol = rows - 5, cols - 3                              # flat index 2.35e9 > 2^31
    x[prow, pcol] = -7.5
    s, iv, am = empty(1, torch.float32), empty(1, torch.float32), empty(1, torch.float32)
    w = ws(Q.qsync_absmax_workspace_bytes(rows, cols, Q.PER_TENSOR))
    Q.qsync_absmax_scale(x, rows, cols, cols, Q.PER_TENSOR, 8, s, iv, am, None, w)
    q = torch.empty(rows, cols, dtype=torch.int8, device="cuda")
    qT = torch.empty(cols, rows, dtype=torch.int8, device="cuda")
    Q.qsync_quantize(x, rows, cols, cols, Q.INT8, 8, Q.PER_TENSOR, Q.ROUND_STOCHASTIC, 21, 5, iv, q, qT)
    torch.cuda.synchronize()
    picks = _sample_rows(rows, cols) + [prow]
    xs = np.stack([host(x[r]) for r in picks])
    assert orc.absmax(xs, "tensor")[0] == np.float32(7.5)       # the planted element is in the sample; the rest is below 1
    assert_bits_equal(host(am), np.asarray([7.5], np.float32), "maximum found beyond 2^31 elements")
    so, io = orc.scales_from_amax(np.asarray([7.5], np.float32))
    assert_bits_equal(host(s), so, "scale")
    assert_bits_equal(host(iv), io, "inverse scale")
    for r, xr in zip(picks, xs):
        # the oracle numbers the Philox draws by flat element index: give it the row at its true position
        want = orc.quantize_int(xr[None, :], io, "tensor", "stochastic", 21, 5 + (r * cols) // 8)
        assert_bits_equal(host(q[r])[None, :], want, f"codes of row {r}")
        assert_bits_equal(host(qT[:, r])[None, :], want, f"transposed codes of row {r}")
    # the row-major-only form (streaming kernel: group indices beyond 2^28, byte offsets beyond 2^32) gives the same codes
    del qT
    q1 = torch.empty(rows, cols, dtype=torch.int8, device="cuda")
    Q.qsync_quantize(x, rows, cols, cols, Q.INT8, 8, Q.PER_TENSOR, Q.ROUND_STOCHASTIC, 21, 5, iv, q1, None)
    torch.cuda.synchronize()
    for r in picks:
        assert torch.equal(q1[r], q[r]), f"row-major-only codes of row {r}"
    assert torch.equal(q1[rows // 2:rows // 2 + 4096], q[rows // 2:rows // 2 + 4096])
    del x, q, q1


def test_forward_gemm_with_more_than_2_to_31_outputs():
    M, N, K = 71680, 32768, 64                                   # 2.35e9 outputs
    say("large index: forward GEMM", M, N, K)
    rng = np.random.default_rng(3)
    xq = rng.integers(-127, 128, (M, K), dtype=np.int8)
    wq = rng.integers(-127, 128, (N, K), dtype=np.int8)
    sw = (rng.random(N).astype(np.float32) + 0.5) * 1e-3
    bias = rng.standard_normal(N).astype(np.float32)
    sx = np.asarray([2e-2], np.float32)
    y = torch.empty(M, N, dtype=torch.float16, device="cuda")
    to = lambda a: torch.from_numpy(a).cuda()
    wsp = ws(Q.qsync_qlinear_workspace_bytes(Q.INT8, M, N, K))
    Q.qsync_qlinear_fwd(Q.INT8, M, N, K, to(xq), to(sx), to(wq), to(sw), Q.PER_ROW, to(bias), y, None, wsp)
    torch.cuda.synchronize()
    for r in _sample_rows(M, N):
        want = orc.qlinear_fwd(Q.INT8, xq[r:r + 1], sx, wq, sw, bias, out_dtype=np.float64)[0]
        assert_close(host(y[r])[None, :], want, f"Y row {r}")
    del y


def test_cast_and_dequantize_over_more_than_2_to_31_elements():
    rows, cols = 71680, 32768
    say("large index: fp16 cast with transposed copy, dequantize", rows, cols)
    g = torch.Generator(device="cuda")
    g.manual_seed(11)
    picks = _sample_rows(rows, cols)
    # binary16 cast of fp32 input, with the transposed copy
    x = torch.empty(rows, cols, dtype=torch.float32, device="cuda")
    for r0 in range(0, rows, 8192):
        n = min(8192, rows - r0)
        x[r0:r0 + n] = torch.randn(n, cols, device="cuda", generator=g)
    h = torch.empty(rows, cols, dtype=torch.float16, device="cuda")
    hT = torch.empty(cols, rows, dtype=torch.float16, device="cuda")
    Q.qsync_quantize(x, rows, cols, cols, Q.FP16, 0, 0, 0, 0, 0, None, h, hT)
    torch.cuda.synchronize()
    for r in picks:
        want = orc.cast_fp16(host(x[r])[None, :])
        assert_bits_equal(host(h[r])[None, :], want, f"cast row {r}")
        assert_bits_equal(host(hT[:, r])[None, :], want, f"transposed cast row {r}")
    del h, hT
    # int32 accumulators -> binary16 with column scales and bias (reusing x's memory as the int32 input)
    acc = x.view(torch.int32)
    acc.random_(-(1 << 20), 1 << 20, generator=g)
    cs = (torch.rand(cols, device="cuda", generator=g) + 0.5) * 1e-4
    cb = torch.randn(cols, device="cuda", generator=g)
    y = torch.empty(rows, cols, dtype=torch.float16, device="cuda")
    Q.qsync_dequantize(acc, rows, cols, cols, None, cs, 0.5, cb, y)
    torch.cuda.synchronize()
    for r in picks:
        want = orc.dequantize(host(acc[r])[None, :], 0.5, None, host(cs), host(cb), out_dtype=np.float64)
        assert_close(host(y[r])[None, :], want, f"dequantized row {r}")
    del x, y
