"""A whole operator step (conversions, forward, backward) captured in a HIP graph and replayed (GPU).

The library only enqueues kernels on the caller's stream (no allocation, no memset, no host copy), so a
step can be captured; every replay must reproduce the eager result bit for bit, also with eager work
and synchronisations between the replays.
"""
import numpy as np
import pytest
import torch

from paper_2407_02327_amd import qsync as Q
from paper_2407_02327_amd import workloads as wl
from paper_2407_02327_amd.operator import QLinear
from tests.gpu_util import GRAN, RND, dev, host, say

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("tag", [Q.INT8, Q.FP16])
def test_graph_replays_equal_eager(tag):
    case = wl.ragged_case(528, 272, 400, seed=91, dtype=np.float16)
    M, N, K = case.mnk
    x, w, dy = dev(case.x), dev(case.w), dev(case.dy)

    def make():
        op = QLinear(tag, M, N, K, x_dtype=torch.float16, y_dtype=torch.float32, dx_dtype=torch.float16,
                     w_gran=GRAN[case.w_gran], dy_round=RND[case.dy_round], philox_seed=case.philox_seed)
        op.bias.copy_(dev(case.bias))
        return op

    def step(op, stream):
        op.offset = 0                          # the same Philox counters every time
        op.forward(x, w, stream)
        op.backward(dy, stream)

    eager = make()
    step(eager, torch.cuda.current_stream())
    torch.cuda.synchronize()
    want = [host(t).copy() for t in (eager.y, eager.dx, eager.dw, eager.db)]

    op = make()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step(op, side)                         # warm-up on the capture stream (function attributes, lazy loading)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step(op, torch.cuda.current_stream())
    for replay in range(4):
        say("graph replay", tag, replay)
        for t in (op.y, op.dx, op.dw, op.db):
            t.zero_()                          # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name, t, ref in zip(("y", "dx", "dw", "db"), (op.y, op.dx, op.dw, op.db), want):
            got = host(t)
            assert got.tobytes() == ref.tobytes(), f"replay {replay}: {name} differs from the eager step"
