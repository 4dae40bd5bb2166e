"""GPU parity of the quantized linear operator (forward + both backward GEMMs) against the CPU oracle.

Bar: INT8 codes, scales and int32 accumulators bit-exact; FP16 / FP32 and every dequantized
output within rtol 1e-3 and atol 1e-3 * max|reference|.
"""
import numpy as np
import pytest
import torch

from oracle import qsync_oracle as orc
from paper_2407_02327_amd import qsync as Q
from paper_2407_02327_amd import workloads as wl
from paper_2407_02327_amd.operator import QLinear
from tests.gpu_util import GRAN, RND, assert_bits_equal, assert_close, dev, host, say

pytestmark = pytest.mark.gpu
TORCH = {np.dtype(np.float32): torch.float32, np.dtype(np.float16): torch.float16}


def run_case(case: wl.LinearCase, tag: int, y_dtype=np.float32, dx_dtype=np.float16, dw_dtype=np.float32,
             check_codes=True, dump_acc=True, transposed_copies=None):
    """Runs one operator fwd+bwd on the GPU and compares every stage with the oracle.

    dump_acc=True asks the INT8 GEMMs for their raw int32 accumulators (compared bit for bit); a GEMM that
    dumps takes the element-wise store path.  dump_acc=False is the production launch (what the benchmark
    times): dequantize in registers, staged 16-byte stores, no accumulators in memory; Y, dX, dW, db are then
    compared element by element with the oracle to the output tolerance."""
    M, N, K = case.mnk
    say(case.name, "tag", tag, "MNK", M, N, K, "w_gran", case.w_gran, "dy_round", case.dy_round)
    op = QLinear(tag, M, N, K, x_dtype=TORCH[case.x.dtype], w_dtype=TORCH[case.w.dtype],
                 dy_dtype=TORCH[case.dy.dtype], y_dtype=TORCH[np.dtype(y_dtype)], dx_dtype=TORCH[np.dtype(dx_dtype)],
                 dw_dtype=TORCH[np.dtype(dw_dtype)], w_gran=GRAN[case.w_gran], dy_round=RND[case.dy_round],
                 philox_seed=case.philox_seed, dump_acc=dump_acc, transposed_copies=transposed_copies)
    op.offset = 12345
    op.bias.copy_(dev(case.bias))
    xd, wd, dyd = dev(case.x), dev(case.w), dev(case.dy)
    op.forward(xd, wd)
    op.backward(dyd)
    ref = orc.operator_fwd_bwd(tag, case.x, case.w, case.bias, case.dy, case.w_gran, case.dy_round,
                               seed=case.philox_seed, offset=12345, y_dtype=np.float64, dx_dtype=np.float64,
                               dw_dtype=np.float64)
    assert not ref["overflow"]
    if tag == Q.INT8:
        assert_bits_equal(host(op.sx), ref["sx"], "sx")
        assert_bits_equal(host(op.sw), ref["sw"], "sw")
        assert_bits_equal(host(op.sdy), ref["sdy"], "sdy")
        assert_bits_equal(host(op.swb), ref["swb"], "swb")
        if check_codes:
            assert_bits_equal(host(op.xq), ref["xq"], "xq")
            if op.xqT is not None:
                assert_bits_equal(host(op.xqT), ref["xq"].T, "xqT")
            assert_bits_equal(host(op.wq), ref["wq"], "wq")
            assert_bits_equal(host(op.wqbT), ref["wqb"].T, "wqbT")
            assert_bits_equal(host(op.dyq), ref["dyq"], "dyq")
            if op.dyqT is not None:
                assert_bits_equal(host(op.dyqT), ref["dyq"].T, "dyqT")
        if dump_acc:
            assert_bits_equal(host(op.acc), ref["acc"], "fwd accumulators")
            assert_bits_equal(host(op.acc_dx), ref["acc_dx"], "dX accumulators")
            assert_bits_equal(host(op.acc_dw), ref["acc_dw"], "dW accumulators")
        else:
            assert op.acc is None and op.acc_dx is None and op.acc_dw is None
    elif check_codes:
        assert_bits_equal(host(op.xq), ref["xq"], "x cast")
        assert_bits_equal(host(op.wqbT), ref["wq"].T, "w cast transposed")
        assert_bits_equal(host(op.dyq), ref["dyq"], "dy cast")
        if op.dyqT is not None:
            assert_bits_equal(host(op.dyqT), ref["dyq"].T, "dy cast transposed")
        if op.xqT is not None:
            assert_bits_equal(host(op.xqT), ref["xq"].T, "x cast transposed")
    assert_close(host(op.y), ref["y"], "Y")
    assert_close(host(op.dx), ref["dx"], "dX")
    assert_close(host(op.dw), ref["dw"], "dW")
    assert_close(host(op.db), ref["db"], "db", rtol=1e-3, atol_rel=1e-3)
    return op, ref


def test_config1_small_int8_everything_bit_exact():
    run_case(wl.config1(), Q.INT8, y_dtype=np.float32, dx_dtype=np.float32)


@pytest.mark.parametrize("tag", [Q.INT8, Q.FP16, Q.FP32])
@pytest.mark.parametrize("shape", [(64, 64, 64), (32, 48, 80), (208, 144, 272), (272, 528, 144), (528, 272, 400),
                                   (16, 16, 2064), (1040, 784, 528)])
def test_ragged_shapes_span_tiles_and_tails(tag, shape):
    m, n, k = shape
    case = wl.ragged_case(m, n, k, seed=m + n + k, dtype=np.float16 if tag != Q.FP32 else np.float32)
    run_case(case, tag, y_dtype=np.float16 if tag == Q.FP16 else np.float32)


def test_seeded_random_shapes_with_the_planners_own_choices():
    """Forty operator shapes drawn from a seeded generator (multiples of 16, from one tile to several tile rows
    and K tiles, narrow and wide outputs), each with a drawn tag, weight granularity, rounding, input dtype and
    epilogue; tile and K splits are the planner's.  Every stage is compared with the oracle as in `run_case`."""
    import random
    rnd = random.Random(2407)
    for i in range(40):
        m = rnd.choice([128, 256, 384, 512, 640, 1024, 1152, 2048, 3200, 144, 528, 1008, 4096])
        n = rnd.choice([64, 128, 192, 256, 576, 768, 1024, 1536, 80, 208, 1344])
        k = rnd.choice([64, 128, 256, 384, 640, 1024, 2048, 3072, 208, 336])
        tag = rnd.choice([Q.INT8, Q.INT8, Q.FP16])
        dump = rnd.choice([True, False])
        case = wl.ragged_case(m, n, k, seed=1000 + i, dtype=rnd.choice([np.float32, np.float16]))
        case.w_gran = rnd.choice(["tensor", "row"])
        case.dy_round = rnd.choice(["nearest", "stochastic"])
        run_case(case, tag, y_dtype=np.float16 if not dump else np.float32, dump_acc=dump)


@pytest.mark.parametrize("tile", [0, 1, 2])
@pytest.mark.parametrize("tag", [Q.INT8, Q.FP16, Q.FP32])
def test_every_gemm_tile_shape_on_ragged_operators(tile, tag):
    """The planner picks small tiles for small outputs; pin each tile shape in turn (with the K splits the planner
    then chooses for it) so that the 256x256 and 128x128 kernels also see ragged M, N and K tails."""
    Q.qsync_debug_set_gemm_tile(tile)
    try:
        for (m, n, k) in [(208, 144, 272), (528, 272, 400), (16, 16, 2064), (1040, 784, 528), (48, 2064, 64)]:
            case = wl.ragged_case(m, n, k, seed=m + n + k + tile, dtype=np.float16 if tag != Q.FP32 else np.float32)
            run_case(case, tag, y_dtype=np.float16 if tag == Q.FP16 else np.float32)
    finally:
        Q.qsync_debug_set_gemm_tile(-1)


@pytest.mark.parametrize("ydt,dxdt,dwdt", [(np.float16, np.float16, np.float32), (np.float32, np.float32, np.float16)])
def test_production_epilogue_on_ragged_shapes_int8(ydt, dxdt, dwdt):
    """INT8 without accumulator dumps: the staged-store epilogue (and the split-K reduction) on ragged shapes
    whose row lengths are 16-byte multiples in both output types, planner's choice of tile."""
    for (m, n, k) in [(64, 64, 64), (208, 144, 272), (272, 528, 144), (528, 272, 400), (16, 16, 2064), (1040, 784, 528),
                      (48, 2064, 64)]:
        case = wl.ragged_case(m, n, k, seed=m + n + k + 9, dtype=np.float16)
        run_case(case, Q.INT8, y_dtype=ydt, dx_dtype=dxdt, dw_dtype=dwdt, dump_acc=False)


@pytest.mark.parametrize("tile", [0, 1, 2])
def test_production_epilogue_every_tile_shape_int8(tile):
    Q.qsync_debug_set_gemm_tile(tile)
    try:
        for (m, n, k) in [(208, 144, 272), (528, 272, 400), (1040, 784, 528), (48, 2064, 64), (784, 1040, 272)]:
            case = wl.ragged_case(m, n, k, seed=m + n + k + tile + 17, dtype=np.float16)
            run_case(case, Q.INT8, y_dtype=np.float16, dump_acc=False)
    finally:
        Q.qsync_debug_set_gemm_tile(-1)


def test_per_tensor_weights_share_codes_between_forward_and_backward():
    case = wl.ragged_case(144, 96, 160, seed=21)
    case.w_gran = "tensor"
    op, ref = run_case(case, Q.INT8)
    assert op.swb is op.sw


def test_bias_gradient_from_the_backward_call():
    """db requested from qsync_qlinear_bwd itself (not from the fused absmax pass)."""
    case = wl.ragged_case(208, 144, 80, seed=31, dtype=np.float16)
    say("db via qlinear_bwd")
    M, N, K = case.mnk
    for dy in (case.dy, case.dy.astype(np.float32)):
        db = torch.empty(N, dtype=torch.float32, device="cuda")
        w = torch.empty(Q.qsync_qlinear_bwd_workspace_bytes(Q.INT8, M, N, K), dtype=torch.uint8, device="cuda")
        Q.qsync_qlinear_bwd(Q.INT8, M, N, K, None, None, None, None, None, None, None, Q.PER_TENSOR, None, None, db,
                            dev(dy), None, None, w)
        assert_close(host(db), dy.astype(np.float64).sum(axis=0), "db")


def test_fp32_tag_equals_plain_matmul():
    case = wl.ragged_case(100, 60, 75, seed=5)               # K with no alignment at all
    say("fp32 plain matmul")
    op = QLinear(Q.FP32, 100, 60, 75, x_dtype=torch.float32, y_dtype=torch.float32, dx_dtype=torch.float32)
    op.bias.copy_(dev(case.bias))
    op.forward(dev(case.x), dev(case.w))
    want = orc.naive_matmul_nt_f32(case.x, case.w) + case.bias
    np.testing.assert_allclose(host(op.y), want, rtol=2e-6, atol=2e-6)


def test_fp32_tag_on_the_matrix_cores_stays_fp32_accurate():
    """Rows that are 16-byte multiples run the fp32 matrix instructions (the K axis is summed in another order
    than the textbook loop): the result must stay within fp32 rounding of the naive fp32 product."""
    case = wl.ragged_case(96, 80, 256, seed=8)
    say("fp32 on matrix cores")
    op = QLinear(Q.FP32, 96, 80, 256, x_dtype=torch.float32, y_dtype=torch.float32, dx_dtype=torch.float32)
    op.bias.copy_(dev(case.bias))
    op.forward(dev(case.x), dev(case.w))
    want = orc.naive_matmul_nt_f32(case.x, case.w) + case.bias
    np.testing.assert_allclose(host(op.y), want, rtol=1e-5, atol=1e-5)
    exact = case.x.astype(np.float64) @ case.w.astype(np.float64).T + case.bias
    np.testing.assert_allclose(host(op.y), exact, rtol=1e-5, atol=1e-5)


def test_fp32_tag_any_shape_forward_and_backward():
    run_case(wl.ragged_case(100, 60, 75, seed=6, dtype=np.float32), Q.FP32, dx_dtype=np.float32)
    run_case(wl.ragged_case(1, 1, 1, seed=7, dtype=np.float32), Q.FP32, dx_dtype=np.float32)


def test_config2_bert_base_ffn_full_size():
    run_case(wl.config2(), Q.INT8, y_dtype=np.float16)


@pytest.mark.parametrize("transposed_copies", [False, True])
def test_config2_with_and_without_transposed_copies(transposed_copies):
    """Both weight-gradient paths at full size: one row-major copy of the X and dY codes read as they are, and the
    quantizer writing xqT / dyqT for the NT GEMM; codes and accumulators exact either way."""
    op, _ = run_case(wl.config2(), Q.INT8, y_dtype=np.float16, transposed_copies=transposed_copies)
    assert op.rowmajor_bwd == (not transposed_copies) and (op.xqT is None) == (not transposed_copies)
    assert (op.dyqT is None) == (not transposed_copies)


def test_config2_bert_base_ffn_full_size_production_epilogue():
    run_case(wl.config2(), Q.INT8, y_dtype=np.float16, dump_acc=False)


def test_config2_fp32_outputs_and_split_k_paths():
    case = wl.config2(tokens=1024)
    run_case(case, Q.INT8, y_dtype=np.float32, dx_dtype=np.float32)
    run_case(case, Q.FP16, y_dtype=np.float16)


@pytest.mark.parametrize("tag", [Q.INT8, Q.FP16])
def test_config3_resnet_conv_reduced_batch(tag):
    """Batch 4 of the im2col GEMM (M = 12544): element-by-element, including the split-K dW."""
    run_case(wl.config3(batch=4), tag, y_dtype=np.float16 if tag == Q.FP16 else np.float32)


def test_int32_wraparound_matches_oracle():
    """Contraction long enough to leave the int32 range: both sides wrap mod 2^32."""
    say("wraparound")
    M, N, K = 16, 16, 133152
    a = np.full((M, K), 127, np.int8); a[1::2] = -127
    b = np.full((N, K), 127, np.int8)
    one = dev(np.ones(1, np.float32))
    y = torch.empty((M, N), dtype=torch.float32, device="cuda")
    acc = torch.empty((M, N), dtype=torch.int32, device="cuda")
    w = torch.empty(max(Q.qsync_qlinear_workspace_bytes(Q.INT8, M, N, K), 256), dtype=torch.uint8, device="cuda")
    Q.qsync_qlinear_fwd(Q.INT8, M, N, K, dev(a), one, dev(b), one, Q.PER_TENSOR, None, y, acc, w)
    want, ovf = orc.int_gemm_nt(a, b)
    assert ovf
    assert_bits_equal(host(acc), want, "wrapped accumulators")


@pytest.mark.parametrize("tokens,epilogue_maxima", [(2048, False), (8192, False), (8192, True)])
def test_config4_mixed_precision_mlp_chain(tokens, epilogue_maxima):
    """12 linears (width -> hidden -> width, GELU in between), per-layer precision tags; fwd then bwd
    (8192 tokens is the configuration's full size).  With `epilogue_maxima` every layer whose output feeds the
    next layer as it is (no GELU in between: the odd layers) collects max |Y| in its GEMM epilogue and the
    consumer takes its activation scale from that word; every comparison below stays the same.

    Parity is asserted per operator on identical input bits: each layer's actual GPU input and
    incoming gradient are downloaded and given to the oracle.  GELU and its derivative are not part
    of the operator path; the harness evaluates them with torch between the operators.
    """
    chain = wl.config4(tokens=tokens)
    M = chain.x.shape[0]
    say("config4 chain, tags", chain.tags)
    assert set(chain.tags) == {Q.INT8, Q.FP16, Q.FP32}
    ops, acts, pre = [], [dev(chain.x)], []
    wd = [dev(w) for w in chain.weights]
    for l, (w, tag) in enumerate(zip(chain.weights, chain.tags)):
        N, K = w.shape
        feeds_next_directly = epilogue_maxima and l % 2 == 1 and l + 1 < len(chain.weights)
        op = QLinear(tag, M, N, K, x_dtype=torch.float32, y_dtype=torch.float32, dx_dtype=torch.float32,
                     w_gran=Q.PER_ROW, dy_round=Q.ROUND_STOCHASTIC, philox_seed=chain.philox_seed, dump_acc=True,
                     collect_y_amax=feeds_next_directly)
        producer = ops[-1] if ops else None
        x_amax = producer.y_amax if (producer is not None and producer.y_amax is not None and tag == Q.INT8) else None
        y = op.forward(acts[-1], wd[l], x_amax=x_amax)
        ops.append(op)
        pre.append(y)
        acts.append(torch.nn.functional.gelu(y) if l % 2 == 0 else y)
    grads = [None] * len(ops)
    g = dev(chain.dy_last)
    offset = 0
    offsets = [0] * len(ops)
    for l in reversed(range(len(ops))):
        if l % 2 == 0:                                       # through the GELU that follows layer l
            t = pre[l].detach().clone().requires_grad_(True)
            torch.nn.functional.gelu(t).backward(g)
            g = t.grad
        grads[l] = g
        ops[l].offset = offsets[l] = offset
        dx, dw, db = ops[l].backward(g)
        if chain.tags[l] == Q.INT8:
            offset += (M * chain.weights[l].shape[0] + 7) // 8
        g = dx
    torch.cuda.synchronize()
    for l, op in enumerate(ops):
        say("config4 layer", l, "tag", chain.tags[l])
        x_l, g_l = host(acts[l]), host(grads[l])
        ref = orc.operator_fwd_bwd(chain.tags[l], x_l, chain.weights[l], None, g_l, "row", "stochastic",
                                   seed=chain.philox_seed, offset=offsets[l], y_dtype=np.float64,
                                   dx_dtype=np.float64, dw_dtype=np.float64)
        if chain.tags[l] == Q.INT8:
            assert_bits_equal(host(op.xq), ref["xq"], "xq")
            assert_bits_equal(host(op.dyq), ref["dyq"], "dyq")
            assert_bits_equal(host(op.acc), ref["acc"], "fwd accumulators")
            assert_bits_equal(host(op.acc_dx), ref["acc_dx"], "dX accumulators")
            assert_bits_equal(host(op.acc_dw), ref["acc_dw"], "dW accumulators")
            assert not ref["overflow"]
        assert_close(host(op.y), ref["y"], "Y")
        assert_close(host(op.dx), ref["dx"], "dX")
        assert_close(host(op.dw), ref["dw"], "dW")
        assert_close(host(op.db), ref["db"], "db")
    # the chain as a whole stays close to the unquantized fp64 network (sanity, not parity)
    a = chain.x.astype(np.float64)
    for l, w in enumerate(chain.weights):
        a = a @ w.astype(np.float64).T
        if l % 2 == 0:
            a = orc.gelu(a)
    out = host(acts[-1]).astype(np.float64)
    assert np.abs(out - a).max() <= 0.1 * np.abs(a).max()


@pytest.mark.parametrize("which", ["up", "down"])
def test_config5_bert_large_full_size_int8(which):
    """Full-size BERT-large-scale linears with the raw accumulators of all three GEMMs compared bit for bit
    (a GEMM that dumps its accumulators stores element-wise)."""
    case = wl.config5()[which]
    run_case(case, Q.INT8, y_dtype=np.float16)


@pytest.mark.parametrize("which", ["up", "down"])
def test_config5_bert_large_full_size_int8_as_benchmarked(which):
    """The launch configuration the benchmark times: no accumulator dumps, so every GEMM leaves through the
    production epilogue (dequantize in registers, staged stores; split-K reduction for dW).  Y, dX, dW and db
    element by element against the oracle; codes and scales bit for bit."""
    case = wl.config5()[which]
    run_case(case, Q.INT8, y_dtype=np.float16, dump_acc=False)


@pytest.mark.parametrize("which", ["up", "down"])
def test_config5_fp16_tag_full_size(which):
    run_case(wl.config5()[which], Q.FP16, y_dtype=np.float16)


def test_config3_resnet_conv_full_size_int8():
    """M = 200704: split-K dW over a contraction of 200704, HBM-bound forward and dX."""
    run_case(wl.config3(), Q.INT8, y_dtype=np.float16)


def test_config3_resnet_conv_full_size_int8_production_epilogue():
    run_case(wl.config3(), Q.INT8, y_dtype=np.float16, dump_acc=False)


def test_config3_resnet_conv_full_size_fp16_tag():
    """Config 3 with the FP16 precision tag at full size (M = 200704), cast operands compared bit for bit."""
    run_case(wl.config3(), Q.FP16, y_dtype=np.float16)


def run_case_fp16_backward(case: wl.LinearCase, y_dtype=np.float32, transposed_copies=None):
    """INT8 forward with the paper's FP16 backward on the dequantized saved codes, stage by stage."""
    M, N, K = case.mnk
    say(case.name, "INT8 forward / FP16 backward", "MNK", M, N, K, "w_gran", case.w_gran)
    op = QLinear(Q.INT8, M, N, K, x_dtype=TORCH[case.x.dtype], w_dtype=TORCH[case.w.dtype],
                 dy_dtype=TORCH[case.dy.dtype], y_dtype=TORCH[np.dtype(y_dtype)], dx_dtype=torch.float16,
                 dw_dtype=torch.float32, w_gran=GRAN[case.w_gran], philox_seed=case.philox_seed, bwd_tag=Q.FP16,
                 transposed_copies=transposed_copies)
    op.bias.copy_(dev(case.bias))
    op.forward(dev(case.x), dev(case.w))
    op.backward(dev(case.dy))
    ref = orc.operator_fwd_bwd(Q.INT8, case.x, case.w, case.bias, case.dy, case.w_gran, y_dtype=np.float64,
                               dx_dtype=np.float64, dw_dtype=np.float64, bwd_tag=Q.FP16)
    assert_bits_equal(host(op.xq), ref["xq"], "xq")
    assert_bits_equal(host(op.wq), ref["wq"], "wq")
    # dequantized binary16 operands: the exact product code * scale rounded once to binary16
    if op.rowmajor_bwd:       # the weight gradient reads x_hat and dY16 as they are: no transposed operands exist
        assert op.xqT is None and op.dyhT is None
        assert_bits_equal(host(op.xh), ref["xh"], "x_hat")
    else:
        assert_bits_equal(host(op.xhT), ref["xh"].T, "x_hat transposed")
        assert_bits_equal(host(op.dyhT), ref["dyh"].T, "dY cast transposed")
    assert_bits_equal(host(op.wh), ref["wh"], "w_hat")
    assert_bits_equal(host(op.whT), ref["wh"].T, "w_hat transposed")
    assert_bits_equal(host(op.dyh), ref["dyh"], "dY cast")
    assert_close(host(op.y), ref["y"], "Y")
    assert_close(host(op.dx), ref["dx"], "dX (FP16 backward)")
    assert_close(host(op.dw), ref["dw"], "dW (FP16 backward)")
    assert_close(host(op.db), ref["db"], "db", rtol=1e-3, atol_rel=1e-3)
    return op, ref


@pytest.mark.parametrize("w_gran", ["row", "tensor"])
def test_int8_forward_fp16_backward_small_and_ragged(w_gran):
    for shape in [(64, 128, 128), (208, 144, 272), (528, 272, 400)]:
        case = wl.ragged_case(*shape, seed=sum(shape) + 1)
        case.w_gran = w_gran
        run_case_fp16_backward(case)


@pytest.mark.parametrize("transposed_copies", [False, True])
def test_int8_forward_fp16_backward_config2_full_size(transposed_copies):
    """Both operand forms of the FP16 backward: x_hat [M,K] and dY16 read row-major by the weight-gradient GEMM, and the
    transposed copies x_hat^T, dY16^T for the NT GEMM."""
    op, _ = run_case_fp16_backward(wl.config2(), y_dtype=np.float16, transposed_copies=transposed_copies)
    assert op.rowmajor_bwd == (not transposed_copies)


def test_int8_forward_fp16_backward_row_major_small():
    for shape in [(128, 128, 128), (256, 144, 272), (640, 272, 400)]:
        run_case_fp16_backward(wl.ragged_case(*shape, seed=sum(shape) + 2), transposed_copies=False)


def test_conv_activation_quantized_once_then_expanded():
    """Config 3 through the NHWC path: absmax + quantize of the activation, int8 im2col, then the same GEMMs;
    codes, scales and accumulators equal those of quantizing the fp16 patch matrix (the oracle's operator)."""
    case = wl.config3(batch=4)
    M, N, K = case.mnk
    op = QLinear(Q.INT8, M, N, K, x_dtype=torch.float16, w_dtype=torch.float32, dy_dtype=torch.float16,
                 y_dtype=torch.float16, w_gran=GRAN[case.w_gran], dy_round=RND[case.dy_round],
                 philox_seed=case.philox_seed, dump_acc=True)
    op.bias.copy_(dev(case.bias))
    op.convert_w(dev(case.w))
    op.convert_x_nhwc(dev(case.nhwc))
    op.gemm_fwd()
    op.backward(dev(case.dy))
    ref = orc.operator_fwd_bwd(Q.INT8, case.x, case.w, case.bias, case.dy, case.w_gran, case.dy_round,
                               seed=case.philox_seed, offset=0, y_dtype=np.float64, dx_dtype=np.float64,
                               dw_dtype=np.float64)
    assert_bits_equal(host(op.sx), ref["sx"], "sx")
    assert_bits_equal(host(op.xq), ref["xq"], "xq")
    if op.xqT is not None:
        assert_bits_equal(host(op.xqT), ref["xq"].T, "xqT")
    assert_bits_equal(host(op.acc), ref["acc"], "fwd accumulators")
    assert_bits_equal(host(op.acc_dw), ref["acc_dw"], "dW accumulators")
    assert_close(host(op.y), ref["y"], "Y")
    assert_close(host(op.dw), ref["dw"], "dW")


@pytest.mark.parametrize("tile", [0, 1, 2])
@pytest.mark.parametrize("tag,ydt", [(Q.INT8, torch.float16), (Q.INT8, torch.float32), (Q.FP16, torch.float16),
                                     (Q.FP32, torch.float32)])
def test_forward_epilogue_collects_the_output_maximum(tile, tag, ydt):
    """qsync_qlinear_fwd_amax: same Y as qsync_qlinear_fwd bit for bit, and the collected word is max |Y| of the
    stored values exactly (a maximum has no rounding); against the oracle's Y it holds to the output tolerance.
    Shapes cover the 16-byte store path, the element-wise path (odd N), ragged tiles and split K (where the
    reduction pass takes the maximum); the word accumulates."""
    Q.qsync_debug_set_gemm_tile(tile)
    try:
        shapes = [(300, 264, 272), (257, 131, 144), (64, 128, 128), (192, 264, 4096), (96, 101, 4096)]   # the last two split K
        if tag == Q.FP32:
            shapes.append((130, 70, 50))          # rows that are not 16-byte multiples: the any-shape kernel
        for (M, N, K) in shapes:
            rng = np.random.default_rng(M * 7 + N)
            x = rng.standard_normal((M, K)).astype(np.float32)
            w = (rng.standard_normal((N, K)) * 0.05).astype(np.float32)
            b = rng.standard_normal(N).astype(np.float32)
            say("fwd_amax tile", tile, "tag", tag, "ydt", ydt, "MNK", M, N, K)
            mk = lambda: QLinear(tag, M, N, K, x_dtype=torch.float32, y_dtype=ydt, w_gran=Q.PER_ROW)
            plain, fused = mk(), QLinear(tag, M, N, K, x_dtype=torch.float32, y_dtype=ydt, w_gran=Q.PER_ROW,
                                         collect_y_amax=True)
            for op in (plain, fused):
                op.bias.copy_(dev(b))
                op.forward(dev(x), dev(w))
            torch.cuda.synchronize()
            assert torch.equal(plain.y, fused.y), "Y changes when the maximum is collected"
            want = fused.y.float().abs().max().item()
            assert fused.y_amax.item() == want, (fused.y_amax.item(), want)
            ref = orc.operator_fwd_bwd(tag, x, w, b, np.zeros((M, N), np.float32), "row", "nearest", y_dtype=np.float64)
            ref_amax = np.abs(ref["y"]).max()
            assert abs(fused.y_amax.item() - ref_amax) <= 2e-3 * ref_amax
            # the word is a running maximum: a larger value survives the next collection, then it is consumed
            fused.y_amax.fill_(want * 4.0)
            fused.gemm_fwd()
            torch.cuda.synchronize()
            assert fused.y_amax.item() == want * 4.0
            s_, i_ = torch.empty(1, device="cuda"), torch.empty(1, device="cuda")
            fused.y_amax.fill_(want)
            Q.qsync_scale_from_amax(fused.y_amax, 8, s_, i_, True)
            s2, i2, a2 = torch.empty(1, device="cuda"), torch.empty(1, device="cuda"), torch.empty(1, device="cuda")
            yf = fused.y.float().contiguous()
            ws = torch.zeros(max(256, Q.qsync_absmax_workspace_bytes(M, N, Q.PER_TENSOR)), dtype=torch.uint8, device="cuda")
            Q.qsync_absmax_scale(yf, M, N, N, Q.PER_TENSOR, 8, s2, i2, a2, None, ws)
            torch.cuda.synchronize()
            assert fused.y_amax.item() == 0.0
            assert_bits_equal(host(s_), host(s2), "scale from the collected maximum")
            assert_bits_equal(host(i_), host(i2), "inverse scale from the collected maximum")
            sref, iref = orc.scales_from_amax(np.asarray([want], np.float32), 8)
            assert_bits_equal(host(s_), sref, "scale vs oracle arithmetic")
            assert_bits_equal(host(i_), iref, "inverse scale vs oracle arithmetic")
    finally:
        Q.qsync_debug_set_gemm_tile(-1)


def test_chained_operator_takes_its_scale_from_the_producers_epilogue():
    """Two linears back to back (no nonlinearity in between, as after every odd layer of config 4): the consumer
    quantizes the producer's Y with the maximum the producer's epilogue collected.  Its codes, scales and
    accumulators equal those of a consumer that finds the maximum itself, and the oracle's on the same Y."""
    rng = np.random.default_rng(5)
    M, K0, N0, N1 = 1000, 256, 528, 264
    x = rng.standard_normal((M, K0)).astype(np.float32)
    w0 = (rng.standard_normal((N0, K0)) * 0.05).astype(np.float32)
    w1 = (rng.standard_normal((N1, N0)) * 0.05).astype(np.float32)
    prod = QLinear(Q.INT8, M, N0, K0, x_dtype=torch.float32, y_dtype=torch.float16, collect_y_amax=True, bias=False)
    cons = QLinear(Q.INT8, M, N1, N0, x_dtype=torch.float16, y_dtype=torch.float32, dump_acc=True, bias=False)
    base = QLinear(Q.INT8, M, N1, N0, x_dtype=torch.float16, y_dtype=torch.float32, dump_acc=True, bias=False)
    for step in range(2):            # twice: the consumed maximum starts the next step at zero
        y0 = prod.forward(dev(x), dev(w0))
        cons.forward(y0, dev(w1), x_amax=prod.y_amax)
        base.forward(y0, dev(w1))
        torch.cuda.synchronize()
        assert prod.y_amax.item() == 0.0
        for name in ("sx", "ix", "xq", "acc", "y"):
            assert torch.equal(getattr(cons, name), getattr(base, name)), (step, name)
    ref = orc.operator_fwd_bwd(Q.INT8, host(y0), w1, None, np.zeros((M, N1), np.float32), "row", "nearest",
                               y_dtype=np.float64)
    assert_bits_equal(host(cons.sx), ref["sx"], "sx")
    assert_bits_equal(host(cons.xq), ref["xq"], "xq")
    assert_bits_equal(host(cons.acc), ref["acc"], "accumulators")
    assert_close(host(cons.y), ref["y"], "Y")


@pytest.mark.parametrize("tag", [Q.INT8, Q.FP16])
def test_persistent_gemm_kernel_against_oracle_and_per_tile_kernel(tag):
    """The persistent 256x256 kernel (loader / storer wavefronts, next tile prefetched behind the epilogue) on
    outputs with fewer tiles than compute units, exactly as many, and more (some workgroups then walk two or
    three tiles): Y against the oracle's contraction element by element, and bit for bit against the per-tile
    kernel, which dequantizes with the same fused multiply-add."""
    rng = np.random.default_rng(90)
    try:
        for (M, N, K) in [(256, 256, 256), (512, 768, 512), (4096, 4096, 256), (8192, 2304, 256), (4352, 4352, 768),
                          (2816, 6656, 1280)]:
            say("persistent gemm", tag, M, N, K)
            bias = rng.standard_normal(N).astype(np.float32)
            if tag == Q.INT8:
                a = rng.integers(-127, 128, (M, K)).astype(np.int8)
                b = rng.integers(-127, 128, (N, K)).astype(np.int8)
                sx = np.array([0.004], np.float32)
                sw = (rng.random(N) * 0.002 + 0.0005).astype(np.float32)
                acc, ovf = orc.int_gemm_nt(a, b)
                assert not ovf
                want = acc.astype(np.float64) * float(sx[0]) * sw.astype(np.float64).reshape(1, -1) + bias.astype(np.float64)
                args = (dev(a), dev(sx), dev(b), dev(sw), Q.PER_ROW)
            else:
                a = rng.standard_normal((M, K)).astype(np.float16)
                b = (rng.standard_normal((N, K)) * 0.05).astype(np.float16)
                want = orc.float_gemm_nt(a, b) + bias.astype(np.float64)
                args = (dev(a), None, dev(b), None, Q.PER_TENSOR)
            w = torch.zeros(max(Q.qsync_qlinear_workspace_bytes(tag, M, N, K), 256), dtype=torch.uint8, device="cuda")
            ys = []
            for mode in (0, 1):
                Q.qsync_debug_set_gemm_persistent(mode)
                Q.qsync_debug_set_gemm_tile(0)
                y = torch.full((M, N), 7.0, dtype=torch.float16, device="cuda")
                Q.qsync_qlinear_fwd(tag, M, N, K, args[0], args[1], args[2], args[3], args[4], dev(bias), y, None, w)
                ys.append(host(y))
            assert_close(ys[1], want, "Y from the persistent kernel")
            assert_close(ys[0], want, "Y from the per-tile kernel")
            assert_bits_equal(ys[1], ys[0], "persistent against per-tile kernel")
    finally:
        Q.qsync_debug_set_gemm_persistent(-1)
        Q.qsync_debug_set_gemm_tile(-1)


@pytest.mark.parametrize("tile", [-1, 0, 1, 2])
@pytest.mark.parametrize("tag,ydt", [(Q.INT8, torch.float16), (Q.INT8, torch.float32), (Q.FP16, torch.float16),
                                     (Q.FP32, torch.float32)])
def test_forward_epilogue_writes_the_consumers_codes(tile, tag, ydt):
    """qsync_qlinear_fwd_codes: Y unchanged bit for bit; the codes equal the oracle's quantizer applied to the
    GPU's Y bits with the given inverse scale (both sides decide in fp32 on the stored value), and equal what
    qsync_quantize makes of that Y.  Shapes: 16-byte store path, element-wise path (N not a multiple of 16),
    ragged tiles, split K (the reduction pass writes the codes); a scale that clamps part of the values."""
    Q.qsync_debug_set_gemm_tile(tile)
    try:
        for (M, N, K) in [(300, 272, 272), (257, 136, 144), (64, 128, 128), (192, 272, 4096), (96, 104, 4096), (528, 1040, 400)]:
            rng = np.random.default_rng(M * 11 + N)
            x = rng.standard_normal((M, K)).astype(np.float32)
            w = (rng.standard_normal((N, K)) * 0.05).astype(np.float32)
            b = rng.standard_normal(N).astype(np.float32)
            say("fwd_codes tile", tile, "tag", tag, "ydt", ydt, "MNK", M, N, K)
            op = QLinear(tag, M, N, K, x_dtype=torch.float32, y_dtype=ydt, w_gran=Q.PER_ROW, collect_y_amax=True)
            op.bias.copy_(dev(b))
            op.forward(dev(x), dev(w))
            y_plain = host(op.y).copy()
            amax = float(np.abs(y_plain.astype(np.float32)).max())
            for bits, slack in ((8, 1.0), (8, 0.6), (5, 1.0)):            # slack < 1: the scale clamps the largest values
                qmax = (1 << (bits - 1)) - 1
                inv = np.array([np.float32(qmax) / np.float32(amax * slack)], np.float32)
                yq = torch.full((M, N), 99, dtype=torch.int8, device="cuda")
                op.y.fill_(0)
                op.y_amax.zero_()
                Q.qsync_qlinear_fwd_codes(tag, M, N, K, op.xq, op.sx, op.wq, op.sw, op.w_gran, op.bias, op.y, bits, dev(inv), yq,
                                          op.y_amax, op.ws_fwd)
                got_y = host(op.y)
                if N % 16 == 0:                       # same store path as the plain forward: the same bits
                    assert_bits_equal(got_y, y_plain, "Y with code output")
                    assert float(host(op.y_amax)[0]) == amax
                else:                                 # element-wise stores: a tie of the binary16 output may fall the other way
                    assert_close(got_y, y_plain.astype(np.float64), "Y with code output")
                    assert float(host(op.y_amax)[0]) == float(np.abs(got_y.astype(np.float32)).max())
                want = orc.quantize_int(got_y.astype(np.float32), inv, "tensor", "nearest", bits=bits)
                assert_bits_equal(host(yq), want, "codes from the epilogue")
                if slack < 1.0:
                    assert (np.abs(want) == qmax).sum() > 1
                q2 = torch.empty((M, N), dtype=torch.int8, device="cuda")
                Q.qsync_quantize(op.y, M, N, N, Q.INT8, bits, Q.PER_TENSOR, Q.ROUND_NEAREST, 0, 0, dev(inv), q2, None)
                assert torch.equal(q2, yq), "epilogue codes against the quantizer on the same Y"
    finally:
        Q.qsync_debug_set_gemm_tile(-1)


def test_transpose_of_codes():
    rng = np.random.default_rng(17)
    for rows, cols in [(16, 16), (128, 128), (1024, 4096), (272, 144), (48, 8208), (5, 7), (17, 64), (130, 66)]:
        say("transpose i8", rows, cols)
        a = rng.integers(-128, 128, (rows, cols)).astype(np.int8)
        out = torch.full((cols, rows), 3, dtype=torch.int8, device="cuda")
        Q.qsync_transpose_i8(dev(a), rows, cols, out)
        assert_bits_equal(host(out), np.ascontiguousarray(a.T), "transposed codes")


def test_chained_operator_consumes_codes_from_the_producers_epilogue():
    """Two INT8 linears back to back.  Step 0 runs the consumer's own quantizer and leaves its scale; in step 1 the
    producer's epilogue writes the consumer's codes with that scale (the activations barely move between steps, as
    in training), the consumer only transposes them.  Codes against the oracle's quantizer on the producer's Y bits;
    the consumer's accumulators and Y against the oracle's GEMM on those codes; its dW against the oracle too."""
    rng = np.random.default_rng(6)
    M, K0, N0, N1 = 1024, 256, 528, 272
    w0 = (rng.standard_normal((N0, K0)) * 0.05).astype(np.float32)
    w1 = (rng.standard_normal((N1, N0)) * 0.05).astype(np.float32)
    prod = QLinear(Q.INT8, M, N0, K0, x_dtype=torch.float32, y_dtype=torch.float16, collect_y_amax=True, bias=False)
    cons = QLinear(Q.INT8, M, N1, N0, x_dtype=torch.float16, y_dtype=torch.float32, dump_acc=True, bias=False)
    x0 = rng.standard_normal((M, K0)).astype(np.float32)
    y0 = prod.forward(dev(x0), dev(w0))
    cons.forward(y0, dev(w1))                                   # step 0: the consumer finds its own scale
    inv0 = host(cons.ix).copy()
    x1 = (x0 * 0.98).astype(np.float32)                         # step 1: slightly smaller activations, nothing clamps
    prod.convert_x(dev(x1)); prod.convert_w(dev(w0))
    prod.y_amax.zero_()
    prod.gemm_fwd_codes(cons)
    cons.forward_from_codes(dev(w1))
    dy = (rng.standard_normal((M, N1)) * 1e-2).astype(np.float32)
    cons.backward(dev(dy))
    y1 = host(prod.y)
    want_codes = orc.quantize_int(y1.astype(np.float32), inv0, "tensor", "nearest")
    assert float(host(prod.y_amax)[0]) * float(inv0[0]) <= 127.5
    assert_bits_equal(host(cons.xq), want_codes, "consumer codes written by the producer")
    if cons.xqT is not None:
        assert_bits_equal(host(cons.xqT), np.ascontiguousarray(want_codes.T), "their transpose")
    ref_w = orc.scales_from_amax(orc.absmax(w1, "row"))
    wq = orc.quantize_int(w1, ref_w[1], "row", "nearest")
    acc, ovf = orc.int_gemm_nt(want_codes, wq)
    assert not ovf
    assert_bits_equal(host(cons.acc), acc, "consumer accumulators")
    sx0 = host(cons.sx).astype(np.float64)
    assert_close(host(cons.y), acc.astype(np.float64) * sx0[0] * ref_w[0].astype(np.float64).reshape(1, -1), "consumer Y")
    ady = orc.absmax(dy, "tensor"); sdy, idy = orc.scales_from_amax(ady)
    dyq = orc.quantize_int(dy, idy, "tensor", "stochastic", cons.seed, cons.last_dy_offset)
    acc_dw, _ = orc.int_gemm_nt(np.ascontiguousarray(dyq.T), np.ascontiguousarray(want_codes.T))
    assert_bits_equal(host(cons.acc_dw), acc_dw, "consumer weight-gradient accumulators")


@pytest.mark.parametrize("tile", [-1, 0, 1, 2])
def test_weight_gradient_from_row_major_codes(tile):
    """qsync_qlinear_bwd_rm: dW = dY^T X from the row-major codes (no transposed copies; the GEMM transposes on the
    way from LDS into the matrix instructions), dX as before.  int32 accumulators bit for bit against the oracle,
    dW and dX values in tolerance, on every tile shape, ragged N and K (multiples of 16), one and several K tiles,
    split K."""
    rng = np.random.default_rng(123)
    Q.qsync_debug_set_gemm_tile(tile)
    try:
        for (M, N, K) in [(128, 16, 16), (128, 256, 256), (256, 272, 144), (384, 48, 528), (1024, 528, 272), (4096, 144, 80),
                          (8192, 1040, 784), (2048, 2064, 64)]:
            say("bwd_rm tile", tile, "MNK", M, N, K)
            dyq = rng.integers(-127, 128, (M, N)).astype(np.int8)
            xq = rng.integers(-127, 128, (M, K)).astype(np.int8)
            wqb = rng.integers(-127, 128, (N, K)).astype(np.int8)
            sdy, sx = np.array([3e-5], np.float32), np.array([0.01], np.float32)
            swb = (rng.random(K) * 0.002 + 0.0005).astype(np.float32)
            acc_dw, o1 = orc.int_gemm_nt(np.ascontiguousarray(dyq.T), np.ascontiguousarray(xq.T))
            acc_dx, o2 = orc.int_gemm_nt(dyq, np.ascontiguousarray(wqb.T))
            assert not (o1 or o2)
            dx, dw = torch.empty((M, K), dtype=torch.float16, device="cuda"), torch.empty((N, K), dtype=torch.float32, device="cuda")
            adx, adw = torch.empty((M, K), dtype=torch.int32, device="cuda"), torch.empty((N, K), dtype=torch.int32, device="cuda")
            w = torch.zeros(max(Q.qsync_qlinear_bwd_rm_workspace_bytes(Q.INT8, M, N, K), 256), dtype=torch.uint8, device="cuda")
            wqbT = dev(np.ascontiguousarray(wqb.T))
            Q.qsync_qlinear_bwd_rm(Q.INT8, M, N, K, dev(dyq), dev(sdy), dev(xq), dev(sx), wqbT, dev(swb), Q.PER_ROW, dx, dw, None, None,
                                   adx, adw, w)
            assert_bits_equal(host(adw), acc_dw, "dW accumulators (row-major operands)")
            assert_bits_equal(host(adx), acc_dx, "dX accumulators")
            want_dw = acc_dw.astype(np.float64) * float(sdy[0]) * float(sx[0])
            assert_close(host(dw), want_dw, "dW")
            # the production epilogue (no accumulator dump), fp32 and binary16 outputs
            for dt in (torch.float32, torch.float16):
                dw2 = torch.empty((N, K), dtype=dt, device="cuda")
                Q.qsync_qlinear_bwd_rm(Q.INT8, M, N, K, dev(dyq), dev(sdy), dev(xq), dev(sx), None, None, Q.PER_ROW, None, dw2, None, None,
                                       None, None, w)
                assert_close(host(dw2), want_dw, f"dW {dt} without dump")
    finally:
        Q.qsync_debug_set_gemm_tile(-1)


@pytest.mark.parametrize("tile", [-1, 0, 1, 2])
def test_weight_gradient_from_row_major_binary16_operands(tile):
    """qsync_qlinear_bwd_rm under the FP16 tag: dW = dY^T X from the row-major binary16 operands (16-bit transposing
    LDS reads), dX and db as in qsync_qlinear_bwd; against the oracle's float64 sums of the same binary16 values, on
    every tile shape, ragged N and K (multiples of 8), one and several K tiles, split K."""
    rng = np.random.default_rng(321)
    Q.qsync_debug_set_gemm_tile(tile)
    try:
        for (M, N, K) in [(128, 8, 8), (128, 256, 256), (256, 264, 136), (384, 40, 520), (1024, 520, 264), (4096, 136, 72),
                          (8192, 1032, 776), (2048, 2056, 64)]:
            say("bwd_rm fp16 tile", tile, "MNK", M, N, K)
            dyh = (rng.standard_normal((M, N)) * 0.01).astype(np.float16)
            xh = rng.standard_normal((M, K)).astype(np.float16)
            wh = (rng.standard_normal((N, K)) * 0.05).astype(np.float16)
            want_dw = orc.float_gemm_nt(np.ascontiguousarray(dyh.T), np.ascontiguousarray(xh.T))
            want_dx = orc.float_gemm_nt(dyh, np.ascontiguousarray(wh.T))
            want_db = dyh.astype(np.float64).sum(axis=0)
            dx, dw = torch.empty((M, K), dtype=torch.float16, device="cuda"), torch.empty((N, K), dtype=torch.float32, device="cuda")
            db = torch.empty(N, dtype=torch.float32, device="cuda")
            w = torch.zeros(max(Q.qsync_qlinear_bwd_rm_workspace_bytes(Q.FP16, M, N, K), 256), dtype=torch.uint8, device="cuda")
            d_dy = dev(dyh)
            Q.qsync_qlinear_bwd_rm(Q.FP16, M, N, K, d_dy, None, dev(xh), None, dev(np.ascontiguousarray(wh.T)), None, Q.PER_TENSOR,
                                   dx, dw, db, d_dy, None, None, w)
            assert_close(host(dw), want_dw, "dW (row-major binary16 operands)")
            assert_close(host(dx), want_dx, "dX")
            assert_close(host(db), want_db, "db")
            dw16 = torch.empty((N, K), dtype=torch.float16, device="cuda")
            Q.qsync_qlinear_bwd_rm(Q.FP16, M, N, K, d_dy, None, dev(xh), None, None, None, Q.PER_TENSOR, None, dw16, None, None,
                                   None, None, w)
            assert_close(host(dw16), want_dw, "dW binary16 output")
    finally:
        Q.qsync_debug_set_gemm_tile(-1)
