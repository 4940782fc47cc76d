"""GPU parity of the single-read paths: mxfp4_quantize_dual (row-wise and column-wise quantisation of
one tensor from one pass, App. D layouts) and the training pair mxfp4_linear_fwd_save /
mxfp4_linear_bwd_saved (Fig. 3: X and W feed Fprop and both backward GEMMs).  Every quantised byte is
compared with the oracle's two independent single-axis quantisations; GEMM outputs as in the other
linear tests."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_09825_amd as mx
from paper_2605_09825_amd import synth
from gpu_util import first_mismatch
from test_gpu_gemm import assert_close, structured_check
from test_gpu_linear import ws_slices

pytestmark = pytest.mark.gpu

HADS = [mx.HAD_NONE, mx.HAD_DET, mx.HAD_RANDSIGN, mx.HAD_DET16, mx.HAD_RANDSIGN16]
RNDS = [mx.RNE, mx.SR]


def check_dual(t_cpu, had, rnd, seed=0, x_gpu=None):
    x = t_cpu.to("cuda:0") if x_gpu is None else x_gpu
    ql, sl, qf, sf = mx.mxfp4_quantize_dual(x, had, rnd, seed)
    torch.cuda.synchronize()
    xb = synth.as_u16(t_cpu.contiguous())
    for name, axis, q, s in (("last", mx.AXIS_LAST, ql, sl), ("first", mx.AXIS_FIRST, qf, sf)):
        qo, so = oracle.quantize(xb, axis, had, rnd, seed)
        assert np.array_equal(s.cpu().numpy(), so), f"{name} scales: " + first_mismatch(s.cpu().numpy(), so)
        assert np.array_equal(q.cpu().numpy(), qo), f"{name} codes: " + first_mismatch(q.cpu().numpy(), qo)


@pytest.mark.parametrize("had", HADS)
@pytest.mark.parametrize("rnd", RNDS)
@pytest.mark.parametrize("shape", [(256, 128), (32, 32), (96, 160), (288, 416), (1056, 256), (512, 1024)])
def test_dual_modes_and_ragged_shapes(shape, had, rnd):
    check_dual(synth.normal(shape[0], shape[1], 1.0, 4, synth.STREAM_DY), had, rnd, seed=987654321)


@pytest.mark.parametrize("had", [mx.HAD_NONE, mx.HAD_DET])
def test_dual_leading_dimension(had):
    base = synth.normal(320, 640, 1.0, 5, synth.STREAM_X)
    view = base[32:288, 64:576]
    xg = base.to("cuda:0")[32:288, 64:576]
    check_dual(view, had, mx.RNE, x_gpu=xg)
    check_dual(view, had, mx.SR, seed=5, x_gpu=xg)


@pytest.mark.parametrize("had", HADS)
def test_dual_value_distributions(had):
    check_dual(synth.normal_with_outlier_channels(512, 1024, 6, synth.STREAM_X, fraction=0.004), had, mx.RNE)
    check_dual(synth.student_t3(512, 512, 1e-3, 6, synth.STREAM_DY), had, mx.RNE)
    check_dual(synth.from_bits(np.arange(65536, dtype=np.uint16).reshape(256, 256)), had, mx.RNE)
    check_dual(synth.from_bits(np.arange(65536, dtype=np.uint16).reshape(256, 256)), had, mx.SR, seed=9)


def test_dual_empty_and_argument_errors():
    z = torch.empty((0, 64), dtype=torch.bfloat16, device="cuda:0")
    ql, sl, qf, sf = mx.mxfp4_quantize_dual(z)
    assert ql.numel() == 0 and qf.numel() == 0
    x = torch.zeros((48, 64), dtype=torch.bfloat16, device="cuda:0")  # rows not a multiple of 32
    with pytest.raises(mx.Mxfp4Error) as e:
        mx.mxfp4_quantize_dual(x)
    assert e.value.status == mx.ESHAPE
    x = torch.zeros((64, 48), dtype=torch.bfloat16, device="cuda:0")  # cols not a multiple of 32
    with pytest.raises(mx.Mxfp4Error) as e:
        mx.mxfp4_quantize_dual(x)
    assert e.value.status == mx.ESHAPE


def saved_slices(saved, M, N, K):
    off = mx.mxfp4_linear_saved_layout(M, N, K)
    b = saved.cpu().numpy()
    out = []
    for k, (R, C) in enumerate([(K, N), (K, M)]):
        q = b[off[2 * k]: off[2 * k] + R * C // 2].reshape(R, C // 2)
        s = b[off[2 * k + 1]: off[2 * k + 1] + R * C // 32].reshape(R, C // 32)
        out.append((q, s))
    return out


def run_pair(x, w, dy, had, rnd, seed, full):
    """fwd_save + bwd_saved; byte parity of all six operands; outputs in full or on samples."""
    M, K = x.shape
    N = w.shape[0]
    cfg = mx.make_cfg(had, rnd, seed, y_dtype=mx.OUT_FP32, dx_dtype=mx.OUT_FP32, dw_dtype=mx.OUT_FP32)
    xg, wg, dyg = x.to("cuda:0"), w.to("cuda:0"), dy.to("cuda:0")
    y, ws_f, saved = mx.mxfp4_linear_fwd_save(xg, wg, cfg)
    del xg, wg  # the backward call must not need them
    dx, dw, ws_b = mx.mxfp4_linear_bwd_saved(dyg, saved, K, cfg)
    torch.cuda.synchronize()
    xb, wb, dyb = synth.as_u16(x), synth.as_u16(w), synth.as_u16(dy)
    ops_f = oracle.linear_fwd_operands(xb, wb, had, rnd, seed)
    ops_d = oracle.linear_dgrad_operands(dyb, wb, had, rnd, seed)
    ops_w = oracle.linear_wgrad_operands(dyb, xb, had, rnd, seed)
    fw = ws_slices(ws_f, M, N, K, False)
    bw = ws_slices(ws_b, M, N, K, True)
    sv = saved_slices(saved, M, N, K)
    got = {"X": fw[0], "W": fw[1], "dY": bw[0], "W^T": sv[0], "dY^T": bw[2], "X^T": sv[1]}
    want = {"X": ops_f[0], "W": ops_f[1], "dY": ops_d[0], "W^T": ops_d[1], "dY^T": ops_w[0], "X^T": ops_w[1]}
    for name in got:
        assert np.array_equal(got[name][1], want[name][1]), f"{name}: scale bytes differ"
        assert np.array_equal(got[name][0], want[name][0]), f"{name}: packed codes differ"
    if full:
        yo, ya = oracle.linear_fwd(xb, wb, had, rnd, seed)
        (dxo, dxa), (dwo, dwa) = oracle.linear_bwd(dyb, xb, wb, had, rnd, seed)
        assert_close(y.cpu().numpy(), yo, ya)
        assert_close(dx.cpu().numpy(), dxo, dxa)
        assert_close(dw.cpu().numpy(), dwo, dwa)
    else:
        rng = np.random.default_rng(11)
        for out, ((aq, as_), (bq, bs)) in ((y, ops_f), (dx, ops_d), (dw, ops_w)):
            structured_check(out.cpu().numpy(), (aq, as_), (bq, bs), rng)


@pytest.mark.parametrize("had,rnd", [(mx.HAD_NONE, mx.RNE), (mx.HAD_DET, mx.RNE), (mx.HAD_RANDSIGN, mx.RNE),
                                     (mx.HAD_NONE, mx.SR), (mx.HAD_DET16, mx.RNE), (mx.HAD_RANDSIGN16, mx.SR)])
@pytest.mark.parametrize("shape", [(256, 512, 512), (96, 160, 224)])
def test_training_pair(shape, had, rnd):
    M, N, K = shape
    run_pair(synth.normal(M, K, 1.0, 1, synth.STREAM_X), synth.normal(N, K, 0.02, 1, synth.STREAM_W),
             synth.normal(M, N, 1e-3, 1, synth.STREAM_DY), had, rnd, 77, full=True)


def test_training_pair_one_gradient_only_and_accumulate():
    M, N, K = 256, 512, 512
    x = synth.normal(M, K, 1.0, 2, synth.STREAM_X)
    w = synth.normal(N, K, 0.02, 2, synth.STREAM_W)
    dy = synth.normal(M, N, 1e-3, 2, synth.STREAM_DY)
    cfg = mx.make_cfg(mx.HAD_DET, dx_dtype=mx.OUT_FP32, dw_dtype=mx.OUT_FP32)
    _, _, saved = mx.mxfp4_linear_fwd_save(x.to("cuda:0"), w.to("cuda:0"), cfg)
    dyg = dy.to("cuda:0")
    dx_ref, dw_ref, _ = mx.mxfp4_linear_bwd_saved(dyg, saved, K, cfg)
    dx_only, none_dw, _ = mx.mxfp4_linear_bwd_saved(dyg, saved, K, cfg, need_dw=False)
    none_dx, dw_only, _ = mx.mxfp4_linear_bwd_saved(dyg, saved, K, cfg, need_dx=False)
    assert none_dw is None and none_dx is None
    assert torch.equal(dx_only, dx_ref) and torch.equal(dw_only, dw_ref)
    acc = mx.make_cfg(mx.HAD_DET, dx_dtype=mx.OUT_FP32, dw_dtype=mx.OUT_FP32, dw_accumulate=True)
    dw_acc = torch.ones((N, K), dtype=torch.float32, device="cuda:0")
    mx.mxfp4_linear_bwd_saved(dyg, saved, K, acc, dw=dw_acc, need_dx=False)
    torch.cuda.synchronize()
    assert torch.equal(dw_acc, dw_ref + 1.0)


def test_training_pair_config2_full_size():
    # Llama-3.1-8B fused QKV projection, deterministic Hadamard, RNE: the shape bench.py times
    M, K, N = 8192, 4096, 6144
    run_pair(synth.normal(M, K, 1.0, 0, synth.STREAM_X), synth.normal(N, K, 0.02, 0, synth.STREAM_W),
             synth.normal(M, N, 1e-3, 0, synth.STREAM_DY), mx.HAD_DET, mx.RNE, 0, full=False)
