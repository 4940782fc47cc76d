"""GPU parity of the 32 x 32 block-scaling geometry (App. D): mxfp4_quantize_2d against the oracle's
2D quantiser, byte for byte, and the linear calls with geometry = MXFP4_GEOM_2D against the oracle's
composition."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_09825_amd as mx
from paper_2605_09825_amd import synth
from gpu_util import first_mismatch
from test_gpu_gemm import assert_close, structured_check
from test_gpu_linear import ws_slices
from test_gpu_dual import saved_slices

pytestmark = pytest.mark.gpu

HADS = [mx.HAD_NONE, mx.HAD_DET, mx.HAD_RANDSIGN, mx.HAD_DET16, mx.HAD_RANDSIGN16]
RNDS = [mx.RNE, mx.SR]


def check_2d(t_cpu, had, rnd, seed=0, x_gpu=None, want_last=True, want_first=True):
    x = t_cpu.to("cuda:0") if x_gpu is None else x_gpu
    ql, sl, qf, sf = mx.mxfp4_quantize_2d(x, had, rnd, seed, want_last, want_first)
    torch.cuda.synchronize()
    xb = synth.as_u16(t_cpu.contiguous())
    assert (ql is None) == (not want_last) and (qf is None) == (not want_first)
    for name, axis, q, s in (("last", mx.AXIS_LAST, ql, sl), ("first", mx.AXIS_FIRST, qf, sf)):
        if q is None:
            continue
        qo, so = oracle.quantize_2d(xb, axis, had, rnd, seed)
        assert np.array_equal(s.cpu().numpy(), so), f"{name} scales: " + first_mismatch(s.cpu().numpy(), so)
        assert np.array_equal(q.cpu().numpy(), qo), f"{name} codes: " + first_mismatch(q.cpu().numpy(), qo)


@pytest.mark.parametrize("had", HADS)
@pytest.mark.parametrize("rnd", RNDS)
@pytest.mark.parametrize("shape", [(256, 128), (32, 32), (96, 160), (288, 416), (1056, 256), (512, 1024)])
def test_2d_modes_and_ragged_shapes(shape, had, rnd):
    check_2d(synth.student_t3(shape[0], shape[1], 1.0, 4, synth.STREAM_DY), had, rnd, seed=192837465)


@pytest.mark.parametrize("want", [(True, False), (False, True)])
@pytest.mark.parametrize("had", [mx.HAD_NONE, mx.HAD_DET])
def test_2d_single_output(want, had):
    check_2d(synth.normal(288, 416, 1.0, 5, synth.STREAM_X), had, mx.RNE, want_last=want[0], want_first=want[1])
    check_2d(synth.normal(288, 416, 1.0, 5, synth.STREAM_X), had, mx.SR, seed=3, want_last=want[0], want_first=want[1])


def test_2d_leading_dimension_and_distributions():
    base = synth.normal(320, 640, 1.0, 5, synth.STREAM_X)
    check_2d(base[32:288, 64:576], mx.HAD_DET, mx.RNE, x_gpu=base.to("cuda:0")[32:288, 64:576])
    check_2d(synth.normal_with_outlier_channels(512, 1024, 6, synth.STREAM_X, fraction=0.004), mx.HAD_NONE, mx.RNE)
    bits = np.arange(65536, dtype=np.uint16).reshape(256, 256)  # every bf16 pattern, NaN and Inf included
    for had in HADS:
        check_2d(synth.from_bits(bits), had, mx.RNE)
        check_2d(synth.from_bits(bits), had, mx.SR, seed=9)


def test_2d_transposition_invariance_on_the_gpu():
    x = synth.normal(256, 384, 1.0, 7, synth.STREAM_W).to("cuda:0")
    ql, sl, qf, sf = mx.mxfp4_quantize_2d(x)
    ql, qf = ql.cpu().numpy(), qf.cpu().numpy()
    unpack = lambda q: np.stack([q & 15, q >> 4], axis=-1).reshape(q.shape[0], -1)
    assert np.array_equal(unpack(qf), unpack(ql).T)
    slr, sfr = sl.cpu().numpy(), sf.cpu().numpy()
    for rb in range(8):
        for cb in range(12):
            assert slr[rb * 32, cb] == sfr[cb * 32, rb]


def test_2d_argument_errors():
    x = torch.zeros((48, 64), dtype=torch.bfloat16, device="cuda:0")
    with pytest.raises(mx.Mxfp4Error) as e:
        mx.mxfp4_quantize_2d(x)
    assert e.value.status == mx.ESHAPE
    x = torch.zeros((64, 64), dtype=torch.bfloat16, device="cuda:0")
    with pytest.raises(mx.Mxfp4Error) as e:
        mx.mxfp4_quantize_2d(x, want_last=False, want_first=False)
    assert e.value.status == mx.EINVAL
    z = torch.empty((0, 64), dtype=torch.bfloat16, device="cuda:0")
    assert mx.mxfp4_quantize_2d(z)[0].numel() == 0


def run_linear_2d(x, w, dy, had, rnd, seed, full, saved_path):
    M, K = x.shape
    N = w.shape[0]
    cfg = mx.make_cfg(had, rnd, seed, y_dtype=mx.OUT_FP32, dx_dtype=mx.OUT_FP32, dw_dtype=mx.OUT_FP32,
                      geometry=mx.GEOM_2D)
    xg, wg, dyg = x.to("cuda:0"), w.to("cuda:0"), dy.to("cuda:0")
    if saved_path:
        y, ws_f, saved = mx.mxfp4_linear_fwd_save(xg, wg, cfg)
        dx, dw, ws_b = mx.mxfp4_linear_bwd_saved(dyg, saved, K, cfg)
    else:
        y, ws_f = mx.mxfp4_linear_fwd(xg, wg, cfg)
        dx, dw, ws_b = mx.mxfp4_linear_bwd(dyg, xg, wg, cfg)
    torch.cuda.synchronize()
    xb, wb, dyb = synth.as_u16(x), synth.as_u16(w), synth.as_u16(dy)
    g2 = oracle.GEOM_2D
    ops_f = oracle.linear_fwd_operands(xb, wb, had, rnd, seed, g2)
    ops_d = oracle.linear_dgrad_operands(dyb, wb, had, rnd, seed, g2)
    ops_w = oracle.linear_wgrad_operands(dyb, xb, had, rnd, seed, g2)
    fw, bw = ws_slices(ws_f, M, N, K, False), ws_slices(ws_b, M, N, K, True)
    if saved_path:
        sv = saved_slices(saved, M, N, K)
        got = {"X": fw[0], "W": fw[1], "dY": bw[0], "W^T": sv[0], "dY^T": bw[2], "X^T": sv[1]}
    else:
        got = {"X": fw[0], "W": fw[1], "dY": bw[0], "W^T": bw[1], "dY^T": bw[2], "X^T": bw[3]}
    want = {"X": ops_f[0], "W": ops_f[1], "dY": ops_d[0], "W^T": ops_d[1], "dY^T": ops_w[0], "X^T": ops_w[1]}
    for name in got:
        assert np.array_equal(got[name][1], want[name][1]), f"{name}: scale bytes differ"
        assert np.array_equal(got[name][0], want[name][0]), f"{name}: packed codes differ"
    if full:
        yo, ya = oracle.linear_fwd(xb, wb, had, rnd, seed, g2)
        (dxo, dxa), (dwo, dwa) = oracle.linear_bwd(dyb, xb, wb, had, rnd, seed, g2)
        assert_close(y.cpu().numpy(), yo, ya)
        assert_close(dx.cpu().numpy(), dxo, dxa)
        assert_close(dw.cpu().numpy(), dwo, dwa)
    else:
        rng = np.random.default_rng(13)
        for out, ((aq, as_), (bq, bs)) in ((y, ops_f), (dx, ops_d), (dw, ops_w)):
            structured_check(out.cpu().numpy(), (aq, as_), (bq, bs), rng)


@pytest.mark.parametrize("saved_path", [False, True])
@pytest.mark.parametrize("had,rnd", [(mx.HAD_NONE, mx.RNE), (mx.HAD_DET, mx.RNE), (mx.HAD_NONE, mx.SR)])
@pytest.mark.parametrize("shape", [(256, 512, 512), (96, 160, 224)])
def test_linear_with_2d_geometry(shape, had, rnd, saved_path):
    M, N, K = shape
    run_linear_2d(synth.normal(M, K, 1.0, 1, synth.STREAM_X), synth.normal(N, K, 0.02, 1, synth.STREAM_W),
                  synth.normal(M, N, 1e-3, 1, synth.STREAM_DY), had, rnd, 77, True, saved_path)


def test_linear_2d_rejects_ragged_shapes():
    cfg = mx.make_cfg(geometry=mx.GEOM_2D)
    x = torch.zeros((48, 64), dtype=torch.bfloat16, device="cuda:0")
    w = torch.zeros((64, 64), dtype=torch.bfloat16, device="cuda:0")
    with pytest.raises(mx.Mxfp4Error) as e:
        mx.mxfp4_linear_fwd(x, w, cfg)
    assert e.value.status == mx.ESHAPE


def test_linear_2d_config2_full_size():
    # the benchmark shape with 2D scaling and no rotation: W's two quantisations are transposes of each other
    M, K, N = 8192, 4096, 6144
    run_linear_2d(synth.normal(M, K, 1.0, 0, synth.STREAM_X), synth.normal(N, K, 0.02, 0, synth.STREAM_W),
                  synth.normal(M, N, 1e-3, 0, synth.STREAM_DY), mx.HAD_NONE, mx.RNE, 0, False, True)
