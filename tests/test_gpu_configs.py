"""GPU parity at the full sizes of the benchmark configurations 3, 4 and 5 (Llama-3.1-8B linear
shapes, Sec. 2.2): every quantised byte of every operand is compared with the oracle; GEMM outputs
are compared on complete K-sums at a 16x16 patch inside every 256x256 output tile, 64 whole rows and
64 whole columns (the oracle cannot finish the 0.4-1.9 TFLOP products of configurations 3-5; configuration 2
is compared whole).  Inputs are the seeded synthetic stand-ins for the paper's training tensors."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_09825_amd as mx
from paper_2605_09825_amd import synth
from test_gpu_gemm import assert_close, structured_check
from test_gpu_linear import ws_slices

pytestmark = pytest.mark.gpu


def check_linear(x, w, dy, had, rnd=mx.RNE, seed=0, tag=""):
    """fwd + bwd through the fused calls; byte parity of all six quantised operands; Y, dX, dW on a patch in
    every output tile plus whole rows and columns."""
    M, K = x.shape
    N = w.shape[0]
    print(f"[{tag}] M={M} N={N} K={K} had={had} rnd={rnd}", flush=True)
    cfg = mx.make_cfg(had, rnd, seed, y_dtype=mx.OUT_FP32, dx_dtype=mx.OUT_FP32, dw_dtype=mx.OUT_FP32)
    xg, wg, dyg = x.to("cuda:0"), w.to("cuda:0"), dy.to("cuda:0")
    y, ws_f = mx.mxfp4_linear_fwd(xg, wg, cfg)
    dx, dw, ws_b = mx.mxfp4_linear_bwd(dyg, xg, wg, cfg)
    torch.cuda.synchronize()
    del xg, wg, dyg
    xb, wb, dyb = synth.as_u16(x), synth.as_u16(w), synth.as_u16(dy)
    ops_f = oracle.linear_fwd_operands(xb, wb, had, rnd, seed)
    ops_d = oracle.linear_dgrad_operands(dyb, wb, had, rnd, seed)
    ops_w = oracle.linear_wgrad_operands(dyb, xb, had, rnd, seed)
    names = ["X", "W", "dY", "W^T", "dY^T", "X^T"]
    got = ws_slices(ws_f, M, N, K, False) + ws_slices(ws_b, M, N, K, True)
    for name, (q, s), (qo, so) in zip(names, got, list(ops_f) + list(ops_d) + list(ops_w)):
        assert np.array_equal(s, so), f"{tag} {name}: scale bytes differ"
        assert np.array_equal(q, qo), f"{tag} {name}: packed codes differ"
    rng = np.random.default_rng(7)
    for name, out, ((aq, as_), (bq, bs)) in (("Y", y, ops_f), ("dX", dx, ops_d), ("dW", dw, ops_w)):
        structured_check(out.cpu().numpy(), (aq, as_), (bq, bs), rng)


@pytest.mark.parametrize("had", [mx.HAD_DET, mx.HAD_NONE])
def test_config3_mlp_gate_up_with_outlier_channels(had):
    # fused gate/up projection: K=4096, N=28672, M=8192; 0.1 % of the activation channels x100
    M, K, N = 8192, 4096, 28672
    x = synth.normal_with_outlier_channels(M, K, 0, synth.STREAM_X)
    w = synth.normal(N, K, 0.02, 0, synth.STREAM_W)
    dy = synth.normal(M, N, 1e-3, 0, synth.STREAM_DY)
    check_linear(x, w, dy, had, tag="cfg3 gate/up")


@pytest.mark.parametrize("had", [mx.HAD_DET, mx.HAD_NONE])
def test_config3_mlp_down_with_outlier_channels(had):
    M, K, N = 8192, 14336, 4096
    x = synth.normal_with_outlier_channels(M, K, 1, synth.STREAM_X)
    w = synth.normal(N, K, 0.02, 1, synth.STREAM_W)
    dy = synth.normal(M, N, 1e-3, 1, synth.STREAM_DY)
    check_linear(x, w, dy, had, tag="cfg3 down")


def test_config3_hadamard_lowers_the_error_with_outliers():
    # informational direction check of App. A.2's claim on the config-3 activations (smaller slice)
    M, K, N = 1024, 4096, 1024
    x = synth.normal_with_outlier_channels(M, K, 0, synth.STREAM_X)
    w = synth.normal(N, K, 0.02, 0, synth.STREAM_W)
    ref = x.to(torch.float64) @ w.to(torch.float64).T
    errs = {}
    for had in (mx.HAD_NONE, mx.HAD_DET):
        cfg = mx.make_cfg(had, y_dtype=mx.OUT_FP32)
        y, _ = mx.mxfp4_linear_fwd(x.to("cuda:0"), w.to("cuda:0"), cfg)
        torch.cuda.synchronize()
        errs[had] = float(torch.linalg.norm(y.cpu().to(torch.float64) - ref) / torch.linalg.norm(ref))
    assert errs[mx.HAD_DET] < errs[mx.HAD_NONE], errs


@pytest.mark.parametrize("had,rnd", [(mx.HAD_DET, mx.RNE), (mx.HAD_RANDSIGN, mx.RNE), (mx.HAD_NONE, mx.SR)])
def test_config4_wgrad_stress(had, rnd):
    # dW = dY^T X contracting over 16384 tokens; heavy-tailed gradients; both operands quantised
    # down the token axis
    M, N, K = 16384, 4096, 14336
    seed = 2024
    dy = synth.student_t3(M, N, 1e-3, 0, synth.STREAM_DY)
    x = synth.normal(M, K, 1.0, 0, synth.STREAM_X)
    print(f"[cfg4] had={had} rnd={rnd}", flush=True)
    cfg = mx.make_cfg(had, rnd, seed, dw_dtype=mx.OUT_FP32)
    dyg, xg = dy.to("cuda:0"), x.to("cuda:0")
    _, dw, ws = mx.mxfp4_linear_bwd(dyg, xg, None, cfg, need_dx=False)
    torch.cuda.synchronize()
    del dyg, xg
    (gtq, gts), (xtq, xts) = oracle.linear_wgrad_operands(synth.as_u16(dy), synth.as_u16(x), had, rnd, seed)
    got = ws_slices(ws, M, N, K, True)
    assert np.array_equal(got[2][1], gts) and np.array_equal(got[2][0], gtq), "dY^T"
    assert np.array_equal(got[3][1], xts) and np.array_equal(got[3][0], xtq), "X^T"
    assert dw.shape == (N, K)
    structured_check(dw.cpu().numpy(), (gtq, gts), (xtq, xts), np.random.default_rng(3))


LAYER = [  # Llama-3.1-8B decoder layer linears: name, in-features K, out-features N
    ("q", 4096, 4096), ("k", 4096, 1024), ("v", 4096, 1024), ("o", 4096, 4096),
    ("gate", 4096, 14336), ("up", 4096, 14336), ("down", 14336, 4096),
]


@pytest.mark.parametrize("name,K,N", LAYER)
def test_config5_decoder_layer_linear(name, K, N):
    # seq 8192 x batch 1; deterministic Hadamard; Fprop + Dgrad + Wgrad of each of the 7 linears
    M = 8192
    idx = [n for n, _, _ in LAYER].index(name)
    x = synth.normal(M, K, 1.0, 5, synth.STREAM_X + 16 * (K == 14336))  # q,k,v share X; gate,up share X
    w = synth.normal(N, K, 0.02, 5 + idx, synth.STREAM_W)
    dy = synth.normal(M, N, 1e-3, 5 + idx, synth.STREAM_DY)
    check_linear(x, w, dy, mx.HAD_DET, tag=f"cfg5 {name}")


def test_config2_all_stages_whole_outputs():
    # Llama-3.1-8B fused QKV projection (M=8192, K=4096, N=6144, deterministic H32, RNE), the workload bench.py
    # times: every element of Y, dX and dW, through the plain calls and through the training pair (whose
    # backward call runs Dgrad and Wgrad side by side in one launch), against the oracle's fp64 sums
    M, K, N = 8192, 4096, 6144
    x = synth.normal(M, K, 1.0, 0, synth.STREAM_X)
    w = synth.normal(N, K, 0.02, 0, synth.STREAM_W)
    dy = synth.normal(M, N, 1e-3, 0, synth.STREAM_DY)
    cfg = mx.make_cfg(mx.HAD_DET, mx.RNE, 0, y_dtype=mx.OUT_FP32, dx_dtype=mx.OUT_FP32, dw_dtype=mx.OUT_FP32)
    xg, wg, dyg = x.to("cuda:0"), w.to("cuda:0"), dy.to("cuda:0")
    y, ws_f = mx.mxfp4_linear_fwd(xg, wg, cfg)
    dx, dw, ws_b = mx.mxfp4_linear_bwd(dyg, xg, wg, cfg)
    y2, _, saved = mx.mxfp4_linear_fwd_save(xg, wg, cfg)
    dx2, dw2, _ = mx.mxfp4_linear_bwd_saved(dyg, saved, K, cfg)
    dx1, _, _ = mx.mxfp4_linear_bwd(dyg, xg, wg, cfg, need_dw=False)     # each gradient alone: one launch each
    _, dw1, _ = mx.mxfp4_linear_bwd(dyg, xg, wg, cfg, need_dx=False)
    torch.cuda.synchronize()
    assert torch.equal(y, y2) and torch.equal(dx, dx2) and torch.equal(dw, dw2)
    assert torch.equal(dx, dx1) and torch.equal(dw, dw1)
    xb, wb, dyb = synth.as_u16(x), synth.as_u16(w), synth.as_u16(dy)
    stages = (("Y", y, oracle.linear_fwd_operands(xb, wb, mx.HAD_DET)),
              ("dX", dx, oracle.linear_dgrad_operands(dyb, wb, mx.HAD_DET)),
              ("dW", dw, oracle.linear_wgrad_operands(dyb, xb, mx.HAD_DET)))
    got_ops = ws_slices(ws_f, M, N, K, False) + ws_slices(ws_b, M, N, K, True)
    k = 0
    for name, out, (a, b) in stages:
        for (q, s_), (qo, so) in zip(got_ops[k:k + 2], (a, b)):
            assert np.array_equal(s_, so) and np.array_equal(q, qo), f"{name}: quantised operand differs"
        k += 2
        print(f"[cfg2 whole output] {name}", flush=True)
        want, absum = oracle.gemm(a[0], a[1], b[0], b[1])
        assert_close(out.cpu().numpy(), want, absum)
        del want, absum
