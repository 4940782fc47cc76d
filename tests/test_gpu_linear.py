"""GPU parity of the fused linear calls against the oracle's composition of quantise and GEMM,
stage by stage (App. C.1 Fprop, C.2 Dgrad, C.3 Wgrad)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_09825_amd as mx
from paper_2605_09825_amd import synth
from test_gpu_gemm import assert_close, structured_check

pytestmark = pytest.mark.gpu


def ws_slices(ws, M, N, K, bwd):
    off = mx.mxfp4_linear_workspace_layout(M, N, K, bwd)
    w = ws.cpu().numpy()
    if not bwd:
        dims = [(M, K), (N, K)]
    else:
        dims = [(M, N), (K, N), (N, M), (K, M)]
    out = []
    for k, (R, C) in enumerate(dims):
        q = w[off[2 * k]: off[2 * k] + R * C // 2].reshape(R, C // 2)
        s = w[off[2 * k + 1]: off[2 * k + 1] + R * C // 32].reshape(R, C // 32)
        out.append((q, s))
    return out


@pytest.mark.parametrize("had,rnd", [(mx.HAD_NONE, mx.RNE), (mx.HAD_DET, mx.RNE), (mx.HAD_RANDSIGN, mx.RNE),
                                     (mx.HAD_NONE, mx.SR), (mx.HAD_DET16, mx.RNE), (mx.HAD_RANDSIGN16, mx.SR)])
@pytest.mark.parametrize("shape", [(256, 512, 512), (96, 160, 224)])
def test_linear_fwd_and_bwd(shape, had, rnd):
    M, N, K = shape
    seed = 77
    x = synth.normal(M, K, 1.0, 1, synth.STREAM_X)
    w = synth.normal(N, K, 0.02, 1, synth.STREAM_W)
    dy = synth.normal(M, N, 1e-3, 1, synth.STREAM_DY)
    cfg = mx.make_cfg(had, rnd, seed, y_dtype=mx.OUT_FP32, dx_dtype=mx.OUT_FP32, dw_dtype=mx.OUT_FP32)
    xg, wg, dyg = x.to("cuda:0"), w.to("cuda:0"), dy.to("cuda:0")
    y, ws_f = mx.mxfp4_linear_fwd(xg, wg, cfg)
    dx, dw, ws_b = mx.mxfp4_linear_bwd(dyg, xg, wg, cfg)
    torch.cuda.synchronize()
    xb, wb, dyb = synth.as_u16(x), synth.as_u16(w), synth.as_u16(dy)

    # operands left in the workspace: byte parity with the oracle's quantiser
    ops_f = oracle.linear_fwd_operands(xb, wb, had, rnd, seed)
    for (q, s), (qo, so) in zip(ws_slices(ws_f, M, N, K, False), ops_f):
        assert np.array_equal(q, qo) and np.array_equal(s, so)
    ops_b = list(oracle.linear_dgrad_operands(dyb, wb, had, rnd, seed)) + \
        list(oracle.linear_wgrad_operands(dyb, xb, had, rnd, seed))
    for (q, s), (qo, so) in zip(ws_slices(ws_b, M, N, K, True), ops_b):
        assert np.array_equal(q, qo) and np.array_equal(s, so)

    yo, ya = oracle.linear_fwd(xb, wb, had, rnd, seed)
    (dxo, dxa), (dwo, dwa) = oracle.linear_bwd(dyb, xb, wb, had, rnd, seed)
    assert y.shape == (M, N) and dx.shape == (M, K) and dw.shape == (N, K)
    assert_close(y.cpu().numpy(), yo, ya)
    assert_close(dx.cpu().numpy(), dxo, dxa)
    assert_close(dw.cpu().numpy(), dwo, dwa)


def test_bwd_skips_and_accumulates():
    M, N, K = 64, 96, 128
    x = synth.normal(M, K, 1.0, 2, synth.STREAM_X).to("cuda:0")
    w = synth.normal(N, K, 0.02, 2, synth.STREAM_W).to("cuda:0")
    dy = synth.normal(M, N, 1e-3, 2, synth.STREAM_DY).to("cuda:0")
    cfg = mx.make_cfg(mx.HAD_DET, dx_dtype=mx.OUT_BF16, dw_dtype=mx.OUT_FP32)
    dx, dw, _ = mx.mxfp4_linear_bwd(dy, x, w, cfg)
    dx_only, none_dw, _ = mx.mxfp4_linear_bwd(dy, None, w, cfg, need_dw=False)
    none_dx, dw_only, _ = mx.mxfp4_linear_bwd(dy, x, None, cfg, need_dx=False)
    torch.cuda.synchronize()
    assert none_dw is None and none_dx is None
    assert torch.equal(dx, dx_only) and torch.equal(dw, dw_only)
    acc = mx.make_cfg(mx.HAD_DET, dx_dtype=mx.OUT_BF16, dw_dtype=mx.OUT_FP32, dw_accumulate=True)
    dw2 = dw.clone()
    mx.mxfp4_linear_bwd(dy, x, w, acc, dw=dw2, need_dx=False)
    torch.cuda.synchronize()
    assert torch.allclose(dw2, 2 * dw, rtol=1e-6, atol=0)


def test_operands_of_a_gemm_round_under_their_own_streams_and_share_the_sign_diagonal():
    # random-sign rotation + stochastic rounding, seed with bits in its stream field: each of the six operands
    # must equal the single-tensor quantiser's output under seed ^ (k << 48)
    M, N, K = 128, 160, 96
    seed = 0xABCD_1234_5678_9ABC
    x = synth.normal(M, K, 1.0, 3, synth.STREAM_X)
    w = synth.normal(N, K, 0.02, 3, synth.STREAM_W)
    dy = synth.normal(M, N, 1e-3, 3, synth.STREAM_DY)
    cfg = mx.make_cfg(mx.HAD_RANDSIGN, mx.SR, seed, y_dtype=mx.OUT_FP32, dx_dtype=mx.OUT_FP32, dw_dtype=mx.OUT_FP32)
    xg, wg, dyg = x.to("cuda:0"), w.to("cuda:0"), dy.to("cuda:0")
    _, ws_f = mx.mxfp4_linear_fwd(xg, wg, cfg)
    _, _, ws_b = mx.mxfp4_linear_bwd(dyg, xg, wg, cfg)
    torch.cuda.synchronize()
    got = ws_slices(ws_f, M, N, K, False) + ws_slices(ws_b, M, N, K, True)
    src = [(xg, mx.AXIS_LAST), (wg, mx.AXIS_LAST), (dyg, mx.AXIS_LAST), (wg, mx.AXIS_FIRST), (dyg, mx.AXIS_FIRST),
           (xg, mx.AXIS_FIRST)]
    cpu = {id(xg): x, id(wg): w, id(dyg): dy}
    for k, ((t, axis), (q, s)) in enumerate(zip(src, got)):
        sk = seed ^ (k << 48)
        q1, s1 = mx.mxfp4_quantize(t, axis, mx.HAD_RANDSIGN, mx.SR, sk)
        qo, so = oracle.quantize(synth.as_u16(cpu[id(t)]), axis, oracle.HAD_RANDSIGN, oracle.SR, sk)
        assert np.array_equal(q, q1.cpu().numpy()) and np.array_equal(s, s1.cpu().numpy()), k
        assert np.array_equal(q, qo) and np.array_equal(s, so), k
    # (same base seed, so the same diagonal: operands 0 and 1 differ from a run with another stream only in rounding)
    assert oracle.sign_mask(seed) == oracle.sign_mask(seed ^ (5 << 48))


def test_config2_all_three_stages_every_tile():
    # Llama-3.1-8B fused QKV: M=8192, K=4096, N=6144, deterministic Hadamard, RNE
    M, N, K = 8192, 6144, 4096
    x = synth.normal(M, K, 1.0, 0, synth.STREAM_X)
    w = synth.normal(N, K, 0.02, 0, synth.STREAM_W)
    dy = synth.normal(M, N, 1e-3, 0, synth.STREAM_DY)
    cfg = mx.make_cfg(mx.HAD_DET, y_dtype=mx.OUT_FP32, dx_dtype=mx.OUT_FP32, dw_dtype=mx.OUT_FP32)
    xg, wg, dyg = x.to("cuda:0"), w.to("cuda:0"), dy.to("cuda:0")
    y, _ = mx.mxfp4_linear_fwd(xg, wg, cfg)
    dx, dw, _ = mx.mxfp4_linear_bwd(dyg, xg, wg, cfg)
    torch.cuda.synchronize()
    xb, wb, dyb = synth.as_u16(x), synth.as_u16(w), synth.as_u16(dy)
    rng = np.random.default_rng(1)
    stages = [
        (y, oracle.linear_fwd_operands(xb, wb, mx.HAD_DET)),
        (dx, oracle.linear_dgrad_operands(dyb, wb, mx.HAD_DET)),
        (dw, oracle.linear_wgrad_operands(dyb, xb, mx.HAD_DET)),
    ]
    for out, ((aq, as_), (bq, bs)) in stages:
        structured_check(out.cpu().numpy(), (aq, as_), (bq, bs), rng)


def test_calls_enqueue_on_the_stream_they_are_given_and_nowhere_else():
    # The calls only enqueue on the caller's stream.  A side stream is held busy by a spin kernel, the forward and
    # backward calls are given that stream while the default stream is current: as long as the spin kernel runs
    # none of their outputs may have been touched, and once the side stream has drained they must be complete.
    M, N, K = 512, 768, 1024
    dev = "cuda:0"
    cfg = mx.make_cfg(mx.HAD_DET, mx.RNE, 3, y_dtype=mx.OUT_FP32, dx_dtype=mx.OUT_FP32, dw_dtype=mx.OUT_FP32)
    x = synth.normal(M, K, 1.0, 4, synth.STREAM_X).to(dev)
    w = synth.normal(N, K, 0.02, 4, synth.STREAM_W).to(dev)
    dy = synth.normal(M, N, 1e-3, 4, synth.STREAM_DY).to(dev)
    y_ref, _ = mx.mxfp4_linear_fwd(x, w, cfg)
    dx_ref, dw_ref, _ = mx.mxfp4_linear_bwd(dy, x, w, cfg)
    y = torch.full((M, N), 7.0, dtype=torch.float32, device=dev)
    dx = torch.full((M, K), 7.0, dtype=torch.float32, device=dev)
    dw = torch.full((N, K), 7.0, dtype=torch.float32, device=dev)
    ws_f = torch.empty(mx.mxfp4_linear_workspace_bytes(M, N, K, cfg, False), dtype=torch.uint8, device=dev)
    ws_b = torch.empty(mx.mxfp4_linear_workspace_bytes(M, N, K, cfg, True), dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        torch.cuda._sleep(int(4e8))   # a bounded spin (a fraction of a second) that keeps the side stream busy
    mx.mxfp4_linear_fwd(x, w, cfg, y=y, workspace=ws_f, stream=side)
    mx.mxfp4_linear_bwd(dy, x, w, cfg, dx=dx, dw=dw, workspace=ws_b, stream=side)
    torch.cuda.current_stream().synchronize()          # whatever went to the default stream has run by now
    untouched = all(bool((t == 7.0).all()) for t in (y, dx, dw))
    still_spinning = not side.query()
    side.synchronize()
    if still_spinning:
        assert untouched, "a call ran ahead of the work queued before it on its stream"
    assert torch.equal(y, y_ref) and torch.equal(dx, dx_ref) and torch.equal(dw, dw_ref)
