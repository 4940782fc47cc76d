"""The library calls only enqueue kernels on the caller's stream (no allocation, no memset, no
synchronisation), so a training step can be recorded into a HIP graph.  A recorded step (Fig. 3:
Fprop, then Dgrad and Wgrad) is replayed several times with new inputs, eager work in between, and
every replay must reproduce the eager result bit for bit."""
import pytest
import torch

import paper_2605_09825_amd as mx
from paper_2605_09825_amd import synth

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("shape,had,rnd", [((512, 768, 1024), mx.HAD_DET, mx.RNE),
                                           ((512, 768, 1024), mx.HAD_NONE, mx.SR),
                                           ((96, 160, 224), mx.HAD_RANDSIGN, mx.RNE)])
def test_recorded_training_step_replays_bit_exactly(shape, had, rnd):
    M, N, K = shape
    dev = "cuda:0"
    cfg = mx.make_cfg(had, rnd, 5, y_dtype=mx.OUT_BF16, dx_dtype=mx.OUT_BF16, dw_dtype=mx.OUT_FP32)
    inputs = [(synth.normal(M, K, 1.0, i, synth.STREAM_X).to(dev), synth.normal(N, K, 0.02, i, synth.STREAM_W).to(dev),
               synth.normal(M, N, 1e-3, i, synth.STREAM_DY).to(dev)) for i in range(3)]

    def eager(x, w, dy):
        y, _, saved = mx.mxfp4_linear_fwd_save(x, w, cfg)
        dx, dw, _ = mx.mxfp4_linear_bwd_saved(dy, saved, K, cfg)
        torch.cuda.synchronize()
        return y.clone(), dx.clone(), dw.clone()

    want = [eager(*t) for t in inputs]

    # static buffers of the recorded step
    x, w, dy = (torch.empty_like(t) for t in inputs[0])
    y = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
    dx = torch.empty((M, K), dtype=torch.bfloat16, device=dev)
    dw = torch.empty((N, K), dtype=torch.float32, device=dev)
    ws_f = torch.empty(mx.mxfp4_linear_workspace_bytes(M, N, K, cfg, False), dtype=torch.uint8, device=dev)
    ws_b = torch.empty(mx.mxfp4_linear_workspace_bytes(M, N, K, cfg, True), dtype=torch.uint8, device=dev)
    saved = torch.empty(mx.mxfp4_linear_saved_bytes(M, N, K, cfg), dtype=torch.uint8, device=dev)

    def step():
        mx.mxfp4_linear_fwd_save(x, w, cfg, y=y, workspace=ws_f, saved=saved)
        mx.mxfp4_linear_bwd_saved(dy, saved, K, cfg, dx=dx, dw=dw, workspace=ws_b)

    for src, dst in zip(inputs[0], (x, w, dy)):
        dst.copy_(src)
    step()  # once outside the recording
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for i in (1, 2, 0, 1):
        for src, dst in zip(inputs[i], (x, w, dy)):
            dst.copy_(src)
        for t in (y, dx, dw, ws_f, ws_b, saved):
            t.fill_(0x5A if t.dtype == torch.uint8 else 3.0)  # eager work between replays; stale outputs gone
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, want[i][0]), f"replay with inputs {i}: Y differs"
        assert torch.equal(dx, want[i][1]), f"replay with inputs {i}: dX differs"
        assert torch.equal(dw, want[i][2]), f"replay with inputs {i}: dW differs"


def test_recorded_forward_on_the_static_scratch_replays_bit_exactly():
    # mxfp4_linear_fwd_static is there for code under graph capture that may not allocate or pass a workspace: after
    # one call outside the recording (which looks the scratch array's address up) the call is recorded and replayed
    # with new inputs; a different, smaller call on the same scratch runs eagerly between the replays
    M, N, K = 768, 1024, 1280     # 3 x 4 tiles: the 256 x 128-tile GEMM
    dev = "cuda:0"
    cfg = mx.make_cfg(mx.HAD_DET, mx.RNE, 9, y_dtype=mx.OUT_BF16)
    inputs = [(synth.normal(M, K, 1.0, 10 + i, synth.STREAM_X).to(dev), synth.normal(N, K, 0.02, 10 + i, synth.STREAM_W).to(dev))
              for i in range(3)]
    want = []
    for x_, w_ in inputs:
        y_, _ = mx.mxfp4_linear_fwd(x_, w_, cfg)
        torch.cuda.synchronize()
        want.append(y_.clone())
    x, w = (torch.empty_like(t) for t in inputs[0])
    y = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
    xs, ws_ = synth.normal(96, 224, 1.0, 3, synth.STREAM_X).to(dev), synth.normal(160, 224, 0.02, 3, synth.STREAM_W).to(dev)
    ys = torch.empty((96, 160), dtype=torch.bfloat16, device=dev)
    ys_want, _ = mx.mxfp4_linear_fwd(xs, ws_, cfg)
    x.copy_(inputs[0][0])
    w.copy_(inputs[0][1])
    mx.mxfp4_linear_fwd_static(x, w, cfg, y)   # outside the recording
    torch.cuda.synchronize()
    assert torch.equal(y, want[0])
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        mx.mxfp4_linear_fwd_static(x, w, cfg, y)
    for i in (1, 2, 0):
        x.copy_(inputs[i][0])
        w.copy_(inputs[i][1])
        y.fill_(3.0)
        mx.mxfp4_linear_fwd_static(xs, ws_, cfg, ys)   # eager, on the same scratch array, before the replay
        torch.cuda.synchronize()
        assert torch.equal(ys, ys_want)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, want[i]), f"replay with inputs {i}: Y differs"


def test_recorded_gemm_with_a_part_filled_last_round_replays_bit_exactly():
    # 320 tiles of 256 x 256 on 256 compute units: one round of 256 x 256 tiles, then 256 x 128 tiles on the rest
    Ra, Rb, C = 256 * 40, 256 * 8, 1024
    dev = "cuda:0"
    g = torch.Generator(device=dev)
    g.manual_seed(1)
    ops = [tuple(torch.randint(lo, hi, shape, dtype=torch.uint8, device=dev, generator=g)
                 for lo, hi, shape in ((0, 256, (Ra, C // 2)), (118, 132, (Ra, C // 32)), (0, 256, (Rb, C // 2)),
                                       (118, 132, (Rb, C // 32)))) for _ in range(2)]
    want = [mx.mxfp4_gemm(*o, out_dtype=mx.OUT_FP32).clone() for o in ops]
    torch.cuda.synchronize()
    bufs = tuple(torch.empty_like(t) for t in ops[0])
    out = torch.empty((Ra, Rb), dtype=torch.float32, device=dev)
    for s_, d_ in zip(ops[0], bufs):
        d_.copy_(s_)
    mx.mxfp4_gemm(*bufs, out=out, out_dtype=mx.OUT_FP32)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        mx.mxfp4_gemm(*bufs, out=out, out_dtype=mx.OUT_FP32)
    for i in (1, 0, 1):
        for s_, d_ in zip(ops[i], bufs):
            d_.copy_(s_)
        out.fill_(5.0)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, want[i])
