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
