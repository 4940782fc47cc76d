"""The forward call that allocates nothing (mxfp4_linear_fwd_static: operands staged in the library's static
device array) against mxfp4_linear_fwd, called through the C ABI with raw pointers: outputs must be equal bit
for bit on two calls in a row, the second with a smaller input, and sizes beyond the array are refused."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2605_09825_amd as mx
from paper_2605_09825_amd import synth

pytestmark = pytest.mark.gpu


def fwd_both_ways(M, N, K, had, rnd, y_dtype, seed):
    L = mx.lib()
    dev = torch.device("cuda:0")
    x = synth.normal(M, K, 1.0, seed, synth.STREAM_X).to(dev)
    w = synth.normal(N, K, 0.02, seed, synth.STREAM_W).to(dev)
    cfg = mx.make_cfg(had, rnd, 1234 + seed, y_dtype=y_dtype)
    tdt = torch.float32 if y_dtype == mx.OUT_FP32 else torch.bfloat16
    need = L.mxfp4_linear_workspace_bytes(M, N, K, ctypes.byref(cfg), 0)
    ws = torch.empty(need, dtype=torch.uint8, device=dev)
    y_ref = torch.zeros((M, N), dtype=tdt, device=dev)
    y_new = torch.full((M, N), 7.0, dtype=tdt, device=dev)
    st = torch.cuda.current_stream().cuda_stream
    torch.cuda.synchronize()
    rc = L.mxfp4_linear_fwd(x.data_ptr(), w.data_ptr(), y_ref.data_ptr(), M, N, K, ctypes.byref(cfg),
                            ws.data_ptr(), need, st)
    assert rc == mx.OK
    before = torch.cuda.memory_allocated()
    rc = L.mxfp4_linear_fwd_static(x.data_ptr(), w.data_ptr(), y_new.data_ptr(), M, N, K, ctypes.byref(cfg), st)
    assert rc == mx.OK, mx.status_string(rc)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    a = y_ref.view(torch.int32 if y_dtype == mx.OUT_FP32 else torch.int16).cpu().numpy()
    b = y_new.view(torch.int32 if y_dtype == mx.OUT_FP32 else torch.int16).cpu().numpy()
    return a, b


def test_static_scratch_forward_equals_workspace_forward_twice():
    # first call: 3 x 3 tiles of the tiled GEMM plus ragged edges, rotated, fp32 out; the second is smaller
    # (its operands overwrite only the front of the array, the rest still holds the first call's bytes)
    a, b = fwd_both_ways(800, 832, 1280, mx.HAD_DET, mx.RNE, mx.OUT_FP32, 1)
    assert np.array_equal(a, b)
    a, b = fwd_both_ways(96, 160, 224, mx.HAD_RANDSIGN, mx.SR, mx.OUT_BF16, 2)
    assert np.array_equal(a, b)
    # and a larger one again after the small one
    a, b = fwd_both_ways(512, 768, 2048, mx.HAD_DET16, mx.RNE, mx.OUT_BF16, 3)
    assert np.array_equal(a, b)


def test_static_scratch_limit_and_argument_errors():
    L = mx.lib()
    cfg = mx.make_cfg(mx.HAD_DET, mx.RNE, 0)
    P = 0x10000
    # 8192 x 4096 and 6144 x 4096 operands need 29.75 MiB: accepted sizes end at 32 MiB
    assert L.mxfp4_linear_workspace_bytes(8192, 6144, 4096, ctypes.byref(cfg), 0) <= mx.STATIC_SCRATCH_BYTES
    assert L.mxfp4_linear_fwd_static(P, P, P, 16384, 6144, 4096, ctypes.byref(cfg), None) == mx.EWORKSPACE
    assert L.mxfp4_linear_fwd_static(P, P, P, 1 << 40, 1 << 40, 1 << 40, ctypes.byref(cfg), None) == mx.EWORKSPACE
    assert L.mxfp4_linear_fwd_static(P, P, P, 64, 64, 48, ctypes.byref(cfg), None) == mx.ESHAPE
    assert L.mxfp4_linear_fwd_static(None, P, P, 64, 64, 64, ctypes.byref(cfg), None) == mx.EINVAL
    assert L.mxfp4_linear_fwd_static(P, P, P, 64, 64, 64, None, None) == mx.EINVAL
