"""Helpers shared by the GPU parity tests: move seeded host tensors to the device, call the
library through its Python binding (= the C ABI), bring results back as numpy."""
import numpy as np
import torch

import paper_2605_09825_amd as mx
from paper_2605_09825_amd import synth


def dev():
    return torch.device("cuda:0")


def to_gpu_bf16(t_cpu: torch.Tensor) -> torch.Tensor:
    assert t_cpu.dtype == torch.bfloat16
    return t_cpu.to(dev())


def gpu_quantize(t_cpu: torch.Tensor, axis=mx.AXIS_LAST, had=mx.HAD_NONE, rnd=mx.RNE, seed=0):
    """Quantise a CPU bf16 tensor (possibly a strided row view) on the GPU; numpy (q, s) back."""
    if t_cpu.is_contiguous():
        x = to_gpu_bf16(t_cpu)
    else:  # keep the leading dimension: copy the base storage, then take the same view
        base = t_cpu._base
        assert base is not None and base.dim() == 2
        off = t_cpu.storage_offset() - base.storage_offset()
        r0, c0 = divmod(off, base.stride(0))
        x = to_gpu_bf16(base)[r0:r0 + t_cpu.shape[0], c0:c0 + t_cpu.shape[1]]
    q, s = mx.mxfp4_quantize(x, axis, had, rnd, seed)
    torch.cuda.synchronize()
    return q.cpu().numpy(), s.cpu().numpy()


def first_mismatch(a: np.ndarray, b: np.ndarray) -> str:
    if a.shape != b.shape:
        return f"shape {a.shape} vs {b.shape}"
    bad = np.argwhere(a != b)
    if bad.size == 0:
        return "equal"
    i = tuple(bad[0])
    return f"{len(bad)} of {a.size} differ; first at {i}: gpu {a[i]:#x} vs oracle {b[i]:#x}"
