"""GPU parity of mxfp4_quantize against the CPU oracle: packed codes and scale bytes must be
bit-exact (App. A.1 eq. (1), App. A.2, App. D)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_09825_amd as mx
from paper_2605_09825_amd import synth
from gpu_util import first_mismatch, gpu_quantize

pytestmark = pytest.mark.gpu

HADS = [mx.HAD_NONE, mx.HAD_DET, mx.HAD_RANDSIGN, mx.HAD_DET16, mx.HAD_RANDSIGN16]
RNDS = [mx.RNE, mx.SR]


def check(t_cpu, axis, had, rnd, seed=0):
    q, s = gpu_quantize(t_cpu, axis, had, rnd, seed)
    xb = synth.as_u16(t_cpu.contiguous()) if not t_cpu.is_contiguous() else synth.as_u16(t_cpu)
    qo, so = oracle.quantize(xb, axis, had, rnd, seed)
    assert np.array_equal(s, so), "scales: " + first_mismatch(s, so)
    assert np.array_equal(q, qo), "codes: " + first_mismatch(q, qo)


def test_config1_operands_bit_exact():
    # X [256,512] ~ N(0,1), W [512,512] ~ N(0, 0.02), seed 0; blocks along K, RNE, no rotation
    check(synth.normal(256, 512, 1.0, 0, synth.STREAM_X), mx.AXIS_LAST, mx.HAD_NONE, mx.RNE)
    check(synth.normal(512, 512, 0.02, 0, synth.STREAM_W), mx.AXIS_LAST, mx.HAD_NONE, mx.RNE)


@pytest.mark.parametrize("had", HADS)
@pytest.mark.parametrize("rnd", RNDS)
@pytest.mark.parametrize("shape", [(256, 512), (37, 96), (1, 32), (300, 4096)])
def test_rows_modes_and_ragged_shapes(shape, had, rnd):
    check(synth.normal(shape[0], shape[1], 1.0, 3, synth.STREAM_X), mx.AXIS_LAST, had, rnd, seed=1234567891011)


@pytest.mark.parametrize("had", HADS)
@pytest.mark.parametrize("rnd", RNDS)
@pytest.mark.parametrize("shape", [(256, 128), (96, 74), (32, 2), (288, 130), (1056, 258), (512, 1024)])
def test_cols_modes_and_ragged_shapes(shape, had, rnd):
    check(synth.normal(shape[0], shape[1], 1.0, 4, synth.STREAM_DY), mx.AXIS_FIRST, had, rnd, seed=987654321)


@pytest.mark.parametrize("axis", [mx.AXIS_LAST, mx.AXIS_FIRST])
@pytest.mark.parametrize("had", [mx.HAD_NONE, mx.HAD_DET])
def test_leading_dimension(axis, had):
    base = synth.normal(320, 640, 1.0, 5, synth.STREAM_X)
    check(base[32:288, 64:576], axis, had, mx.RNE)
    check(base[32:288, 64:576], axis, had, mx.SR, seed=5)


@pytest.mark.parametrize("axis", [mx.AXIS_LAST, mx.AXIS_FIRST])
@pytest.mark.parametrize("had", HADS)
def test_value_distributions(axis, had):
    check(synth.normal_with_outlier_channels(512, 1024, 6, synth.STREAM_X, fraction=0.004), axis, had, mx.RNE)
    check(synth.student_t3(512, 512, 1e-3, 6, synth.STREAM_DY), axis, had, mx.RNE)
    check(synth.normal(256, 512, 1e-30, 6, synth.STREAM_W), axis, had, mx.RNE)
    check(synth.normal(256, 512, 1e30, 6, synth.STREAM_W), axis, had, mx.RNE)
    check(synth.small_integers(256, 256, -8, 8, 6, synth.STREAM_X), axis, had, mx.RNE)


@pytest.mark.parametrize("axis", [mx.AXIS_LAST, mx.AXIS_FIRST])
@pytest.mark.parametrize("had", HADS)
@pytest.mark.parametrize("rnd", RNDS)
def test_every_bf16_bit_pattern(axis, had, rnd):
    # all 65536 patterns, in natural order (neighbours share an exponent: every mantissa and every
    # rounding tie of the FP4 cast occurs) -- includes zeros, subnormals, infinities and NaNs
    bits = np.arange(65536, dtype=np.uint16).reshape(256, 256)
    check(synth.from_bits(bits), axis, had, rnd, seed=42)
    # and shuffled, so that blocks mix magnitudes (finite patterns only)
    finite = bits.reshape(-1)[(bits.reshape(-1) & 0x7F80) != 0x7F80]
    rng = np.random.default_rng(0)
    mixed = rng.permutation(finite)[: 254 * 256].reshape(254 * 256 // 512, 512)
    check(synth.from_bits(mixed[:96]), axis, had, rnd, seed=43)


@pytest.mark.parametrize("axis", [mx.AXIS_LAST, mx.AXIS_FIRST])
def test_tiny_and_signed_zero_blocks(axis):
    x = np.zeros((64, 64), dtype=np.float32)
    x[0, :32] = -0.0
    x[1, 3] = 1.5 * 2.0**-126
    x[1, 4] = -(2.0**-127)
    x[2, 7] = 2.0**-133          # smallest bf16 subnormal
    x[3, :] = -1e-38
    x[40, 40] = 3.3895e38        # near the largest bf16
    t = torch.from_numpy(x).to(torch.bfloat16)
    for had in HADS:
        check(t, axis, had, mx.RNE)
        check(t, axis, had, mx.SR, seed=9)


def test_empty_calls_are_accepted():
    z = torch.empty((0, 64), dtype=torch.bfloat16, device="cuda:0")
    q, s = mx.mxfp4_quantize(z)
    assert q.shape == (0, 32) and s.shape == (0, 2)
    z2 = torch.empty((64, 0), dtype=torch.bfloat16, device="cuda:0")
    q, s = mx.mxfp4_quantize(z2, axis=mx.AXIS_FIRST)
    assert q.shape == (0, 32) and s.shape == (0, 2)


def test_seed_changes_stochastic_modes_only():
    t = synth.normal(128, 256, 1.0, 8, synth.STREAM_X)
    a = gpu_quantize(t, mx.AXIS_LAST, mx.HAD_DET, mx.RNE, seed=1)
    b = gpu_quantize(t, mx.AXIS_LAST, mx.HAD_DET, mx.RNE, seed=2)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    c = gpu_quantize(t, mx.AXIS_LAST, mx.HAD_NONE, mx.SR, seed=1)
    d = gpu_quantize(t, mx.AXIS_LAST, mx.HAD_NONE, mx.SR, seed=2)
    assert not np.array_equal(c[0], d[0])


def test_repeat_runs_are_bitwise_identical():
    t = synth.normal(1024, 1024, 1.0, 10, synth.STREAM_X)
    ref = gpu_quantize(t, mx.AXIS_FIRST, mx.HAD_DET, mx.SR, seed=3)
    for _ in range(3):
        again = gpu_quantize(t, mx.AXIS_FIRST, mx.HAD_DET, mx.SR, seed=3)
        assert np.array_equal(ref[0], again[0]) and np.array_equal(ref[1], again[1])


# ---- full-size tensors of the benchmark configurations (never sampled: every byte compared)
@pytest.mark.parametrize("axis", [mx.AXIS_LAST, mx.AXIS_FIRST])
def test_config2_full_size(axis):
    check(synth.normal(8192, 4096, 1.0, 0, synth.STREAM_X), axis, mx.HAD_DET, mx.RNE)
    check(synth.normal(6144, 4096, 0.02, 0, synth.STREAM_W), axis, mx.HAD_DET, mx.RNE)
    check(synth.normal(8192, 6144, 1e-3, 0, synth.STREAM_DY), axis, mx.HAD_DET, mx.RNE)


def test_config4_wgrad_operands_full_size():
    dy = synth.student_t3(16384, 4096, 1e-3, 0, synth.STREAM_DY)
    check(dy, mx.AXIS_FIRST, mx.HAD_DET, mx.RNE)
    check(dy, mx.AXIS_FIRST, mx.HAD_RANDSIGN, mx.RNE, seed=4)
    check(dy, mx.AXIS_FIRST, mx.HAD_NONE, mx.SR, seed=4)
    x = synth.normal(16384, 14336, 1.0, 0, synth.STREAM_X)
    check(x, mx.AXIS_FIRST, mx.HAD_DET, mx.RNE)
    check(x, mx.AXIS_LAST, mx.HAD_DET, mx.RNE)   # (448 MiB: the row-wise kernel's variant for tensors beyond the cache)


def test_more_than_2_32_elements_stochastic_rounding_counters():
    # 131104 x 32768 = 4.296e9 elements (8.6 GB of bf16): block and byte offsets beyond 2^31 and
    # stochastic-rounding counters beyond 2^32 (the high word of the counter enters the hash)
    rows, cols = 131072 + 32, 32768
    block = synth.as_u16(synth.normal(4097, cols, 1.0, 12, synth.STREAM_X))
    x = np.tile(block, (32, 1))
    assert x.shape == (rows, cols) and x.size > 2**32
    t = synth.from_bits(x)
    q, s = gpu_quantize(t, mx.AXIS_LAST, mx.HAD_NONE, mx.SR, seed=77)
    qo, so = oracle.quantize(x, oracle.AXIS_LAST, oracle.HAD_NONE, oracle.SR, 77)
    assert np.array_equal(s, so)
    assert np.array_equal(q, qo), "codes: " + first_mismatch(q, qo)
    # the same values at different positions round differently (the counter, not the value, decides)
    assert not np.array_equal(q[:4097], q[-4097:])


def test_blocks_that_expose_the_rotation_rounding_order(golden_dir):
    # the input blocks of tests/golden/rotation_sensitive_blocks.txt sit next to an FP4 rounding threshold after the
    # rotation: a multiply placed before the butterflies, a constant one ulp off or another stage order changes
    # their codes.  Row-wise (one block per row) and column-wise (one block per column, padded to 2 columns)
    import os
    rows = []
    for line in open(os.path.join(golden_dir, "rotation_sensitive_blocks.txt")):
        if line.startswith("#") or not line.strip():
            continue
        rows.append([int(h, 16) for h in line.split()[1:]])
    blocks = synth.from_bits(np.array(rows, dtype=np.uint16))        # [16][32]
    assert blocks.shape[1] == 32 and blocks.shape[0] % 2 == 0
    for had in (mx.HAD_DET, mx.HAD_RANDSIGN):
        check(blocks, mx.AXIS_LAST, had, mx.RNE, seed=0 if had == mx.HAD_DET else 99)
    check(blocks.t().contiguous(), mx.AXIS_FIRST, mx.HAD_DET, mx.RNE)
    # both ways at once: the blocks as the 32 columns of a 32 x 32 tensor (the 16 of them twice)
    sq = torch.cat([blocks, blocks], dim=0).t().contiguous()
    ql, sl, qf, sf = mx.mxfp4_quantize_dual(sq.to("cuda:0"), mx.HAD_DET)
    torch.cuda.synchronize()
    qo, so = oracle.quantize(synth.as_u16(sq), oracle.AXIS_FIRST, oracle.HAD_DET)
    assert np.array_equal(qf.cpu().numpy(), qo) and np.array_equal(sf.cpu().numpy(), so)
    qo, so = oracle.quantize(synth.as_u16(sq), oracle.AXIS_LAST, oracle.HAD_DET)
    assert np.array_equal(ql.cpu().numpy(), qo) and np.array_equal(sl.cpu().numpy(), so)
