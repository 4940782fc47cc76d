"""GPU parity of mxfp4_gemm against the CPU oracle (plain fp64 sum of decoded products).
Tolerance, written out: |gpu - oracle| <= 1e-5 * sum_c |a_c||b_c| on the fp32 output."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_09825_amd as mx
from paper_2605_09825_amd import synth

pytestmark = pytest.mark.gpu
RTOL = 1e-5


def rand_operand(rng, R, C, s_lo=115, s_hi=135):
    q = rng.integers(0, 256, size=(R, C // 2), dtype=np.uint8)
    s = rng.integers(s_lo, s_hi, size=(R, C // 32), dtype=np.uint8)
    return q, s


def gpu(t):
    return torch.from_numpy(np.ascontiguousarray(t)).to("cuda:0")


def run_gemm(aq, as_, bq, bs, **kw):
    out = mx.mxfp4_gemm(gpu(aq), gpu(as_), gpu(bq), gpu(bs), **kw)
    torch.cuda.synchronize()
    return out


def assert_close(got, want, absum):
    err = np.abs(got.astype(np.float64) - want)
    bound = RTOL * absum
    worst = np.argmax(err - bound)
    assert (err <= bound).all(), (f"max err/absum {np.max(err / np.maximum(absum, 1e-300)):.3e}; "
                                  f"at {np.unravel_index(worst, err.shape)} got {got.flat[worst]} want {want.flat[worst]}")


@pytest.mark.parametrize("shape", [(64, 64, 128), (16, 16, 32), (37, 53, 96), (1, 1, 32), (256, 512, 512),
                                   (130, 70, 1024), (512, 384, 4096), (100, 260, 160), (512, 768, 1536),
                                   (256, 256, 1024), (768, 512, 2560), (512, 256, 1280), (256, 768, 1792)])
def test_random_codes_fp32(shape):
    Ra, Rb, C = shape
    rng = np.random.default_rng(Ra * 7 + Rb * 3 + C)
    aq, as_ = rand_operand(rng, Ra, C)
    bq, bs = rand_operand(rng, Rb, C)
    want, absum = oracle.gemm(aq, as_, bq, bs)
    got = run_gemm(aq, as_, bq, bs, out_dtype=mx.OUT_FP32).cpu().numpy()
    assert_close(got, want, absum)


@pytest.mark.parametrize("shape", [(300, 520, 1024), (544, 784, 1536), (320, 256, 2048), (256, 257, 1024),
                                   (1030, 513, 1024), (300, 520, 1280)])
def test_ragged_rows_and_columns_around_whole_tiles(shape):
    # row / column counts that leave edge strips beside a 256-aligned interior (different kernels write the
    # interior and the strips): every output element once, nothing outside
    Ra, Rb, C = shape
    rng = np.random.default_rng(Ra * 5 + Rb * 11 + C)
    aq, as_ = rand_operand(rng, Ra, C)
    bq, bs = rand_operand(rng, Rb, C)
    want, absum = oracle.gemm(aq, as_, bq, bs)
    ld = Rb + 8 - Rb % 8 + 8  # padded rows: the padding must stay untouched
    canvas = torch.full((Ra + 1, ld), 7.0, dtype=torch.float32, device="cuda:0")
    mx.mxfp4_gemm(gpu(aq), gpu(as_), gpu(bq), gpu(bs), out=canvas[:Ra, :Rb], out_dtype=mx.OUT_FP32)
    torch.cuda.synchronize()
    c = canvas.cpu().numpy()
    assert_close(c[:Ra, :Rb], want, absum)
    assert np.all(c[:Ra, Rb:] == 7.0) and np.all(c[Ra] == 7.0)
    # accumulate on top, and bf16 output = RNE of the fp32 result
    mx.mxfp4_gemm(gpu(aq), gpu(as_), gpu(bq), gpu(bs), out=canvas[:Ra, :Rb], out_dtype=mx.OUT_FP32, accumulate=True)
    b16 = run_gemm(aq, as_, bq, bs, out_dtype=mx.OUT_BF16)
    torch.cuda.synchronize()
    first = torch.from_numpy(c[:Ra, :Rb].copy())
    assert torch.equal(canvas[:Ra, :Rb].cpu(), first + first)
    assert torch.equal(b16.cpu(), first.to(torch.bfloat16))


def test_wide_scale_range_and_exactness_on_small_sums():
    # one block per row (C = 32): at most 32 products, partial sums < 2^24 in units of the
    # smallest product: the fp32 result must be exact
    # (scale bytes chosen so that every result stays inside fp32's normal range)
    rng = np.random.default_rng(1)
    aq, as_ = rand_operand(rng, 64, 32, 80, 175)
    bq, bs = rand_operand(rng, 48, 32, 80, 175)
    want, _ = oracle.gemm(aq, as_, bq, bs)
    got = run_gemm(aq, as_, bq, bs, out_dtype=mx.OUT_FP32).cpu().numpy()
    bad = np.argwhere(got.astype(np.float64) != want)
    assert bad.size == 0, (len(bad), bad[0], got[tuple(bad[0])], want[tuple(bad[0])])


def test_bf16_output_is_rne_of_the_fp32_output():
    rng = np.random.default_rng(2)
    aq, as_ = rand_operand(rng, 96, 256)
    bq, bs = rand_operand(rng, 80, 256)
    f32 = run_gemm(aq, as_, bq, bs, out_dtype=mx.OUT_FP32)
    b16 = run_gemm(aq, as_, bq, bs, out_dtype=mx.OUT_BF16)
    assert b16.dtype == torch.bfloat16
    want_bits = oracle.f32_to_bf16_rne(f32.cpu().numpy())
    got_bits = b16.cpu().view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got_bits, want_bits)
    assert torch.equal(b16, f32.to(torch.bfloat16))


def test_accumulate_and_leading_dimension():
    rng = np.random.default_rng(3)
    aq, as_ = rand_operand(rng, 70, 128)
    bq, bs = rand_operand(rng, 50, 128)
    want, absum = oracle.gemm(aq, as_, bq, bs)
    big = torch.full((70, 64), 7.0, dtype=torch.float32, device="cuda:0")
    view = big[:, :50]
    mx.mxfp4_gemm(gpu(aq), gpu(as_), gpu(bq), gpu(bs), out=view, out_dtype=mx.OUT_FP32, accumulate=True)
    torch.cuda.synchronize()
    got = big.cpu().numpy()
    assert (got[:, 50:] == 7.0).all()                      # padding untouched
    assert_close(got[:, :50] - 7.0, want, absum + 1e-6 * 7.0 / RTOL)
    mx.mxfp4_gemm(gpu(aq), gpu(as_), gpu(bq), gpu(bs), out=view, out_dtype=mx.OUT_FP32, accumulate=False)
    torch.cuda.synchronize()
    assert_close(big.cpu().numpy()[:, :50], want, absum)


def test_empty_and_zero_length_contraction():
    e = torch.empty((0, 16), dtype=torch.uint8, device="cuda:0")
    es = torch.empty((0, 1), dtype=torch.uint8, device="cuda:0")
    b = torch.zeros((8, 16), dtype=torch.uint8, device="cuda:0")
    bs = torch.full((8, 1), 127, dtype=torch.uint8, device="cuda:0")
    assert mx.mxfp4_gemm(e, es, b, bs).shape == (0, 8)
    assert mx.mxfp4_gemm(b, bs, e, es).shape == (8, 0)
    # C = 0: the empty sum
    a0 = torch.empty((5, 0), dtype=torch.uint8, device="cuda:0")
    b0 = torch.empty((6, 0), dtype=torch.uint8, device="cuda:0")
    out = mx.mxfp4_gemm(a0, a0, b0, b0)
    torch.cuda.synchronize()
    assert out.shape == (5, 6) and (out == 0).all()


def test_quantised_real_operands_config1():
    # config 1 end to end through the two calls: quantise (RNE, no rotation), then GEMM
    x = synth.normal(256, 512, 1.0, 0, synth.STREAM_X)
    w = synth.normal(512, 512, 0.02, 0, synth.STREAM_W)
    xq, xs = mx.mxfp4_quantize(x.to("cuda:0"))
    wq, ws = mx.mxfp4_quantize(w.to("cuda:0"))
    y = mx.mxfp4_gemm(xq, xs, wq, ws, out_dtype=mx.OUT_FP32)
    torch.cuda.synchronize()
    want, absum = oracle.linear_fwd(synth.as_u16(x), synth.as_u16(w))
    assert y.shape == (256, 512)
    assert_close(y.cpu().numpy(), want, absum)


def sample_positions(rng, Ra, Rb, n_rows=4, n_cols=4, n_tiles=24):
    ii, jj = [], []
    for r in list(rng.integers(0, Ra, n_rows)) + [0, Ra - 1]:
        ii += [r] * Rb
        jj += list(range(Rb))
    for c in list(rng.integers(0, Rb, n_cols)) + [0, Rb - 1]:
        ii += list(range(Ra))
        jj += [c] * Ra
    for _ in range(n_tiles):
        r0, c0 = rng.integers(0, Ra - 15), rng.integers(0, Rb - 15)
        g = np.mgrid[0:16, 0:16]
        ii += list((r0 + g[0]).ravel())
        jj += list((c0 + g[1]).ravel())
    return np.array(ii, dtype=np.int64), np.array(jj, dtype=np.int64)


@pytest.mark.parametrize("C", [1024, 1280, 2304])
@pytest.mark.parametrize("out_dtype", [mx.OUT_FP32, mx.OUT_BF16])
def test_many_tiles_per_workgroup_sampled(out_dtype, C):
    # 17 x 17 = 289 tiles of 256 x 256 (more than one per CU, not a multiple of 8); 4, 5 and 9 K-stages of 256
    # (with an odd count the stage buffers swap roles from one tile of a workgroup to the next)
    Ra = Rb = 256 * 17
    rng = np.random.default_rng(5)
    aq, as_ = rand_operand(rng, Ra, C)
    bq, bs = rand_operand(rng, Rb, C)
    out = run_gemm(aq, as_, bq, bs, out_dtype=out_dtype)
    ii, jj = sample_positions(rng, Ra, Rb, n_rows=3, n_cols=3, n_tiles=64)
    want, absum = oracle.gemm_at(aq, as_, bq, bs, ii, jj)
    got = out.float().cpu().numpy()[ii, jj]
    if out_dtype == mx.OUT_FP32:
        assert_close(got, want, absum)
    else:
        assert (np.abs(got - want) <= 1e-5 * absum + 2.0**-8 * np.abs(want)).all()


def test_config2_shape_sampled():
    # 8192 x 6144 x 4096 (fused QKV Fprop): complete K-sums at whole rows, whole columns and tiles
    x = synth.normal(8192, 4096, 1.0, 0, synth.STREAM_X)
    w = synth.normal(6144, 4096, 0.02, 0, synth.STREAM_W)
    xq, xs = mx.mxfp4_quantize(x.to("cuda:0"), hadamard=mx.HAD_DET)
    wq, ws = mx.mxfp4_quantize(w.to("cuda:0"), hadamard=mx.HAD_DET)
    y = mx.mxfp4_gemm(xq, xs, wq, ws, out_dtype=mx.OUT_FP32)
    torch.cuda.synchronize()
    ii, jj = sample_positions(np.random.default_rng(0), 8192, 6144)
    want, absum = oracle.gemm_at(xq.cpu().numpy(), xs.cpu().numpy(), wq.cpu().numpy(), ws.cpu().numpy(), ii, jj)
    got = y.cpu().numpy()[ii, jj]
    assert_close(got, want, absum)
