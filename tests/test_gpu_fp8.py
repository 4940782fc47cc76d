"""GPU parity of the MXFP8 (E4M3) pieces used by the stages of the stage-wise recipe that stay in 8 bits
(Table 1, "MXFP4 GEMMs (others FP8)"): the quantiser must match the oracle byte for byte.  The GEMM is compared
with the oracle's exact fp64 sum under the tolerance the matrix unit's arithmetic allows: with an E4M3 operand
the unit adds the products of 8 consecutive K-elements after aligning them to the largest of the 8 and dropping
what lies below 2^-13 of it (probed), i.e. up to 7 * 2^-13 of a group's sum |a||b| is lost; when the products of
every group span less than 2^13 nothing is lost and the MXFP4 bound 1e-5 * sum|a||b| holds."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_09825_amd as mx
from paper_2605_09825_amd import synth
from gpu_util import first_mismatch
from test_gpu_gemm import assert_close, close_bf16, gpu, structured_check

pytestmark = pytest.mark.gpu
FP8_RTOL = 7 * 2.0 ** -13 + 1e-5

HADS = [mx.HAD_NONE, mx.HAD_DET, mx.HAD_RANDSIGN, mx.HAD_DET16, mx.HAD_RANDSIGN16]


def check_q(t_cpu, axis, had, seed=0, x_gpu=None):
    x = t_cpu.to("cuda:0") if x_gpu is None else x_gpu
    q, s = mx.mxfp4_quantize_fp8(x, axis, had, seed)
    torch.cuda.synchronize()
    qo, so = oracle.quantize_fp8(synth.as_u16(t_cpu.contiguous()), axis, had, seed)
    assert np.array_equal(s.cpu().numpy(), so), "scales: " + first_mismatch(s.cpu().numpy(), so)
    assert np.array_equal(q.cpu().numpy(), qo), "codes: " + first_mismatch(q.cpu().numpy(), qo)


@pytest.mark.parametrize("had", HADS)
@pytest.mark.parametrize("shape", [(256, 512), (37, 96), (1, 32), (300, 4096)])
def test_rows(shape, had):
    check_q(synth.student_t3(shape[0], shape[1], 1.0, 3, synth.STREAM_X), mx.AXIS_LAST, had, seed=11)


@pytest.mark.parametrize("had", HADS)
@pytest.mark.parametrize("shape", [(256, 128), (96, 74), (32, 2), (288, 130), (1056, 258), (512, 1024)])
def test_cols(shape, had):
    check_q(synth.student_t3(shape[0], shape[1], 1.0, 4, synth.STREAM_DY), mx.AXIS_FIRST, had, seed=12)


@pytest.mark.parametrize("had", HADS)
@pytest.mark.parametrize("shape", [(256, 128), (32, 32), (96, 160), (288, 416), (1056, 2080), (2048, 1024)])
def test_dual_axis_call_equals_the_oracle_on_both_outputs(shape, had):
    # one pass over the tensor, both MXFP8 layouts (ragged tiles: rows not in whole 256s, columns not in whole 128s)
    t = synth.student_t3(shape[0], shape[1], 1.0, 6, synth.STREAM_DY)
    xb = synth.as_u16(t)
    ql, sl, qf, sf = mx.mxfp4_quantize_fp8_dual(t.to("cuda:0"), had, seed=13)
    torch.cuda.synchronize()
    for axis, q, s_ in ((mx.AXIS_LAST, ql, sl), (mx.AXIS_FIRST, qf, sf)):
        qo, so = oracle.quantize_fp8(xb, axis, had, 13)
        assert np.array_equal(s_.cpu().numpy(), so), f"axis {axis} scales: " + first_mismatch(s_.cpu().numpy(), so)
        assert np.array_equal(q.cpu().numpy(), qo), f"axis {axis} codes: " + first_mismatch(q.cpu().numpy(), qo)


def test_dual_axis_call_on_a_strided_view_and_special_values():
    u = synth.as_u16(synth.normal(96, 320, 1.0, 8, synth.STREAM_X)).copy()
    u[5, 40] = 0x7F80            # +inf
    u[70, 200] = 0x7FC1          # a NaN
    u[33, 64:96] = 0             # an all-zero block
    big = synth.from_bits(u)
    xb = u[:, 32:288]            # ld = 320, cols = 256
    ql, sl, qf, sf = mx.mxfp4_quantize_fp8_dual(big.to("cuda:0")[:, 32:288], mx.HAD_DET)
    torch.cuda.synchronize()
    for axis, q, s_ in ((mx.AXIS_LAST, ql, sl), (mx.AXIS_FIRST, qf, sf)):
        qo, so = oracle.quantize_fp8(xb, axis, mx.HAD_DET, 0)
        assert np.array_equal(s_.cpu().numpy(), so) and np.array_equal(q.cpu().numpy(), qo)
        assert (so == 0xFF).sum() >= 2


@pytest.mark.parametrize("axis", [mx.AXIS_LAST, mx.AXIS_FIRST])
@pytest.mark.parametrize("had", HADS)
def test_every_bf16_bit_pattern_and_distributions(axis, had):
    bits = np.arange(65536, dtype=np.uint16).reshape(256, 256)  # includes zeros, subnormals, infinities, NaNs
    check_q(synth.from_bits(bits), axis, had)
    finite = bits.reshape(-1)[(bits.reshape(-1) & 0x7F80) != 0x7F80]
    mixed = np.random.default_rng(0).permutation(finite)[: 96 * 512].reshape(96, 512)
    check_q(synth.from_bits(mixed), axis, had)
    check_q(synth.normal_with_outlier_channels(512, 1024, 6, synth.STREAM_X, fraction=0.004), axis, had)
    check_q(synth.normal(256, 512, 1e-30, 6, synth.STREAM_W), axis, had)
    check_q(synth.normal(256, 512, 1e30, 6, synth.STREAM_W), axis, had)
    base = synth.normal(320, 640, 1.0, 5, synth.STREAM_X)
    check_q(base[32:288, 64:576], axis, had, x_gpu=base.to("cuda:0")[32:288, 64:576])


def rand_fp8(rng, R, C):
    q = rng.integers(0, 127, size=(R, C), dtype=np.uint8) | (rng.integers(0, 2, size=(R, C), dtype=np.uint8) << 7)
    return q, rng.integers(115, 135, size=(R, C // 32), dtype=np.uint8)


def rand_fp4(rng, R, C):
    return rng.integers(0, 256, size=(R, C // 2), dtype=np.uint8), rng.integers(115, 135, size=(R, C // 32), dtype=np.uint8)


@pytest.mark.parametrize("fmts", [(1, 1), (1, 0), (0, 1)])
@pytest.mark.parametrize("shape", [(64, 64, 128), (37, 53, 96), (1, 1, 32), (256, 512, 512), (130, 70, 1024),
                                   (512, 768, 1536), (300, 520, 1024), (256, 256, 1024), (768, 512, 2560),
                                   (512, 256, 1280)])
def test_gemm_random_codes(shape, fmts):
    Ra, Rb, C = shape
    rng = np.random.default_rng(Ra * 7 + Rb * 3 + C + 100 * fmts[0] + 10 * fmts[1])
    aq, as_ = (rand_fp8 if fmts[0] else rand_fp4)(rng, Ra, C)
    bq, bs = (rand_fp8 if fmts[1] else rand_fp4)(rng, Rb, C)
    want, absum = oracle.gemm_fmt(aq, as_, fmts[0], bq, bs, fmts[1])
    got = mx.mxfp4_gemm(gpu(aq), gpu(as_), gpu(bq), gpu(bs), out_dtype=mx.OUT_FP32, a_format=fmts[0], b_format=fmts[1])
    torch.cuda.synchronize()
    assert np.all(np.abs(got.cpu().numpy() - want) <= FP8_RTOL * absum)
    b16 = mx.mxfp4_gemm(gpu(aq), gpu(as_), gpu(bq), gpu(bs), out_dtype=mx.OUT_BF16, a_format=fmts[0], b_format=fmts[1])
    acc = got.clone()
    mx.mxfp4_gemm(gpu(aq), gpu(as_), gpu(bq), gpu(bs), out=acc, out_dtype=mx.OUT_FP32, accumulate=True,
                  a_format=fmts[0], b_format=fmts[1])
    torch.cuda.synchronize()
    assert torch.equal(b16.cpu(), got.cpu().to(torch.bfloat16)) and torch.equal(acc, got + got)


@pytest.mark.parametrize("fmts", [(1, 1), (1, 0), (0, 1)])
@pytest.mark.parametrize("shape", [(64, 64, 128), (37, 53, 96), (256, 512, 512), (300, 520, 1024),
                                   (256, 256, 1024), (512, 768, 1536), (768, 512, 2560), (512, 256, 1280),
                                   (1280, 1024, 4096)])
def test_gemm_narrow_exponent_range_meets_the_mxfp4_bound(shape, fmts):
    # E4M3 exponent fields 5..9 (magnitudes 0.25 .. 7.5), any E2M1 code but zero excluded from neither: the
    # products inside a group of 8 then span at most 2^5 * 15 * 12 < 2^13, so no bit is dropped
    Ra, Rb, C = shape
    rng = np.random.default_rng(Ra + Rb + C + 7 * fmts[0] + fmts[1])

    def narrow_fp8(R):
        q = (rng.integers(5, 10, size=(R, C), dtype=np.uint8) << 3) | rng.integers(0, 8, size=(R, C), dtype=np.uint8)
        q |= rng.integers(0, 2, size=(R, C), dtype=np.uint8) << 7
        return q.astype(np.uint8), np.full((R, C // 32), 127, dtype=np.uint8) + rng.integers(0, 2, size=(R, C // 32), dtype=np.uint8) * 0

    def fp4_nonzero(R):
        codes = rng.integers(1, 8, size=(R, C), dtype=np.uint8) | (rng.integers(0, 2, size=(R, C), dtype=np.uint8) << 3)
        return (codes[:, 0::2] | (codes[:, 1::2] << 4)).astype(np.uint8), np.full((R, C // 32), 127, dtype=np.uint8)

    aq, as_ = (narrow_fp8 if fmts[0] else fp4_nonzero)(Ra)
    bq, bs = (narrow_fp8 if fmts[1] else fp4_nonzero)(Rb)
    # per-row scales that differ between rows (not inside a row: a group of 8 lies inside one block anyway,
    # but keep the spread argument simple)
    as_ = (as_ + rng.integers(-6, 7, size=(Ra, 1))).astype(np.uint8)
    bs = (bs + rng.integers(-6, 7, size=(Rb, 1))).astype(np.uint8)
    want, absum = oracle.gemm_fmt(aq, as_, fmts[0], bq, bs, fmts[1])
    got = mx.mxfp4_gemm(gpu(aq), gpu(as_), gpu(bq), gpu(bs), out_dtype=mx.OUT_FP32, a_format=fmts[0], b_format=fmts[1])
    torch.cuda.synchronize()
    assert_close(got.cpu().numpy(), want, absum)


@pytest.mark.parametrize("C", [1024, 2304, 1152, 1408])  # 8, 18, 9 and 11 K-stages of 128
def test_fp8_many_tiles_per_workgroup_whole_output(C):
    # 17 x 17 = 289 tiles of 256 x 256: more than one tile per CU, so tiles hand over inside a workgroup;
    # narrow exponent range, so the MXFP4 bound applies; every element compared
    Ra = Rb = 256 * 17
    rng = np.random.default_rng(C)

    def narrow(R):
        q = (rng.integers(5, 10, size=(R, C), dtype=np.uint8) << 3) | rng.integers(0, 8, size=(R, C), dtype=np.uint8)
        q |= rng.integers(0, 2, size=(R, C), dtype=np.uint8) << 7
        srow = (127 + rng.integers(-6, 7, size=(R, 1))).astype(np.uint8)  # one scale per row (see above)
        return q.astype(np.uint8), np.ascontiguousarray(np.broadcast_to(srow, (R, C // 32)))

    aq, as_ = narrow(Ra)
    bq, bs = narrow(Rb)
    want, absum = oracle.gemm_fmt(aq, as_, 1, bq, bs, 1)
    f32 = mx.mxfp4_gemm(gpu(aq), gpu(as_), gpu(bq), gpu(bs), out_dtype=mx.OUT_FP32, a_format=1, b_format=1)
    b16 = mx.mxfp4_gemm(gpu(aq), gpu(as_), gpu(bq), gpu(bs), out_dtype=mx.OUT_BF16, a_format=1, b_format=1)
    torch.cuda.synchronize()
    assert_close(f32.cpu().numpy(), want, absum)
    assert torch.equal(b16, f32.to(torch.bfloat16))


def test_fp8_linear_stage_on_real_operands():
    # Fprop of a small layer entirely in MXFP8, deterministic rotation: quantise both operands, multiply
    M, K, N = 256, 512, 384
    x = synth.normal(M, K, 1.0, 1, synth.STREAM_X)
    w = synth.normal(N, K, 0.02, 1, synth.STREAM_W)
    xq, xs = mx.mxfp4_quantize_fp8(x.to("cuda:0"), mx.AXIS_LAST, mx.HAD_DET)
    wq, ws = mx.mxfp4_quantize_fp8(w.to("cuda:0"), mx.AXIS_LAST, mx.HAD_DET)
    y = mx.mxfp4_gemm(xq, xs, wq, ws, out_dtype=mx.OUT_FP32, a_format=mx.FMT_E4M3, b_format=mx.FMT_E4M3)
    torch.cuda.synchronize()
    xo = oracle.quantize_fp8(synth.as_u16(x), oracle.AXIS_LAST, oracle.HAD_DET)
    wo = oracle.quantize_fp8(synth.as_u16(w), oracle.AXIS_LAST, oracle.HAD_DET)
    want, absum = oracle.gemm_fmt(xo[0], xo[1], 1, wo[0], wo[1], 1)
    assert np.all(np.abs(y.cpu().numpy() - want) <= FP8_RTOL * absum)
    # and it is much closer to the real product than the MXFP4 version of the same layer
    ref = x.to(torch.float64) @ w.to(torch.float64).T
    e8 = float(torch.linalg.norm(y.cpu().to(torch.float64) - ref) / torch.linalg.norm(ref))
    y4, _ = mx.mxfp4_linear_fwd(x.to("cuda:0"), w.to("cuda:0"), mx.make_cfg(mx.HAD_DET, y_dtype=mx.OUT_FP32))
    e4 = float(torch.linalg.norm(y4.cpu().to(torch.float64) - ref) / torch.linalg.norm(ref))
    assert e8 < 0.05 and e8 < e4 / 3, (e8, e4)


def test_fp8_argument_errors():
    x = torch.zeros((64, 48), dtype=torch.bfloat16, device="cuda:0")
    with pytest.raises(mx.Mxfp4Error) as e:
        mx.mxfp4_quantize_fp8(x)
    assert e.value.status == mx.ESHAPE
    q = torch.zeros((16, 32), dtype=torch.uint8, device="cuda:0")
    s = torch.zeros((16, 1), dtype=torch.uint8, device="cuda:0")
    out = torch.zeros((16, 16), dtype=torch.float32, device="cuda:0")
    rc = mx.lib().mxfp4_gemm_fmt(q.data_ptr(), s.data_ptr(), 5, q.data_ptr(), s.data_ptr(), 1, 16, 16, 32,
                                 out.data_ptr(), 16, mx.OUT_FP32, 0, None)
    assert rc == mx.EINVAL


# ---- the stage-wise recipe: MXFP4 in some stages, MXFP8 in the others (Table 1) -------------------
def _slices(buf, offs, dims, fmts):
    b = buf.cpu().numpy()
    out = []
    for k, ((R, C), f) in enumerate(zip(dims, fmts)):
        nq = R * (C if f else C // 2)
        out.append((b[offs[2 * k]: offs[2 * k] + nq].reshape(R, -1),
                    b[offs[2 * k + 1]: offs[2 * k + 1] + R * C // 32].reshape(R, C // 32)))
    return out


def _oracle_q(x, axis, fmt, had, rnd, seed):
    if fmt:
        return oracle.quantize_fp8(x, axis, oracle.HAD_NONE, seed)
    return oracle.quantize(x, axis, had, rnd, seed)


@pytest.mark.parametrize("saved_path", [False, True])
@pytest.mark.parametrize("fmts", [(0, 1, 1), (0, 0, 1), (1, 1, 1), (1, 0, 0), (0, 1, 0)])
@pytest.mark.parametrize("shape,had,rnd", [((256, 512, 1024), mx.HAD_DET, mx.RNE), ((96, 160, 224), mx.HAD_DET, mx.RNE),
                                           ((288, 416, 352), mx.HAD_RANDSIGN16, mx.SR)])
def test_linear_with_stage_formats(shape, had, rnd, fmts, saved_path):
    M, N, K = shape
    seed = 31
    fF, fD, fW = fmts
    x = synth.normal(M, K, 1.0, 1, synth.STREAM_X)
    w = synth.normal(N, K, 0.02, 1, synth.STREAM_W)
    dy = synth.normal(M, N, 1e-3, 1, synth.STREAM_DY)
    cfg = mx.make_cfg(had, rnd, seed, y_dtype=mx.OUT_FP32, dx_dtype=mx.OUT_FP32, dw_dtype=mx.OUT_FP32,
                      fprop_format=fF, dgrad_format=fD, wgrad_format=fW)
    xg, wg, dyg = x.to("cuda:0"), w.to("cuda:0"), dy.to("cuda:0")
    if saved_path:
        y, ws_f, saved = mx.mxfp4_linear_fwd_save(xg, wg, cfg)
        dx, dw, ws_b = mx.mxfp4_linear_bwd_saved(dyg, saved, K, cfg)
    else:
        y, ws_f = mx.mxfp4_linear_fwd(xg, wg, cfg)
        dx, dw, ws_b = mx.mxfp4_linear_bwd(dyg, xg, wg, cfg)
    torch.cuda.synchronize()
    xb, wb, dyb = synth.as_u16(x), synth.as_u16(w), synth.as_u16(dy)
    L, F = oracle.AXIS_LAST, oracle.AXIS_FIRST
    sd = lambda stream: oracle.seed_with_stream(seed, stream)   # every operand rounds under its own stream
    want = {"X": _oracle_q(xb, L, fF, had, rnd, sd(oracle.STREAM_X)), "W": _oracle_q(wb, L, fF, had, rnd, sd(oracle.STREAM_W)),
            "dY": _oracle_q(dyb, L, fD, had, rnd, sd(oracle.STREAM_DY)),
            "W^T": _oracle_q(wb, F, fD, had, rnd, sd(oracle.STREAM_WT)),
            "dY^T": _oracle_q(dyb, F, fW, had, rnd, sd(oracle.STREAM_DYT)),
            "X^T": _oracle_q(xb, F, fW, had, rnd, sd(oracle.STREAM_XT))}
    fw = _slices(ws_f, mx.mxfp4_linear_workspace_layout(M, N, K, False, cfg), [(M, K), (N, K)], [fF, fF])
    bw = _slices(ws_b, mx.mxfp4_linear_workspace_layout(M, N, K, True, cfg), [(M, N), (K, N), (N, M), (K, M)],
                 [fD, fD, fW, fW])
    got = {"X": fw[0], "W": fw[1], "dY": bw[0], "dY^T": bw[2]}
    if saved_path:
        sv = _slices(saved, mx.mxfp4_linear_saved_layout(M, N, K, cfg), [(K, N), (K, M)], [fD, fW])
        got["W^T"], got["X^T"] = sv[0], sv[1]
    else:
        got["W^T"], got["X^T"] = bw[1], bw[3]
    for name in got:
        assert np.array_equal(got[name][1], want[name][1]), f"{name}: scale bytes differ"
        assert np.array_equal(got[name][0], want[name][0]), f"{name}: codes differ"
    for out, a, b, f in ((y, "X", "W", fF), (dx, "dY", "W^T", fD), (dw, "dY^T", "X^T", fW)):
        o, absum = oracle.gemm_fmt(want[a][0], want[a][1], f, want[b][0], want[b][1], f)
        tol = FP8_RTOL if f else 1e-5
        assert np.all(np.abs(out.cpu().numpy() - o) <= tol * absum), (a, b)


@pytest.mark.parametrize("fmts", [(0, 1, 1), (0, 0, 1)])
def test_backward_side_by_side_launch_with_mxfp8_stages(fmts):
    # M = N = K = 4096: Dgrad and Wgrad have 256 tiles each, enough for the launch that runs them side by side
    # (bf16 dX, fp32 dW), with Dgrad in MXFP8 or MXFP4 and Wgrad in MXFP8.  Bit-equal to each gradient asked for
    # alone (launches of their own), and against the oracle on a patch in every tile plus whole rows and columns.
    M = N = K = 4096
    fF, fD, fW = fmts
    x = synth.normal(M, K, 1.0, 2, synth.STREAM_X)
    w = synth.normal(N, K, 0.02, 2, synth.STREAM_W)
    dy = synth.normal(M, N, 1e-3, 2, synth.STREAM_DY)
    cfg = mx.make_cfg(mx.HAD_DET, mx.RNE, 5, y_dtype=mx.OUT_BF16, dx_dtype=mx.OUT_BF16, dw_dtype=mx.OUT_FP32,
                      fprop_format=fF, dgrad_format=fD, wgrad_format=fW)
    xg, wg, dyg = x.to("cuda:0"), w.to("cuda:0"), dy.to("cuda:0")
    dx, dw, ws_b = mx.mxfp4_linear_bwd(dyg, xg, wg, cfg)
    dx1, _, _ = mx.mxfp4_linear_bwd(dyg, xg, wg, cfg, need_dw=False)
    _, dw1, _ = mx.mxfp4_linear_bwd(dyg, xg, wg, cfg, need_dx=False)
    # ... and with dW accumulated into what the buffer already holds
    cfg_acc = mx.make_cfg(mx.HAD_DET, mx.RNE, 5, y_dtype=mx.OUT_BF16, dx_dtype=mx.OUT_BF16, dw_dtype=mx.OUT_FP32,
                          dw_accumulate=True, fprop_format=fF, dgrad_format=fD, wgrad_format=fW)
    dw_acc = torch.full((N, K), 0.125, dtype=torch.float32, device="cuda:0")
    dx2, _, _ = mx.mxfp4_linear_bwd(dyg, xg, wg, cfg_acc, dw=dw_acc)
    torch.cuda.synchronize()
    assert torch.equal(dx, dx1) and torch.equal(dw, dw1)
    assert torch.equal(dx2, dx) and torch.equal(dw_acc, dw + 0.125)
    ops = _slices(ws_b, mx.mxfp4_linear_workspace_layout(M, N, K, True, cfg), [(M, N), (K, N), (N, M), (K, M)],
                  [fD, fD, fW, fW])
    rng = np.random.default_rng(4)

    def close_fp8_bf16(got, want, absum):
        assert (np.abs(got - want) <= FP8_RTOL * absum + 2.0**-8 * np.abs(want)).all()

    def close_fp8(got, want, absum):
        assert (np.abs(got - want) <= FP8_RTOL * absum).all()
    structured_check(dx.float().cpu().numpy().astype(np.float64), ops[0], ops[1], rng, fmts=(fD, fD), n_lines=16,
                     close=close_fp8_bf16 if fD else close_bf16)
    structured_check(dw.cpu().numpy().astype(np.float64), ops[2], ops[3], rng, fmts=(fW, fW), n_lines=16,
                     close=close_fp8)


def test_stage_formats_reject_2d_geometry():
    cfg = mx.make_cfg(geometry=mx.GEOM_2D, wgrad_format=mx.FMT_E4M3)
    x = torch.zeros((64, 64), dtype=torch.bfloat16, device="cuda:0")
    with pytest.raises(mx.Mxfp4Error) as e:
        mx.mxfp4_linear_fwd(x, x, cfg)
    assert e.value.status == mx.ENOTIMPL


# ---- where the FP8-stage tolerance comes from: what the matrix unit does with E4M3 products ---------------------
E4M3_ONE, E4M3_256 = 0x38, 0x78


def _e4m3(v):
    """E4M3 code of a positive value that the format holds exactly (taken from the oracle's decoder)."""
    for c in range(127):
        if oracle.e4m3_decode(c) == v:
            return c
    raise ValueError(v)


@pytest.mark.parametrize("shape", [(16, 16, 128), (256, 256, 1024)])  # any-shape kernel, tiled kernel
def test_e4m3_products_below_2_to_minus_13_of_their_group_maximum_are_dropped(shape):
    # One row of A holds 256 at k = 0 and a small value at k = k0, everything else 0; B is all ones.  The exact result
    # is 256 + small.  Observed on the MI355X matrix unit and asserted here: inside a group of 8 consecutive K-elements
    # the products are aligned to the exponent of the largest and what lies below 2^-13 of that power of two is
    # truncated (not rounded); products of different groups are added in fp32 without loss.  Hence the tolerance of
    # the FP8 stages, 7 * 2^-13 * sum|a||b| + the MXFP4 bound: seven of a group's eight products can each lose
    # less than 2^-13 of the largest.
    Ra, Rb, C = shape
    ones = np.full((Rb, C), E4M3_ONE, dtype=np.uint8)
    s127a = np.full((Ra, C // 32), 127, dtype=np.uint8)
    s127b = np.full((Rb, C // 32), 127, dtype=np.uint8)

    def result(small, k0):
        a = np.zeros((Ra, C), dtype=np.uint8)
        a[0, 0] = E4M3_256
        a[0, k0] = _e4m3(small)
        out = mx.mxfp4_gemm(gpu(a), gpu(s127a), gpu(ones), gpu(s127b), out_dtype=mx.OUT_FP32, a_format=1, b_format=1)
        torch.cuda.synchronize()
        o = out.cpu().numpy()
        assert np.all(o[0] == o[0, 0]) and np.all(o[1:] == 0)
        want, absum = oracle.gemm_fmt(a, s127a, 1, ones, s127b, 1)
        assert want[0, 0] == 256.0 + small
        assert abs(float(o[0, 0]) - want[0, 0]) <= FP8_RTOL * absum[0, 0]     # the documented bound always holds
        return float(o[0, 0])

    if shape[2] == 128:  # the 16x16x128 instruction of the any-shape kernel: the probed facts themselves
        for k0 in range(1, 8):                                    # same group of 8 as k = 0
            assert result(2.0 ** -5, k0) == 256.0 + 2.0 ** -5     # 2^-13 of 2^8: kept
            assert result(2.0 ** -6, k0) == 256.0                 # below: dropped
            assert result(3 * 2.0 ** -6, k0) == 256.0 + 2.0 ** -5  # truncated, not rounded (would be 256.0625)
        for k0 in (8, 9, 15, 16, 31, 32, 64, 127):                # another group: an exact fp32 addition
            assert result(2.0 ** -6, k0) == 256.0 + 2.0 ** -6
    else:                # the 32x32x64 instruction of the tiled kernel: the bound, and exactness above 2^-13
        for k0 in (1, 7, 8, 33, 500, 1023):
            assert result(2.0 ** -5, k0) == 256.0 + 2.0 ** -5
            got = result(2.0 ** -6, k0)
            assert got in (256.0, 256.0 + 2.0 ** -6)
