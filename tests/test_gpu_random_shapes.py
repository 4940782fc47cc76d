"""Seeded sweep over random shapes, modes, seeds and magnitudes: every quantiser entry point bit-exact
against the oracle (App. A.1 eq. (1), App. A.2, App. D), every GEMM path (whole tiles, ragged edges
around tiles, small odd shapes; E2M1 and E4M3 operands) within its bound."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_09825_amd as mx
from paper_2605_09825_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
FP8_RTOL = 7 * 2.0 ** -13 + 1e-5  # the matrix unit truncates E4M3 products inside groups of 8 (see test_gpu_fp8)


def same(gpu_pair, want_pair):
    return all(np.array_equal(g.cpu().numpy(), w) for g, w in zip(gpu_pair, want_pair))


@pytest.mark.parametrize("kind", ["single", "dual", "2d", "fp8", "strided"])
def test_quantisers_on_random_shapes(kind):
    rng = np.random.default_rng(["single", "dual", "2d", "fp8", "strided"].index(kind) + 100)
    for it in range(16):
        rows, cols = int(rng.integers(1, 40)) * 32, int(rng.integers(1, 40)) * 32
        had, rnd, seed = int(rng.integers(0, 4)), int(rng.integers(0, 2)), int(rng.integers(0, 2 ** 40))
        scale = float(10.0 ** rng.uniform(-6, 6))
        tag = f"{kind} #{it}: {rows}x{cols} had {had} rnd {rnd} seed {seed} scale {scale:.3g}"
        x = synth.normal(rows, cols, scale, it, synth.STREAM_X)
        xb, xg = synth.as_u16(x), x.to(DEV)
        if kind == "single":
            for axis in (mx.AXIS_LAST, mx.AXIS_FIRST):
                got = mx.mxfp4_quantize(xg, axis, had, rnd, seed)
                assert same(got, oracle.quantize(xb, axis, had, rnd, seed)), tag
        elif kind == "dual":
            got = mx.mxfp4_quantize_dual(xg, had, rnd, seed)
            want = oracle.quantize(xb, mx.AXIS_LAST, had, rnd, seed) + oracle.quantize(xb, mx.AXIS_FIRST, had, rnd, seed)
            assert same(got, want), tag
        elif kind == "2d":
            got = mx.mxfp4_quantize_2d(xg, had, rnd, seed)
            want = (oracle.quantize_2d(xb, mx.AXIS_LAST, had, rnd, seed) +
                    oracle.quantize_2d(xb, mx.AXIS_FIRST, had, rnd, seed))
            assert same(got, want), tag
        elif kind == "fp8":
            for axis in (mx.AXIS_LAST, mx.AXIS_FIRST):
                got = mx.mxfp4_quantize_fp8(xg, axis, had, seed)
                assert same(got, oracle.quantize_fp8(xb, axis, had, seed)), tag
        else:  # a view with a leading dimension and an offset
            base = synth.normal(rows + 32, cols + 64, scale, it, synth.STREAM_W)
            view, view_gpu = base[32:, 64:], base.to(DEV)[32:, 64:]
            vb = synth.as_u16(view.contiguous())
            for axis in (mx.AXIS_LAST, mx.AXIS_FIRST):
                got = mx.mxfp4_quantize(view_gpu, axis, had, rnd, seed)
                assert same(got, oracle.quantize(vb, axis, had, rnd, seed)), tag
                got = mx.mxfp4_quantize_fp8(view_gpu, axis, had, seed)
                assert same(got, oracle.quantize_fp8(vb, axis, had, seed)), tag + " (fp8)"
            got = mx.mxfp4_quantize_dual(view_gpu, had, rnd, seed)
            want = oracle.quantize(vb, mx.AXIS_LAST, had, rnd, seed) + oracle.quantize(vb, mx.AXIS_FIRST, had, rnd, seed)
            assert same(got, want), tag + " (dual)"
            got = mx.mxfp4_quantize_2d(view_gpu, had, rnd, seed)
            want = (oracle.quantize_2d(vb, mx.AXIS_LAST, had, rnd, seed) +
                    oracle.quantize_2d(vb, mx.AXIS_FIRST, had, rnd, seed))
            assert same(got, want), tag + " (2d)"


@pytest.mark.parametrize("kind", ["tiles", "ragged", "small"])
def test_gemms_on_random_shapes(kind):
    rng = np.random.default_rng(["tiles", "ragged", "small"].index(kind) + 200)
    for it in range(14):
        if kind == "tiles":    # whole 256 x 256 tiles, any whole number of K stages
            Ra, Rb, C = int(rng.integers(1, 4)) * 256, int(rng.integers(1, 4)) * 256, int(rng.integers(4, 13)) * 256
        elif kind == "ragged":  # edge strips beside a tiled interior
            Ra, Rb, C = int(rng.integers(200, 900)), int(rng.integers(25, 112)) * 8, int(rng.integers(4, 10)) * 256
        else:
            Ra, Rb, C = int(rng.integers(1, 300)), int(rng.integers(1, 300)), int(rng.integers(1, 40)) * 32
        fa = int(rng.integers(0, 2))
        fb = fa if it % 2 else int(rng.integers(0, 2))

        def operand(R, fmt):
            if fmt == mx.FMT_E2M1:
                return (rng.integers(0, 256, size=(R, C // 2), dtype=np.uint8),
                        rng.integers(115, 135, size=(R, C // 32), dtype=np.uint8))
            q = (rng.integers(5, 10, size=(R, C), dtype=np.uint8) << 3) | rng.integers(0, 8, size=(R, C), dtype=np.uint8)
            q |= rng.integers(0, 2, size=(R, C), dtype=np.uint8) << 7  # finite E4M3 codes of either sign
            s = rng.integers(121, 134, size=(R, C // 32), dtype=np.uint8)
            return q.astype(np.uint8), s

        aq, as_ = operand(Ra, fa)
        bq, bs = operand(Rb, fb)
        want, absum = oracle.gemm_fmt(aq, as_, fa, bq, bs, fb)
        got = mx.mxfp4_gemm(*(torch.from_numpy(t).to(DEV) for t in (aq, as_, bq, bs)), out_dtype=mx.OUT_FP32,
                            a_format=fa, b_format=fb)
        torch.cuda.synchronize()
        err = np.abs(got.cpu().numpy().astype(np.float64) - want)
        tol = 1e-5 if fa == fb == mx.FMT_E2M1 else FP8_RTOL
        assert (err <= tol * absum).all(), (f"{kind} #{it}: {Ra}x{Rb}x{C} formats {fa}{fb}: "
                                            f"max err/sum|a||b| {np.max(err / np.maximum(absum, 1e-300)):.3e}")


def test_linear_calls_on_random_recipes():
    # random shapes, rotation, rounding, seed, geometry, stage formats and output dtypes: the training pair must
    # reproduce the plain forward / backward calls bit for bit (Fig. 3: same three GEMMs), and all-MXFP4 recipes
    # must match the oracle within the GEMM bound (App. C.1-C.3)
    rng = np.random.default_rng(300)
    for it in range(24):
        M, N, K = (int(rng.integers(1, 12)) * 32 for _ in range(3))
        if it % 8 == 0:
            M, N, K = 512, 256, 1024  # whole tiles: the tiled GEMM and the side-by-side backward launch
        had, rnd, seed = int(rng.integers(0, 4)), int(rng.integers(0, 2)), int(rng.integers(0, 2 ** 40))
        geom = int(rng.integers(0, 2))
        fm = [int(rng.integers(0, 2)) for _ in range(3)] if geom == mx.GEOM_1D and it % 2 else [0, 0, 0]
        ydt, dxdt = int(rng.integers(0, 2)), int(rng.integers(0, 2))
        cfg = mx.make_cfg(had, rnd, seed, y_dtype=ydt, dx_dtype=dxdt, dw_dtype=mx.OUT_FP32, geometry=geom,
                          fprop_format=fm[0], dgrad_format=fm[1], wgrad_format=fm[2])
        tag = f"#{it}: M {M} N {N} K {K} had {had} rnd {rnd} geometry {geom} formats {fm} y {ydt} dx {dxdt}"
        x = synth.normal(M, K, 1.0, it, synth.STREAM_X)
        w = synth.normal(N, K, 0.02, it, synth.STREAM_W)
        dy = synth.normal(M, N, 1e-3, it, synth.STREAM_DY)
        xg, wg, dyg = x.to(DEV), w.to(DEV), dy.to(DEV)
        y0, _ = mx.mxfp4_linear_fwd(xg, wg, cfg)
        dx0, dw0, _ = mx.mxfp4_linear_bwd(dyg, xg, wg, cfg)
        y1, _, saved = mx.mxfp4_linear_fwd_save(xg, wg, cfg)
        dx1, dw1, _ = mx.mxfp4_linear_bwd_saved(dyg, saved, K, cfg)
        torch.cuda.synchronize()
        assert torch.equal(y0, y1) and torch.equal(dx0, dx1) and torch.equal(dw0, dw1), tag
        if fm != [0, 0, 0]:
            continue
        xb, wb, dyb = synth.as_u16(x), synth.as_u16(w), synth.as_u16(dy)
        yo, ya = oracle.linear_fwd(xb, wb, had, rnd, seed, geom)
        (dxo, dxa), (dwo, dwa) = oracle.linear_bwd(dyb, xb, wb, had, rnd, seed, geom)
        for got, want, absum, bf16 in ((y0, yo, ya, ydt == mx.OUT_BF16), (dx0, dxo, dxa, dxdt == mx.OUT_BF16),
                                       (dw0, dwo, dwa, False)):
            err = np.abs(got.float().cpu().numpy().astype(np.float64) - want)
            assert (err <= 1e-5 * absum + (2.0 ** -8 * np.abs(want) if bf16 else 0.0)).all(), tag
