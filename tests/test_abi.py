"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header declares,
and every argument error is caught on the host before anything is launched."""
import ctypes
import os
import re

import pytest

import paper_2605_09825_amd as mx

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(mx.LIB_PATH):
        from paper_2605_09825_amd.build import build
        build()
    return mx.lib()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "mxfp4.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mxfp4_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported(L):
    names = declared_symbols()
    assert set(names) == set(mx.EXPORTS)
    for n in names:
        assert getattr(L, n) is not None


def test_status_strings(L):
    seen = set()
    for code in range(7):
        s = mx.status_string(code)
        assert s and s not in seen
        seen.add(s)
    assert mx.status_string(99) == "unknown status"


P = 0x10000  # a fake, 16-byte aligned, non-null device address: never dereferenced on the host


def test_quantize_argument_errors(L):
    q = L.mxfp4_quantize
    assert q(P, 64, 64, 64, 2, 0, 0, 0, P, P, None) == mx.EINVAL          # axis
    assert q(P, 64, 64, 64, 0, 9, 0, 0, P, P, None) == mx.EINVAL          # hadamard
    assert q(P, 64, 64, 64, 0, mx.HAD_RANDSIGN16 + 1, 0, 0, P, P, None) == mx.EINVAL
    assert q(P, 64, 64, 64, 0, 0, 2, 0, P, P, None) == mx.EINVAL          # rounding
    assert q(None, 64, 64, 64, 0, 0, 0, 0, P, P, None) == mx.EINVAL
    assert q(P, 64, 64, 64, 0, 0, 0, 0, None, P, None) == mx.EINVAL
    assert q(P, 64, 64, 64, 0, 0, 0, 0, P, None, None) == mx.EINVAL
    assert q(P, -1, 64, 64, 0, 0, 0, 0, P, P, None) == mx.ESHAPE
    assert q(P, 64, 48, 48, 0, 0, 0, 0, P, P, None) == mx.ESHAPE          # cols % 32
    assert q(P, 48, 64, 64, 1, 0, 0, 0, P, P, None) == mx.ESHAPE          # rows % 32 for AXIS_FIRST
    assert q(P, 64, 63, 64, 1, 0, 0, 0, P, P, None) == mx.ESHAPE          # odd cols for AXIS_FIRST
    assert q(P, 64, 64, 32, 0, 0, 0, 0, P, P, None) == mx.ESHAPE          # ld < cols
    assert q(P + 2, 64, 64, 64, 0, 0, 0, 0, P, P, None) == mx.EALIGN
    assert q(P, 64, 64, 64, 0, 0, 0, 0, P + 8, P, None) == mx.EALIGN
    assert q(P, 64, 64, 68, 0, 0, 0, 0, P, P, None) == mx.EALIGN          # ld % 8
    assert q(P, 64, 64, 65, 1, 0, 0, 0, P, P, None) == mx.EALIGN          # ld % 2 for AXIS_FIRST
    assert q(P + 2, 64, 64, 64, 1, 0, 0, 0, P, P, None) == mx.EALIGN
    assert q(None, 0, 64, 64, 0, 0, 0, 0, None, None, None) == mx.OK      # empty


def test_quantize_fp8_dual_argument_errors(L):
    d = L.mxfp4_quantize_fp8_dual
    assert d(P, 64, 64, 64, 9, 0, P, P, P, P, None) == mx.EINVAL          # hadamard
    assert d(P, 64, 64, 64, 0, 0, P, P, None, P, None) == mx.EINVAL
    assert d(P, 64, 48, 64, 0, 0, P, P, P, P, None) == mx.ESHAPE          # cols % 32
    assert d(P, 48, 64, 64, 0, 0, P, P, P, P, None) == mx.ESHAPE          # rows % 32
    assert d(P, 64, 64, 68, 0, 0, P, P, P, P, None) == mx.EALIGN          # ld % 8
    assert d(P, 64, 64, 64, 0, 0, P + 8, P, P, P, None) == mx.EALIGN
    assert d(None, 0, 64, 64, 0, 0, None, None, None, None, None) == mx.OK  # empty


def test_gemm_argument_errors(L):
    g = L.mxfp4_gemm
    assert g(P, P, P, P, 16, 16, 32, P, 16, 5, 0, None) == mx.EINVAL      # dtype
    assert g(P, P, P, P, 16, 16, 32, P, 16, mx.OUT_BF16, 1, None) == mx.EINVAL  # accumulate into bf16
    assert g(P, P, P, P, 16, 16, 32, P, 16, mx.OUT_FP32, 2, None) == mx.EINVAL
    assert g(P, P, P, P, 16, 16, 48, P, 16, 1, 0, None) == mx.ESHAPE      # C % 32
    assert g(P, P, P, P, -1, 16, 32, P, 16, 1, 0, None) == mx.ESHAPE
    assert g(P, P, P, P, 16, 16, 32, P, 8, 1, 0, None) == mx.ESHAPE       # ld < R_b
    assert g(None, P, P, P, 16, 16, 32, P, 16, 1, 0, None) == mx.EINVAL
    assert g(P, P, P, P, 16, 16, 32, None, 16, 1, 0, None) == mx.EINVAL
    assert g(P + 4, P, P, P, 16, 16, 32, P, 16, 1, 0, None) == mx.EALIGN
    assert g(P, P, P, P, 0, 16, 32, None, 16, 1, 0, None) == mx.OK        # empty


def test_gemm_pair_argument_errors(L):
    g = L.mxfp4_gemm_pair
    ok0 = (P, P, P, P, 16, 16, 32, P, 16, mx.OUT_BF16)
    ok1 = (P, P, P, P, 16, 16, 32, P, 16, mx.OUT_FP32, 0)
    assert g(*ok0[:9], 5, *ok1, None) == mx.EINVAL                         # dtype of problem 0
    assert g(*ok0, *ok1[:9], mx.OUT_BF16, 1, None) == mx.EINVAL            # problem 1 accumulating into bf16
    assert g(*ok0[:6], 48, *ok0[7:], *ok1, None) == mx.ESHAPE              # C0 % 32
    assert g(*ok0, P, P, P, P, 16, 16, 32, P, 8, mx.OUT_FP32, 0, None) == mx.ESHAPE   # ld1 < R_b1
    assert g(*ok0, None, P, P, P, 16, 16, 32, P, 16, mx.OUT_FP32, 0, None) == mx.EINVAL
    assert g(P + 4, *ok0[1:], *ok1, None) == mx.EALIGN
    empty0 = (None, None, None, None, 0, 16, 32, None, 16, mx.OUT_BF16)
    empty1 = (None, None, None, None, 16, 0, 32, None, 16, mx.OUT_FP32, 0)
    assert g(*empty0, *empty1, None) == mx.OK                              # both empty: nothing to enqueue
    assert g(*empty0, *ok1[:9], mx.OUT_BF16, 1, None) == mx.EINVAL         # the other problem is still checked


def test_linear_argument_errors_and_workspace(L):
    cfg = mx.make_cfg()
    M, N, K = 64, 96, 128
    need_f = mx.mxfp4_linear_workspace_bytes(M, N, K, cfg, False)
    need_b = mx.mxfp4_linear_workspace_bytes(M, N, K, cfg, True)
    assert need_f >= (M + N) * (K // 2 + K // 32)
    assert need_b >= (M + K) * (N // 2 + N // 32) + (N + K) * (M // 2 + M // 32)
    off = mx.mxfp4_linear_workspace_layout(M, N, K, True)
    assert off == sorted(off) and all(o % 256 == 0 for o in off) and off[-1] + K * (M // 32) <= need_b
    W = 0x100000
    f, b = L.mxfp4_linear_fwd, L.mxfp4_linear_bwd
    c = ctypes.byref(cfg)
    assert f(P, P, P, M, N, K, None, W, need_f, None) == mx.EINVAL
    assert f(P, P, P, M, N, 100, c, W, need_f, None) == mx.ESHAPE
    assert f(P, P, P, 0, N, K, c, W, need_f, None) == mx.ESHAPE
    assert f(None, P, P, M, N, K, c, W, need_f, None) == mx.EINVAL
    assert f(P, P, P, M, N, K, c, W, need_f - 1, None) == mx.EWORKSPACE
    assert f(P, P, P, M, N, K, c, W + 16, need_f, None) == mx.EALIGN
    bad = mx.make_cfg(dw_dtype=mx.OUT_BF16, dw_accumulate=True)
    assert f(P, P, P, M, N, K, ctypes.byref(bad), W, need_f, None) == mx.EINVAL
    assert b(P, P, P, P, P, M, N, K, c, W, need_b - 1, None) == mx.EWORKSPACE
    assert b(P, P, P, P, P, M, 100, K, c, W, need_b, None) == mx.ESHAPE   # Dgrad needs N % 32
    assert b(P, P, P, None, P, 48, N, K, c, W, need_b, None) == mx.ESHAPE  # Wgrad needs M % 32
    assert b(P, None, P, P, P, M, N, K, c, W, need_b, None) == mx.EINVAL  # x needed for dW
    assert b(P, P, None, P, P, M, N, K, c, W, need_b, None) == mx.EINVAL  # w needed for dX
    assert b(P, P, P, None, None, M, N, K, c, W, need_b, None) == mx.OK   # nothing asked


def test_dual_and_saved_argument_errors(L):
    d = L.mxfp4_quantize_dual
    assert d(P, 64, 64, 64, 9, 0, 0, P, P, P, P, None) == mx.EINVAL       # hadamard
    assert d(P, 64, 64, 64, 0, 0, 0, P, P, None, P, None) == mx.EINVAL
    assert d(P, 64, 64, 64, 0, 0, 0, None, P, P, P, None) == mx.EINVAL
    assert d(P, 48, 64, 64, 0, 0, 0, P, P, P, P, None) == mx.ESHAPE       # rows % 32
    assert d(P, 64, 48, 48, 0, 0, 0, P, P, P, P, None) == mx.ESHAPE       # cols % 32
    assert d(P, 64, 64, 68, 0, 0, 0, P, P, P, P, None) == mx.EALIGN       # ld % 8
    assert d(P + 4, 64, 64, 64, 0, 0, 0, P, P, P, P, None) == mx.EALIGN
    assert d(P, 64, 64, 64, 0, 0, 0, P, P, P + 8, P, None) == mx.EALIGN
    assert d(None, 64, 0, 64, 0, 0, 0, None, None, None, None, None) == mx.OK  # empty
    cfg = mx.make_cfg()
    c = ctypes.byref(cfg)
    M, N, K = 64, 96, 128
    need_f = mx.mxfp4_linear_workspace_bytes(M, N, K, cfg, False)
    need_b = mx.mxfp4_linear_workspace_bytes(M, N, K, cfg, True)
    need_s = mx.mxfp4_linear_saved_bytes(M, N, K)
    assert need_s >= K * (N // 2 + N // 32) + K * (M // 2 + M // 32)
    off = mx.mxfp4_linear_saved_layout(M, N, K)
    assert off == sorted(off) and all(o % 256 == 0 for o in off) and off[-1] + K * (M // 32) <= need_s
    W, S = 0x100000, 0x200000
    f, b = L.mxfp4_linear_fwd_save, L.mxfp4_linear_bwd_saved
    assert f(P, P, P, M, N, K, c, W, need_f, S, need_s - 1, None) == mx.EWORKSPACE
    assert f(P, P, P, M, N, K, c, W, need_f - 1, S, need_s, None) == mx.EWORKSPACE
    assert f(P, P, P, 48, N, K, c, W, need_f, S, need_s, None) == mx.ESHAPE   # M % 32
    assert f(P, P, P, M, 100, K, c, W, need_f, S, need_s, None) == mx.ESHAPE  # N % 32
    assert f(P, P, P, M, N, K, c, W, need_f, None, need_s, None) == mx.EINVAL
    assert f(P, P, P, M, N, K, c, W, need_f, S + 16, need_s, None) == mx.EALIGN
    assert b(P, S, need_s - 1, P, P, M, N, K, c, W, need_b, None) == mx.EWORKSPACE
    assert b(P, S, need_s, P, P, M, N, K, c, W, need_b - 1, None) == mx.EWORKSPACE
    assert b(P, None, need_s, P, P, M, N, K, c, W, need_b, None) == mx.EINVAL
    assert b(None, S, need_s, P, P, M, N, K, c, W, need_b, None) == mx.EINVAL
    assert b(P, S, need_s, P, P, M, N, 100, c, W, need_b, None) == mx.ESHAPE
    assert b(P, S, need_s, None, None, M, N, K, c, W, need_b, None) == mx.OK  # nothing asked


def test_2d_geometry_argument_errors(L):
    d = L.mxfp4_quantize_2d
    assert d(P, 64, 64, 64, 9, 0, 0, P, P, P, P, None) == mx.EINVAL        # hadamard
    assert d(P, 64, 64, 64, 0, 0, 0, None, None, None, None, None) == mx.EINVAL  # no output asked
    assert d(P, 64, 64, 64, 0, 0, 0, P, None, None, None, None) == mx.EINVAL     # half a pair
    assert d(P, 48, 64, 64, 0, 0, 0, P, P, None, None, None) == mx.ESHAPE  # rows % 32 even for the row-wise output
    assert d(P, 64, 48, 48, 0, 0, 0, None, None, P, P, None) == mx.ESHAPE
    assert d(P, 64, 64, 68, 0, 0, 0, P, P, None, None, None) == mx.EALIGN
    assert d(P + 4, 64, 64, 64, 0, 0, 0, None, None, P, P, None) == mx.EALIGN
    assert d(None, 0, 64, 64, 0, 0, 0, None, None, None, None, None) == mx.OK
    bad = mx.make_cfg(geometry=7)
    W = 0x100000
    need = mx.mxfp4_linear_workspace_bytes(64, 96, 128, bad, False)
    assert L.mxfp4_linear_fwd(P, P, P, 64, 96, 128, ctypes.byref(bad), W, need, None) == mx.EINVAL
    g2 = mx.make_cfg(geometry=mx.GEOM_2D)
    assert L.mxfp4_linear_fwd(P, P, P, 48, 96, 128, ctypes.byref(g2), W, need, None) == mx.ESHAPE
    needb = mx.mxfp4_linear_workspace_bytes(64, 96, 128, g2, True)
    assert L.mxfp4_linear_bwd(P, P, P, P, None, 64, 96, 136, ctypes.byref(g2), W, needb, None) == mx.ESHAPE


def test_fp8_and_stage_format_argument_errors(L):
    q = L.mxfp4_quantize_fp8
    assert q(P, 64, 64, 64, 2, 0, 0, P, P, None) == mx.EINVAL          # axis
    assert q(P, 64, 64, 64, 0, 9, 0, P, P, None) == mx.EINVAL          # hadamard
    assert q(P, 64, 48, 48, 0, 0, 0, P, P, None) == mx.ESHAPE
    assert q(P, 48, 64, 64, 1, 0, 0, P, P, None) == mx.ESHAPE
    assert q(P + 2, 64, 64, 64, 0, 0, 0, P, P, None) == mx.EALIGN
    assert q(None, 0, 64, 64, 0, 0, 0, None, None, None) == mx.OK
    g = L.mxfp4_gemm_fmt
    assert g(P, P, 2, P, P, 0, 16, 16, 32, P, 16, 1, 0, None) == mx.EINVAL
    assert g(P, P, 1, P, P, -1, 16, 16, 32, P, 16, 1, 0, None) == mx.EINVAL
    assert g(P, P, 1, P, P, 1, 16, 16, 48, P, 16, 1, 0, None) == mx.ESHAPE
    assert g(P, P, 1, P, P, 1, 0, 16, 32, None, 16, 1, 0, None) == mx.OK
    M, N, K = 64, 96, 128
    all4, all8 = mx.make_cfg(), mx.make_cfg(fprop_format=1, dgrad_format=1, wgrad_format=1)
    mixed = mx.make_cfg(dgrad_format=1)
    # an 8-bit stage doubles the code bytes of its operands, scale bytes stay
    f4, f8 = (mx.mxfp4_linear_workspace_bytes(M, N, K, c, False) for c in (all4, all8))
    assert f8 - f4 == (M + N) * K // 2
    b4, bm = (mx.mxfp4_linear_workspace_bytes(M, N, K, c, True) for c in (all4, mixed))
    assert bm - b4 == (M + K) * N // 2
    assert mx.mxfp4_linear_saved_bytes(M, N, K, mixed) - mx.mxfp4_linear_saved_bytes(M, N, K, all4) == K * N // 2
    assert mx.mxfp4_linear_saved_bytes(M, N, K, None) == mx.mxfp4_linear_saved_bytes(M, N, K, all4)
    assert mx.mxfp4_linear_workspace_layout(M, N, K, True, None) == mx.mxfp4_linear_workspace_layout(M, N, K, True, all4)
    bad = mx.make_cfg(wgrad_format=3)
    W = 0x100000
    assert L.mxfp4_linear_fwd(P, P, P, M, N, K, ctypes.byref(bad), W, f8, None) == mx.EINVAL
    g2 = mx.make_cfg(geometry=mx.GEOM_2D, fprop_format=1)
    assert L.mxfp4_linear_fwd(P, P, P, M, N, K, ctypes.byref(g2), W, f8, None) == mx.ENOTIMPL
    assert L.mxfp4_linear_fwd(P, P, P, M, N, K, ctypes.byref(all8), W, f4, None) == mx.EWORKSPACE


def test_missing_library_is_a_loud_error(monkeypatch, tmp_path):
    monkeypatch.setattr(mx, "_lib", None)
    monkeypatch.setattr(mx, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        mx.lib()


def test_static_scratch_forward_argument_errors(L):
    # the call that allocates nothing: sizes beyond its 32 MiB array and bad arguments are refused on the host
    cfg = mx.make_cfg(mx.HAD_DET, mx.RNE, 0)
    f = L.mxfp4_linear_fwd_static
    assert L.mxfp4_linear_workspace_bytes(8192, 6144, 4096, ctypes.byref(cfg), 0) <= mx.STATIC_SCRATCH_BYTES
    assert f(P, P, P, 16384, 6144, 4096, ctypes.byref(cfg), None) == mx.EWORKSPACE
    assert f(P, P, P, 1 << 40, 1 << 40, 1 << 40, ctypes.byref(cfg), None) == mx.EWORKSPACE
    assert f(P, P, P, 64, 64, 48, ctypes.byref(cfg), None) == mx.ESHAPE
    assert f(None, P, P, 64, 64, 64, ctypes.byref(cfg), None) == mx.EINVAL
    assert f(P, P, P, 64, 64, 64, None, None) == mx.EINVAL


def test_gemm_plan_host_logic(L):
    # which kernels a product is cut into (256 compute units): no device is touched
    A, T256, T128, TAIL = mx.GEMM_ANY, mx.GEMM_TILED_256, mx.GEMM_TILED_128, mx.GEMM_TILED_256_TAIL_128
    plan = mx.mxfp4_gemm_plan
    # the headline GEMMs: 768 and 512 tiles = whole rounds of 256 x 256 tiles
    assert plan(8192, 6144, 4096) == [(T256, 0, 8192, 0, 6144, 0)]
    assert plan(8192, 4096, 6144) == [(T256, 0, 8192, 0, 4096, 0)]
    # its Wgrad, 384 tiles: one whole round on 256 x 256 tiles, then the other 128 in halves, in one launch
    assert plan(6144, 4096, 8192) == [(TAIL, 0, 6144, 0, 4096, 256)]
    # fewer tiles than compute units (Llama's k / v projections), columns in whole 128s only
    assert plan(8192, 1024, 4096) == [(T128, 0, 8192, 0, 1024, 0)]
    assert plan(1024, 4096, 8192) == [(T128, 0, 1024, 0, 4096, 0)]
    assert plan(4352, 2176, 1280) == [(T128, 0, 4352, 0, 2176, 0)]
    # three and a half rounds (the Wgrad stress shape): three rounds whole, the last in halves
    assert plan(4096, 14336, 16384) == [(TAIL, 0, 4096, 0, 14336, 768)]
    # more than four whole rounds in front (1320 tiles), or a last round more than half full: no halves
    assert plan(256 * 40, 256 * 33, 2048) == [(T256, 0, 256 * 40, 0, 256 * 33, 0)]
    assert plan(256 * 28, 256 * 16, 4096) == [(T256, 0, 256 * 28, 0, 256 * 16, 0)]     # 448 tiles: 192 in the last
    # 289 tiles (17 x 17): 33 in the last round
    assert plan(4352, 4352, 1024) == [(TAIL, 0, 4352, 0, 4352, 256)]
    # ragged edges: tiled interior + strips on the any-shape kernel
    assert plan(8224, 6144, 4096) == [(T256, 0, 8192, 0, 6144, 0), (A, 8192, 32, 0, 6144, 0)]
    assert plan(300, 520, 1024) == [(T128, 0, 256, 0, 512, 0), (A, 0, 300, 512, 8, 0), (A, 256, 44, 0, 512, 0)]
    assert plan(6144 + 5, 4096, 8192) == [(TAIL, 0, 6144, 0, 4096, 256), (A, 6144, 5, 0, 4096, 0)]
    # contraction too short or not in whole stages, mixed formats, misaligned rows: any-shape kernel
    assert plan(512, 512, 512) == [(A, 0, 512, 0, 512, 0)]
    assert plan(512, 512, 1024 + 32) == [(A, 0, 512, 0, 512, 0)]
    assert plan(512, 512, 2048, mx.FMT_E4M3, mx.FMT_E2M1) == [(A, 0, 512, 0, 512, 0)]
    assert plan(512, 512, 2048, ld_out=516) == [(A, 0, 512, 0, 512, 0)]
    # MXFP8 stays on 256 x 256 tiles; a smaller chip changes the rounds
    assert plan(512, 512, 2048, mx.FMT_E4M3, mx.FMT_E4M3) == [(T256, 0, 512, 0, 512, 0)]
    assert plan(6144, 4096, 8192, mx.FMT_E4M3, mx.FMT_E4M3) == [(T256, 0, 6144, 0, 4096, 0)]
    assert plan(6144, 4096, 8192, compute_units=128) == [(T256, 0, 6144, 0, 4096, 0)]
    assert plan(0, 16, 32) == []
    n = ctypes.c_int(0)
    parts = (ctypes.c_int64 * 24)()
    assert L.mxfp4_gemm_plan(16, 16, 48, 0, 0, 16, 256, ctypes.byref(n), parts) == mx.ESHAPE
    assert L.mxfp4_gemm_plan(16, 16, 32, 0, 0, 16, 0, ctypes.byref(n), parts) == mx.EINVAL
    assert L.mxfp4_gemm_plan(16, 16, 32, 7, 0, 16, 256, ctypes.byref(n), parts) == mx.EINVAL
    assert L.mxfp4_gemm_plan(16, 16, 32, 0, 0, 16, 256, None, parts) == mx.EINVAL
