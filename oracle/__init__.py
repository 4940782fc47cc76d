"""CPU oracle for the MXFP4 linear-layer hot path (TEST INFRASTRUCTURE ONLY).

Thin ctypes loader around ``mxfp4_oracle.c`` plus the compositions that need
no arithmetic of their own (linear forward/backward = quantise, then GEMM, with
the axes of App. C.1-C.3).  Only tests, the smoke check and the benchmark's
``cpu_baseline`` leg may import this package; the product path never does.

All arrays are numpy, on the host.  bf16 tensors travel as uint16 bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mxfp4_oracle.c")
_LIB = os.path.join(_HERE, "libmxfp4_oracle.so")

AXIS_LAST, AXIS_FIRST = 0, 1
HAD_NONE, HAD_DET, HAD_RANDSIGN, HAD_DET16, HAD_RANDSIGN16 = 0, 1, 2, 3, 4
RNE, SR = 0, 1
FMT_E2M1, FMT_E4M3 = 0, 1


# MXFP4_ORACLE_SANITIZE=1 builds and loads an AddressSanitizer + UndefinedBehaviorSanitizer build of the oracle
# instead (the interpreter must then be started with the ASan runtime preloaded):
#   MXFP4_ORACLE_SANITIZE=1 LD_PRELOAD=$(gcc -print-file-name=libasan.so) ASAN_OPTIONS=detect_leaks=0 \
#       python -m pytest tests -q -m "not gpu"
_SANITIZE = os.environ.get("MXFP4_ORACLE_SANITIZE", "") not in ("", "0")
if _SANITIZE:
    _LIB = os.path.join(_HERE, "libmxfp4_oracle_san.so")


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-fno-fast-math", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        if _SANITIZE:
            cmd[1:2] = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                        "-fno-omit-frame-pointer"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib: Optional[ctypes.CDLL] = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        u8p = ctypes.POINTER(ctypes.c_uint8)
        u16p = ctypes.POINTER(ctypes.c_uint16)
        f64p = ctypes.POINTER(ctypes.c_double)
        i64p = ctypes.POINTER(ctypes.c_int64)
        i64 = ctypes.c_int64
        L.orc_rand32.restype = ctypes.c_uint32
        L.orc_rand32.argtypes = [ctypes.c_uint64, ctypes.c_uint64]
        L.orc_rand32_array.restype = None
        L.orc_rand32_array.argtypes = [ctypes.c_uint64, ctypes.c_uint64, i64, ctypes.POINTER(ctypes.c_uint32)]
        L.orc_sign_mask.restype = ctypes.c_uint32
        L.orc_sign_mask.argtypes = [ctypes.c_uint64]
        L.orc_seed_with_stream.restype = ctypes.c_uint64
        L.orc_seed_with_stream.argtypes = [ctypes.c_uint64, ctypes.c_uint]
        L.orc_bf16_to_f32.restype = ctypes.c_float
        L.orc_bf16_to_f32.argtypes = [ctypes.c_uint16]
        L.orc_e2m1_decode.restype = ctypes.c_double
        L.orc_e2m1_decode.argtypes = [ctypes.c_uint]
        L.orc_e2m1_encode_rne.restype = ctypes.c_uint
        L.orc_e2m1_encode_rne.argtypes = [ctypes.c_double]
        L.orc_e2m1_encode_sr.restype = ctypes.c_uint
        L.orc_e2m1_encode_sr.argtypes = [ctypes.c_double, ctypes.c_uint32]
        L.orc_e8m0_from_amax_bits.restype = ctypes.c_uint
        L.orc_e8m0_from_amax_bits.argtypes = [ctypes.c_uint32]
        L.orc_wht.restype = None
        L.orc_wht.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_int]
        L.orc_quantize.restype = ctypes.c_int
        L.orc_quantize.argtypes = [u16p, i64, i64, i64, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                   ctypes.c_uint64, u8p, u8p]
        L.orc_quantize_2d.restype = ctypes.c_int
        L.orc_quantize_2d.argtypes = [u16p, i64, i64, i64, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                      ctypes.c_uint64, u8p, u8p]
        L.orc_e4m3_decode.restype = ctypes.c_double
        L.orc_e4m3_decode.argtypes = [ctypes.c_uint]
        L.orc_e4m3_encode_rne.restype = ctypes.c_uint
        L.orc_e4m3_encode_rne.argtypes = [ctypes.c_double]
        L.orc_e8m0_from_amax_bits_fp8.restype = ctypes.c_uint
        L.orc_e8m0_from_amax_bits_fp8.argtypes = [ctypes.c_uint32]
        L.orc_quantize_fp8.restype = ctypes.c_int
        L.orc_quantize_fp8.argtypes = [u16p, i64, i64, i64, ctypes.c_int, ctypes.c_int, ctypes.c_uint64, u8p, u8p]
        L.orc_gemm_fmt.restype = ctypes.c_int
        L.orc_gemm_fmt.argtypes = [u8p, u8p, ctypes.c_int, u8p, u8p, ctypes.c_int, i64, i64, i64, f64p, f64p]
        L.orc_gemm_at_fmt.restype = ctypes.c_int
        L.orc_gemm_at_fmt.argtypes = [u8p, u8p, ctypes.c_int, u8p, u8p, ctypes.c_int, i64, i64, i64, i64p, i64p, i64,
                                      f64p, f64p]
        L.orc_dequantize.restype = None
        L.orc_dequantize.argtypes = [u8p, u8p, i64, i64, f64p]
        L.orc_gemm.restype = ctypes.c_int
        L.orc_gemm.argtypes = [u8p, u8p, u8p, u8p, i64, i64, i64, f64p, f64p]
        L.orc_gemm_at.restype = ctypes.c_int
        L.orc_gemm_at.argtypes = [u8p, u8p, u8p, u8p, i64, i64, i64, i64p, i64p, i64, f64p, f64p]
        L.orc_f32_to_bf16_rne.restype = ctypes.c_uint16
        L.orc_f32_to_bf16_rne.argtypes = [ctypes.c_float]
        L.orc_num_threads.restype = ctypes.c_int
        L.orc_num_threads.argtypes = []
        _lib = L
    return _lib


def _p(a: np.ndarray, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct))


# ---------------------------------------------------------------------------
# scalar helpers (used by the pins)
# ---------------------------------------------------------------------------
def rand32(seed: int, idx: int) -> int:
    return int(lib().orc_rand32(seed & (2**64 - 1), idx & (2**64 - 1)))


def rand32_array(seed: int, idx0: int, n: int) -> np.ndarray:
    out = np.empty(n, dtype=np.uint32)
    lib().orc_rand32_array(seed & (2**64 - 1), idx0 & (2**64 - 1), n, _p(out, ctypes.c_uint32))
    return out


def sign_mask(seed: int) -> int:
    return int(lib().orc_sign_mask(seed & (2**64 - 1)))


def e2m1_decode(code: int) -> float:
    return float(lib().orc_e2m1_decode(code))


def e2m1_encode_rne(t: float) -> int:
    return int(lib().orc_e2m1_encode_rne(float(t)))


def e2m1_encode_sr(t: float, r: int) -> int:
    return int(lib().orc_e2m1_encode_sr(float(t), r & 0xFFFFFFFF))


def e8m0_from_amax_bits(bits: int) -> int:
    return int(lib().orc_e8m0_from_amax_bits(bits & 0xFFFFFFFF))


def wht(v: np.ndarray) -> np.ndarray:
    """Unnormalised fp32 Walsh-Hadamard butterfly of a length-16 or -32 vector."""
    out = np.ascontiguousarray(v, dtype=np.float32).copy()
    assert out.ndim == 1 and out.size in (16, 32)
    lib().orc_wht(_p(out, ctypes.c_float), out.size)
    return out


def num_threads() -> int:
    return int(lib().orc_num_threads())


# ---------------------------------------------------------------------------
# tensors
# ---------------------------------------------------------------------------
def quantize(x_bf16: np.ndarray, axis: int = AXIS_LAST, had: int = HAD_NONE, rnd: int = RNE,
             seed: int = 0) -> Tuple[np.ndarray, np.ndarray]:
    """x_bf16: uint16 [rows][cols] (row-major view allowed: last stride 1).

    Returns (q uint8 [R][C/2], s uint8 [R][C/32]); R, C as in orc_quantize."""
    assert x_bf16.dtype == np.uint16 and x_bf16.ndim == 2
    assert x_bf16.strides[1] == 2 and x_bf16.strides[0] % 2 == 0
    rows, cols = x_bf16.shape
    ld = x_bf16.strides[0] // 2
    R, C = (rows, cols) if axis == AXIS_LAST else (cols, rows)
    if C % 32 != 0:
        raise ValueError("contraction length must be a multiple of 32")
    q = np.empty((R, C // 2), dtype=np.uint8)
    s = np.empty((R, C // 32), dtype=np.uint8)
    rc = lib().orc_quantize(_p(x_bf16, ctypes.c_uint16), rows, cols, ld, axis, had, rnd,
                            seed & (2**64 - 1), _p(q, ctypes.c_uint8), _p(s, ctypes.c_uint8))
    if rc != 0:
        raise RuntimeError(f"orc_quantize failed: {rc}")
    return q, s


def quantize_2d(x_bf16: np.ndarray, axis: int = AXIS_LAST, had: int = HAD_NONE, rnd: int = RNE,
                seed: int = 0) -> Tuple[np.ndarray, np.ndarray]:
    """As quantize(), with one scale per 32 x 32 region (orc_quantize_2d)."""
    assert x_bf16.dtype == np.uint16 and x_bf16.ndim == 2
    assert x_bf16.strides[1] == 2 and x_bf16.strides[0] % 2 == 0
    rows, cols = x_bf16.shape
    ld = x_bf16.strides[0] // 2
    R, C = (rows, cols) if axis == AXIS_LAST else (cols, rows)
    if C % 32 != 0 or R % 32 != 0:
        raise ValueError("both lengths must be multiples of 32")
    q = np.empty((R, C // 2), dtype=np.uint8)
    s = np.empty((R, C // 32), dtype=np.uint8)
    rc = lib().orc_quantize_2d(_p(x_bf16, ctypes.c_uint16), rows, cols, ld, axis, had, rnd,
                               seed & (2**64 - 1), _p(q, ctypes.c_uint8), _p(s, ctypes.c_uint8))
    if rc != 0:
        raise RuntimeError(f"orc_quantize_2d failed: {rc}")
    return q, s


def dequantize(q: np.ndarray, s: np.ndarray) -> np.ndarray:
    q = np.ascontiguousarray(q, dtype=np.uint8)
    s = np.ascontiguousarray(s, dtype=np.uint8)
    R, C = q.shape[0], q.shape[1] * 2
    assert s.shape == (R, C // 32)
    out = np.empty((R, C), dtype=np.float64)
    lib().orc_dequantize(_p(q, ctypes.c_uint8), _p(s, ctypes.c_uint8), R, C, _p(out, ctypes.c_double))
    return out


def gemm(aq, as_, bq, bs, want_absum: bool = True):
    """out[i][j] = sum_c A[i][c] B[j][c] in double; also sum |a||b| if asked."""
    aq, as_, bq, bs = (np.ascontiguousarray(t, dtype=np.uint8) for t in (aq, as_, bq, bs))
    Ra, C = aq.shape[0], aq.shape[1] * 2
    Rb = bq.shape[0]
    assert bq.shape[1] * 2 == C and as_.shape == (Ra, C // 32) and bs.shape == (Rb, C // 32)
    out = np.empty((Ra, Rb), dtype=np.float64)
    ab = np.empty((Ra, Rb), dtype=np.float64) if want_absum else None
    rc = lib().orc_gemm(_p(aq, ctypes.c_uint8), _p(as_, ctypes.c_uint8), _p(bq, ctypes.c_uint8),
                        _p(bs, ctypes.c_uint8), Ra, Rb, C, _p(out, ctypes.c_double),
                        _p(ab, ctypes.c_double) if want_absum else None)
    if rc != 0:
        raise RuntimeError(f"orc_gemm failed: {rc}")
    return (out, ab) if want_absum else out


def gemm_at(aq, as_, bq, bs, ii, jj):
    """The GEMM sum at the output positions (ii[k], jj[k]) only."""
    aq, as_, bq, bs = (np.ascontiguousarray(t, dtype=np.uint8) for t in (aq, as_, bq, bs))
    ii = np.ascontiguousarray(ii, dtype=np.int64)
    jj = np.ascontiguousarray(jj, dtype=np.int64)
    Ra, C = aq.shape[0], aq.shape[1] * 2
    Rb = bq.shape[0]
    assert bq.shape[1] * 2 == C and ii.shape == jj.shape and ii.ndim == 1
    out = np.empty(ii.shape, dtype=np.float64)
    ab = np.empty(ii.shape, dtype=np.float64)
    rc = lib().orc_gemm_at(_p(aq, ctypes.c_uint8), _p(as_, ctypes.c_uint8), _p(bq, ctypes.c_uint8),
                           _p(bs, ctypes.c_uint8), Ra, Rb, C, _p(ii, ctypes.c_int64), _p(jj, ctypes.c_int64),
                           ii.size, _p(out, ctypes.c_double), _p(ab, ctypes.c_double))
    if rc != 0:
        raise RuntimeError(f"orc_gemm_at failed: {rc}")
    return out, ab


def e4m3_decode(code: int) -> float:
    return float(lib().orc_e4m3_decode(int(code)))


def e4m3_encode_rne(t: float) -> int:
    return int(lib().orc_e4m3_encode_rne(float(t)))


def e8m0_from_amax_bits_fp8(bits: int) -> int:
    return int(lib().orc_e8m0_from_amax_bits_fp8(int(bits)))


def quantize_fp8(x_bf16: np.ndarray, axis: int = AXIS_LAST, had: int = HAD_NONE,
                 seed: int = 0) -> Tuple[np.ndarray, np.ndarray]:
    """MXFP8 (E4M3 elements): returns (q8 uint8 [R][C], s uint8 [R][C/32])."""
    assert x_bf16.dtype == np.uint16 and x_bf16.ndim == 2
    assert x_bf16.strides[1] == 2 and x_bf16.strides[0] % 2 == 0
    rows, cols = x_bf16.shape
    ld = x_bf16.strides[0] // 2
    R, C = (rows, cols) if axis == AXIS_LAST else (cols, rows)
    if C % 32 != 0:
        raise ValueError("contraction length must be a multiple of 32")
    q = np.empty((R, C), dtype=np.uint8)
    s = np.empty((R, C // 32), dtype=np.uint8)
    rc = lib().orc_quantize_fp8(_p(x_bf16, ctypes.c_uint16), rows, cols, ld, axis, had, seed & (2**64 - 1),
                                _p(q, ctypes.c_uint8), _p(s, ctypes.c_uint8))
    if rc != 0:
        raise RuntimeError(f"orc_quantize_fp8 failed: {rc}")
    return q, s


def _contraction_length(q: np.ndarray, fmt: int) -> int:
    return q.shape[1] * (2 if fmt == FMT_E2M1 else 1)


def gemm_fmt(aq, as_, afmt, bq, bs, bfmt):
    """gemm() with each operand in its own element format; returns (out, absum)."""
    aq, as_, bq, bs = (np.ascontiguousarray(t, dtype=np.uint8) for t in (aq, as_, bq, bs))
    Ra, Rb, C = aq.shape[0], bq.shape[0], _contraction_length(aq, afmt)
    assert _contraction_length(bq, bfmt) == C and as_.shape == (Ra, C // 32) and bs.shape == (Rb, C // 32)
    out = np.empty((Ra, Rb), dtype=np.float64)
    ab = np.empty((Ra, Rb), dtype=np.float64)
    rc = lib().orc_gemm_fmt(_p(aq, ctypes.c_uint8), _p(as_, ctypes.c_uint8), afmt, _p(bq, ctypes.c_uint8),
                            _p(bs, ctypes.c_uint8), bfmt, Ra, Rb, C, _p(out, ctypes.c_double),
                            _p(ab, ctypes.c_double))
    if rc != 0:
        raise RuntimeError(f"orc_gemm_fmt failed: {rc}")
    return out, ab


def gemm_at_fmt(aq, as_, afmt, bq, bs, bfmt, ii, jj):
    aq, as_, bq, bs = (np.ascontiguousarray(t, dtype=np.uint8) for t in (aq, as_, bq, bs))
    ii = np.ascontiguousarray(ii, dtype=np.int64)
    jj = np.ascontiguousarray(jj, dtype=np.int64)
    Ra, Rb, C = aq.shape[0], bq.shape[0], _contraction_length(aq, afmt)
    assert _contraction_length(bq, bfmt) == C and ii.shape == jj.shape and ii.ndim == 1
    out = np.empty(ii.shape, dtype=np.float64)
    ab = np.empty(ii.shape, dtype=np.float64)
    rc = lib().orc_gemm_at_fmt(_p(aq, ctypes.c_uint8), _p(as_, ctypes.c_uint8), afmt, _p(bq, ctypes.c_uint8),
                               _p(bs, ctypes.c_uint8), bfmt, Ra, Rb, C, _p(ii, ctypes.c_int64),
                               _p(jj, ctypes.c_int64), ii.size, _p(out, ctypes.c_double), _p(ab, ctypes.c_double))
    if rc != 0:
        raise RuntimeError(f"orc_gemm_at_fmt failed: {rc}")
    return out, ab


def f32_to_bf16_rne(x: np.ndarray) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape, dtype=np.uint16)
    f = lib().orc_f32_to_bf16_rne
    flat_in, flat_out = x.reshape(-1), out.reshape(-1)
    for k in range(flat_in.size):
        flat_out[k] = f(float(flat_in[k]))
    return out


# ---------------------------------------------------------------------------
# the three training-stage GEMMs of one linear layer (App. C.1-C.3)
# ---------------------------------------------------------------------------
GEOM_1D, GEOM_2D = 0, 1


def _q(geom):
    return quantize_2d if geom == GEOM_2D else quantize


# Rounding stream of each of the six quantised operands of a linear layer (high 16 bits of the seed): the two
# operands of every GEMM round under different streams, the random-sign diagonal (low 48 bits) is shared.
STREAM_X, STREAM_W, STREAM_DY, STREAM_WT, STREAM_DYT, STREAM_XT = range(6)


def seed_with_stream(seed: int, stream: int) -> int:
    return int(lib().orc_seed_with_stream(seed & (2**64 - 1), stream))


def linear_fwd_operands(x, w, had=HAD_NONE, rnd=RNE, seed=0, geom=GEOM_1D):
    """Fprop Y = X W^T: both operands rotated/quantised along K (App. C.1)."""
    return (_q(geom)(x, AXIS_LAST, had, rnd, seed_with_stream(seed, STREAM_X)),
            _q(geom)(w, AXIS_LAST, had, rnd, seed_with_stream(seed, STREAM_W)))


def linear_fwd(x, w, had=HAD_NONE, rnd=RNE, seed=0, geom=GEOM_1D):
    (xq, xs), (wq, ws) = linear_fwd_operands(x, w, had, rnd, seed, geom)
    return gemm(xq, xs, wq, ws)


def linear_dgrad_operands(dy, w, had=HAD_NONE, rnd=RNE, seed=0, geom=GEOM_1D):
    """Dgrad dX = dY W: contraction over N; dY[M,N] along its last axis, W[N,K]
    along its first axis (giving W^T rows) (App. C.2)."""
    return (_q(geom)(dy, AXIS_LAST, had, rnd, seed_with_stream(seed, STREAM_DY)),
            _q(geom)(w, AXIS_FIRST, had, rnd, seed_with_stream(seed, STREAM_WT)))


def linear_wgrad_operands(dy, x, had=HAD_NONE, rnd=RNE, seed=0, geom=GEOM_1D):
    """Wgrad dW = dY^T X: contraction over tokens M; both operands quantised down
    their first axis (App. C.3)."""
    return (_q(geom)(dy, AXIS_FIRST, had, rnd, seed_with_stream(seed, STREAM_DYT)),
            _q(geom)(x, AXIS_FIRST, had, rnd, seed_with_stream(seed, STREAM_XT)))


def linear_bwd(dy, x, w, had=HAD_NONE, rnd=RNE, seed=0, geom=GEOM_1D):
    """Returns ((dX, absum_dX), (dW, absum_dW))."""
    (gq, gs), (wtq, wts) = linear_dgrad_operands(dy, w, had, rnd, seed, geom)
    dx = gemm(gq, gs, wtq, wts)
    (gtq, gts), (xtq, xts) = linear_wgrad_operands(dy, x, had, rnd, seed, geom)
    dw = gemm(gtq, gts, xtq, xts)
    return dx, dw
