// C ABI of the library (see include/mxfp4.h): argument checks on the host, then launches.
#include <hip/hip_runtime.h>
#include <string.h>

#include <mutex>

#include "../../include/mxfp4.h"
#include "mxfp4_internal.h"

namespace {

using namespace mxfp4;

bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// The kernels are built for gfx950 only: refuse to launch anywhere else (checked once per process
// and device).
int device_ok()
{
    static int cached[64];  // 0 unknown, 1 ok, 2 bad
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (dev < 0 || dev >= 64) return 0;
    if (cached[dev] == 0) {
        hipDeviceProp_t prop;
        if (hipGetDeviceProperties(&prop, dev) != hipSuccess) return 0;
        cached[dev] = (strncmp(prop.gcnArchName, "gfx950", 6) == 0) ? 1 : 2;
    }
    return cached[dev] == 1;
}

int check_quantize(const void *x, int64_t rows, int64_t cols, int64_t ld, int axis, int had, int rnd,
                   const void *q, const void *s)
{
    if (axis != MXFP4_AXIS_LAST && axis != MXFP4_AXIS_FIRST) return MXFP4_EINVAL;
    if (had < MXFP4_HAD_NONE || had > MXFP4_HAD_RANDSIGN16) return MXFP4_EINVAL;
    if (rnd != MXFP4_RNE && rnd != MXFP4_SR) return MXFP4_EINVAL;
    if (rows < 0 || cols < 0) return MXFP4_ESHAPE;
    if (rows == 0 || cols == 0) return MXFP4_OK;
    if (!x || !q || !s) return MXFP4_EINVAL;
    if (ld < cols) return MXFP4_ESHAPE;
    if (axis == MXFP4_AXIS_LAST && (cols % 32) != 0) return MXFP4_ESHAPE;
    if (axis == MXFP4_AXIS_FIRST && ((rows % 32) != 0 || (cols % 2) != 0)) return MXFP4_ESHAPE;
    if (rows > (int64_t(1) << 40) || cols > (int64_t(1) << 40)) return MXFP4_ESHAPE;
    {   // the 1-D launch grids hold at most 2^31 - 1 workgroups
        const int64_t groups = (axis == MXFP4_AXIS_LAST) ? (rows * (cols / 32) + 255) / 256
                                                         : ((cols + 127) / 128) * ((rows / 32 + 7) / 8);
        if (groups >= (int64_t(1) << 31)) return MXFP4_ESHAPE;
    }
    if (!aligned(q, 16)) return MXFP4_EALIGN;
    if (axis == MXFP4_AXIS_LAST && (!aligned(x, 16) || (ld % 8) != 0)) return MXFP4_EALIGN;
    if (axis == MXFP4_AXIS_FIRST && (!aligned(x, 4) || (ld % 2) != 0)) return MXFP4_EALIGN;
    return -1;  // go
}

int check_gemm(const void *aq, const void *as, const void *bq, const void *bs, int64_t Ra, int64_t Rb, int64_t C,
               const void *out, int64_t ld, int dt, int acc)
{
    if (dt != MXFP4_OUT_BF16 && dt != MXFP4_OUT_FP32) return MXFP4_EINVAL;
    if (acc != 0 && acc != 1) return MXFP4_EINVAL;
    if (acc == 1 && dt != MXFP4_OUT_FP32) return MXFP4_EINVAL;
    if (Ra < 0 || Rb < 0 || C < 0 || (C % 32) != 0) return MXFP4_ESHAPE;
    if (Ra == 0 || Rb == 0) return MXFP4_OK;
    if (!out) return MXFP4_EINVAL;
    if (ld < Rb) return MXFP4_ESHAPE;
    if (C > 0 && (!aq || !as || !bq || !bs)) return MXFP4_EINVAL;
    if (Ra > (int64_t(1) << 36) || Rb > (int64_t(65535) * 64)) return MXFP4_ESHAPE;
    if (!aligned(aq, 16) || !aligned(bq, 16) || !aligned(out, 16)) return MXFP4_EALIGN;
    return -1;
}

// element format of each stage's operands (null cfg: all MXFP4)
struct StageFormats {
    int fprop, dgrad, wgrad;
};
StageFormats stage_formats(const mxfp4_linear_cfg *cfg)
{
    if (!cfg) return StageFormats{MXFP4_FMT_E2M1, MXFP4_FMT_E2M1, MXFP4_FMT_E2M1};
    return StageFormats{cfg->fprop_format, cfg->dgrad_format, cfg->wgrad_format};
}
// bytes of the code array of an operand with R rows and contraction length C
size_t q_bytes(int64_t R, int64_t C, int fmt) { return (size_t)R * (size_t)(fmt == MXFP4_FMT_E4M3 ? C : C / 2); }

struct FwdLayout {
    size_t xq, xs, wq, ws, total;
};
FwdLayout fwd_layout(int64_t M, int64_t N, int64_t K, const StageFormats &f)
{
    FwdLayout L;
    size_t o = 0;
    L.xq = o; o = round_up(o + q_bytes(M, K, f.fprop), 256);
    L.xs = o; o = round_up(o + (size_t)M * (K / 32), 256);
    L.wq = o; o = round_up(o + q_bytes(N, K, f.fprop), 256);
    L.ws = o; o = round_up(o + (size_t)N * (K / 32), 256);
    L.total = o;
    return L;
}

struct BwdLayout {
    size_t gq, gs, wtq, wts, gtq, gts, xtq, xts, total;
};
BwdLayout bwd_layout(int64_t M, int64_t N, int64_t K, const StageFormats &f)
{
    BwdLayout L;
    size_t o = 0;
    L.gq = o;  o = round_up(o + q_bytes(M, N, f.dgrad), 256);
    L.gs = o;  o = round_up(o + (size_t)M * (N / 32), 256);
    L.wtq = o; o = round_up(o + q_bytes(K, N, f.dgrad), 256);
    L.wts = o; o = round_up(o + (size_t)K * (N / 32), 256);
    L.gtq = o; o = round_up(o + q_bytes(N, M, f.wgrad), 256);
    L.gts = o; o = round_up(o + (size_t)N * (M / 32), 256);
    L.xtq = o; o = round_up(o + q_bytes(K, M, f.wgrad), 256);
    L.xts = o; o = round_up(o + (size_t)K * (M / 32), 256);
    L.total = o;
    return L;
}

struct SavedLayout {
    size_t wtq, wts, xtq, xts, total;
};
SavedLayout saved_layout(int64_t M, int64_t N, int64_t K, const StageFormats &f)
{
    SavedLayout L;
    size_t o = 0;
    L.wtq = o; o = round_up(o + q_bytes(K, N, f.dgrad), 256);
    L.wts = o; o = round_up(o + (size_t)K * (N / 32), 256);
    L.xtq = o; o = round_up(o + q_bytes(K, M, f.wgrad), 256);
    L.xts = o; o = round_up(o + (size_t)K * (M / 32), 256);
    L.total = o;
    return L;
}

int check_cfg(const mxfp4_linear_cfg *cfg)
{
    if (!cfg) return MXFP4_EINVAL;
    if (cfg->hadamard < MXFP4_HAD_NONE || cfg->hadamard > MXFP4_HAD_RANDSIGN16) return MXFP4_EINVAL;
    if (cfg->rounding != MXFP4_RNE && cfg->rounding != MXFP4_SR) return MXFP4_EINVAL;
    const int32_t dts[3] = {cfg->y_dtype, cfg->dx_dtype, cfg->dw_dtype};
    for (int i = 0; i < 3; ++i)
        if (dts[i] != MXFP4_OUT_BF16 && dts[i] != MXFP4_OUT_FP32) return MXFP4_EINVAL;
    if (cfg->dw_accumulate != 0 && cfg->dw_accumulate != 1) return MXFP4_EINVAL;
    if (cfg->dw_accumulate == 1 && cfg->dw_dtype != MXFP4_OUT_FP32) return MXFP4_EINVAL;
    if (cfg->geometry != MXFP4_GEOM_1D && cfg->geometry != MXFP4_GEOM_2D) return MXFP4_EINVAL;
    const int32_t fm[3] = {cfg->fprop_format, cfg->dgrad_format, cfg->wgrad_format};
    for (int i = 0; i < 3; ++i) {
        if (fm[i] != MXFP4_FMT_E2M1 && fm[i] != MXFP4_FMT_E4M3) return MXFP4_EINVAL;
        // the 8-bit stages know only the 1x32 geometry
        if (fm[i] == MXFP4_FMT_E4M3 && cfg->geometry == MXFP4_GEOM_2D) return MXFP4_ENOTIMPL;
    }
    return MXFP4_OK;
}

}  // namespace

extern "C" {

const char *mxfp4_status_string(int status)
{
    switch (status) {
        case MXFP4_OK: return "ok";
        case MXFP4_EINVAL: return "invalid argument (null pointer, unknown enum value or flag combination)";
        case MXFP4_ESHAPE: return "bad shape (negative size, contraction length not a multiple of 32, ld too small)";
        case MXFP4_EALIGN: return "misaligned pointer or leading dimension";
        case MXFP4_EWORKSPACE: return "workspace too small";
        case MXFP4_EDEVICE: return "HIP launch error or device is not gfx950";
        case MXFP4_ENOTIMPL: return "not implemented";
        default: return "unknown status";
    }
}

int mxfp4_quantize(const void *x_bf16, int64_t rows, int64_t cols, int64_t ld_elems, int axis, int hadamard,
                   int rounding, uint64_t seed, void *q_out, void *s_out, void *hip_stream)
{
    int rc = check_quantize(x_bf16, rows, cols, ld_elems, axis, hadamard, rounding, q_out, s_out);
    if (rc >= 0) return rc;
    if (!device_ok()) return MXFP4_EDEVICE;
    QuantArgs a{static_cast<const uint16_t *>(x_bf16), rows, cols, ld_elems, hadamard, rounding, seed,
                static_cast<uint8_t *>(q_out), static_cast<uint8_t *>(s_out)};
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    hipError_t e = (axis == MXFP4_AXIS_LAST) ? launch_quantize_rows(a, st) : launch_quantize_cols(a, st);
    return e == hipSuccess ? MXFP4_OK : MXFP4_EDEVICE;
}

// Argument checks of the two-output calls.  Return -1 and fill `a` when a launch is due, else the status to
// hand back (MXFP4_OK for an empty tensor).
static int prep_dual(const void *x_bf16, int64_t rows, int64_t cols, int64_t ld_elems, int hadamard, int rounding,
                     uint64_t seed_last, uint64_t seed_first, void *q_last, void *s_last, void *q_first,
                     void *s_first, QuantArgs &a)
{
    // the union of the two single-axis argument rules
    int rc = check_quantize(x_bf16, rows, cols, ld_elems, MXFP4_AXIS_LAST, hadamard, rounding, q_last, s_last);
    int rc2 = check_quantize(x_bf16, rows, cols, ld_elems, MXFP4_AXIS_FIRST, hadamard, rounding, q_first, s_first);
    if (rc > 0) return rc;
    if (rc2 > 0) return rc2;
    if (rc == 0 || rc2 == 0) return MXFP4_OK;
    a = QuantArgs{static_cast<const uint16_t *>(x_bf16), rows, cols, ld_elems, hadamard, rounding, seed_first,
                  static_cast<uint8_t *>(q_first), static_cast<uint8_t *>(s_first)};
    a.q_row = static_cast<uint8_t *>(q_last);
    a.s_row = static_cast<uint8_t *>(s_last);
    a.seed_row = seed_last;
    return -1;
}

static int prep_2d(const void *x_bf16, int64_t rows, int64_t cols, int64_t ld_elems, int hadamard, int rounding,
                   uint64_t seed_last, uint64_t seed_first, void *q_last, void *s_last, void *q_first,
                   void *s_first, QuantArgs &a)
{
    const bool want_last = q_last || s_last, want_first = q_first || s_first;
    if (hadamard < MXFP4_HAD_NONE || hadamard > MXFP4_HAD_RANDSIGN16) return MXFP4_EINVAL;
    if (rounding != MXFP4_RNE && rounding != MXFP4_SR) return MXFP4_EINVAL;
    if (rows < 0 || cols < 0) return MXFP4_ESHAPE;
    if (rows == 0 || cols == 0) return MXFP4_OK;
    if (!want_last && !want_first) return MXFP4_EINVAL;
    if ((rows % 32) != 0 || (cols % 32) != 0) return MXFP4_ESHAPE;
    // per requested output, the single-axis argument rules
    if (want_last) {
        int rc = check_quantize(x_bf16, rows, cols, ld_elems, MXFP4_AXIS_LAST, hadamard, rounding, q_last, s_last);
        if (rc >= 0) return rc;
    }
    if (want_first) {
        int rc = check_quantize(x_bf16, rows, cols, ld_elems, MXFP4_AXIS_FIRST, hadamard, rounding, q_first, s_first);
        if (rc >= 0) return rc;
    }
    if (!aligned(x_bf16, 16) || (ld_elems % 8) != 0) return MXFP4_EALIGN;
    a = QuantArgs{static_cast<const uint16_t *>(x_bf16), rows, cols, ld_elems, hadamard, rounding, seed_first,
                  static_cast<uint8_t *>(q_first), static_cast<uint8_t *>(s_first)};
    a.q_row = static_cast<uint8_t *>(q_last);
    a.s_row = static_cast<uint8_t *>(s_last);
    a.seed_row = seed_last;
    return -1;
}

// the two-output quantisers with a seed per output (the linear calls give every operand its own rounding stream)
static int quantize_dual_seeds(const void *x_bf16, int64_t rows, int64_t cols, int64_t ld_elems, int hadamard,
                               int rounding, uint64_t seed_last, uint64_t seed_first, void *q_last, void *s_last,
                               void *q_first, void *s_first, bool geom_2d, void *hip_stream)
{
    QuantArgs a;
    int rc = (geom_2d ? prep_2d : prep_dual)(x_bf16, rows, cols, ld_elems, hadamard, rounding, seed_last, seed_first,
                                             q_last, s_last, q_first, s_first, a);
    if (rc >= 0) return rc;
    if (!device_ok()) return MXFP4_EDEVICE;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    hipError_t e = geom_2d ? launch_quantize_2d(a, nullptr, st) : launch_quantize_dual(a, nullptr, st);
    return e == hipSuccess ? MXFP4_OK : MXFP4_EDEVICE;
}

int mxfp4_quantize_dual(const void *x_bf16, int64_t rows, int64_t cols, int64_t ld_elems, int hadamard,
                        int rounding, uint64_t seed, void *q_last, void *s_last, void *q_first, void *s_first,
                        void *hip_stream)
{
    return quantize_dual_seeds(x_bf16, rows, cols, ld_elems, hadamard, rounding, seed, seed, q_last, s_last, q_first,
                               s_first, false, hip_stream);
}

int mxfp4_quantize_2d(const void *x_bf16, int64_t rows, int64_t cols, int64_t ld_elems, int hadamard,
                      int rounding, uint64_t seed, void *q_last, void *s_last, void *q_first, void *s_first,
                      void *hip_stream)
{
    return quantize_dual_seeds(x_bf16, rows, cols, ld_elems, hadamard, rounding, seed, seed, q_last, s_last, q_first,
                               s_first, true, hip_stream);
}

int mxfp4_quantize_fp8(const void *x_bf16, int64_t rows, int64_t cols, int64_t ld_elems, int axis, int hadamard,
                       uint64_t seed, void *q8_out, void *s_out, void *hip_stream)
{
    int rc = check_quantize(x_bf16, rows, cols, ld_elems, axis, hadamard, MXFP4_RNE, q8_out, s_out);
    if (rc >= 0) return rc;
    if (!device_ok()) return MXFP4_EDEVICE;
    QuantArgs a{static_cast<const uint16_t *>(x_bf16), rows, cols, ld_elems, hadamard, MXFP4_RNE, seed,
                static_cast<uint8_t *>(q8_out), static_cast<uint8_t *>(s_out)};
    hipError_t e = launch_quantize_fp8(a, axis == MXFP4_AXIS_FIRST, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? MXFP4_OK : MXFP4_EDEVICE;
}

int mxfp4_quantize_fp8_dual(const void *x_bf16, int64_t rows, int64_t cols, int64_t ld_elems, int hadamard,
                            uint64_t seed, void *q8_last, void *s_last, void *q8_first, void *s_first,
                            void *hip_stream)
{
    // the union of the two single-axis argument rules
    int rc = check_quantize(x_bf16, rows, cols, ld_elems, MXFP4_AXIS_LAST, hadamard, MXFP4_RNE, q8_last, s_last);
    int rc2 = check_quantize(x_bf16, rows, cols, ld_elems, MXFP4_AXIS_FIRST, hadamard, MXFP4_RNE, q8_first, s_first);
    if (rc > 0) return rc;
    if (rc2 > 0) return rc2;
    if (rc == 0 || rc2 == 0) return MXFP4_OK;
    if (!device_ok()) return MXFP4_EDEVICE;
    QuantArgs a{static_cast<const uint16_t *>(x_bf16), rows, cols, ld_elems, hadamard, MXFP4_RNE, seed,
                static_cast<uint8_t *>(q8_first), static_cast<uint8_t *>(s_first)};
    a.q_row = static_cast<uint8_t *>(q8_last);
    a.s_row = static_cast<uint8_t *>(s_last);
    hipError_t e = launch_quantize_fp8_dual(a, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? MXFP4_OK : MXFP4_EDEVICE;
}

int mxfp4_gemm_fmt(const void *a_q, const void *a_s, int a_format, const void *b_q, const void *b_s, int b_format,
                   int64_t R_a, int64_t R_b, int64_t C, void *out, int64_t ld_out, int out_dtype, int accumulate,
                   void *hip_stream)
{
    if ((a_format != MXFP4_FMT_E2M1 && a_format != MXFP4_FMT_E4M3) ||
        (b_format != MXFP4_FMT_E2M1 && b_format != MXFP4_FMT_E4M3))
        return MXFP4_EINVAL;
    int rc = check_gemm(a_q, a_s, b_q, b_s, R_a, R_b, C, out, ld_out, out_dtype, accumulate);
    if (rc >= 0) return rc;
    if (!device_ok()) return MXFP4_EDEVICE;
    GemmArgs g{static_cast<const uint8_t *>(a_q), static_cast<const uint8_t *>(a_s),
               static_cast<const uint8_t *>(b_q), static_cast<const uint8_t *>(b_s),
               R_a, R_b, C, out, ld_out, out_dtype == MXFP4_OUT_FP32, accumulate, a_format, b_format};
    hipError_t e = launch_gemm(g, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? MXFP4_OK : MXFP4_EDEVICE;
}

int mxfp4_gemm_pair(const void *a0_q, const void *a0_s, const void *b0_q, const void *b0_s, int64_t R_a0,
                    int64_t R_b0, int64_t C0, void *out0, int64_t ld_out0, int out_dtype0,
                    const void *a1_q, const void *a1_s, const void *b1_q, const void *b1_s, int64_t R_a1,
                    int64_t R_b1, int64_t C1, void *out1, int64_t ld_out1, int out_dtype1, int accumulate1,
                    void *hip_stream)
{
    const int rc0 = check_gemm(a0_q, a0_s, b0_q, b0_s, R_a0, R_b0, C0, out0, ld_out0, out_dtype0, 0);
    if (rc0 > 0) return rc0;
    const int rc1 = check_gemm(a1_q, a1_s, b1_q, b1_s, R_a1, R_b1, C1, out1, ld_out1, out_dtype1, accumulate1);
    if (rc1 > 0) return rc1;
    if (rc0 == 0 && rc1 == 0) return MXFP4_OK;  // both empty
    if (!device_ok()) return MXFP4_EDEVICE;
    const GemmArgs g0{static_cast<const uint8_t *>(a0_q), static_cast<const uint8_t *>(a0_s),
                      static_cast<const uint8_t *>(b0_q), static_cast<const uint8_t *>(b0_s),
                      R_a0, R_b0, C0, out0, ld_out0, out_dtype0 == MXFP4_OUT_FP32, 0, MXFP4_FMT_E2M1, MXFP4_FMT_E2M1};
    const GemmArgs g1{static_cast<const uint8_t *>(a1_q), static_cast<const uint8_t *>(a1_s),
                      static_cast<const uint8_t *>(b1_q), static_cast<const uint8_t *>(b1_s),
                      R_a1, R_b1, C1, out1, ld_out1, out_dtype1 == MXFP4_OUT_FP32, accumulate1, MXFP4_FMT_E2M1,
                      MXFP4_FMT_E2M1};
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    hipError_t e;
    if (rc0 == 0) e = launch_gemm(g1, st);        // one of the two is empty: the other alone
    else if (rc1 == 0) e = launch_gemm(g0, st);
    else e = launch_gemm_pair(g0, g1, st);
    return e == hipSuccess ? MXFP4_OK : MXFP4_EDEVICE;
}

int mxfp4_gemm_plan(int64_t R_a, int64_t R_b, int64_t C, int a_format, int b_format, int64_t ld_out,
                    int compute_units, int *n_parts, int64_t parts[24])
{
    if (!n_parts || !parts || compute_units <= 0) return MXFP4_EINVAL;
    if ((a_format != MXFP4_FMT_E2M1 && a_format != MXFP4_FMT_E4M3) ||
        (b_format != MXFP4_FMT_E2M1 && b_format != MXFP4_FMT_E4M3))
        return MXFP4_EINVAL;
    if (R_a < 0 || R_b < 0 || C < 0 || (C % 32) != 0 || ld_out < R_b) return MXFP4_ESHAPE;
    *n_parts = 0;
    if (R_a == 0 || R_b == 0) return MXFP4_OK;
    // (operand pointers as well aligned as the call itself demands; the plan depends on them no further)
    const GemmArgs g{nullptr, nullptr, nullptr, nullptr, R_a, R_b, C, nullptr, ld_out, 1, 0, a_format, b_format};
    const GemmPlan plan = plan_gemm(g, compute_units);
    for (int i = 0; i < plan.n; ++i) {
        const GemmPart &p = plan.part[i];
        const int64_t row[6] = {p.kind, p.r0, p.rows, p.c0, p.cols, p.main_tiles};
        memcpy(parts + 6 * i, row, sizeof(row));
    }
    *n_parts = plan.n;
    return MXFP4_OK;
}

int mxfp4_gemm(const void *a_q, const void *a_s, const void *b_q, const void *b_s, int64_t R_a, int64_t R_b,
               int64_t C, void *out, int64_t ld_out, int out_dtype, int accumulate, void *hip_stream)
{
    return mxfp4_gemm_fmt(a_q, a_s, MXFP4_FMT_E2M1, b_q, b_s, MXFP4_FMT_E2M1, R_a, R_b, C, out, ld_out, out_dtype,
                          accumulate, hip_stream);
}

// Rounding stream of each quantised operand of a layer (the high 16 bits of its seed).  Both operands of every
// GEMM get different streams: with a shared one, A[i][c] and B[i][c] of out[i][j] = sum_c A[i][c] B[j][c] would
// draw the same stochastic-rounding variate and the diagonal of the product would be biased, which defeats the
// purpose of stochastic rounding (Sec. 3.1).  The random-sign diagonal comes from the low 48 bits and stays
// common to all six, as the cancellation of App. C requires.
enum OperandStream { STREAM_X = 0, STREAM_W = 1, STREAM_DY = 2, STREAM_WT = 3, STREAM_DYT = 4, STREAM_XT = 5 };
static uint64_t operand_seed(const mxfp4_linear_cfg *cfg, int stream) { return cfg->seed ^ ((uint64_t)stream << 48); }

// One dense tensor of a linear layer: the row-wise output (q_last, s_last) in format fmt_last, the column-wise
// one (q_first, s_first) in fmt_first, or both (a null pair = not wanted); st_last / st_first: their OperandStream.
// MXFP4 outputs follow the layer's rotation, rounding and geometry, and come from one pass over the tensor when
// both are MXFP4; an MXFP8 output is unrotated and rounded to nearest (the rotation and the rounding mode are
// stabilisers of the MXFP4 GEMMs, Table 1).
static int quantize_operand(const mxfp4_linear_cfg *cfg, const void *x, int64_t rows, int64_t cols, int fmt_last,
                            int st_last, uint8_t *q_last, uint8_t *s_last, int fmt_first, int st_first,
                            uint8_t *q_first, uint8_t *s_first, void *hip_stream)
{
    const uint64_t seed_last = operand_seed(cfg, st_last), seed_first = operand_seed(cfg, st_first);
    if (q_last && q_first && fmt_last == MXFP4_FMT_E4M3 && fmt_first == MXFP4_FMT_E4M3)  // both in 8 bits: one pass
        return mxfp4_quantize_fp8_dual(x, rows, cols, cols, MXFP4_HAD_NONE, seed_last, q_last, s_last, q_first, s_first,
                                       hip_stream);
    if (q_last && q_first && fmt_last == MXFP4_FMT_E2M1 && fmt_first == MXFP4_FMT_E4M3 &&
        cfg->geometry == MXFP4_GEOM_1D) {
        // row-wise MXFP4 and column-wise MXFP8 (the stage-wise recipes between "Fprop only" and "all three"): one pass
        QuantArgs a;
        int rc = prep_dual(x, rows, cols, cols, cfg->hadamard, cfg->rounding, seed_last, seed_first, q_last, s_last,
                           q_first, s_first, a);
        if (rc >= 0) return rc;
        if (!device_ok()) return MXFP4_EDEVICE;
        hipError_t e = launch_quantize_mxfp4_rows_mxfp8_cols(a, static_cast<hipStream_t>(hip_stream));
        return e == hipSuccess ? MXFP4_OK : MXFP4_EDEVICE;
    }
    if (q_last && fmt_last == MXFP4_FMT_E4M3) {
        int rc = mxfp4_quantize_fp8(x, rows, cols, cols, MXFP4_AXIS_LAST, MXFP4_HAD_NONE, seed_last, q_last, s_last,
                                    hip_stream);
        if (rc != MXFP4_OK) return rc;
        q_last = s_last = nullptr;
    }
    if (q_first && fmt_first == MXFP4_FMT_E4M3) {
        int rc = mxfp4_quantize_fp8(x, rows, cols, cols, MXFP4_AXIS_FIRST, MXFP4_HAD_NONE, seed_first, q_first,
                                    s_first, hip_stream);
        if (rc != MXFP4_OK) return rc;
        q_first = s_first = nullptr;
    }
    if (!q_last && !q_first) return MXFP4_OK;
    if (cfg->geometry == MXFP4_GEOM_2D || (q_last && q_first))
        return quantize_dual_seeds(x, rows, cols, cols, cfg->hadamard, cfg->rounding, seed_last, seed_first, q_last,
                                   s_last, q_first, s_first, cfg->geometry == MXFP4_GEOM_2D, hip_stream);
    if (q_last)
        return mxfp4_quantize(x, rows, cols, cols, MXFP4_AXIS_LAST, cfg->hadamard, cfg->rounding, seed_last, q_last,
                              s_last, hip_stream);
    return mxfp4_quantize(x, rows, cols, cols, MXFP4_AXIS_FIRST, cfg->hadamard, cfg->rounding, seed_first, q_first,
                          s_first, hip_stream);
}

// Both MXFP4 outputs of the two dense tensors X and W of a forward call that also saves for the backward call,
// in one launch.
static int quantize_operand_pair(const mxfp4_linear_cfg *cfg, const void *x0, int64_t rows0, int64_t cols0,
                                 uint8_t *ql0, uint8_t *sl0, uint8_t *qf0, uint8_t *sf0, const void *x1,
                                 int64_t rows1, int64_t cols1, uint8_t *ql1, uint8_t *sl1, uint8_t *qf1,
                                 uint8_t *sf1, void *hip_stream)
{
    const bool g2 = cfg->geometry == MXFP4_GEOM_2D;
    QuantArgs a, b;
    auto prep = g2 ? prep_2d : prep_dual;
    int rc = prep(x0, rows0, cols0, cols0, cfg->hadamard, cfg->rounding, operand_seed(cfg, STREAM_X),
                  operand_seed(cfg, STREAM_XT), ql0, sl0, qf0, sf0, a);
    if (rc > 0) return rc;
    int rc1 = prep(x1, rows1, cols1, cols1, cfg->hadamard, cfg->rounding, operand_seed(cfg, STREAM_W),
                   operand_seed(cfg, STREAM_WT), ql1, sl1, qf1, sf1, b);
    if (rc1 > 0) return rc1;
    if (rc == 0 && rc1 == 0) return MXFP4_OK;
    if (!device_ok()) return MXFP4_EDEVICE;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    hipError_t e;
    auto tiles = [](const QuantArgs &t) { return ((t.cols + 127) / 128) * ((t.rows / 32 + 7) / 8); };
    if (rc == 0 || rc1 == 0) {  // one of them is empty
        e = g2 ? launch_quantize_2d(rc == 0 ? b : a, nullptr, st) : launch_quantize_dual(rc == 0 ? b : a, nullptr, st);
    } else if (tiles(a) + tiles(b) >= (int64_t(1) << 31)) {  // too many workgroups for one grid
        e = g2 ? launch_quantize_2d(a, nullptr, st) : launch_quantize_dual(a, nullptr, st);
        if (e == hipSuccess) e = g2 ? launch_quantize_2d(b, nullptr, st) : launch_quantize_dual(b, nullptr, st);
    } else {
        e = g2 ? launch_quantize_2d(a, &b, st) : launch_quantize_dual(a, &b, st);
    }
    return e == hipSuccess ? MXFP4_OK : MXFP4_EDEVICE;
}

// The column-wise MXFP4 quantisations of two dense tensors (W and X of a backward call) in one launch.
static int quantize_cols_pair(const mxfp4_linear_cfg *cfg, const void *x0, int64_t rows0, int64_t cols0, int st0,
                              uint8_t *q0, uint8_t *s0, const void *x1, int64_t rows1, int64_t cols1, int st1,
                              uint8_t *q1, uint8_t *s1, void *hip_stream)
{
    int rc = check_quantize(x0, rows0, cols0, cols0, MXFP4_AXIS_FIRST, cfg->hadamard, cfg->rounding, q0, s0);
    if (rc >= 0) return rc;  // (an error; the linear calls pass no empty tensors)
    rc = check_quantize(x1, rows1, cols1, cols1, MXFP4_AXIS_FIRST, cfg->hadamard, cfg->rounding, q1, s1);
    if (rc >= 0) return rc;
    const int64_t groups = ((cols0 + 127) / 128) * ((rows0 / 32 + 7) / 8) + ((cols1 + 127) / 128) * ((rows1 / 32 + 7) / 8);
    if (groups >= (int64_t(1) << 31)) return MXFP4_ESHAPE;  // the two grids share one launch
    if (!device_ok()) return MXFP4_EDEVICE;
    const QuantArgs a{static_cast<const uint16_t *>(x0), rows0, cols0, cols0, cfg->hadamard, cfg->rounding,
                      operand_seed(cfg, st0), q0, s0};
    const QuantArgs b{static_cast<const uint16_t *>(x1), rows1, cols1, cols1, cfg->hadamard, cfg->rounding,
                      operand_seed(cfg, st1), q1, s1};
    hipError_t e = launch_quantize_cols(a, static_cast<hipStream_t>(hip_stream), &b);
    return e == hipSuccess ? MXFP4_OK : MXFP4_EDEVICE;
}

// Dgrad and Wgrad of one layer: two GEMMs on the same stream that do not depend on each other.
static int gemm_pair(const GemmArgs &g0, int dt0, const GemmArgs &g1, int dt1, void *hip_stream)
{
    int rc = check_gemm(g0.aq, g0.as, g0.bq, g0.bs, g0.Ra, g0.Rb, g0.C, g0.out, g0.ld, dt0, g0.accumulate);
    if (rc > 0) return rc;
    int rc1 = check_gemm(g1.aq, g1.as, g1.bq, g1.bs, g1.Ra, g1.Rb, g1.C, g1.out, g1.ld, dt1, g1.accumulate);
    if (rc1 > 0) return rc1;
    if (!device_ok()) return MXFP4_EDEVICE;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    hipError_t e = hipSuccess;
    if (rc < 0 && rc1 < 0)
        e = launch_gemm_pair(g0, g1, st);
    else if (rc < 0)
        e = launch_gemm(g0, st);
    else if (rc1 < 0)
        e = launch_gemm(g1, st);
    return e == hipSuccess ? MXFP4_OK : MXFP4_EDEVICE;
}

size_t mxfp4_linear_workspace_bytes(int64_t M, int64_t N, int64_t K, const mxfp4_linear_cfg *cfg, int bwd)
{
    if (M < 0 || N < 0 || K < 0) return 0;
    const StageFormats f = stage_formats(cfg);
    return bwd ? bwd_layout(M, N, K, f).total : fwd_layout(M, N, K, f).total;
}

int mxfp4_linear_workspace_layout(int64_t M, int64_t N, int64_t K, const mxfp4_linear_cfg *cfg, int bwd,
                                  size_t offsets[8])
{
    if (!offsets || M < 0 || N < 0 || K < 0) return MXFP4_EINVAL;
    const StageFormats f = stage_formats(cfg);
    if (bwd) {
        BwdLayout L = bwd_layout(M, N, K, f);
        const size_t o[8] = {L.gq, L.gs, L.wtq, L.wts, L.gtq, L.gts, L.xtq, L.xts};
        memcpy(offsets, o, sizeof(o));
    } else {
        FwdLayout L = fwd_layout(M, N, K, f);
        const size_t o[8] = {L.xq, L.xs, L.wq, L.ws, 0, 0, 0, 0};
        memcpy(offsets, o, sizeof(o));
    }
    return MXFP4_OK;
}

int mxfp4_linear_fwd(const void *x, const void *w, void *y, int64_t M, int64_t N, int64_t K,
                     const mxfp4_linear_cfg *cfg, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    int rc = check_cfg(cfg);
    if (rc != MXFP4_OK) return rc;
    if (M <= 0 || N <= 0 || K <= 0 || (K % 32) != 0) return MXFP4_ESHAPE;
    if (cfg->geometry == MXFP4_GEOM_2D && ((M % 32) != 0 || (N % 32) != 0)) return MXFP4_ESHAPE;
    if (!x || !w || !y || !workspace) return MXFP4_EINVAL;
    const StageFormats F = stage_formats(cfg);
    const FwdLayout L = fwd_layout(M, N, K, F);
    if (workspace_bytes < L.total) return MXFP4_EWORKSPACE;
    if (!aligned(workspace, 256) || !aligned(x, 16) || !aligned(w, 16) || !aligned(y, 16)) return MXFP4_EALIGN;
    uint8_t *ws = static_cast<uint8_t *>(workspace);
    rc = quantize_operand(cfg, x, M, K, F.fprop, STREAM_X, ws + L.xq, ws + L.xs, 0, 0, nullptr, nullptr, hip_stream);
    if (rc != MXFP4_OK) return rc;
    rc = quantize_operand(cfg, w, N, K, F.fprop, STREAM_W, ws + L.wq, ws + L.ws, 0, 0, nullptr, nullptr, hip_stream);
    if (rc != MXFP4_OK) return rc;
    return mxfp4_gemm_fmt(ws + L.xq, ws + L.xs, F.fprop, ws + L.wq, ws + L.ws, F.fprop, M, N, K, y, N, cfg->y_dtype, 0,
                          hip_stream);
}

// ---- forward call on the library's own scratch (for callers that cannot allocate) -----------------------
// The quantised operands of the forward call are staged in this array instead of a caller's workspace.
// In host code the array's name is only a stand-in for the symbol: its device address is asked for once per
// device (each GPU holds its own copy) and only that address is ever handed to kernels.
static __device__ __align__(256) uint8_t scratch[MXFP4_STATIC_SCRATCH_BYTES];

static void *static_scratch_ptr()
{
    static std::mutex mu;
    static void *ptr[64];  // per device, null until asked
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) {
            (void)hipGetLastError();  // (leave no sticky error behind for the caller's next HIP call)
            return nullptr;
        }
        ptr[dev] = p;
    }
    return ptr[dev];
}

int mxfp4_linear_fwd_static(const void *x, const void *w, void *y, int64_t M, int64_t N, int64_t K,
                            const mxfp4_linear_cfg *cfg, void *hip_stream)
{
    int rc = check_cfg(cfg);
    if (rc != MXFP4_OK) return rc;
    if (M <= 0 || N <= 0 || K <= 0 || (K % 32) != 0) return MXFP4_ESHAPE;
    // (each dimension is bounded on its own first, so that the byte count below cannot overflow)
    if (M > (int64_t)MXFP4_STATIC_SCRATCH_BYTES || N > (int64_t)MXFP4_STATIC_SCRATCH_BYTES ||
        K > (int64_t)MXFP4_STATIC_SCRATCH_BYTES)
        return MXFP4_EWORKSPACE;
    if (fwd_layout(M, N, K, stage_formats(cfg)).total > (size_t)MXFP4_STATIC_SCRATCH_BYTES) return MXFP4_EWORKSPACE;
    if (!x || !w || !y) return MXFP4_EINVAL;  // (before the device is touched: argument errors need no GPU)
    if (!device_ok()) return MXFP4_EDEVICE;
    void *ws = static_scratch_ptr();
    if (!ws) return MXFP4_EDEVICE;
    return mxfp4_linear_fwd(x, w, y, M, N, K, cfg, ws, (size_t)MXFP4_STATIC_SCRATCH_BYTES, hip_stream);
}

int mxfp4_linear_bwd(const void *dy, const void *x, const void *w, void *dx, void *dw, int64_t M, int64_t N,
                     int64_t K, const mxfp4_linear_cfg *cfg, void *workspace, size_t workspace_bytes,
                     void *hip_stream)
{
    int rc = check_cfg(cfg);
    if (rc != MXFP4_OK) return rc;
    if (M <= 0 || N <= 0 || K <= 0) return MXFP4_ESHAPE;
    if (dx && ((N % 32) != 0 || (K % 2) != 0)) return MXFP4_ESHAPE;
    if (dw && ((M % 32) != 0 || (N % 2) != 0 || (K % 2) != 0)) return MXFP4_ESHAPE;
    if (cfg->geometry == MXFP4_GEOM_2D && ((M % 32) != 0 || (N % 32) != 0 || (K % 32) != 0)) return MXFP4_ESHAPE;
    if (!dx && !dw) return MXFP4_OK;
    if (!dy || !workspace) return MXFP4_EINVAL;
    if ((dx && !w) || (dw && !x)) return MXFP4_EINVAL;
    const StageFormats F = stage_formats(cfg);
    const BwdLayout L = bwd_layout(M, N, K, F);
    if (workspace_bytes < L.total) return MXFP4_EWORKSPACE;
    if (!aligned(workspace, 256) || !aligned(dy, 16) || (dx && (!aligned(dx, 16) || !aligned(w, 16))) ||
        (dw && (!aligned(dw, 16) || !aligned(x, 16))))
        return MXFP4_EALIGN;
    if ((N % 8) != 0 || (K % 8) != 0) return MXFP4_EALIGN;  // dense bf16 rows must stay 16-byte aligned
    uint8_t *ws = static_cast<uint8_t *>(workspace);
    // dY is needed row-wise for Dgrad and column-wise for Wgrad: one pass when both are asked
    rc = quantize_operand(cfg, dy, M, N, F.dgrad, STREAM_DY, dx ? ws + L.gq : nullptr, dx ? ws + L.gs : nullptr,
                          F.wgrad, STREAM_DYT, dw ? ws + L.gtq : nullptr, dw ? ws + L.gts : nullptr, hip_stream);
    if (rc != MXFP4_OK) return rc;
    if (dx && dw && F.dgrad == MXFP4_FMT_E2M1 && F.wgrad == MXFP4_FMT_E2M1 && cfg->geometry == MXFP4_GEOM_1D) {
        // W and X, both column-wise in MXFP4: one launch for the two tensors
        rc = quantize_cols_pair(cfg, w, N, K, STREAM_WT, ws + L.wtq, ws + L.wts, x, M, K, STREAM_XT, ws + L.xtq,
                                ws + L.xts, hip_stream);
        if (rc != MXFP4_OK) return rc;
    } else {
        if (dx) {
            rc = quantize_operand(cfg, w, N, K, 0, 0, nullptr, nullptr, F.dgrad, STREAM_WT, ws + L.wtq, ws + L.wts,
                                  hip_stream);
            if (rc != MXFP4_OK) return rc;
        }
        if (dw) {
            rc = quantize_operand(cfg, x, M, K, 0, 0, nullptr, nullptr, F.wgrad, STREAM_XT, ws + L.xtq, ws + L.xts,
                                  hip_stream);
            if (rc != MXFP4_OK) return rc;
        }
    }
    const GemmArgs gd{ws + L.gq, ws + L.gs, ws + L.wtq, ws + L.wts, M, K, N, dx, K, cfg->dx_dtype == MXFP4_OUT_FP32, 0,
                      F.dgrad, F.dgrad};
    const GemmArgs gw{ws + L.gtq, ws + L.gts, ws + L.xtq, ws + L.xts, N, K, M, dw, K,
                      cfg->dw_dtype == MXFP4_OUT_FP32, cfg->dw_accumulate, F.wgrad, F.wgrad};
    if (dx && dw) return gemm_pair(gd, cfg->dx_dtype, gw, cfg->dw_dtype, hip_stream);
    if (dx)
        return mxfp4_gemm_fmt(gd.aq, gd.as, F.dgrad, gd.bq, gd.bs, F.dgrad, M, K, N, dx, K, cfg->dx_dtype, 0, hip_stream);
    return mxfp4_gemm_fmt(gw.aq, gw.as, F.wgrad, gw.bq, gw.bs, F.wgrad, N, K, M, dw, K, cfg->dw_dtype,
                          cfg->dw_accumulate, hip_stream);
}

size_t mxfp4_linear_saved_bytes(int64_t M, int64_t N, int64_t K, const mxfp4_linear_cfg *cfg)
{
    if (M < 0 || N < 0 || K < 0) return 0;
    return saved_layout(M, N, K, stage_formats(cfg)).total;
}

int mxfp4_linear_saved_layout(int64_t M, int64_t N, int64_t K, const mxfp4_linear_cfg *cfg, size_t offsets[4])
{
    if (!offsets || M < 0 || N < 0 || K < 0) return MXFP4_EINVAL;
    const SavedLayout L = saved_layout(M, N, K, stage_formats(cfg));
    const size_t o[4] = {L.wtq, L.wts, L.xtq, L.xts};
    memcpy(offsets, o, sizeof(o));
    return MXFP4_OK;
}

int mxfp4_linear_fwd_save(const void *x, const void *w, void *y, int64_t M, int64_t N, int64_t K,
                          const mxfp4_linear_cfg *cfg, void *workspace, size_t workspace_bytes, void *saved,
                          size_t saved_bytes, void *hip_stream)
{
    int rc = check_cfg(cfg);
    if (rc != MXFP4_OK) return rc;
    if (M <= 0 || N <= 0 || K <= 0 || (M % 32) != 0 || (N % 32) != 0 || (K % 32) != 0) return MXFP4_ESHAPE;
    if (!x || !w || !y || !workspace || !saved) return MXFP4_EINVAL;
    const StageFormats F = stage_formats(cfg);
    const FwdLayout L = fwd_layout(M, N, K, F);
    const SavedLayout S = saved_layout(M, N, K, F);
    if (workspace_bytes < L.total || saved_bytes < S.total) return MXFP4_EWORKSPACE;
    if (!aligned(workspace, 256) || !aligned(saved, 256) || !aligned(x, 16) || !aligned(w, 16) || !aligned(y, 16))
        return MXFP4_EALIGN;
    uint8_t *ws = static_cast<uint8_t *>(workspace);
    uint8_t *sv = static_cast<uint8_t *>(saved);
    if (F.fprop == MXFP4_FMT_E2M1 && F.dgrad == MXFP4_FMT_E2M1 && F.wgrad == MXFP4_FMT_E2M1) {
        rc = quantize_operand_pair(cfg, x, M, K, ws + L.xq, ws + L.xs, sv + S.xtq, sv + S.xts, w, N, K, ws + L.wq,
                                   ws + L.ws, sv + S.wtq, sv + S.wts, hip_stream);
        if (rc != MXFP4_OK) return rc;
    } else {
        rc = quantize_operand(cfg, x, M, K, F.fprop, STREAM_X, ws + L.xq, ws + L.xs, F.wgrad, STREAM_XT, sv + S.xtq,
                              sv + S.xts, hip_stream);
        if (rc != MXFP4_OK) return rc;
        rc = quantize_operand(cfg, w, N, K, F.fprop, STREAM_W, ws + L.wq, ws + L.ws, F.dgrad, STREAM_WT, sv + S.wtq,
                              sv + S.wts, hip_stream);
        if (rc != MXFP4_OK) return rc;
    }
    return mxfp4_gemm_fmt(ws + L.xq, ws + L.xs, F.fprop, ws + L.wq, ws + L.ws, F.fprop, M, N, K, y, N, cfg->y_dtype, 0,
                          hip_stream);
}

int mxfp4_linear_bwd_saved(const void *dy, const void *saved, size_t saved_bytes, void *dx, void *dw, int64_t M,
                           int64_t N, int64_t K, const mxfp4_linear_cfg *cfg, void *workspace,
                           size_t workspace_bytes, void *hip_stream)
{
    int rc = check_cfg(cfg);
    if (rc != MXFP4_OK) return rc;
    if (M <= 0 || N <= 0 || K <= 0 || (M % 32) != 0 || (N % 32) != 0 || (K % 32) != 0) return MXFP4_ESHAPE;
    if (!dx && !dw) return MXFP4_OK;
    if (!dy || !saved || !workspace) return MXFP4_EINVAL;
    const StageFormats F = stage_formats(cfg);
    const BwdLayout L = bwd_layout(M, N, K, F);
    const SavedLayout S = saved_layout(M, N, K, F);
    if (workspace_bytes < L.total || saved_bytes < S.total) return MXFP4_EWORKSPACE;
    if (!aligned(workspace, 256) || !aligned(saved, 256) || !aligned(dy, 16) || (dx && !aligned(dx, 16)) ||
        (dw && !aligned(dw, 16)))
        return MXFP4_EALIGN;
    uint8_t *ws = static_cast<uint8_t *>(workspace);
    const uint8_t *sv = static_cast<const uint8_t *>(saved);
    rc = quantize_operand(cfg, dy, M, N, F.dgrad, STREAM_DY, dx ? ws + L.gq : nullptr, dx ? ws + L.gs : nullptr,
                          F.wgrad, STREAM_DYT, dw ? ws + L.gtq : nullptr, dw ? ws + L.gts : nullptr, hip_stream);
    if (rc != MXFP4_OK) return rc;
    const GemmArgs gd{ws + L.gq, ws + L.gs, sv + S.wtq, sv + S.wts, M, K, N, dx, K, cfg->dx_dtype == MXFP4_OUT_FP32, 0,
                      F.dgrad, F.dgrad};
    const GemmArgs gw{ws + L.gtq, ws + L.gts, sv + S.xtq, sv + S.xts, N, K, M, dw, K,
                      cfg->dw_dtype == MXFP4_OUT_FP32, cfg->dw_accumulate, F.wgrad, F.wgrad};
    if (dx && dw) return gemm_pair(gd, cfg->dx_dtype, gw, cfg->dw_dtype, hip_stream);
    if (dx)
        return mxfp4_gemm_fmt(gd.aq, gd.as, F.dgrad, gd.bq, gd.bs, F.dgrad, M, K, N, dx, K, cfg->dx_dtype, 0, hip_stream);
    return mxfp4_gemm_fmt(gw.aq, gw.as, F.wgrad, gw.bq, gw.bs, F.wgrad, N, K, M, dw, K, cfg->dw_dtype,
                          cfg->dw_accumulate, hip_stream);
}

}  // extern "C"
