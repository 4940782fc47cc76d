// Internal launch interface between the C ABI (api.hip) and the gfx950 kernels.
// Every launcher assumes its arguments were validated by the caller and returns the
// hipError_t of the launch.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mxfp4 {

struct QuantArgs {
    const uint16_t *x;  // bf16 [rows][ld]
    int64_t rows, cols, ld;
    int hadamard, rounding;
    uint64_t seed;
    uint8_t *q, *s;
    uint8_t *q_row = nullptr, *s_row = nullptr;  // launch_quantize_dual / _2d only: the row-wise outputs
    uint64_t seed_row = 0;                       // ... and the seed their stochastic rounding draws from
};

// A seed's low 48 bits (the base seed) fix the random-sign diagonal; its high 16 bits only select the stream of
// stochastic-rounding variates, so the two operands of a GEMM can share the diagonal and still round independently.
constexpr uint64_t SEED_BASE_MASK = 0xFFFFFFFFFFFFull;

// blocks along rows (1x32): q[rows][cols/2], s[rows][cols/32]
hipError_t launch_quantize_rows(const QuantArgs &a, hipStream_t st);
// blocks down columns (32x1): q[cols][rows/2], s[cols][rows/32]
// (b, if not null: a second tensor in the same launch, same hadamard, rounding and base seed)
hipError_t launch_quantize_cols(const QuantArgs &a, hipStream_t st, const QuantArgs *b = nullptr);
// both from one pass over x: q, s as launch_quantize_cols; q_row, s_row as launch_quantize_rows
// (b, if not null: a second tensor in the same launch, same hadamard, rounding and seed; the two grids together
// must stay below 2^31 workgroups)
hipError_t launch_quantize_dual(const QuantArgs &a, const QuantArgs *b, hipStream_t st);
// one scale per 32 x 32 region; the pair q, s (column-wise layout) or the pair q_row, s_row (row-wise layout)
// may be null
hipError_t launch_quantize_2d(const QuantArgs &a, const QuantArgs *b, hipStream_t st);

// MXFP8 (E4M3) output, round to nearest even: q[R][C] one byte per element, s[R][C/32]; cols_axis selects the
// column-wise (32x1, transposed output) layout
hipError_t launch_quantize_fp8(const QuantArgs &a, bool cols_axis, hipStream_t st);
// both MXFP8 layouts from one pass over x: q, s column-wise (q[cols][rows]); q_row, s_row row-wise (q_row[rows][cols])
hipError_t launch_quantize_fp8_dual(const QuantArgs &a, hipStream_t st);
// one pass over x for a tensor that feeds one MXFP4 and one MXFP8 GEMM: q_row, s_row = the row-wise MXFP4 output
// (rotation a.hadamard, rounding a.rounding under a.seed_row; the sign diagonal from a.seed), q, s = the column-wise
// MXFP8 output (unrotated, round to nearest)
hipError_t launch_quantize_mxfp4_rows_mxfp8_cols(const QuantArgs &a, hipStream_t st);

struct GemmArgs {
    const uint8_t *aq, *as, *bq, *bs;
    int64_t Ra, Rb, C;
    void *out;
    int64_t ld;
    int out_fp32, accumulate;
    int a_fmt = 0, b_fmt = 0;  // element format of each operand: 0 = E2M1 (q[R][C/2]), 1 = E4M3 (q[R][C])
};

// The kernels one GEMM is cut into: the tiled kernel on 256 x 256 or on 256 x 128 tiles for whole-tile blocks of the
// output (one launch may run whole rounds of 256 x 256 tiles and then the last round in 256 x 128 halves), the
// any-shape kernel for edge strips and everything else.  At most four parts.
enum GemmKind { GEMM_ANY = 0, GEMM_TILED_256 = 1, GEMM_TILED_128 = 2, GEMM_TILED_256_TAIL_128 = 3 };
struct GemmPart {
    int kind;
    int64_t r0, rows, c0, cols;  // block of the output: rows of A, rows of B
    int64_t main_tiles;          // GEMM_TILED_256_TAIL_128: tiles on 256 x 256 before the rest runs in halves; else 0
};
struct GemmPlan {
    int n;
    GemmPart part[4];
};
// host logic only (no device call); cus: compute units of the device the launch is planned for
GemmPlan plan_gemm(const GemmArgs &g, int cus);

hipError_t launch_gemm(const GemmArgs &g, hipStream_t st);
// two GEMMs that do not depend on each other (g0.accumulate must be 0); may share one launch
hipError_t launch_gemm_pair(const GemmArgs &g0, const GemmArgs &g1, hipStream_t st);

}  // namespace mxfp4
