/*
 * mxfp4.h -- C ABI of the MI355X (gfx950) MXFP4 linear-layer library.
 *
 * The library implements the hot path of MXFP4 pretraining: for each of the
 * three GEMMs of a transformer linear layer (App. C.1 Fprop Y = X W^T, App. C.2
 * Dgrad dX = dY W, App. C.3 Wgrad dW = dY^T X) both operands are optionally
 * rotated by a block Hadamard transform (App. A.2), quantised to MXFP4 along
 * the contraction axis (App. A.1, eq. (1)) and multiplied on the FP4 matrix
 * units with fp32 accumulation.
 *
 * Conventions common to every call
 *   - Every data pointer is a DEVICE pointer on the current HIP device unless
 *     stated otherwise.  The caller owns all buffers, including workspaces; the
 *     library never allocates, frees or keeps a pointer after a call returns.
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the default
 *     stream).  Calls only enqueue work on that stream and return; they never
 *     synchronise.  Outputs are valid once the stream has reached that point.
 *   - Return value: an mxfp4_status.  Argument errors are detected on the host
 *     before anything is launched, so a failed call has no effect.  No call
 *     throws or aborts.
 *   - bf16 tensors are row-major with a leading dimension in elements.
 *   - Quantised tensor layout ("canonical"): for an operand with R rows and
 *     contraction length C (C % 32 == 0)
 *         q: uint8 [R][C/2]   two E2M1 codes per byte; element c of a row is in
 *                             byte c/2, even c in the low nibble
 *         s: uint8 [R][C/32]  one E8M0 byte per 32 consecutive elements,
 *                             value 2^(byte-127); 0xFF marks a block that held
 *                             a NaN or an infinity (its codes are all 0)
 *     Every GEMM is then out[i][j] = sum_c A[i][c] * B[j][c].
 */
#ifndef MXFP4_H
#define MXFP4_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MXFP4_OK = 0,
    MXFP4_EINVAL = 1,     /* null pointer, unknown enum value, bad flag combination */
    MXFP4_ESHAPE = 2,     /* a dimension <= 0, contraction length not a multiple of 32, ld too small */
    MXFP4_EALIGN = 3,     /* pointer or leading dimension not aligned as documented */
    MXFP4_EWORKSPACE = 4, /* workspace smaller than mxfp4_linear_workspace_bytes() */
    MXFP4_EDEVICE = 5,    /* HIP reported an error at launch, or the device is not gfx950 */
    MXFP4_ENOTIMPL = 6
} mxfp4_status;

/* Which axis of the row-major input the 32-element blocks run along (App. D). */
typedef enum {
    MXFP4_AXIS_LAST = 0, /* 1x32 blocks along a row:     R = rows, C = cols                      */
    MXFP4_AXIS_FIRST = 1 /* 32x1 blocks down a column:   R = cols, C = rows; output is transposed */
} mxfp4_axis;

/* Rotation applied to every block before quantisation (App. A.2; Table 1 rows). */
typedef enum {
    MXFP4_HAD_NONE = 0,
    MXFP4_HAD_DET = 1,      /* deterministic H32/sqrt(32), Sylvester order                       */
    MXFP4_HAD_RANDSIGN = 2, /* H32/sqrt(32) after a seeded +-1 diagonal shared by all blocks     */
    MXFP4_HAD_DET16 = 3,    /* two independent H16/4 per block (the paper's H16 tiling)          */
    MXFP4_HAD_RANDSIGN16 = 4 /* the same +-1 diagonal (32 entries per block), then two H16/4:
                              * Table 1's randomised rotation runs at size 16               */
} mxfp4_hadamard;

/* FP4 cast of eq. (1). */
typedef enum {
    MXFP4_RNE = 0, /* nearest, ties to the even code, saturating at +-6                              */
    MXFP4_SR = 1   /* stochastic: counter hash of (seed, linear index of the element in q's layout) */
} mxfp4_round;

typedef enum { MXFP4_OUT_BF16 = 0, MXFP4_OUT_FP32 = 1 } mxfp4_out;

/* Scale granularity (App. D). */
typedef enum {
    MXFP4_GEOM_1D = 0, /* one scale per 32 elements along the contraction axis (1x32 / 32x1)   */
    MXFP4_GEOM_2D = 1  /* one scale per 32 x 32 region; needs M, N, K all multiples of 32      */
} mxfp4_geometry;

/* Element format of a quantised operand. */
typedef enum {
    MXFP4_FMT_E2M1 = 0, /* MXFP4: two 4-bit codes per byte, q[R][C/2]                           */
    MXFP4_FMT_E4M3 = 1  /* MXFP8: one OCP E4M3 byte per element, q[R][C]                        */
} mxfp4_format;

/* Recipe of one linear layer (one row of Table 1: stabiliser x rounding, all stages MXFP4). */
typedef struct {
    int32_t hadamard;      /* mxfp4_hadamard, used for both operands of every GEMM             */
    int32_t rounding;      /* mxfp4_round                                                       */
    uint64_t seed;         /* random-sign diagonal (low 48 bits) and stochastic-rounding counters: the six
                              quantised operands X, W, dY, W^T, dY^T, X^T of a layer round under the seeds
                              seed ^ (k << 48), k = 0..5 in that order, so that the two operands of every
                              GEMM draw independent variates while sharing the diagonal                  */
    int32_t y_dtype;       /* mxfp4_out for Y                                                   */
    int32_t dx_dtype;      /* mxfp4_out for dX                                                  */
    int32_t dw_dtype;      /* mxfp4_out for dW                                                  */
    int32_t dw_accumulate; /* 1: dW += (fp32 only; gradient accumulation), 0: dW =             */
    int32_t geometry;      /* mxfp4_geometry of every quantisation of the layer (App. D)        */
    int32_t fprop_format;  /* mxfp4_format of both operands of Fprop: the stage-wise recipe of Table 1  */
    int32_t dgrad_format;  /*   ("MXFP4 GEMMs (others FP8)") sets a stage to MXFP4_FMT_E4M3 to keep it  */
    int32_t wgrad_format;  /*   in 8 bits: MXFP8, no rotation, round to nearest, 1D blocks only         */
} mxfp4_linear_cfg;

/*
 * Rotate + quantise one bf16 matrix (App. A.1 eq. (1), App. A.2, App. D).
 *   x        bf16 [rows][ld], ld >= cols
 *   axis     MXFP4_AXIS_LAST : R = rows, C = cols, cols % 32 == 0;
 *                              x 16-byte aligned, ld % 8 == 0
 *            MXFP4_AXIS_FIRST: R = cols, C = rows, rows % 32 == 0, cols % 2 == 0;
 *                              x 4-byte aligned, ld % 2 == 0; q/s hold the quantised transpose
 *   q_out    uint8 [R][C/2], 16-byte aligned      s_out  uint8 [R][C/32]
 *   seed     used by the two random-sign modes and MXFP4_SR only.  Its low 48 bits (the base seed)
 *            determine the random-sign diagonal; all 64 bits key the stochastic-rounding
 *            counters.  Both operands of a GEMM must use the same base seed and mode for the
 *            rotation to cancel in the product, and should differ in the high 16 bits
 *            (MXFP4_SEED_STREAM) when rounding stochastically: the counters of A[i][c] and
 *            B[i][c] coincide, so under one stream both would round the same way and the
 *            diagonal of the product would be biased.
 * Per block: widen to fp32; optional sign flips; fp32 butterflies in the order
 * h = 1,2,4,8,16 then one multiply by fl32(2^-2.5) (H16: h = 1..8, multiply by 1/4);
 * scale byte = clamp(biased exponent of the block maximum - 2, 0, 254); codes = FP4 cast of
 * value * 2^-(byte-127).  Stochastic rounding draws u = (2*(r>>9)+1)/2^24 from the 32-bit
 * counter hash r of (seed, row_of_q * C + column_of_q) and rounds up when u < fraction.
 * rows == 0 or cols == 0 is a valid empty call.
 */
#define MXFP4_SEED_STREAM(base_seed, stream) \
    (((uint64_t)(base_seed) & 0xFFFFFFFFFFFFull) | ((uint64_t)((stream) & 0xFFFF) << 48))
int mxfp4_quantize(const void *x_bf16, int64_t rows, int64_t cols, int64_t ld_elems, int axis, int hadamard,
                   int rounding, uint64_t seed, void *q_out, void *s_out, void *hip_stream);

/*
 * Both quantisations of one bf16 matrix from a single pass over it: the row-wise one a Fprop
 * or Dgrad operand needs and the column-wise one the same tensor needs as a Dgrad or Wgrad
 * operand (App. C.1-C.3; the transposed access is the costly layout of App. D).
 *   x        bf16 [rows][ld], 16-byte aligned, ld % 8 == 0, rows % 32 == 0, cols % 32 == 0
 *   q_last   uint8 [rows][cols/2], s_last uint8 [rows][cols/32]: exactly what mxfp4_quantize
 *            writes for MXFP4_AXIS_LAST with the same hadamard, rounding and seed
 *   q_first  uint8 [cols][rows/2], s_first uint8 [cols][rows/32]: the same for MXFP4_AXIS_FIRST
 *   q_last, q_first 16-byte aligned.  rows == 0 or cols == 0 is a valid empty call.
 *   Both outputs round under the one seed given (they are operands of different GEMMs).
 */
int mxfp4_quantize_dual(const void *x_bf16, int64_t rows, int64_t cols, int64_t ld_elems, int hadamard,
                        int rounding, uint64_t seed, void *q_last, void *s_last, void *q_first, void *s_first,
                        void *hip_stream);

/*
 * 2D block quantisation (App. D, "32 x 32"): one E8M0 scale per 32 x 32 region instead of one per
 * 32-element block.  The scale follows the same rule, applied to the largest magnitude of the
 * region after the rotation (which still runs along each output's contraction axis); it is
 * stored once per row of the region, so both outputs keep the layouts of mxfp4_quantize and feed
 * mxfp4_gemm unchanged.  Without rotation the two outputs hold the same codes and scales,
 * transposed: one quantisation of W serves Fprop and Dgrad.
 *   x        bf16 [rows][ld], 16-byte aligned, ld % 8 == 0, rows % 32 == 0, cols % 32 == 0
 *   q_last / s_last   row-wise output [rows][cols/2], [rows][cols/32], or both NULL
 *   q_first / s_first column-wise output [cols][rows/2], [cols][rows/32], or both NULL
 *   (at least one pair; q pointers 16-byte aligned).  A NaN or an infinity marks its whole
 *   region (byte 0xFF, codes 0).  rows == 0 or cols == 0 is a valid empty call.
 */
int mxfp4_quantize_2d(const void *x_bf16, int64_t rows, int64_t cols, int64_t ld_elems, int hadamard,
                      int rounding, uint64_t seed, void *q_last, void *s_last, void *q_first, void *s_first,
                      void *hip_stream);

/*
 * MXFP8 quantiser for the stages of the stage-wise recipe that stay in 8 bits (Table 1: "MXFP4 GEMMs
 * (others FP8)").  As mxfp4_quantize with OCP E4M3 elements (bias 7, largest finite 448, no infinities):
 * scale byte = clamp(biased exponent of the block maximum - 8, 0, 254); element = value * 2^-(byte-127)
 * rounded to nearest even, saturating at +-448; round-to-nearest only.
 *   q8_out uint8 [R][C], 16-byte aligned     s_out uint8 [R][C/32]
 * axis, hadamard, seed, shapes and alignment rules as for mxfp4_quantize.
 */
int mxfp4_quantize_fp8(const void *x_bf16, int64_t rows, int64_t cols, int64_t ld_elems, int axis, int hadamard,
                       uint64_t seed, void *q8_out, void *s_out, void *hip_stream);

/*
 * Both MXFP8 quantisations of one tensor from one pass over it (what mxfp4_quantize_dual is for MXFP4): the
 * row-wise output q8_last [rows][cols], s_last [rows][cols/32] and the column-wise output q8_first [cols][rows],
 * s_first [cols][rows/32], byte for byte those of two mxfp4_quantize_fp8 calls.
 *   x bf16 [rows][ld], 16-byte aligned, ld % 8 == 0; rows % 32 == 0, cols % 32 == 0; q pointers 16-byte aligned.
 * rows == 0 or cols == 0 is a valid empty call.
 */
int mxfp4_quantize_fp8_dual(const void *x_bf16, int64_t rows, int64_t cols, int64_t ld_elems, int hadamard,
                            uint64_t seed, void *q8_last, void *s_last, void *q8_first, void *s_first,
                            void *hip_stream);

/*
 * mxfp4_gemm with each operand in its own element format (mxfp4_format): the same block-scaled matrix
 * instruction takes E2M1 and E4M3 operands in any combination.
 */
int mxfp4_gemm_fmt(const void *a_q, const void *a_s, int a_format, const void *b_q, const void *b_s, int b_format,
                   int64_t R_a, int64_t R_b, int64_t C, void *out, int64_t ld_out, int out_dtype, int accumulate,
                   void *hip_stream);

/*
 * Block-scaled FP4 GEMM on quantised operands (the MXFP4 GEMM that replaces the FP8 GEMM of
 * the linear layers, Sec. 1 and App. A.2):
 *     out[i][j] (+)= sum_c A[i][c] * B[j][c],  A = a_q/a_s [R_a][C],  B = b_q/b_s [R_b][C]
 * products exact, fp32 accumulation (partial sums of 64 or 128 consecutive elements are formed
 * exactly enough to meet 1e-5 * sum|a||b| against the exact sum and are added in fp32, round to
 * nearest even, with gradual underflow: results below 2^-126 come out as fp32 subnormal numbers,
 * not flushed; results beyond fp32's range come out as infinities).  C % 32 == 0; R_a, R_b >= 0
 * (0 = empty call).
 *   out        [R_a][ld_out] bf16 or fp32 (out_dtype), ld_out >= R_b
 *   accumulate 1: out += result (MXFP4_OUT_FP32 only), 0: out = result
 * All operand pointers 16-byte aligned.  A scale byte of 0xFF (the NaN of the scale format) makes
 * every output of that operand row NaN, whatever the codes under it.
 */
int mxfp4_gemm(const void *a_q, const void *a_s, const void *b_q, const void *b_s, int64_t R_a, int64_t R_b,
               int64_t C, void *out, int64_t ld_out, int out_dtype, int accumulate, void *hip_stream);

/*
 * Two independent MXFP4 GEMMs enqueued together: the Dgrad and the Wgrad product of one layer share no
 * operand buffer and no output (App. C.2, C.3; Fig. 3), so they can run side by side.  Each problem is
 * described as in mxfp4_gemm (E2M1 operands); problem 0 never accumulates, problem 1 may (fp32 output).
 * When both shapes fit the tiled kernel and together fill the chip, one launch runs them on disjoint sets
 * of compute units split in proportion to their work; otherwise the call is mxfp4_gemm on problem 0
 * followed by mxfp4_gemm on problem 1.  Results are bit for bit those of the two separate calls.
 * The two outputs must not overlap each other or any operand.  Arguments are checked for both problems
 * before anything is enqueued.
 */
int mxfp4_gemm_pair(const void *a0_q, const void *a0_s, const void *b0_q, const void *b0_s, int64_t R_a0,
                    int64_t R_b0, int64_t C0, void *out0, int64_t ld_out0, int out_dtype0,
                    const void *a1_q, const void *a1_s, const void *b1_q, const void *b1_s, int64_t R_a1,
                    int64_t R_b1, int64_t C1, void *out1, int64_t ld_out1, int out_dtype1, int accumulate1,
                    void *hip_stream);

/*
 * Which kernels mxfp4_gemm_fmt cuts a product of this shape into on a device with `compute_units` compute
 * units (256 on MI355X), for operands and an output aligned as those calls demand: the tiled kernel of the
 * block-scaled FP4 GEMM (Sec. 2.1) on 256 x 256 tiles or, where those would leave compute units idle, on
 * 256 x 128 tiles, and a slower any-shape kernel for edge strips and for contraction lengths below 1024 or
 * not in whole 256s (MXFP8: 128s).  Host-only: touches no device.
 *   parts[6 * i ..] = kind, first row, rows, first column, columns of block i of the output, main tiles;
 *   kind: 0 any-shape, 1 tiled 256 x 256, 2 tiled 256 x 128, 3 one launch that runs `main tiles` tiles (whole
 *   rounds over the compute units) on 256 x 256 and the rest of the block, a last round at most half full, as
 *   twice as many 256 x 128 tiles; main tiles is 0 for the other kinds.
 *   *n_parts <= 4 receives the number of blocks (0 for an empty product).
 * Returns MXFP4_OK, MXFP4_EINVAL or MXFP4_ESHAPE as the GEMM call would.
 */
int mxfp4_gemm_plan(int64_t R_a, int64_t R_b, int64_t C, int a_format, int b_format, int64_t ld_out,
                    int compute_units, int *n_parts, int64_t parts[24]);

/*
 * Fprop of one linear layer (App. C.1): Y[M][N] = Q(X H) Q(W H)^T, contraction over K.
 *   x bf16 [M][K], w bf16 [N][K] (both dense: ld = K), y [M][N] dense, dtype cfg->y_dtype
 *   workspace: device scratch of at least mxfp4_linear_workspace_bytes(M,N,K,cfg,0) bytes,
 *   256-byte aligned.  On return (after the stream completes) it holds the canonical
 *   q/s of X then W at the offsets reported by mxfp4_linear_workspace_layout.
 * M, N, K >= 1 and K % 32 == 0 (else MXFP4_ESHAPE).
 */
int mxfp4_linear_fwd(const void *x, const void *w, void *y, int64_t M, int64_t N, int64_t K,
                     const mxfp4_linear_cfg *cfg, void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * mxfp4_linear_fwd for callers that cannot allocate device memory or hand over a workspace (code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the quantised
 * operands are staged in a device array of MXFP4_STATIC_SCRATCH_BYTES that is part of the library's
 * code object (every GPU the library runs on holds it until the process ends) instead of a caller's
 * workspace.  The call allocates and frees nothing.  Same arguments, checks, kernels and results
 * (bit for bit) as mxfp4_linear_fwd.
 *   Limit: mxfp4_linear_workspace_bytes(M,N,K,cfg,0) <= MXFP4_STATIC_SCRATCH_BYTES, else
 *   MXFP4_EWORKSPACE (32 MiB holds the 8B model's fused QKV forward, M=8192 K=4096 N=6144).
 *   The first call on a device looks the array's address up (hipGetSymbolAddress); make that call
 *   outside any graph capture.  All calls on one GPU share the one array: two calls that overlap
 *   in time on different streams of the same GPU race, and the array keeps the last call's operands
 *   (nothing in it needs clearing: every byte a GEMM reads is written by that call's quantisers first).
 */
#define MXFP4_STATIC_SCRATCH_BYTES (32u << 20)
int mxfp4_linear_fwd_static(const void *x, const void *w, void *y, int64_t M, int64_t N, int64_t K,
                            const mxfp4_linear_cfg *cfg, void *hip_stream);

/*
 * Backward of one linear layer: Dgrad (App. C.2) dX[M][K] = Q(dY H) Q(W^T H)^T, contraction
 * over N, and Wgrad (App. C.3) dW[N][K] = Q(dY^T H) Q(X^T H)^T, contraction over tokens M.
 *   dy bf16 [M][N], x bf16 [M][K], w bf16 [N][K], all dense.
 *   dx or dw may be NULL to skip that GEMM (x may be NULL if dw is, w if dx is).
 *   M, N, K >= 1; N % 8 == 0 and K % 8 == 0 (16-byte rows); Dgrad needs N % 32 == 0, Wgrad
 *   needs M % 32 == 0.
 *   workspace as for the forward call, sized with bwd = 1.
 */
int mxfp4_linear_bwd(const void *dy, const void *x, const void *w, void *dx, void *dw, int64_t M, int64_t N,
                     int64_t K, const mxfp4_linear_cfg *cfg, void *workspace, size_t workspace_bytes,
                     void *hip_stream);

/*
 * Training pair with each tensor read once (Fig. 3: the same X and W feed Fprop and the two
 * backward GEMMs).  mxfp4_linear_fwd_save computes Y as mxfp4_linear_fwd does and, from the
 * same pass over X and W, also stores their column-wise quantisations W^T (for Dgrad) and
 * X^T (for Wgrad) in `saved`; mxfp4_linear_bwd_saved then needs neither x nor w: it
 * quantises dY both ways in one pass and runs Dgrad and Wgrad against `saved`.  Outputs are
 * bit-identical to mxfp4_linear_fwd / mxfp4_linear_bwd with the same cfg.
 *   saved: device buffer of at least mxfp4_linear_saved_bytes(M,N,K,cfg) bytes, 256-byte aligned,
 *          owned by the caller, kept untouched between the two calls; offsets of q and s of
 *          W^T (rows K, C=N) and X^T (rows K, C=M) from mxfp4_linear_saved_layout.
 *   M % 32 == 0, N % 32 == 0, K % 32 == 0, all >= 1 (else MXFP4_ESHAPE).
 *   workspace: as for mxfp4_linear_fwd (bwd = 0) and mxfp4_linear_bwd (bwd = 1).
 *   dx or dw may be NULL to skip that GEMM.
 */
int mxfp4_linear_fwd_save(const void *x, const void *w, void *y, int64_t M, int64_t N, int64_t K,
                          const mxfp4_linear_cfg *cfg, void *workspace, size_t workspace_bytes, void *saved,
                          size_t saved_bytes, void *hip_stream);
int mxfp4_linear_bwd_saved(const void *dy, const void *saved, size_t saved_bytes, void *dx, void *dw, int64_t M,
                           int64_t N, int64_t K, const mxfp4_linear_cfg *cfg, void *workspace,
                           size_t workspace_bytes, void *hip_stream);
size_t mxfp4_linear_saved_bytes(int64_t M, int64_t N, int64_t K, const mxfp4_linear_cfg *cfg);
/* offsets[4]: q, s of W^T then q, s of X^T inside `saved` (cfg: the stage formats; NULL = all MXFP4).  Host-only. */
int mxfp4_linear_saved_layout(int64_t M, int64_t N, int64_t K, const mxfp4_linear_cfg *cfg, size_t offsets[4]);

/* Bytes of workspace the fused calls need (bwd = 0: forward, 1: backward).  Host-only. */
size_t mxfp4_linear_workspace_bytes(int64_t M, int64_t N, int64_t K, const mxfp4_linear_cfg *cfg, int bwd);

/*
 * Byte offsets, inside the workspace, of the canonical quantised operands the fused calls
 * leave behind (for byte-parity tests).  offsets[8] receives, in order, q and s of:
 *   bwd = 0: X (rows M, C=K), W (rows N, C=K); entries 4..7 are 0
 *   bwd = 1: dY (rows M, C=N), W^T (rows K, C=N), dY^T (rows N, C=M), X^T (rows K, C=M)
 * The code array of an operand of an MXFP8 stage holds one byte per element (cfg: the stage formats;
 * NULL = all MXFP4).  Host-only.  Returns MXFP4_OK or MXFP4_EINVAL.
 */
int mxfp4_linear_workspace_layout(int64_t M, int64_t N, int64_t K, const mxfp4_linear_cfg *cfg, int bwd,
                                  size_t offsets[8]);

/* Human-readable name of a status code; pointer to static storage, never NULL.  Host-only. */
const char *mxfp4_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* MXFP4_H */
