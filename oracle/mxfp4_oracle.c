/*
 * mxfp4_oracle.c -- plain CPU reference for the MXFP4 linear-layer hot path.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may call this file;
 * it exists so that the GPU kernels can be compared with something that can be
 * checked against the paper by eye.  It shares no code with the GPU path.
 *
 * What it follows
 *   - MXFP4 micro-scaled block quantisation: App. A.1, eq. (1), with the OCP MX
 *     rules the paper cites there for the shared exponent and the FP4 cast
 *     (E2M1 elements, one E8M0 power-of-two scale per 32 elements).
 *   - Hadamard rotation before quantisation: App. A.2 and App. C (H orthogonal
 *     with +-1 entries; H H^T = I after the 1/sqrt(32) normalisation).
 *   - Which axis is rotated/quantised in each stage: App. C.1 (Fprop, along K),
 *     App. C.2 (Dgrad, along N), App. C.3 (Wgrad, along the token axis M).
 *   - Row-wise 1x32 and column-wise 32x1 block geometry: App. D.
 *   - Stochastic rounding and random-sign Hadamard: named in Sec. 3.1 (H2) and
 *     Table 1 only; the definitions used here are this build's readings.
 *
 * Arithmetic
 *   The quantiser is an encoding, so it is written as the algorithm, step by
 *   step, in the precision the method uses (fp32 butterflies, then an exact
 *   power-of-two scaling evaluated in double).  The GEMM has a plain
 *   definition (a sum of products of decoded values), written out in double.
 *
 * Parity pins: every function here is pinned by tests/test_oracle_*.py against
 * closed forms, exhaustive enumeration or brute force.  The paper prints no
 * worked numeric example, so parity against the authors' own kernels is
 * unpinned (their tie rule, scale rule and Hadamard ordering are not stated).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define MX_BLOCK 32

enum { ORC_AXIS_LAST = 0, ORC_AXIS_FIRST = 1 };
enum { ORC_HAD_NONE = 0, ORC_HAD_DET = 1, ORC_HAD_RANDSIGN = 2, ORC_HAD_DET16 = 3, ORC_HAD_RANDSIGN16 = 4 };
enum { ORC_RNE = 0, ORC_SR = 1 };
enum { ORC_FMT_E2M1 = 0, ORC_FMT_E4M3 = 1 };

/* ------------------------------------------------------------------------- */
/* Counter-based random numbers (no state: a pure function of seed and index) */
/* ------------------------------------------------------------------------- */

static uint32_t mix32(uint32_t x)
{
    x ^= x >> 16;
    x *= 0x9E3779B9u;
    x ^= x >> 15;
    x *= 0xBB67AE85u;
    x ^= x >> 16;
    return x;
}

/* 32 random bits for (seed, idx).  Used by stochastic rounding (idx = linear
 * index of the element in the quantised output) and by the random-sign
 * diagonal (idx = all ones). */
uint32_t orc_rand32(uint64_t seed, uint64_t idx)
{
    uint32_t seed_lo = (uint32_t)seed, seed_hi = (uint32_t)(seed >> 32);
    uint32_t idx_lo = (uint32_t)idx, idx_hi = (uint32_t)(idx >> 32);
    uint32_t a = mix32(idx_lo + seed_lo * 0x9E3779B9u);
    uint32_t b = mix32(seed_hi ^ 0x6A09E667u);
    return mix32(a ^ idx_hi ^ b);
}

/* rand32 for n consecutive indices idx0, idx0+1, ... */
void orc_rand32_array(uint64_t seed, uint64_t idx0, int64_t n, uint32_t *out)
{
    for (int64_t k = 0; k < n; ++k) out[k] = orc_rand32(seed, idx0 + (uint64_t)k);
}

/* A 64-bit seed has two parts.  The low 48 bits are the base seed: the random-sign
 * diagonal depends on them alone, so that both operands of a GEMM, which must share
 * the diagonal for the rotation to cancel (App. C), can still differ in the high 16
 * bits, the stream number.  Stochastic rounding uses all 64 bits: operands rounded
 * under different streams draw independent variates.  (With one stream for both
 * operands of out[i][j] = sum_c A[i][c] B[j][c] the elements A[i][c] and B[i][c]
 * would share their variate, and the product of two roundings that move together is
 * biased: unbiasedness is the reason stochastic rounding is tried at all, Sec. 3.1.) */
#define ORC_SEED_BASE_MASK 0xFFFFFFFFFFFFull

uint64_t orc_seed_with_stream(uint64_t seed, unsigned stream)
{
    return seed ^ ((uint64_t)(stream & 0xFFFFu) << 48);
}

/* The +-1 diagonal of the random-sign Hadamard: bit i set means d_i = -1.
 * One mask per call, the same for every block and for both GEMM operands. */
uint32_t orc_sign_mask(uint64_t seed)
{
    return orc_rand32(seed & ORC_SEED_BASE_MASK, 0xFFFFFFFFFFFFFFFFull);
}

/* ------------------------------------------------------------------------- */
/* Number formats                                                            */
/* ------------------------------------------------------------------------- */

float orc_bf16_to_f32(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

static uint32_t f32_bits(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    return u;
}

/* E2M1: 1 sign, 2 exponent (bias 1), 1 mantissa bit.  Magnitudes by code 0..7. */
static const double E2M1_MAG[8] = {0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0};

double orc_e2m1_decode(unsigned code)
{
    double m = E2M1_MAG[code & 7u];
    return (code & 8u) ? -m : m;
}

/* Q_FP4 of eq. (1), round-to-nearest: the representable magnitude closest to
 * |t|; of two equally close ones, the one with an even code (mantissa bit 0);
 * beyond 6, 6.  The sign bit is that of t, also for results of magnitude 0. */
unsigned orc_e2m1_encode_rne(double t)
{
    double a = fabs(t);
    unsigned best = 0;
    double best_d = INFINITY;
    if (a > 6.0) a = 6.0; /* saturate first: far above 6 the distances below would all round alike */
    for (unsigned c = 0; c < 8; ++c) {
        double d = fabs(a - E2M1_MAG[c]);
        if (d < best_d || (d == best_d && (c & 1u) == 0)) {
            best_d = d;
            best = c;
        }
    }
    return (signbit(t) ? 8u : 0u) | best;
}

/* Stochastic rounding of t to E2M1 with the 32 random bits r.
 * |t| is clipped to 6; lo <= |t| <= hi are the neighbouring representable
 * magnitudes; the result is hi with probability (|t|-lo)/(hi-lo).  The uniform
 * variate is u = (2*(r>>9)+1) * 2^-24, an odd multiple of 2^-24 strictly
 * inside (0,1), so an exactly representable |t| never moves. */
unsigned orc_e2m1_encode_sr(double t, uint32_t r)
{
    double a = fabs(t);
    if (a > 6.0) a = 6.0;
    double delta = (a < 2.0) ? 0.5 : (a < 4.0) ? 1.0 : 2.0;
    double q = a / delta;
    double fl = floor(q);
    double f = q - fl;
    double u = (double)(2u * (r >> 9) + 1u) * ldexp(1.0, -24);
    double mag = (fl + ((u < f) ? 1.0 : 0.0)) * delta;
    unsigned c;
    for (c = 0; c < 8; ++c)
        if (E2M1_MAG[c] == mag) break;
    if (c == 8) abort(); /* cannot happen: mag is always on the grid */
    return (signbit(t) ? 8u : 0u) | c;
}

/* E4M3 (OCP 8-bit floating point, the MXFP8 element of the FP8 stages): 1 sign, 4
 * exponent bits (bias 7), 3 mantissa bits; subnormals at exponent field 0; no
 * infinities; the all-ones magnitude (0x7F) is NaN; largest finite 448. */
double orc_e4m3_decode(unsigned code)
{
    unsigned e = (code >> 3) & 15u, m = code & 7u;
    double mag;
    if (e == 15u && m == 7u) return NAN;
    mag = (e == 0u) ? ldexp((double)m, -9) : ldexp(1.0 + (double)m / 8.0, (int)e - 7);
    return (code & 0x80u) ? -mag : mag;
}

/* Round-to-nearest, ties to the even mantissa, saturating at 448; never NaN.
 * The sign bit is that of t, also for results of magnitude 0. */
unsigned orc_e4m3_encode_rne(double t)
{
    double a = fabs(t);
    unsigned best = 0;
    double best_d = INFINITY;
    if (a > 448.0) a = 448.0;
    for (unsigned c = 0; c < 127u; ++c) { /* 0x7F is NaN */
        double d = fabs(a - orc_e4m3_decode(c));
        if (d < best_d || (d == best_d && (c & 1u) == 0)) {
            best_d = d;
            best = c;
        }
    }
    return (signbit(t) ? 0x80u : 0u) | best;
}

/* E8M0 byte of an MXFP8 (E4M3) block: as orc_e8m0_from_amax_bits with the
 * largest E4M3 exponent (8) in place of E2M1's (2). */
unsigned orc_e8m0_from_amax_bits_fp8(uint32_t amax_bits)
{
    int e_b = (int)((amax_bits >> 23) & 0xFFu);
    if (e_b == 255) return 0xFFu;
    int byte = e_b - 8;
    if (byte < 0) byte = 0;
    if (byte > 254) byte = 254;
    return (unsigned)byte;
}

/* E8M0 byte for a block whose largest magnitude has the fp32 bit pattern
 * amax_bits (sign cleared).  OCP MX: shared exponent = floor(log2 amax) minus
 * the largest E2M1 exponent (2); the byte is that exponent plus 127, clamped
 * to [0,254].  0xFF (the E8M0 NaN) marks a block with a NaN or an infinity. */
unsigned orc_e8m0_from_amax_bits(uint32_t amax_bits)
{
    int e_b = (int)((amax_bits >> 23) & 0xFFu);
    if (e_b == 255) return 0xFFu;
    int byte = e_b - 2;
    if (byte < 0) byte = 0;
    if (byte > 254) byte = 254;
    return (unsigned)byte;
}

/* ------------------------------------------------------------------------- */
/* Walsh-Hadamard transforms in fp32                                          */
/* ------------------------------------------------------------------------- */

/* Unnormalised n-point transform (n = 16 or 32), Sylvester order
 * H[i][j] = (-1)^popcount(i&j).  Butterfly stages h = 1,2,4,...; every add and
 * subtract is one fp32 operation rounded to nearest even. */
void orc_wht(float *v, int n)
{
    for (int h = 1; h < n; h <<= 1)
        for (int i = 0; i < n; ++i)
            if ((i & h) == 0) {
                volatile float s = v[i] + v[i + h];
                volatile float d = v[i] - v[i + h];
                v[i] = s;
                v[i + h] = d;
            }
}

/* ------------------------------------------------------------------------- */
/* The block quantiser                                                        */
/* ------------------------------------------------------------------------- */

/* Optional sign flips and rotation of one block v[0..31] (App. A.2), in place. */
static void rotate_block(float *v, int had, uint32_t sign_mask)
{
    /* randomised rotation: the block's +-1 diagonal first (entry i of the 32 for element i of the block,
     * also when two 16-point rotations follow: Table 1 runs the randomised rotation at size 16) */
    if (had == ORC_HAD_RANDSIGN || had == ORC_HAD_RANDSIGN16)
        for (int i = 0; i < MX_BLOCK; ++i)
            if ((sign_mask >> i) & 1u) v[i] = -v[i];

    if (had == ORC_HAD_DET || had == ORC_HAD_RANDSIGN) {
        /* H32 / sqrt(32): 2^-2.5 rounded once to fp32 */
        const volatile float c = 0x1.6a09e6p-3f; /* bits 0x3E3504F3 */
        orc_wht(v, 32);
        for (int i = 0; i < MX_BLOCK; ++i) {
            volatile float p = v[i] * c;
            v[i] = p;
        }
    } else if (had == ORC_HAD_DET16 || had == ORC_HAD_RANDSIGN16) {
        /* two independent H16 / 4 per block */
        orc_wht(v, 16);
        orc_wht(v + 16, 16);
        for (int i = 0; i < MX_BLOCK; ++i) {
            volatile float p = v[i] * 0.25f;
            v[i] = p;
        }
    }
}

/* Largest magnitude of n values as an fp32 bit pattern (NaN and infinity
 * compare above every finite value). */
static uint32_t amax_bits_of(const float *v, int n)
{
    uint32_t amax_bits = 0;
    for (int i = 0; i < n; ++i) {
        uint32_t b = f32_bits(v[i]) & 0x7FFFFFFFu;
        if (b > amax_bits) amax_bits = b;
    }
    return amax_bits;
}

/* FP4 codes of one rotated block under the shared scale byte sb (eq. (1)). */
static void encode_block(const float *v, unsigned sb, int rnd, uint64_t seed, uint64_t idx0, uint8_t *codes)
{
    if (sb == 0xFFu) {
        memset(codes, 0, MX_BLOCK);
        return;
    }
    int E = (int)sb - 127;
    for (int i = 0; i < MX_BLOCK; ++i) {
        double t = ldexp((double)v[i], -E); /* exact */
        codes[i] = (uint8_t)((rnd == ORC_SR) ? orc_e2m1_encode_sr(t, orc_rand32(seed, idx0 + (uint64_t)i))
                                             : orc_e2m1_encode_rne(t));
    }
}

/* v[0..31]: the block, widened to fp32, in order along the contraction axis.
 * idx0: linear index of element 0 of the block in the quantised output. */
static void quantize_block(float *v, int had, int rnd, uint64_t seed, uint32_t sign_mask,
                           uint64_t idx0, uint8_t *codes, uint8_t *scale_byte)
{
    rotate_block(v, had, sign_mask);
    unsigned sb = orc_e8m0_from_amax_bits(amax_bits_of(v, MX_BLOCK));
    *scale_byte = (uint8_t)sb;
    encode_block(v, sb, rnd, seed, idx0, codes);
}

/* Quantise a row-major bf16 matrix x[rows][ld] (cols used per row).
 * AXIS_LAST : blocks run along a row.    R = rows, C = cols.
 * AXIS_FIRST: blocks run down a column.  R = cols, C = rows; the output is the
 *             quantised transpose.
 * Output: q[R][C/2] (element c of a row in byte c/2; even c in the low nibble)
 * and s[R][C/32].  Returns 0, or 1 if C is not a multiple of 32. */
int orc_quantize(const uint16_t *x, int64_t rows, int64_t cols, int64_t ld, int axis, int had, int rnd,
                 uint64_t seed, uint8_t *q, uint8_t *s)
{
    int64_t R = (axis == ORC_AXIS_LAST) ? rows : cols;
    int64_t C = (axis == ORC_AXIS_LAST) ? cols : rows;
    if (C % MX_BLOCK != 0) return 1;
    uint32_t sign_mask = orc_sign_mask(seed);
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < R; ++r) {
        for (int64_t b = 0; b < C / MX_BLOCK; ++b) {
            float v[MX_BLOCK];
            uint8_t codes[MX_BLOCK];
            for (int i = 0; i < MX_BLOCK; ++i) {
                int64_t c = b * MX_BLOCK + i;
                uint16_t h = (axis == ORC_AXIS_LAST) ? x[r * ld + c] : x[c * ld + r];
                v[i] = orc_bf16_to_f32(h);
            }
            quantize_block(v, had, rnd, seed, sign_mask, (uint64_t)(r * C + b * MX_BLOCK), codes,
                           &s[r * (C / MX_BLOCK) + b]);
            for (int i = 0; i < MX_BLOCK; i += 2)
                q[r * (C / 2) + (b * MX_BLOCK + i) / 2] = (uint8_t)(codes[i] | (codes[i + 1] << 4));
        }
    }
    return 0;
}

/* 2D block quantisation (App. D, "32 x 32"): as orc_quantize, but one E8M0
 * scale is shared by a whole 32 x 32 region = 32 consecutive output rows of
 * one 32-element block column.  The scale follows the same rule as in 1D,
 * applied to the largest magnitude of the region (after the rotation, which
 * still runs along the contraction axis of each block); it is stored 32
 * times, once per row, so the output has the 1D layout q[R][C/2], s[R][C/32]
 * and feeds the same GEMM.  A NaN or an infinity anywhere in the region marks
 * all 32 blocks (byte 0xFF, codes 0).  Returns 0, or 1 if R or C is not a
 * multiple of 32. */
int orc_quantize_2d(const uint16_t *x, int64_t rows, int64_t cols, int64_t ld, int axis, int had, int rnd,
                    uint64_t seed, uint8_t *q, uint8_t *s)
{
    int64_t R = (axis == ORC_AXIS_LAST) ? rows : cols;
    int64_t C = (axis == ORC_AXIS_LAST) ? cols : rows;
    if (C % MX_BLOCK != 0 || R % MX_BLOCK != 0) return 1;
    uint32_t sign_mask = orc_sign_mask(seed);
#pragma omp parallel for schedule(static)
    for (int64_t rt = 0; rt < R / MX_BLOCK; ++rt) {
        for (int64_t b = 0; b < C / MX_BLOCK; ++b) {
            float v[MX_BLOCK][MX_BLOCK];
            uint8_t codes[MX_BLOCK];
            for (int rr = 0; rr < MX_BLOCK; ++rr) {
                int64_t r = rt * MX_BLOCK + rr;
                for (int i = 0; i < MX_BLOCK; ++i) {
                    int64_t c = b * MX_BLOCK + i;
                    uint16_t h = (axis == ORC_AXIS_LAST) ? x[r * ld + c] : x[c * ld + r];
                    v[rr][i] = orc_bf16_to_f32(h);
                }
                rotate_block(v[rr], had, sign_mask);
            }
            unsigned sb = orc_e8m0_from_amax_bits(amax_bits_of(&v[0][0], MX_BLOCK * MX_BLOCK));
            for (int rr = 0; rr < MX_BLOCK; ++rr) {
                int64_t r = rt * MX_BLOCK + rr;
                s[r * (C / MX_BLOCK) + b] = (uint8_t)sb;
                encode_block(v[rr], sb, rnd, seed, (uint64_t)(r * C + b * MX_BLOCK), codes);
                for (int i = 0; i < MX_BLOCK; i += 2)
                    q[r * (C / 2) + (b * MX_BLOCK + i) / 2] = (uint8_t)(codes[i] | (codes[i + 1] << 4));
            }
        }
    }
    return 0;
}

/* MXFP8 quantiser for the stages that stay in 8 bits (Table 1, "others FP8"):
 * as orc_quantize with E4M3 elements, one byte each: q8[R][C], s[R][C/32];
 * round-to-nearest-even only.  Returns 0, or 1 if C is not a multiple of 32. */
int orc_quantize_fp8(const uint16_t *x, int64_t rows, int64_t cols, int64_t ld, int axis, int had, uint64_t seed,
                     uint8_t *q8, uint8_t *s)
{
    int64_t R = (axis == ORC_AXIS_LAST) ? rows : cols;
    int64_t C = (axis == ORC_AXIS_LAST) ? cols : rows;
    if (C % MX_BLOCK != 0) return 1;
    uint32_t sign_mask = orc_sign_mask(seed);
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < R; ++r) {
        for (int64_t b = 0; b < C / MX_BLOCK; ++b) {
            float v[MX_BLOCK];
            for (int i = 0; i < MX_BLOCK; ++i) {
                int64_t c = b * MX_BLOCK + i;
                uint16_t h = (axis == ORC_AXIS_LAST) ? x[r * ld + c] : x[c * ld + r];
                v[i] = orc_bf16_to_f32(h);
            }
            rotate_block(v, had, sign_mask);
            unsigned sb = orc_e8m0_from_amax_bits_fp8(amax_bits_of(v, MX_BLOCK));
            s[r * (C / MX_BLOCK) + b] = (uint8_t)sb;
            for (int i = 0; i < MX_BLOCK; ++i) {
                uint8_t code = 0;
                if (sb != 0xFFu) code = (uint8_t)orc_e4m3_encode_rne(ldexp((double)v[i], 127 - (int)sb));
                q8[r * C + b * MX_BLOCK + i] = code;
            }
        }
    }
    return 0;
}

/* Reconstructed values x_MX of eq. (1): code value times 2^(scale byte - 127).
 * A block whose scale byte is 0xFF decodes to NaN. */
void orc_dequantize(const uint8_t *q, const uint8_t *s, int64_t R, int64_t C, double *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < R; ++r)
        for (int64_t c = 0; c < C; ++c) {
            unsigned byte = q[r * (C / 2) + c / 2];
            unsigned code = (c & 1) ? (byte >> 4) : (byte & 15u);
            unsigned sb = s[r * (C / MX_BLOCK) + c / MX_BLOCK];
            out[r * C + c] = (sb == 0xFFu) ? NAN : ldexp(orc_e2m1_decode(code), (int)sb - 127);
        }
}

/* ------------------------------------------------------------------------- */
/* GEMM on quantised operands                                                 */
/* ------------------------------------------------------------------------- */

/* fmt: ORC_FMT_E2M1 (two codes per byte, q[R][C/2]) or ORC_FMT_E4M3 (one byte per element, q[R][C]) */
static void decode_row_fmt(const uint8_t *q, const uint8_t *s, int fmt, int64_t r, int64_t C, double *dst)
{
    for (int64_t c = 0; c < C; ++c) {
        unsigned sb = s[r * (C / MX_BLOCK) + c / MX_BLOCK];
        double val;
        if (fmt == ORC_FMT_E4M3) {
            val = orc_e4m3_decode(q[r * C + c]);
        } else {
            unsigned byte = q[r * (C / 2) + c / 2];
            val = orc_e2m1_decode((c & 1) ? (byte >> 4) : (byte & 15u));
        }
        dst[c] = (sb == 0xFFu) ? NAN : ldexp(val, (int)sb - 127);
    }
}

/* out[i][j] = sum_c A[i][c] * B[j][c] over the decoded operands, in double
 * (every product is exact; only the running sum rounds).  absum, if not NULL,
 * receives sum_c |A[i][c]| |B[j][c]|, the yardstick of the GEMM tolerance.
 * A is [Ra][C], B is [Rb][C], both in the quantiser's output layout. */
int orc_gemm_fmt(const uint8_t *aq, const uint8_t *as, int afmt, const uint8_t *bq, const uint8_t *bs, int bfmt,
                 int64_t Ra, int64_t Rb, int64_t C, double *out, double *absum);

int orc_gemm(const uint8_t *aq, const uint8_t *as, const uint8_t *bq, const uint8_t *bs, int64_t Ra, int64_t Rb,
             int64_t C, double *out, double *absum)
{
    return orc_gemm_fmt(aq, as, ORC_FMT_E2M1, bq, bs, ORC_FMT_E2M1, Ra, Rb, C, out, absum);
}

/* The same sum with each operand in its own element format (MXFP4 or MXFP8). */
int orc_gemm_fmt(const uint8_t *aq, const uint8_t *as, int afmt, const uint8_t *bq, const uint8_t *bs, int bfmt,
                 int64_t Ra, int64_t Rb, int64_t C, double *out, double *absum)
{
    if (C % MX_BLOCK != 0) return 1;
    double *B = (double *)malloc(sizeof(double) * (size_t)Rb * (size_t)C);
    if (!B) return 2;
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < Rb; ++j) decode_row_fmt(bq, bs, bfmt, j, C, B + j * C);
#pragma omp parallel
    {
        double *a = (double *)malloc(sizeof(double) * (size_t)C);
#pragma omp for schedule(static)
        for (int64_t i = 0; i < Ra; ++i) {
            decode_row_fmt(aq, as, afmt, i, C, a);
            for (int64_t j = 0; j < Rb; ++j) {
                const double *b = B + j * C;
                double acc = 0.0, ab = 0.0;
                for (int64_t c = 0; c < C; ++c) {
                    double p = a[c] * b[c];
                    acc += p;
                    ab += fabs(p);
                }
                out[i * Rb + j] = acc;
                if (absum) absum[i * Rb + j] = ab;
            }
        }
        free(a);
    }
    free(B);
    return 0;
}

/* The same sum for n chosen output positions (ii[k], jj[k]) only. */
int orc_gemm_at_fmt(const uint8_t *aq, const uint8_t *as, int afmt, const uint8_t *bq, const uint8_t *bs, int bfmt,
                    int64_t Ra, int64_t Rb, int64_t C, const int64_t *ii, const int64_t *jj, int64_t n, double *out,
                    double *absum);

int orc_gemm_at(const uint8_t *aq, const uint8_t *as, const uint8_t *bq, const uint8_t *bs, int64_t Ra, int64_t Rb,
                int64_t C, const int64_t *ii, const int64_t *jj, int64_t n, double *out, double *absum)
{
    return orc_gemm_at_fmt(aq, as, ORC_FMT_E2M1, bq, bs, ORC_FMT_E2M1, Ra, Rb, C, ii, jj, n, out, absum);
}

int orc_gemm_at_fmt(const uint8_t *aq, const uint8_t *as, int afmt, const uint8_t *bq, const uint8_t *bs, int bfmt,
                    int64_t Ra, int64_t Rb, int64_t C, const int64_t *ii, const int64_t *jj, int64_t n, double *out,
                    double *absum)
{
    if (C % MX_BLOCK != 0) return 1;
    for (int64_t k = 0; k < n; ++k)
        if (ii[k] < 0 || ii[k] >= Ra || jj[k] < 0 || jj[k] >= Rb) return 3;
#pragma omp parallel
    {
        double *a = (double *)malloc(sizeof(double) * (size_t)C);
        double *b = (double *)malloc(sizeof(double) * (size_t)C);
#pragma omp for schedule(dynamic, 16)
        for (int64_t k = 0; k < n; ++k) {
            decode_row_fmt(aq, as, afmt, ii[k], C, a);
            decode_row_fmt(bq, bs, bfmt, jj[k], C, b);
            double acc = 0.0, ab = 0.0;
            for (int64_t c = 0; c < C; ++c) {
                double p = a[c] * b[c];
                acc += p;
                ab += fabs(p);
            }
            out[k] = acc;
            if (absum) absum[k] = ab;
        }
        free(a);
        free(b);
    }
    return 0;
}

/* Round a double to bf16 (nearest even), returning the 16-bit pattern: first to
 * fp32 (the kernel's accumulator type), then fp32 -> bf16.  Used only to state
 * what a bf16 output of a given fp32 value must be. */
uint16_t orc_f32_to_bf16_rne(float f)
{
    uint32_t u = f32_bits(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40u); /* NaN stays NaN */
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7FFFu + lsb;
    return (uint16_t)(u >> 16);
}

/* Number of threads the parallel loops above use. */
int orc_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        n = omp_get_num_threads();
    }
#endif
    return n;
}
