// MXFP8 (E4M3) quantiser kernels for gfx950: the stages of the stage-wise recipe that stay in 8 bits
// (Table 1, "MXFP4 GEMMs (others FP8)").  Same block geometry, rotation and block maximum as the MXFP4 kernels
// (App. A.1, A.2, App. D); one byte per element.
#include "mxfp4_internal.h"
#include "quantize_block.h"

namespace mxfp4 {
namespace {

// ---- MXFP8 (E4M3 elements) for the stages that stay in 8 bits (Table 1, "others FP8") --------------
// Same rotation, same block maximum; scale byte = biased exponent of the maximum - 8 (E4M3's largest
// exponent), one byte per element.  V_CVT_SCALEF32_PK_FP8_F32 divides by the scale and rounds to nearest
// even (probed, subnormals included) but turns everything above 464 into NaN instead of saturating, so
// the values are clamped to +-448 * 2^E first.
typedef short v2s __attribute__((ext_vector_type(2)));

__device__ __forceinline__ void encode_scaled_fp8(const float (&v)[32], uint32_t amax, uint4 &lo, uint4 &hi,
                                                  uint32_t &scale_byte)
{
    const uint32_t eb = amax >> 23;
    const bool bad = (eb == 255u);
    const uint32_t sb = eb > 8u ? eb - 8u : 0u;  // eb <= 254 here, so sb <= 246
    scale_byte = bad ? 0xFFu : sb;
    const float scale = __uint_as_float(sb << 23);
    const float lim = __uint_as_float(((sb + 8u) << 23) | 0x600000u);  // 448 * 2^(sb - 127)
    uint32_t w[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        v2s r = {0, 0};
        r = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(r, __builtin_amdgcn_fmed3f(v[4 * j + 0], -lim, lim),
                                                     __builtin_amdgcn_fmed3f(v[4 * j + 1], -lim, lim), scale, false);
        r = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(r, __builtin_amdgcn_fmed3f(v[4 * j + 2], -lim, lim),
                                                     __builtin_amdgcn_fmed3f(v[4 * j + 3], -lim, lim), scale, true);
        w[j] = (uint32_t)(uint16_t)r.x | ((uint32_t)(uint16_t)r.y << 16);
    }
    lo = bad ? make_uint4(0, 0, 0, 0) : make_uint4(w[0], w[1], w[2], w[3]);
    hi = bad ? make_uint4(0, 0, 0, 0) : make_uint4(w[4], w[5], w[6], w[7]);
}

// row-wise: one lane per block, 32 output bytes per lane
template <int HAD>
__global__ __launch_bounds__(256) void quantize_rows_fp8_kernel(const uint16_t *__restrict__ x, int64_t nblocks,
                                                                int64_t bpr, int64_t ld, int dense,
                                                                uint32_t sign_mask, uint8_t *__restrict__ q,
                                                                uint8_t *__restrict__ s)
{
    int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (g >= nblocks) return;
    const uint16_t *src;
    if (dense) {
        src = x + g * 32;
    } else {
        int64_t row = g / bpr;
        src = x + row * ld + (g - row * bpr) * 32;
    }
    const uint4 *p = reinterpret_cast<const uint4 *>(src);
    uint4 raw[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) raw[j] = p[j];
    float v[32];
    widen(raw, v);
    rotate_block<HAD>(v, sign_mask);
    uint4 lo, hi;
    uint32_t sb;
    encode_scaled_fp8(v, amax_bits(v), lo, hi, sb);
    reinterpret_cast<uint4 *>(q)[2 * g] = lo;
    reinterpret_cast<uint4 *>(q)[2 * g + 1] = hi;
    s[g] = (uint8_t)sb;
}

// column-wise: the tile and lane assignment of quantize_cols_kernel; an output row receives 8 x 32 = 256
// contiguous bytes per tile
template <int HAD>
__global__ __launch_bounds__(512) void quantize_cols_fp8_kernel(const uint16_t *__restrict__ x, int64_t rows,
                                                                int64_t cols, int64_t ld, uint32_t sign_mask,
                                                                uint8_t *__restrict__ q, uint8_t *__restrict__ s,
                                                                uint32_t col_groups)
{
    __shared__ uint4 lds_q[CT_RB][2][CT_COLS + 1];
    __shared__ uint8_t lds_s[CT_COLS][CT_RB];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const uint32_t by = blockIdx.x / col_groups, bx = blockIdx.x - by * col_groups;
    const int64_t c0 = (int64_t)bx * CT_COLS, rb0 = (int64_t)by * CT_RB, nrb = rows >> 5;
    const int64_t rb = rb0 + w, col = c0 + 2 * lane;
    uint32_t raw[32];
    if ((rb < nrb) && (col < cols)) {
        const uint16_t *p = x + (rb * 32) * ld + col;
#pragma unroll
        for (int i = 0; i < 32; ++i) raw[i] = *reinterpret_cast<const uint32_t *>(p + i * ld);
    } else {
#pragma unroll
        for (int i = 0; i < 32; ++i) raw[i] = 0;
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        float v[32];
#pragma unroll
        for (int i = 0; i < 32; ++i) v[i] = j == 0 ? bf16_lo(raw[i]) : bf16_hi(raw[i]);
        rotate_block<HAD>(v, sign_mask);
        uint4 lo, hi;
        uint32_t sb;
        encode_scaled_fp8(v, amax_bits(v), lo, hi, sb);
        lds_q[w][0][2 * lane + j] = lo;
        lds_q[w][1][2 * lane + j] = hi;
        lds_s[2 * lane + j][w] = (uint8_t)sb;
    }
    __syncthreads();
    // 16 consecutive threads write the 256 bytes one output row receives from this tile
#pragma unroll
    for (int pass = 0; pass < 4; ++pass) {
        const int idx = pass * 512 + tid, cl = idx >> 4, k = idx & 15, b = k >> 1, half = k & 1;
        if (c0 + cl < cols && rb0 + b < nrb)
            *reinterpret_cast<uint4 *>(q + (c0 + cl) * rows + (rb0 + b) * 32 + half * 16) = lds_q[b][half][cl];
    }
    if (tid < CT_COLS && c0 + tid < cols) {
        uint8_t *dst = s + (c0 + tid) * nrb + rb0;
#pragma unroll
        for (int k = 0; k < CT_RB; ++k)
            if (rb0 + k < nrb) dst[k] = lds_s[tid][k];
    }
}

// both layouts from one pass over the tensor: the tile and the parking scheme of the dual-axis MXFP4 kernel.
// Each wave parks its 32 x 128 elements in its own LDS slice (the first 16 rows are parked and worked on while
// the other 16 are still in flight), reads them back as row blocks, two per lane and four lanes per row, so that
// a row of the tile leaves as 128 contiguous bytes, and then reuses the slice to regroup its column-wise codes:
// wave w keeps the low 16 bytes of every column's 32 at w * SKEW into its slice and the high 16 bytes FP8_HALF
// further on, which lets the 16 lanes that later gather one output row's 256 bytes from the 8 slices hit every
// bank once.
constexpr int FP8_SLICE = 32 * RAW_PITCH, FP8_HALF = (CT_COLS + 1) * 16, FP8_SKEW = 32;
static_assert(2 * FP8_HALF + (CT_RB - 1) * FP8_SKEW <= FP8_SLICE, "the codes of a wave must fit its slice");

// ROW4: the row-wise output is MXFP4 instead (rotation HAD_ROW, rounding RND_ROW under key_row: what the MXFP4
// kernels write), the column-wise one stays MXFP8 under rotation HAD: a tensor that feeds one MXFP4 and one MXFP8
// GEMM of the stage-wise recipe (X and W when only Fprop is in MXFP4, X and dY when Fprop and Dgrad are).
template <int HAD, bool ROW4, int HAD_ROW, int RND_ROW>
__global__ __launch_bounds__(512) void quantize_dual_fp8_kernel(const uint16_t *__restrict__ x, int64_t rows,
                                                                int64_t cols, int64_t ld, uint32_t sign_mask,
                                                                uint8_t *__restrict__ q, uint8_t *__restrict__ s,
                                                                uint8_t *__restrict__ q_row,
                                                                uint8_t *__restrict__ s_row, uint32_t col_groups,
                                                                int s_row_vec4, RngKey key_row)
{
    __shared__ __attribute__((aligned(16))) uint8_t lds[CT_RB * FP8_SLICE + CT_COLS * CT_RB];
    uint8_t(*lds_s)[CT_RB] = reinterpret_cast<uint8_t(*)[CT_RB]>(lds + CT_RB * FP8_SLICE);
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const uint32_t by = blockIdx.x / col_groups, bx = blockIdx.x - by * col_groups;
    const int64_t c0 = (int64_t)bx * CT_COLS, rb0 = (int64_t)by * CT_RB, nrb = rows >> 5;
    const int64_t rb = rb0 + w, col = c0 + 2 * lane;
    uint32_t raw[32];
    if ((rb < nrb) && (col < cols)) {
        const uint16_t *p = x + (rb * 32) * ld + col;
#pragma unroll
        for (int i = 0; i < 32; ++i) raw[i] = *reinterpret_cast<const uint32_t *>(p + i * ld);
    } else {
#pragma unroll
        for (int i = 0; i < 32; ++i) raw[i] = 0;
    }

    // ---- row-wise output ----
    uint8_t *mine = lds + w * FP8_SLICE;
    const int cb = lane & 3;
    const int64_t colb = c0 + 32 * cb, bpr = cols >> 5;
    const bool on = (rb < nrb) && (colb < cols);
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
#pragma unroll
        for (int i = 16 * pass; i < 16 * pass + 16; ++i)
            *reinterpret_cast<uint32_t *>(mine + i * RAW_PITCH + 4 * lane) = raw[i];
        wave_sync();  // (the slice is written and read by this wave only)
        const int r = (lane >> 2) + 16 * pass;
        const uint4 *p = reinterpret_cast<const uint4 *>(mine + r * RAW_PITCH + 64 * cb);
        uint4 rraw[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) rraw[j] = p[j];
        float v[32];
        widen(rraw, v);
        const int64_t row = rb * 32 + r, g = row * bpr + (colb >> 5);
        uint32_t sb;
        if constexpr (ROW4) {
            rotate_block<HAD_ROW>(v, sign_mask);
            uint4 codes;
            encode_scaled<RND_ROW>(v, amax_bits(v), key_row, (uint64_t)row * (uint64_t)cols + (uint64_t)colb, codes, sb);
            if (on) reinterpret_cast<uint4 *>(q_row)[g] = codes;
        } else {
            rotate_block<HAD>(v, sign_mask);
            uint4 lo, hi;
            encode_scaled_fp8(v, amax_bits(v), lo, hi, sb);
            if (on) {
                reinterpret_cast<uint4 *>(q_row)[2 * g] = lo;
                reinterpret_cast<uint4 *>(q_row)[2 * g + 1] = hi;
            }
        }
        // the four scale bytes of one row of the tile go out as one dword where they can
        uint32_t s4 = sb;
        s4 |= (uint32_t)__shfl_down((int)sb, 1) << 8;
        s4 |= (uint32_t)__shfl_down((int)sb, 2) << 16;
        s4 |= (uint32_t)__shfl_down((int)sb, 3) << 24;
        if (s_row_vec4 && c0 + CT_COLS <= cols) {
            if (on && cb == 0) *reinterpret_cast<uint32_t *>(s_row + g) = s4;
        } else if (on) {
            s_row[g] = (uint8_t)sb;
        }
        __builtin_amdgcn_sched_barrier(0);  // (keep the second half's LDS writes, and with them the wait, down here)
    }
    wave_sync();  // the wave is done with its parked elements: the slice becomes its regrouping buffer

    // ---- column-wise output ----
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        float v[32];
#pragma unroll
        for (int i = 0; i < 32; ++i) v[i] = j == 0 ? bf16_lo(raw[i]) : bf16_hi(raw[i]);
        rotate_block<HAD>(v, sign_mask);
        uint4 lo, hi;
        uint32_t sb;
        encode_scaled_fp8(v, amax_bits(v), lo, hi, sb);
        uint8_t *base = mine + w * FP8_SKEW;
        reinterpret_cast<uint4 *>(base)[2 * lane + j] = lo;
        reinterpret_cast<uint4 *>(base + FP8_HALF)[2 * lane + j] = hi;
        lds_s[2 * lane + j][w] = (uint8_t)sb;
    }
    // workgroup barrier for the LDS traffic only (it does not wait for the row-wise stores still in flight)
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    // 16 consecutive threads write the 256 bytes one output row receives from this tile
#pragma unroll
    for (int pass = 0; pass < 4; ++pass) {
        const int idx = pass * 512 + tid, cl = idx >> 4, k = idx & 15, b = k >> 1, half = k & 1;
        if (c0 + cl < cols && rb0 + b < nrb)
            *reinterpret_cast<uint4 *>(q + (c0 + cl) * rows + (rb0 + b) * 32 + half * 16) =
                *reinterpret_cast<const uint4 *>(lds + b * (FP8_SLICE + FP8_SKEW) + half * FP8_HALF + cl * 16);
    }
    if (tid < CT_COLS && c0 + tid < cols) {
        uint8_t *dst = s + (c0 + tid) * nrb + rb0;
#pragma unroll
        for (int k = 0; k < CT_RB; ++k)
            if (rb0 + k < nrb) dst[k] = lds_s[tid][k];
    }
}

template <int HAD>
hipError_t launch_fp8_h(const QuantArgs &a, bool cols_axis, hipStream_t st)
{
    const uint32_t sign_mask = sign_mask_of(a.seed);
    if (cols_axis) {
        const int64_t nrb = a.rows / 32;
        const uint32_t col_groups = (uint32_t)((a.cols + CT_COLS - 1) / CT_COLS);
        dim3 grid((unsigned)(col_groups * ((nrb + CT_RB - 1) / CT_RB)));
        hipLaunchKernelGGL((quantize_cols_fp8_kernel<HAD>), grid, dim3(512), 0, st, a.x, a.rows, a.cols, a.ld,
                           sign_mask, a.q, a.s, col_groups);
    } else {
        const int64_t bpr = a.cols / 32, nblocks = a.rows * bpr;
        const unsigned grid = (unsigned)((nblocks + 255) / 256);
        hipLaunchKernelGGL((quantize_rows_fp8_kernel<HAD>), dim3(grid), dim3(256), 0, st, a.x, nblocks, bpr, a.ld,
                           (int)(a.ld == a.cols), sign_mask, a.q, a.s);
    }
    return hipGetLastError();
}

template <int HAD, bool ROW4, int HAD_ROW, int RND_ROW>
hipError_t launch_fp8_dual_h(const QuantArgs &a, hipStream_t st)
{
    const int64_t nrb = a.rows / 32;
    const uint32_t col_groups = (uint32_t)((a.cols + CT_COLS - 1) / CT_COLS);
    dim3 grid((unsigned)(col_groups * ((nrb + CT_RB - 1) / CT_RB)));
    const int s_row_vec4 = (((a.cols / 32) % 4) == 0) && ((reinterpret_cast<uintptr_t>(a.s_row) % 4) == 0);
    hipLaunchKernelGGL((quantize_dual_fp8_kernel<HAD, ROW4, HAD_ROW, RND_ROW>), grid, dim3(512), 0, st, a.x, a.rows,
                       a.cols, a.ld, sign_mask_of(a.seed), a.q, a.s, a.q_row, a.s_row, col_groups, s_row_vec4,
                       make_key(a.seed_row));
    return hipGetLastError();
}

template <int HAD_ROW>
hipError_t launch_mixed_h(const QuantArgs &a, hipStream_t st)
{
    return a.rounding == RND_RNE ? launch_fp8_dual_h<HAD_NONE, true, HAD_ROW, RND_RNE>(a, st)
                                 : launch_fp8_dual_h<HAD_NONE, true, HAD_ROW, RND_SR>(a, st);
}

}  // namespace

hipError_t launch_quantize_fp8_dual(const QuantArgs &a, hipStream_t st)
{
    switch (a.hadamard) {
        case HAD_NONE: return launch_fp8_dual_h<HAD_NONE, false, HAD_NONE, RND_RNE>(a, st);
        case HAD_DET: return launch_fp8_dual_h<HAD_DET, false, HAD_NONE, RND_RNE>(a, st);
        case HAD_RANDSIGN: return launch_fp8_dual_h<HAD_RANDSIGN, false, HAD_NONE, RND_RNE>(a, st);
        case HAD_RANDSIGN16: return launch_fp8_dual_h<HAD_RANDSIGN16, false, HAD_NONE, RND_RNE>(a, st);
        default: return launch_fp8_dual_h<HAD_DET16, false, HAD_NONE, RND_RNE>(a, st);
    }
}

hipError_t launch_quantize_mxfp4_rows_mxfp8_cols(const QuantArgs &a, hipStream_t st)
{
    switch (a.hadamard) {
        case HAD_NONE: return launch_mixed_h<HAD_NONE>(a, st);
        case HAD_DET: return launch_mixed_h<HAD_DET>(a, st);
        case HAD_RANDSIGN: return launch_mixed_h<HAD_RANDSIGN>(a, st);
        case HAD_RANDSIGN16: return launch_mixed_h<HAD_RANDSIGN16>(a, st);
        default: return launch_mixed_h<HAD_DET16>(a, st);
    }
}

hipError_t launch_quantize_fp8(const QuantArgs &a, bool cols_axis, hipStream_t st)
{
    switch (a.hadamard) {
        case HAD_NONE: return launch_fp8_h<HAD_NONE>(a, cols_axis, st);
        case HAD_DET: return launch_fp8_h<HAD_DET>(a, cols_axis, st);
        case HAD_RANDSIGN: return launch_fp8_h<HAD_RANDSIGN>(a, cols_axis, st);
        case HAD_RANDSIGN16: return launch_fp8_h<HAD_RANDSIGN16>(a, cols_axis, st);
        default: return launch_fp8_h<HAD_DET16>(a, cols_axis, st);
    }
}

}  // namespace mxfp4
