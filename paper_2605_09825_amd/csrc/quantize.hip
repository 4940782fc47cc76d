// Fused rotate + amax + scale + pack kernels for gfx950 (MXFP4 quantiser).
//
// What is computed per 32-element block is eq. (1) of App. A.1 with the OCP MX scale
// rule, preceded by the Hadamard rotation of App. A.2; the block geometry is the
// 1x32 (row-wise) and 32x1 (column-wise) layouts of App. D.
//
// Design: the work is HBM-bound (2 bytes read, 0.53 bytes written per element), so
// each lane owns one whole block in registers: the five butterfly stages, the block
// maximum, the scale and the packing need no cross-lane traffic at all, and the
// packed output of a lane is one 16-byte store.
//   * row-wise: a lane reads its 64 contiguous bytes with four 16-byte loads; lanes
//     of a wave cover 4 KiB of contiguous memory, so every fetched line is used.
//   * column-wise: a lane owns two adjacent columns over 32 rows (32 dword loads,
//     256 contiguous bytes per wave and row); the eight waves of a workgroup take
//     eight consecutive row blocks, and the packed codes are regrouped through LDS
//     so that each output row receives 128 contiguous bytes.
//   * both at once: the column-wise workgroup tile, whose 256 x 128 elements are also
//     parked in LDS and read back as row-wise blocks; memory delivers the tensor once
//     for the two outputs.
//   * 32 x 32 geometry (App. D): the same kernel with the block maxima reduced over the
//     16 lanes that share a region before the codes are formed.
#include "mxfp4_internal.h"
#include "quantize_block.h"

namespace mxfp4 {
namespace {

constexpr int64_t LLC_BYTES = int64_t(256) << 20;  // MI355X Infinity Cache

// v: the block widened to fp32, in contraction order; 1D scaling (one scale per block).
template <int HAD, int RND>
__device__ __forceinline__ void encode_block(float (&v)[32], uint32_t sign_mask, RngKey key, uint64_t idx0,
                                             uint4 &codes, uint32_t &scale_byte)
{
    rotate_block<HAD>(v, sign_mask);
    encode_scaled<RND>(v, amax_bits(v), key, idx0, codes, scale_byte);
}

// ---- row-wise (1x32) ---------------------------------------------------------------------
// One lane per block.  nblocks = rows * (cols/32); block g is row g / bpr, column block g % bpr.
// STREAM: tensor larger than the last-level cache: non-temporal code stores.
template <int HAD, int RND, int STREAM>
__global__ __launch_bounds__(256) void quantize_rows_kernel(const uint16_t *__restrict__ x, int64_t nblocks,
                                                            int64_t bpr, int64_t ld, int dense,
                                                            uint32_t sign_mask, RngKey key,
                                                            uint8_t *__restrict__ q, uint8_t *__restrict__ s)
{
    constexpr int streaming = STREAM;
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
    uint4 raw[4];  // (plain loads also for tensors beyond the cache: non-temporal 16-byte loads measured 30 % slower
                   // here, whereas the column-wise kernel's dword loads gain 8 % from the hint)
#pragma unroll
    for (int j = 0; j < 4; ++j) raw[j] = p[j];
    float v[32];
    widen(raw, v);
    uint4 codes;
    uint32_t sb;
    encode_block<HAD, RND>(v, sign_mask, key, (uint64_t)g * 32u, codes, sb);
    store_codes(reinterpret_cast<uint4 *>(q) + g, codes, streaming);
    s[g] = (uint8_t)sb;
}

// ---- column-wise (32x1) ------------------------------------------------------------------
// Workgroup tile: 256 rows (8 row blocks, one per wave) x 128 columns (2 per lane).

// MODE_DUAL: additionally emit the row-wise quantisation q_row[rows][cols/2], s_row[rows][cols/32] of the
// same tile (needs cols % 32 == 0).  Each wave parks its 32 x 128 elements in LDS and reads them back as
// 128 row blocks, two per lane, four lanes per row, so the tensor is fetched from memory once.  The parked
// tile and the regrouping buffers of the column-wise output share the same LDS.
// MODE_2D: the 32 x 32 geometry of App. D: one scale per 32 x 32 region (a wave's tile holds four), taken
// from the largest magnitude of the region after the rotation; either output may be switched off (null
// q/s or q_row/s_row).  Each phase runs twice over its data: first the maxima, reduced across the 16 lanes
// that share a region, then the codes.
constexpr int MODE_COLS = 0, MODE_DUAL = 1, MODE_2D = 2;
constexpr int LDS_S_BYTES = CT_COLS * CT_RB;

__device__ __forceinline__ uint32_t max_across(uint32_t m, int xor_mask)
{
    const uint32_t o = (uint32_t)__shfl_xor((int)m, xor_mask);
    return o > m ? o : m;
}

// One tensor's share of a launch.  A launch may carry two tensors (the two operands of a GEMM): workgroups
// 0 .. nblocks-1 of the first job, then those of the second.
struct TileJob {
    const uint16_t *x;
    int64_t rows, cols, ld;
    uint8_t *q, *s, *q_row, *s_row;
    uint32_t col_groups, nblocks, band_rows;
    int s_vec8, s_row_vec4, streaming;
    RngKey key, key_row;  // stochastic-rounding streams of the column-wise and of the row-wise output
};

// STREAM: the tensor is larger than the last-level cache: it is read with non-temporal loads and its codes are
// written with non-temporal stores (a compile-time choice: as a run-time branch around the loads the compiler
// merges the two sides and the hint is lost).
template <int HAD, int RND, int MODE, int STREAM>
__global__ __launch_bounds__(512) void quantize_cols_kernel(const TileJob job0, const TileJob job1,
                                                            uint32_t sign_mask)
{
    const bool second = blockIdx.x >= job0.nblocks;  // uniform: everything below is selected per workgroup
    const uint16_t *__restrict__ x = second ? job1.x : job0.x;
    const int64_t rows = second ? job1.rows : job0.rows, cols = second ? job1.cols : job0.cols;
    const int64_t ld = second ? job1.ld : job0.ld;
    uint8_t *__restrict__ q = second ? job1.q : job0.q;
    uint8_t *__restrict__ s = second ? job1.s : job0.s;
    uint8_t *__restrict__ q_row = second ? job1.q_row : job0.q_row;
    uint8_t *__restrict__ s_row = second ? job1.s_row : job0.s_row;
    const uint32_t col_groups = second ? job1.col_groups : job0.col_groups;
    const uint32_t nb = second ? job1.nblocks : job0.nblocks;
    const uint32_t band_rows = second ? job1.band_rows : job0.band_rows;
    const int s_vec8 = second ? job1.s_vec8 : job0.s_vec8, s_row_vec4 = second ? job1.s_row_vec4 : job0.s_row_vec4;
    constexpr int streaming = STREAM;
    const RngKey key = second ? job1.key : job0.key, key_row = second ? job1.key_row : job0.key_row;
    const uint32_t bid = blockIdx.x - (second ? job0.nblocks : 0u);

    // LDS: per wave one slice that first holds the wave's parked 32 x 128 elements (DUAL, 2D) and then its
    // (CT_COLS + 1) x 16 bytes of column-wise codes waiting to be regrouped; behind the slices the scale bytes
    // of all waves.  A wave only ever touches its own slice until the one barrier before the regrouped stores.
    constexpr bool PARK = (MODE != MODE_COLS);
    constexpr int SLICE = PARK ? 32 * RAW_PITCH : (CT_COLS + 1) * 16;
    // the codes of wave w start w * SKEW bytes into its slice, so that the 8 lanes that later gather one output
    // row from the 8 slices hit different banks (the column-wise-only slice has the odd pitch built in)
    constexpr int SKEW = PARK ? 16 : 0;
    static_assert(SLICE >= CT_COLS * 16 + (CT_RB - 1) * SKEW + (PARK ? 0 : 16), "the codes of a wave must fit its slice");
    __shared__ __attribute__((aligned(16))) uint8_t lds[CT_RB * SLICE + LDS_S_BYTES];
    uint8_t(*lds_s)[CT_RB] = reinterpret_cast<uint8_t(*)[CT_RB]>(lds + CT_RB * SLICE);

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    // Tile order.  A tile contributes only 8 scale bytes per column (4 per row in the row-wise output), far less
    // than the 64 bytes the memory side writes at once, and the 8 XCDs (workgroup id mod 8) have separate L2s
    // that cannot merge each other's partial writes.  With band_rows > 0 each XCD takes a contiguous run of the
    // tile sequence, and the sequence walks the grid in bands of band_rows tile rows, tile rows fastest, so that
    // the tiles completing a 64-byte piece of either scale stream meet in one L2 (measured: write requests fall
    // from 1.18x to 1.00x the algorithmic count; worth 8 % on a 16384 x 14336 tensor, nothing on tensors
    // so small that a CU sees only a few tiles, which keep the plain order band_rows = 0).
    uint32_t by, bx;
    if (band_rows == 0) {
        by = bid / col_groups;
        bx = bid - by * col_groups;
    } else {
        const uint32_t xcd = bid & 7, per = nb >> 3, rem = nb & 7;
        const uint32_t start = xcd < rem ? xcd * (per + 1) : rem * (per + 1) + (xcd - rem) * per;
        const uint32_t lb = start + (bid >> 3);
        const uint32_t row_groups = nb / col_groups, span = band_rows * col_groups;
        const uint32_t band = lb / span, in = lb - band * span;
        const uint32_t left = row_groups - band * band_rows, gm = left < band_rows ? left : band_rows;
        bx = in / gm;
        by = band * band_rows + (in - bx * gm);
    }
    const int64_t c0 = (int64_t)bx * CT_COLS;
    const int64_t rb0 = (int64_t)by * CT_RB;
    const int64_t nrb = rows >> 5;
    const int64_t rb = rb0 + w;
    const int64_t col = c0 + 2 * lane;
    const bool active = (rb < nrb) && (col < cols);
    const bool want_row = (MODE == MODE_DUAL) || (MODE == MODE_2D && q_row != nullptr);
    const bool want_col = (MODE != MODE_2D) || (q != nullptr);

    uint32_t raw[32];
    if (active) {
        const uint16_t *p = x + (rb * 32) * ld + col;
        if constexpr (STREAM) {  // read once: keep it out of the way of the output in the caches
#pragma unroll
            for (int i = 0; i < 32; ++i)
                raw[i] = __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(p + i * ld));
        } else {
#pragma unroll
            for (int i = 0; i < 32; ++i) raw[i] = *reinterpret_cast<const uint32_t *>(p + i * ld);
        }
    } else {
#pragma unroll
        for (int i = 0; i < 32; ++i) raw[i] = 0;
    }

    if (PARK && want_row) {
        // Row pass p (0/1) works on rows 16p .. 16p+15 of the wave's 32: the first half is parked and worked on
        // as soon as its 16 loads are back, under the latency of the other 16.
        uint8_t *mine = lds + w * SLICE;
        auto park = [&](int half) {
#pragma unroll
            for (int i = 16 * half; i < 16 * half + 16; ++i)
                *reinterpret_cast<uint32_t *>(mine + i * RAW_PITCH + 4 * lane) = raw[i];
            wave_sync();  // (the slice is written and read by this wave only)
        };
        const int cb = lane & 3;
        const int64_t colb = c0 + 32 * cb;
        const int64_t bpr = cols >> 5;
        const bool on = (rb < nrb) && (colb < cols);
        auto rotated_row = [&](int pass, float (&v)[32]) {
            const int r = (lane >> 2) + 16 * pass;
            const uint4 *p = reinterpret_cast<const uint4 *>(mine + r * RAW_PITCH + 64 * cb);
            uint4 rraw[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) rraw[j] = p[j];
            widen(rraw, v);
            rotate_block<HAD>(v, sign_mask);
        };
        uint32_t region_max = 0;
        auto row_codes = [&](int pass) {
            const int64_t row = rb * 32 + (lane >> 2) + 16 * pass;
            float v[32];
            rotated_row(pass, v);
            uint4 codes;
            uint32_t sb;
            encode_scaled<RND>(v, MODE == MODE_2D ? region_max : amax_bits(v), key_row,
                               (uint64_t)row * (uint64_t)cols + (uint64_t)colb, codes, sb);
            const int64_t g = row * bpr + (colb >> 5);
            if (on) store_codes(reinterpret_cast<uint4 *>(q_row) + g, codes, streaming);
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
        };
        auto row_max = [&](int pass) {
            float v[32];
            rotated_row(pass, v);
            const uint32_t m = amax_bits(v);
            region_max = m > region_max ? m : region_max;
        };
        park(0);
        if (MODE == MODE_2D) row_max(0); else row_codes(0);
        __builtin_amdgcn_sched_barrier(0);  // (keep the second half's LDS writes, and with them the wait, down here)
        park(1);
        if (MODE == MODE_2D) {
            row_max(1);
            // the 32 rows of one region: the 16 lanes with this lane's (lane & 3), two rows each
            region_max = max_across(region_max, 4);
            region_max = max_across(region_max, 8);
            region_max = max_across(region_max, 16);
            region_max = max_across(region_max, 32);
            row_codes(0);
        }
        row_codes(1);
        wave_sync();  // the wave is done with its parked elements: the slice becomes its regrouping buffer
    }
    if (!want_col) return;  // (uniform over the grid)

    uint32_t region_max = 0;
    if (MODE == MODE_2D) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            float v[32];
#pragma unroll
            for (int i = 0; i < 32; ++i) v[i] = j == 0 ? bf16_lo(raw[i]) : bf16_hi(raw[i]);
            rotate_block<HAD>(v, sign_mask);
            const uint32_t m = amax_bits(v);
            region_max = m > region_max ? m : region_max;
        }
        // the 32 columns of one region: 16 consecutive lanes, two columns each
        region_max = max_across(region_max, 1);
        region_max = max_across(region_max, 2);
        region_max = max_across(region_max, 4);
        region_max = max_across(region_max, 8);
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        float v[32];
#pragma unroll
        for (int i = 0; i < 32; ++i) v[i] = j == 0 ? bf16_lo(raw[i]) : bf16_hi(raw[i]);
        rotate_block<HAD>(v, sign_mask);
        uint4 codes;
        uint32_t sb;
        encode_scaled<RND>(v, MODE == MODE_2D ? region_max : amax_bits(v), key,
                           (uint64_t)(col + j) * (uint64_t)rows + (uint64_t)rb * 32u, codes, sb);
        reinterpret_cast<uint4 *>(lds + w * (SLICE + SKEW))[2 * lane + j] = codes;
        lds_s[2 * lane + j][w] = (uint8_t)sb;
    }
    // workgroup barrier for the LDS traffic only: unlike __syncthreads() it does not make the wave wait for its
    // outstanding global stores (the row-wise output, which nobody in the workgroup reads back)
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");

    // each output row (input column) receives its 8 x 16 bytes from 8 consecutive lanes
    const int ch = tid & 7;
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        const int cl = (tid >> 3) + 64 * pass;
        if (c0 + cl < cols && rb0 + ch < nrb)
            store_codes(reinterpret_cast<uint4 *>(q + (c0 + cl) * (rows >> 1) + (rb0 + ch) * 16),
                        reinterpret_cast<const uint4 *>(lds + ch * (SLICE + SKEW))[cl], streaming);
    }
    if (tid < CT_COLS && c0 + tid < cols) {
        uint8_t *dst = s + (c0 + tid) * nrb + rb0;
        if (s_vec8 && rb0 + CT_RB <= nrb) {
            *reinterpret_cast<uint2 *>(dst) = *reinterpret_cast<const uint2 *>(&lds_s[tid][0]);
        } else {
#pragma unroll
            for (int k = 0; k < CT_RB; ++k)
                if (rb0 + k < nrb) dst[k] = lds_s[tid][k];
        }
    }
}

template <int HAD>
hipError_t launch_rows_h(const QuantArgs &a, hipStream_t st)
{
    const int64_t bpr = a.cols / 32, nblocks = a.rows * bpr;
    const unsigned grid = (unsigned)((nblocks + 255) / 256);
    const RngKey key = make_key(a.seed);
    const uint32_t sign_mask = sign_mask_of(a.seed);
    const int dense = (a.ld == a.cols);
    const int streaming = a.rows * a.cols * 2 > LLC_BYTES;
#define MXFP4_LAUNCH_ROWS(R, S)                                                                              \
    hipLaunchKernelGGL((quantize_rows_kernel<HAD, R, S>), dim3(grid), dim3(256), 0, st, a.x, nblocks, bpr, a.ld, \
                       dense, sign_mask, key, a.q, a.s)
    if (a.rounding == RND_RNE) {
        if (streaming) MXFP4_LAUNCH_ROWS(RND_RNE, 1); else MXFP4_LAUNCH_ROWS(RND_RNE, 0);
    } else {
        if (streaming) MXFP4_LAUNCH_ROWS(RND_SR, 1); else MXFP4_LAUNCH_ROWS(RND_SR, 0);
    }
#undef MXFP4_LAUNCH_ROWS
    return hipGetLastError();
}

template <int MODE>
TileJob make_job(const QuantArgs &a)
{
    const int64_t nrb = a.rows / 32;
    TileJob j;
    j.x = a.x; j.rows = a.rows; j.cols = a.cols; j.ld = a.ld;
    j.q = a.q; j.s = a.s; j.q_row = a.q_row; j.s_row = a.s_row;
    // column groups fastest: neighbouring workgroups read neighbouring memory
    j.col_groups = (uint32_t)((a.cols + CT_COLS - 1) / CT_COLS);
    j.nblocks = (uint32_t)(j.col_groups * ((nrb + CT_RB - 1) / CT_RB));
    j.band_rows = j.nblocks < 2048 ? 0u : (MODE == MODE_COLS ? 16u : 2u);
    j.streaming = a.rows * a.cols * 2 > LLC_BYTES;
    j.s_vec8 = ((nrb % 8) == 0) && ((reinterpret_cast<uintptr_t>(a.s) % 8) == 0);
    j.s_row_vec4 = MODE != MODE_COLS && a.s_row != nullptr && (((a.cols / 32) % 4) == 0) &&
                   ((reinterpret_cast<uintptr_t>(a.s_row) % 4) == 0);
    j.key = make_key(a.seed);
    j.key_row = make_key(a.seed_row);
    return j;
}

// b == nullptr: one tensor.  Otherwise both tensors in one launch (same rotation, rounding and base seed).
template <int HAD, int MODE>
hipError_t launch_cols_h(const QuantArgs &a, const QuantArgs *b, hipStream_t st)
{
    const TileJob j0 = make_job<MODE>(a);
    TileJob j1 = j0;
    j1.nblocks = 0;
    if (b) j1 = make_job<MODE>(*b);
    dim3 grid(j0.nblocks + j1.nblocks);
    const uint32_t sign_mask = sign_mask_of(a.seed);
    const bool streaming = j0.streaming && (!b || j1.streaming);  // (two tensors in one launch: only if both want it)
#define MXFP4_LAUNCH_COLS(R, S) \
    hipLaunchKernelGGL((quantize_cols_kernel<HAD, R, MODE, S>), grid, dim3(512), 0, st, j0, j1, sign_mask)
    if (a.rounding == RND_RNE) {
        if (streaming) MXFP4_LAUNCH_COLS(RND_RNE, 1); else MXFP4_LAUNCH_COLS(RND_RNE, 0);
    } else {
        if (streaming) MXFP4_LAUNCH_COLS(RND_SR, 1); else MXFP4_LAUNCH_COLS(RND_SR, 0);
    }
#undef MXFP4_LAUNCH_COLS
    return hipGetLastError();
}

template <int MODE>
hipError_t launch_cols_mode(const QuantArgs &a, const QuantArgs *b, hipStream_t st)
{
    switch (a.hadamard) {
        case HAD_NONE: return launch_cols_h<HAD_NONE, MODE>(a, b, st);
        case HAD_DET: return launch_cols_h<HAD_DET, MODE>(a, b, st);
        case HAD_RANDSIGN: return launch_cols_h<HAD_RANDSIGN, MODE>(a, b, st);
        case HAD_RANDSIGN16: return launch_cols_h<HAD_RANDSIGN16, MODE>(a, b, st);
        default: return launch_cols_h<HAD_DET16, MODE>(a, b, st);
    }
}

}  // namespace

hipError_t launch_quantize_rows(const QuantArgs &a, hipStream_t st)
{
    switch (a.hadamard) {
        case HAD_NONE: return launch_rows_h<HAD_NONE>(a, st);
        case HAD_DET: return launch_rows_h<HAD_DET>(a, st);
        case HAD_RANDSIGN: return launch_rows_h<HAD_RANDSIGN>(a, st);
        case HAD_RANDSIGN16: return launch_rows_h<HAD_RANDSIGN16>(a, st);
        default: return launch_rows_h<HAD_DET16>(a, st);
    }
}

hipError_t launch_quantize_cols(const QuantArgs &a, hipStream_t st, const QuantArgs *b)
{
    return launch_cols_mode<MODE_COLS>(a, b, st);
}

hipError_t launch_quantize_dual(const QuantArgs &a, const QuantArgs *b, hipStream_t st)
{
    return launch_cols_mode<MODE_DUAL>(a, b, st);
}

hipError_t launch_quantize_2d(const QuantArgs &a, const QuantArgs *b, hipStream_t st)
{
    return launch_cols_mode<MODE_2D>(a, b, st);
}

}  // namespace mxfp4
