// Block-scaled FP4 GEMM for gfx950: out[i][j] (+)= sum_c A[i][c] * B[j][c] on MXFP4
// operands (the MXFP4 GEMM of the linear layers, Sec. 1 / App. A.2; operand axes per
// App. C.1-C.3), on the scaled matrix instructions V_MFMA_SCALE_F32_{16X16X128,32X32X64}_F8F6F4.
//
// Register layout of those instructions with FP4 operands (64 lanes, lane = l; n = 16 or 32 rows):
//   first operand : lane l holds row l%n, the 32 K-elements 32*(l/n) .. +31 as 16 bytes
//                   (4 VGPRs), element k in nibble k%32 (low nibble first); its scale VGPR holds
//                   the E8M0 byte of exactly that 32-element block
//   second operand: the same with "row" = output column
//   result        : 16x16: lane l holds column l%16, rows 4*(l/16) + {0..3};
//                   32x32: register e of lane l holds D[8*(e/4) + 4*(l/32) + e%4][l%32]
// i.e. one lane's operand is precisely one MX block of the canonical layout, so the
// canonical q/s arrays feed the instruction without any repacking.
//
// The kernels pass B's rows as the first operand and A's rows as the second: a lane
// then owns 4 consecutive output columns of one output row.
#include <type_traits>

#include "mxfp4_internal.h"

namespace mxfp4 {
namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint16_t f32_to_bf16(float f)
{
    // round to nearest even on the upper 16 bits; NaN keeps a quiet NaN (branch-free)
    const uint32_t u = __float_as_uint(f);
    const uint32_t rounded = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
    const uint32_t nan = (u >> 16) | 0x40u;
    return (uint16_t)(((u & 0x7FFFFFFFu) > 0x7F800000u) ? nan : rounded);
}

// two floats -> two bf16 in one dword (first in the low half), round to nearest even: one
// V_CVT_PK_BF16_F32
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// ---- any-shape kernel --------------------------------------------------------------------
// 256 threads = 2x2 waves, each wave a 32x32 output tile (2x2 instruction tiles); operands
// come straight from global memory.  Rows beyond the matrix are clamped (their results
// are dropped), K blocks beyond C/32 are fed as zeros.
// AF, BF: element format of each operand, 0 = E2M1 (16 bytes per 32-element block), 1 = E4M3 (32 bytes);
// the instruction's format selectors are 4 for E2M1 and 0 for E4M3.
// One lane's operand registers for the 128 K-elements starting at block k (a multiple of 4), lane group kb.
// E2M1: the lane holds block k + kb, 32 consecutive elements in 16 bytes.  E4M3 (probed on the hardware): the
// lane holds elements 16*kb .. +15 and 64 + 16*kb .. +15 of the 128, 16 bytes each, while its scale register
// still belongs to block k + kb.  Blocks at or beyond nkb read as zeros.
template <int F>
__device__ __forceinline__ v8i load_operand(const uint8_t *q, int64_t row, int64_t C, int64_t nkb, int64_t k, int kb)
{
    const v4i zero = {0, 0, 0, 0};
    if (F == 0) {
        const v4i t = (k + kb < nkb) ? *reinterpret_cast<const v4i *>(q + row * (C >> 1) + (k + kb) * 16) : zero;
        return (v8i){t.x, t.y, t.z, t.w, 0, 0, 0, 0};
    }
    const uint8_t *p = q + row * C + k * 32;
    const v4i t0 = (k + (kb >> 1) < nkb) ? *reinterpret_cast<const v4i *>(p + 16 * kb) : zero;
    const v4i t1 = (k + 2 + (kb >> 1) < nkb) ? *reinterpret_cast<const v4i *>(p + 64 + 16 * kb) : zero;
    return (v8i){t0.x, t0.y, t0.z, t0.w, t1.x, t1.y, t1.z, t1.w};
}

template <bool OUT_FP32, bool ACC, int AF, int BF>
__global__ __launch_bounds__(256) void gemm_any_kernel(const uint8_t *__restrict__ aq, const uint8_t *__restrict__ as,
                                                       const uint8_t *__restrict__ bq, const uint8_t *__restrict__ bs,
                                                       int64_t Ra, int64_t Rb, int64_t C, void *__restrict__ out,
                                                       int64_t ld)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l16 = lane & 15, kb = lane >> 4;
    const int64_t row0 = (int64_t)blockIdx.x * 64 + (wave >> 1) * 32;
    const int64_t col0 = (int64_t)blockIdx.y * 64 + (wave & 1) * 32;
    const int64_t nkb = C >> 5;

    int64_t ar[2], br[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        int64_t r = row0 + 16 * t + l16, c = col0 + 16 * t + l16;
        ar[t] = r < Ra ? r : Ra - 1;
        br[t] = c < Rb ? c : Rb - 1;
    }
    v4f acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = (v4f){0.f, 0.f, 0.f, 0.f};

    for (int64_t k = 0; k < nkb; k += 4) {
        const bool kv = k + kb < nkb;
        v8i a[2], b[2];
        int sa[2], sb[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            a[t] = load_operand<AF>(aq, ar[t], C, nkb, k, kb);
            b[t] = load_operand<BF>(bq, br[t], C, nkb, k, kb);
            sa[t] = kv ? as[ar[t] * nkb + k + kb] : 127;
            sb[t] = kv ? bs[br[t] * nkb + k + kb] : 127;
        }
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(b[j], a[i], acc[i][j], BF ? 0 : 4,
                                                                             AF ? 0 : 4, 0, sb[j], 0, sa[i]);
    }

#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int64_t r = row0 + 16 * i + l16;
        if (r >= Ra) continue;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int64_t c = col0 + 16 * j + 4 * kb + e;
                if (c >= Rb) continue;
                float v = acc[i][j][e];
                if (OUT_FP32) {
                    float *o = reinterpret_cast<float *>(out) + r * ld + c;
                    *o = ACC ? (*o + v) : v;
                } else {
                    reinterpret_cast<uint16_t *>(out)[r * ld + c] = f32_to_bf16(v);
                }
            }
        }
    }
}


// ---- tiled kernel: 256 x 256 output tile per workgroup, K consumed in stages of 256 ---------
// 4 waves (2 x 2), each a 128 x 128 sub-tile = 4 x 4 tiles of V_MFMA_SCALE_F32_32X32X64_F8F6F4
// (256 accumulator registers per lane); a narrow variant works on 256 x 128 tiles (sub-tile 128 x 64, 4 x 2
// instruction tiles) with the same data path, see gemm_tile_body.  With FP4 operands that instruction takes, per lane l,
// the 32 K-elements 32*(l/32).. of row l%32 of each operand (one MX block, 16 bytes) and the
// block's scale byte; the result holds, in register e of lane l, D[8*(e/4) + 4*(l/32) + e%4][l%32].
//
// Data path: packed codes go global -> LDS with the direct-to-LDS loads (no registers), one
// instruction per 8 rows x 128 bytes (whole cache lines: the memory pipeline's cost is per
// request, about 0.45 lines per clock and CU, so partial lines are ruinous).  A wave's 64 lanes
// land at consecutive 16-byte LDS slots, so the lane -> (row, 16-byte chunk) choice on the
// global side fixes the LDS layout; chunk c of row r of an 8-row group g sits at slot
// r*8 + (c ^ r ^ (g&1)), which makes every 16-lane quarter of the later 16-byte fragment reads
// hit all 64 banks once.
// Scale bytes: one row has 8 per stage, far too little for a request of its own, so they
// come in batches of 4 stages (32 bytes per row, two lanes per row), double-buffered; the
// four load instructions of the next batch are spread over the four stages of the current one.
// A byte permute puts the 4 scale bytes a lane needs in one stage into one register, from which
// the instruction's byte selector picks the K-step.
// Two LDS stage buffers; fragments are double-buffered in registers across the 4 K-steps.
// Epilogue: every wave transposes its sub-tile through its own LDS slice so that global
// stores are whole 256- or 512-byte row segments.
constexpr int TILE = 256;                       // output tile edge
constexpr int STAGE_K = 256;                    // K elements per stage = 128 bytes per row
constexpr int OP_BYTES = TILE * STAGE_K / 2;    // 32 KiB per operand and stage
constexpr int STAGE_BYTES = 2 * OP_BYTES;       // 64 KiB
constexpr int OFF_A = 0, OFF_B = OP_BYTES;
constexpr int SCALE_BATCH = 4;                  // stages per scale batch
constexpr int SC_OP_BYTES = TILE * 8 * SCALE_BATCH;  // 8 KiB per operand and batch
constexpr int SC_BUF_BYTES = 2 * SC_OP_BYTES;        // 16 KiB
constexpr int OFF_SC = 2 * STAGE_BYTES;              // scale buffers behind the two stage buffers
constexpr int LDS_BYTES = 2 * STAGE_BYTES + 2 * SC_BUF_BYTES;  // 163840 = all of the CU's LDS
constexpr int GROUP_M = 4;                      // tile rows per rasterisation group
constexpr int NUM_CUS = 256;                    // MI355X: 8 XCDs x 32 CUs

typedef float v16f __attribute__((ext_vector_type(16)));

__device__ __forceinline__ void dma16(uint32_t lds_addr, uint32_t voff, const uint8_t *sbase)
{
    // each lane: 16 bytes from sbase + voff to LDS[lds_addr + 16*lane] (the ISA wants one wait state between a
    // scalar write of M0 and a direct-to-LDS load that reads it)
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2\n\t" ::"s"(lds_addr), "v"(voff), "s"(sbase)
                 : "memory");
}

// A run of such loads under one M0: each lane's 16 bytes from sbase + voff + IMM to LDS[M0 + IMM + 16*lane] (the
// instruction's immediate offset moves both addresses; -4096 <= IMM < 4096).  Only the first load of a run
// (SETM0) writes M0 = lds_base.
template <int IMM, bool SETM0>
__device__ __forceinline__ void dma16_run(uint32_t lds_base, uint32_t voff, const uint8_t *sbase)
{
    static_assert(IMM >= -4096 && IMM < 4096, "13-bit signed instruction offset");
    if (SETM0)
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 offset:%3\n\t" ::"s"(lds_base),
                     "v"(voff), "s"(sbase), "n"(IMM)
                     : "memory");
    else
        asm volatile("global_load_lds_dwordx4 %0, %1 offset:%2\n\t" ::"v"(voff), "s"(sbase), "n"(IMM) : "memory");
}

template <int V>
using IC = std::integral_constant<int, V>;

// Operand rows one wave loads for one tile: rows wave*64 .. +63 of the tile's A rows, B rows and
// of their scale rows.
struct TileSrc {
    const uint8_t *a, *b, *as, *bs;
    int64_t m0, n0;
};

// The whole tiled GEMM as seen by one workgroup: `wg` of `nwg` workgroups share the problem (the ids are
// virtual: a launch may run two problems side by side on disjoint sets of CUs).  smem: the workgroup's
// LDS_BYTES of LDS, lds0 its LDS address.
// FMT: element format of both operands.  0 = E2M1: a stage (128 bytes per row) holds 256 K-elements = 4
// instruction K-steps, one fragment (16 bytes per lane) each.  1 = E4M3: a stage holds 128 K-elements = 2
// instruction K-steps of 32 bytes per lane.  The instruction wants, from lane group h, the elements 16h .. +15
// and 32 + 16h .. +15 of its 64 (probed), which are exactly the two 16-byte fragments the E2M1 path fetches
// for its K-steps 2j and 2j+1: so data movement, LDS layout and fragment reads are the same for both formats,
// and only the matrix instructions differ (16 per two phases instead of 16 per phase, taking two fragments).
// NJ: 32-column groups of a wave's sub-tile.  4: the 256 x 256 tile (wave sub-tile 128 x 128, 16 matrix
// instructions per K-step).  2 (E2M1 only): a 256 x 128 tile (sub-tile 128 x 64, 8 instructions per K-step) for
// outputs that have too few 256 x 256 tiles to fill the chip, and for the part-filled last round of others;
// it moves 1.5 times the operand bytes per flop, so it is only used where compute units would idle otherwise.
// l_lo, l_hi: the body works on tiles l_lo .. l_hi-1 of the tile sequence only (l_hi < 0: all of them).
// HALVES (narrow tile only): tiles_n and the sequence are those of the 256 x 256 grid, and every one of those
// tiles is worked on as two 256 x 128 tiles, left half then right half: the part-filled last round of a launch
// that ran its whole rounds on 256 x 256 tiles.
template <bool OUT_FP32, bool ACC, int FMT, int NJ, bool HALVES = false>
__device__ __forceinline__ void gemm_tile_body(const uint8_t *__restrict__ aq, const uint8_t *__restrict__ as,
                                               const uint8_t *__restrict__ bq, const uint8_t *__restrict__ bs,
                                               int64_t C, void *__restrict__ out, int64_t ld, int tiles_m,
                                               int tiles_n, const uint32_t wg, const uint32_t nwg,
                                               uint8_t *const smem, const uint32_t lds0, const int l_lo = 0,
                                               const int l_hi = -1)
{
    static_assert(!HALVES || NJ == 2, "only the narrow tile works on halves of 256 x 256 tiles");

    static_assert(NJ == 4 || (NJ == 2 && FMT == 0), "the narrow tile is built for E2M1 operands only");
    constexpr int TILE_N = 64 * NJ;          // B rows (output columns) per tile
    constexpr int BROWS = TILE_N / 4;        // B rows one wave loads per stage: 64 or 32
    constexpr int NLOADS = 8 + BROWS / 8;    // direct-to-LDS loads per wave and stage: 16 or 12
    constexpr int NSLOT = 4 * NJ;            // matrix instructions per K-step
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int64_t rowbytes = FMT ? C : (C >> 1), nkb = C >> 5;
    const int nstages = (int)(rowbytes / (STAGE_K / 2));  // >= 4 (E2M1) or >= 8 (E4M3): the host checks
    constexpr int BATCH = FMT ? 8 : 4;   // stages per scale batch (32 scale bytes per row)
    constexpr int SC_STAGE = FMT ? 4 : 8;  // scale bytes per row and stage

    // ---- persistent tile schedule -----------------------------------------------------------
    // Workgroup ids are dealt round-robin to the 8 XCDs (each with its own L2).  XCD x owns a
    // contiguous run of the tile sequence; its workgroups walk that run with a stride equal to
    // their number, so the tiles in flight on one XCD are consecutive in the sequence, and the
    // sequence goes through the tile grid in groups of GROUP_M tile rows: those tiles share
    // A and B panels in the XCD's L2.
    const int T = ((l_hi < 0 ? tiles_m * tiles_n : l_hi) - l_lo) * (HALVES ? 2 : 1), G = (int)nwg;
    const int xcd = wg & 7, lw = wg >> 3;
    const int nwg_x = (G - xcd + 7) >> 3;                      // workgroups living on this XCD
    const int per = T >> 3, rem = T & 7;
    const int count_x = per + (xcd < rem ? 1 : 0);             // tiles owned by this XCD
    const int start_x = xcd < rem ? xcd * (per + 1) : rem * (per + 1) + (xcd - rem) * per;
    auto tile_src = [&](int lloc) {
        const int Lr = start_x + lloc;                       // position in this body's range
        const int L = l_lo + (HALVES ? (Lr >> 1) : Lr);      // position in the tile sequence
        const int span = GROUP_M * tiles_n, grp = L / span, first = grp * GROUP_M;
        const int gm = (tiles_m - first) < GROUP_M ? (tiles_m - first) : GROUP_M;
        const int in = L - grp * span;
        TileSrc t;
        t.m0 = (int64_t)(first + in % gm) * TILE;
        t.n0 = HALVES ? (int64_t)(in / gm) * TILE + (Lr & 1) * TILE_N : (int64_t)(in / gm) * TILE_N;
        t.a = aq + (t.m0 + wave * 64) * rowbytes;
        t.b = bq + (t.n0 + wave * BROWS) * rowbytes;
        t.as = as + (t.m0 + wave * 64) * nkb;
        t.bs = bs + (t.n0 + wave * BROWS) * nkb;
        return t;
    };
    if (lw >= count_x) return;  // (whole workgroup: nothing to do)

    // ---- direct-to-LDS loads: per-lane offsets (fixed for the whole kernel) -----------------
    // dvo[g]: this lane's 16 bytes of 8-row group g of the wave's 64 rows (row 8g + lane/8; the chunk within
    // the row's 128 bytes is swizzled by the row, odd groups one further)
    const int drr = lane >> 3, dcc = lane & 7;
    uint32_t dvo[8];
#pragma unroll
    for (int g = 0; g < 8; ++g)  // (less the immediate offset (g - 4) KiB the load instruction adds back)
        dvo[g] = (uint32_t)((8 * g + drr) * rowbytes) + (uint32_t)((dcc ^ drr ^ (g & 1)) << 4) - (uint32_t)((g - 4) * 1024);
    // the wave's 8 x 1 KiB of A's stage slice and 8 (narrow tile: 4) x 1 KiB of B's
    const uint32_t lds_wave_a = lds0 + OFF_A + (uint32_t)wave * 8192u;
    const uint32_t lds_wave_b = lds0 + OFF_B + (uint32_t)wave * (uint32_t)(BROWS * 128);
    const uint32_t svoff = (uint32_t)((lane >> 1) * nkb) + (uint32_t)((lane & 1) << 4);

    // load n (0..15) of stage s of tile t for this wave, in issue order: n = 0..3 A's 8-row groups 0..3,
    // 4..7 B's groups 0..3, 8..11 A's groups 4..7, 12..15 B's groups 4..7 (the narrow tile has no 12..15: a
    // wave loads only 32 rows of B).  The four loads of a run share one M0
    // (the LDS address of the operand's group 4; the groups sit at immediate offsets (g - 4) KiB from it);
    // `force` makes a load set M0 itself (where scale loads, which set their own, are issued in between).
    auto issue_load = [&](const TileSrc &t, int s, int buf, auto nc, auto force) {
        constexpr int n = decltype(nc)::value, op = (n >> 2) & 1, g = (n >> 3) * 4 + (n & 3);
        static_assert(n < NLOADS, "no such load for this tile shape");
        constexpr bool setm0 = decltype(force)::value || (n & 3) == 0;
        const int64_t koff = (int64_t)s * (STAGE_K / 2);
        dma16_run<(g - 4) * 1024, setm0>((op ? lds_wave_b : lds_wave_a) + buf * STAGE_BYTES + 4096, dvo[g],
                                         (op ? t.b : t.a) + koff);
    };
    using no_force = std::false_type;
    using force_m0 = std::true_type;
    // Scale batch b holds the 32 scale bytes per row of stages first(b) .. first(b)+3, where
    // first(b) = min(4b, nstages-4): the last batch is pulled back so that it never reads past a
    // row's end (batches past the end of K just repeat the last one into the idle buffer).
    auto batch_first = [&](int b) { return (BATCH * b < nstages - BATCH) ? BATCH * b : nstages - BATCH; };
    // instruction j (0..3) of batch b for this wave: j>>1 = operand, j&1 = which 32 of its 64 rows
    // Batch b of a tile lives in scale buffer (b ^ par) & 1; par alternates between tiles so that
    // a tile's first batch never lands in the buffer its predecessor's last batch is still read from.
    // (narrow tile: a wave has only 32 rows of B, so instruction 3 repeats instruction 2: the same bytes to the
    // same place, which keeps the stage bodies free of branches)
    auto scales_dst = [&](int b, int j, int par) {
        if (NJ == 2 && j == 3) j = 2;
        const int rows0 = (j >> 1) ? wave * BROWS : wave * 64;
        return lds0 + OFF_SC + ((b ^ par) & 1) * SC_BUF_BYTES + (j >> 1) * SC_OP_BYTES + (rows0 + (j & 1) * 32) * 32;
    };
    auto scales_src = [&](const TileSrc &t, int b, int j) {
        if (NJ == 2 && j == 3) j = 2;
        return ((j >> 1) ? t.bs : t.as) + (int64_t)(j & 1) * 32 * nkb + batch_first(b) * SC_STAGE;
    };
    auto issue_scales = [&](const TileSrc &t, int b, int j, int par) {
        dma16(scales_dst(b, j, par), svoff, scales_src(t, b, j));
    };

    // ---- fragment reads: per-lane offsets ---------------------------------------------------
    const int fr = lane & 31, fh = lane >> 5;
    const int fm = (fr & 7) ^ ((fr >> 3) & 1);
    const uint32_t fl0 = (uint32_t)((fr >> 3) * 1024 + (fr & 7) * 128);
    uint32_t foff[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) foff[kk] = fl0 + (uint32_t)((((kk << 1) | fh) ^ fm) << 4);
    const uint32_t a_frag0 = OFF_A + wm * 16 * 1024, b_frag0 = OFF_B + wn * (NJ * 4) * 1024;
    const uint32_t sa_frag0 = OFF_SC + (wm * 128 + fr) * 32;
    const uint32_t sb_frag0 = OFF_SC + SC_OP_BYTES + (wn * (32 * NJ) + fr) * 32;
    // scale bytes of one stage -> one register whose byte k is the lane's block in instruction K-step k
    const uint32_t perm_sel = FMT ? (fh ? 0x03010301u : 0x02000200u) : (fh ? 0x07050301u : 0x06040200u);

    v4i fa[FMT ? 4 : 2][4], fb[FMT ? 4 : 2][4];
    uint2 sraw[8];
    int sa_cur[4], sb_cur[4];
    // One fragment fetch (f = 0..7: A0,B0,A1,B1,...) of K-step kk of buffer buf into register set `set`.
    auto read_one = [&](int buf, int kk, int set, int f) {
        const uint8_t *p = smem + buf * STAGE_BYTES + foff[kk] + (f >> 1) * 4096;
        if (f & 1)
            fb[set][f >> 1] = *reinterpret_cast<const v4i *>(p + b_frag0);
        else
            fa[set][f >> 1] = *reinterpret_cast<const v4i *>(p + a_frag0);
    };
    // The 8 scale bytes of stage s for fragment row f (0..7: A0,B0,A1,B1,...), raw.
    auto read_scale_one = [&](int s, int f, int par) {
        const int b = s / BATCH;
        const uint8_t *p = smem + ((b ^ par) & 1) * SC_BUF_BYTES + (s - batch_first(b)) * SC_STAGE + (f >> 1) * 1024;
        if (FMT)
            sraw[f] = make_uint2(*reinterpret_cast<const uint32_t *>(p + ((f & 1) ? sb_frag0 : sa_frag0)), 0u);
        else
            sraw[f] = *reinterpret_cast<const uint2 *>(p + ((f & 1) ? sb_frag0 : sa_frag0));
    };
    // raw scale bytes -> one register per fragment row whose bytes are K blocks fh, 2+fh, 4+fh, 6+fh
    auto permute_scales = [&]() {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            sa_cur[i] = (int)__builtin_amdgcn_perm(sraw[2 * i].y, sraw[2 * i].x, perm_sel);
            if (i < NJ) sb_cur[i] = (int)__builtin_amdgcn_perm(sraw[2 * i + 1].y, sraw[2 * i + 1].x, perm_sel);
        }
    };

    // Stage s of a tile lives in stage buffer (s & 1) ^ bp.  The hand-over loads put the next tile's stage 0
    // into the buffer after the current tile's last one, so with an odd number of stages the parity flips
    // from tile to tile.
    int bp = 0;
    v16f acc[4][4];
    const v16f zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

    // One matrix instruction: tile (n/4, n%4) of the wave's 4 x 4, fragments from register set SET,
    // K-step KK selects the scale byte.
#define MXFP4_MMA(SET, KK, N, FRESH)                                                                            \
    {                                                                                                           \
        constexpr int i_ = (N) / NJ, j_ = (N) % NJ;                                                             \
        v8i fb8 = {fb[SET][j_].x, fb[SET][j_].y, fb[SET][j_].z, fb[SET][j_].w, 0, 0, 0, 0};                     \
        v8i fa8 = {fa[SET][i_].x, fa[SET][i_].y, fa[SET][i_].z, fa[SET][i_].w, 0, 0, 0, 0};                     \
        acc[i_][j_] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fb8, fa8, (FRESH) ? zero16 : acc[i_][j_], \
                                                                      4, 4, KK, sb_cur[j_], KK, sa_cur[i_]);    \
    }
    // E4M3: instruction n (0..15) of instruction K-step KS (0/1): fragments 2*KS (low half) and 2*KS+1
#define MXFP8_MMA(KS, N, FRESH)                                                                                 \
    {                                                                                                           \
        constexpr int i_ = (N) >> 2, j_ = (N) & 3;                                                              \
        v8i fb8 = {fb[2 * (KS)][j_].x, fb[2 * (KS)][j_].y, fb[2 * (KS)][j_].z, fb[2 * (KS)][j_].w,              \
                   fb[2 * (KS) + 1][j_].x, fb[2 * (KS) + 1][j_].y, fb[2 * (KS) + 1][j_].z, fb[2 * (KS) + 1][j_].w}; \
        v8i fa8 = {fa[2 * (KS)][i_].x, fa[2 * (KS)][i_].y, fa[2 * (KS)][i_].z, fa[2 * (KS)][i_].w,              \
                   fa[2 * (KS) + 1][i_].x, fa[2 * (KS) + 1][i_].y, fa[2 * (KS) + 1][i_].z, fa[2 * (KS) + 1][i_].w}; \
        acc[i_][j_] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fb8, fa8, (FRESH) ? zero16 : acc[i_][j_], \
                                                                      0, 0, KS, sb_cur[j_], KS, sa_cur[i_]);    \
    }
    // phase P (0..3) of a stage, slot N (0..15): E2M1 issues instruction N of K-step P; E4M3 issues, in even
    // slots, instruction N/2 (+8 in odd phases) of K-step P/2
#define MXFP4_SLOT_MMA(P, N, FRESH)                                                                             \
    if constexpr (FMT == 0) {                                                                                   \
        if constexpr ((N) < NSLOT) {                                                                            \
            MXFP4_MMA((P) & 1, P, N, FRESH)                                                                     \
        }                                                                                                       \
    } else if constexpr (((N) & 1) == 0) {                                                                      \
        MXFP8_MMA((P) >> 1, ((N) >> 1) + 8 * ((P) & 1), FRESH)                                                  \
    }
#define MXFP4_PIN() __builtin_amdgcn_sched_barrier(0);
    // E2M1: the 8 fragment reads of a K-step go into the even slots, B0..B3 then A0..A3 (instruction n of the
    // next K-step needs A[n/4] and B[n%4]: every fragment is at least 8 slots old when first used), so that LDS
    // reads alternate with the direct-to-LDS loads of the odd slots instead of arriving in bursts.
    // Narrow tile (8 slots per K-step): the 6 fragment reads go into slots 0..5, B0, B1, then A0..A3 (instruction
    // n needs A[n/2] and B[n%2]); the loads take the odd slots of K-step 0 and every slot of K-step 3.
#define MXFP4_FRAG_SLOT(N) (!FMT && (NJ == 4 ? ((N) & 1) == 0 : (N) < 6))
#define MXFP4_FRAG_OF(N)                                                                       \
    (NJ == 4 ? (((N) >> 1) < 4 ? 2 * ((N) >> 1) + 1 : 2 * (((N) >> 1) - 4)) : ((N) < 2 ? 2 * (N) + 1 : 2 * ((N)-2)))
    // load slots of K-step 0 (second half of a stage's loads: 8, 9, ...) and of K-step 3 (first half: 0..7)
    // (the ..._OF values are clamped to an existing load where the slot has none: the call is discarded there, but
    // the compiler still instantiates it)
#define MXFP4_LOAD0_SLOT(N) (((N) & 1) && 8 + ((N) >> 1) < NLOADS)
#define MXFP4_LOAD0_OF(N) (8 + ((N) >> 1) < NLOADS ? 8 + ((N) >> 1) : 8)
#define MXFP4_LOAD3_SLOT(N) (NJ == 4 ? ((N) & 1) : (N) < 8)
#define MXFP4_LOAD3_OF(N) (NJ == 4 ? ((N) >> 1) : ((N) < 8 ? (N) : 0))
#define MXFP4_16(M) M(0) M(1) M(2) M(3) M(4) M(5) M(6) M(7) M(8) M(9) M(10) M(11) M(12) M(13) M(14) M(15)

    // One stage = 4 K-steps of 16 (narrow tile: 8) matrix instructions.  Everything else is threaded between them,
    // one item per matrix instruction, and pinned there with scheduling barriers: with a single
    // wave per SIMD any stall of the wave (a burst of loads filling the memory pipeline's queue,
    // a late fragment) idles the matrix unit, so loads are issued a few at a time.
    //   K-step 0: fragments of K-step 1; second half of the next stage's direct-to-LDS loads
    //   K-step 1: fragments of K-step 2           K-step 2: fragments of K-step 3
    //   barrier (this stage's buffer is free, the next stage has landed)
    //   K-step 3: fragments + scales of the next stage's K-step 0; first half of the loads of
    //             the stage after next, into the buffer just freed; one scale load
    // The main loop's body must stay one basic block (no data-dependent branches), or the matrix
    // instructions get sunk behind the branches; so the last two stages of a tile, which hand
    // over to the next tile, are separate instantiations (MODE 1 and 2).
    //   MODE 3: stage 0: as MODE 0, and its first K-step starts the accumulators from zero
    //   MODE 0: stage 1 <= s <= nstages-3 of tile `cur`
    //   MODE 1: stage nstages-2: its K-step 3 starts loading stage 0 and scale batch 0 of tile `nxt`
    //   MODE 2: stage nstages-1: its K-step 0 finishes stage 0; K-step 3 issues the first load of
    //           nxt's scale batch 1 and fetches nothing (the epilogue follows)
    auto stage = [&](const TileSrc &cur, const TileSrc &nxt, int par, int par_nxt, int s, auto mode) {
        constexpr int MODE = decltype(mode)::value;
        const int buf = (s & 1) ^ bp;
        // destination and source of the stage's one scale load: worked out in idle slots of K-step 1, used
        // in K-step 3
        uint32_t sc_dst = 0;
        const uint8_t *sc_src = nullptr;
#define MXFP4_K0(N)                                                                              \
        if (FMT && (N) < 8) read_one(buf, 2, 2, (N));                                            \
        if (MXFP4_FRAG_SLOT(N)) read_one(buf, 1, 1, MXFP4_FRAG_OF(N));                           \
        if constexpr (MODE != 2 && MXFP4_LOAD0_SLOT(N)) issue_load(cur, s + 1, buf ^ 1, IC<MXFP4_LOAD0_OF(N)>{}, no_force{}); \
        if constexpr (MODE == 2 && MXFP4_LOAD0_SLOT(N)) issue_load(nxt, 0, buf ^ 1, IC<MXFP4_LOAD0_OF(N)>{}, no_force{});     \
        MXFP4_SLOT_MMA(0, N, MODE == 3) MXFP4_PIN()
        MXFP4_16(MXFP4_K0)
#undef MXFP4_K0
#define MXFP4_K1(N)                                                                              \
        if (FMT && (N) < 8) read_one(buf, 3, 3, (N));                                            \
        if (MXFP4_FRAG_SLOT(N)) read_one(buf, 2, 0, MXFP4_FRAG_OF(N));                           \
        if ((MODE == 0 || MODE == 3) && (N) == (NJ == 4 ? 9 : 4)) {                              \
            sc_dst = scales_dst((s + 1) / BATCH + 1, (s + 1) & 3, par);                          \
            asm volatile("" : "+s"(sc_dst));                                                     \
        }                                                                                        \
        if ((MODE == 0 || MODE == 3) && (N) == (NJ == 4 ? 12 : 6)) {                             \
            sc_src = scales_src(cur, (s + 1) / BATCH + 1, (s + 1) & 3);                          \
            asm volatile("" : "+s"(sc_src));                                                     \
        }                                                                                        \
        MXFP4_SLOT_MMA(1, N, FMT && MODE == 3) MXFP4_PIN()
        MXFP4_16(MXFP4_K1)
#undef MXFP4_K1
#define MXFP4_K2(N)                                                                              \
        if (!FMT && NJ == 4 && (N) < 8) read_one(buf, 3, 1, (N)); /* (early: the barrier below waits for them) */ \
        if (NJ == 2 && MXFP4_FRAG_SLOT(N)) read_one(buf, 3, 1, MXFP4_FRAG_OF(N));                \
        MXFP4_SLOT_MMA(2, N, false) MXFP4_PIN()
        MXFP4_16(MXFP4_K2)
#undef MXFP4_K2
        // every wave has fetched its last fragments of this buffer, and this wave's loads of the
        // next stage have landed: after the barrier the buffer may be refilled and the other read
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
#define MXFP4_K3(N)                                                                              \
        if (FMT && MODE != 2 && (N) < 8) read_one(buf ^ 1, 0, 0, (N));                            \
        if (MODE != 2 && MXFP4_FRAG_SLOT(N)) read_one(buf ^ 1, 0, 0, MXFP4_FRAG_OF(N));           \
        if (FMT && MODE != 2 && (N) < 8) read_one(buf ^ 1, 1, 1, (N));                            \
        if (MODE != 2 && NJ == 4 && (N) < 8) read_scale_one(s + 1, (N), par);                     \
        if (MODE != 2 && NJ == 2 && (N) < 6) read_scale_one(s + 1, MXFP4_FRAG_OF(N), par);        \
        if ((MODE == 0 || MODE == 3) && (N) == 0) dma16(sc_dst, svoff, sc_src);                  \
        if constexpr ((MODE == 0 || MODE == 3) && MXFP4_LOAD3_SLOT(N))                           \
            issue_load(cur, s + 2, buf, IC<MXFP4_LOAD3_OF(N)>{}, no_force{});                    \
        if (MODE != 2 && NJ == 4 && (N) == 13) __builtin_amdgcn_s_waitcnt(FMT ? 0xC07F : 0xC37F); /* lgkmcnt(0 / 3): see below */ \
        if (MODE != 2 && NJ == 2 && (N) == 6) __builtin_amdgcn_s_waitcnt(0xC07F); /* lgkmcnt(0) */ \
        if constexpr (MODE == 1 && MXFP4_LOAD3_SLOT(N))                                          \
            issue_load(nxt, 0, buf, IC<MXFP4_LOAD3_OF(N)>{}, force_m0{});                        \
        if (MODE == 1 && !((N) & 1) && (N) < 2 * (NJ == 4 ? 4 : 3)) issue_scales(nxt, 0, (N) >> 1, par_nxt); \
        if (MODE == 2 && (N) == 1) issue_scales(nxt, 1, 0, par_nxt);                             \
        MXFP4_SLOT_MMA(3, N, false) MXFP4_PIN()
        MXFP4_16(MXFP4_K3)
#undef MXFP4_K3
        // (the scale bytes were fetched in the first half of K-step 3 and have long landed: the explicit wait
        // in slot 13 -- for everything but the E2M1 schedule's three younger fragment reads -- tells the compiler
        // so, which otherwise puts a counter wait in front of every permute)
        if (MODE != 2) permute_scales();
    };
    using mode_main = std::integral_constant<int, 0>;
    using mode_penult = std::integral_constant<int, 1>;
    using mode_last = std::integral_constant<int, 2>;
    using mode_first = std::integral_constant<int, 3>;

    // ---- first tile: fill the pipeline --------------------------------------------------------
    // all of stage 0, the first 8 loads of stage 1, scale batch 0 and the first load of batch 1
    TileSrc cur = tile_src(lw);
#define MXFP4_FILL(N) if constexpr ((N) < NLOADS) issue_load(cur, 0, 0, IC<((N) < NLOADS ? (N) : 0)>{}, no_force{});
    MXFP4_16(MXFP4_FILL)
#undef MXFP4_FILL
#pragma unroll
    for (int j = 0; j < (NJ == 4 ? 4 : 3); ++j) issue_scales(cur, 0, j, 0);
    issue_scales(cur, 1, 0, 0);
    int par = 0;
    const int b_last = (nstages - 1) / BATCH;

    for (int lloc = lw; lloc < count_x; lloc += nwg_x) {
        const int par_nxt = (b_last ^ par ^ 1) & 1;
        // the tile after this one; after the last tile the hand-over loads simply fetch that tile's
        // first stage again into buffers that are idle by then (no branches in the stage bodies)
        const TileSrc nxt = (lloc + nwg_x < count_x) ? tile_src(lloc + nwg_x) : cur;
        // entering a tile: its stage 0 and first scale batch have landed (first tile: wait for them
        // here); after the barrier start stage 1's first half and fetch the first fragments
        if (lloc == lw) asm volatile("s_waitcnt vmcnt(1)" ::: "memory");  // (later tiles waited before the epilogue)
        __syncthreads();
#define MXFP4_FILL(N) if constexpr ((N) < 8) issue_load(cur, 1, bp ^ 1, IC<((N) & 7)>{}, no_force{});
        MXFP4_16(MXFP4_FILL)
#undef MXFP4_FILL
#pragma unroll
        for (int f = 0; f < 8; ++f) {
            if ((f & 1) && (f >> 1) >= NJ) continue;  // (narrow tile: two B fragments only)
            read_one(bp, 0, 0, f);
            if (FMT) read_one(bp, 1, 1, f);
            read_scale_one(0, f, par);
        }
        permute_scales();

        stage(cur, nxt, par, par_nxt, 0, mode_first{});
        for (int s = 1; s + 2 < nstages; ++s) stage(cur, nxt, par, par_nxt, s, mode_main{});
        stage(cur, nxt, par, par_nxt, nstages - 2, mode_penult{});
        stage(cur, nxt, par, par_nxt, nstages - 1, mode_last{});
        __builtin_amdgcn_sched_barrier(0);
        // the next tile's stage 0 and scale batch 0 have been on their way for at least two K-steps: make
        // sure they have landed now, before any store is issued (only the one scale load of batch 1 issued
        // a moment ago may stay out), so that nothing later has to wait for the stores to drain
        asm volatile("s_waitcnt vmcnt(1)" ::: "memory");

        // ---- epilogue ---------------------------------------------------------------------------
        // The output is stored non-temporally: it is not read again here, and written the ordinary way it
        // pushes the operands of the kernels that follow (the next quantisers, the next GEMM) out of the
        // last-level cache -- measured on the 8B fused-QKV layer: 10 % of a whole forward + backward step.
        // A lane owns row fr of each 32-row group and, per 32-column group, columns 8*q + 4*fh + {0..3}.
        // The last stage's buffer is free (all waves passed the last barrier; the other one may already hold
        // the next tile's stage 0): each wave transposes its sub-tile through its own 16 KiB slice of it, 64
        // (bf16) or 32 (fp32) rows at a time, and writes whole 256- / 512-byte row segments.  Rows are
        // stored unpadded; 16-byte chunk c of row r sits at chunk c ^ (r & 15) (bf16: and its two 8-byte
        // halves swap when r & 16), which keeps both the 8/16-byte writes and the 16-byte reads
        // conflict-free.
        uint8_t *epi = smem + ((((nstages - 1) & 1) ^ bp) ? STAGE_BYTES : 0) + wave * 16384;
        const int64_t row0 = cur.m0 + wm * 128, col0 = cur.n0 + wn * (32 * NJ);
        if constexpr (NJ == 2 && !OUT_FP32) {
            // Narrow tile, bf16: the wave's 128 rows x 64 columns are 16 KiB, one pass.  A row is 8 chunks of 16
            // bytes; chunk c of row r sits at position c ^ ((r >> 1) & 7): the 8-byte writes of a quarter wave
            // (16 rows, one chunk) and the 16-byte reads (2 rows x 8 chunks) then cover all banks evenly.
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                    for (int qd = 0; qd < 4; ++qd) {
                        const int r = i * 32 + fr, c = j * 4 + qd;
                        uint2 pk;
                        pk.x = pack_bf16(acc[i][j][4 * qd + 0], acc[i][j][4 * qd + 1]);
                        pk.y = pack_bf16(acc[i][j][4 * qd + 2], acc[i][j][4 * qd + 3]);
                        *reinterpret_cast<uint2 *>(epi + r * 128 + ((c ^ ((r >> 1) & 7)) << 4) + (fh << 3)) = pk;
                        if (qd == 3) __builtin_amdgcn_sched_barrier(0);
                    }
            // 8 lanes x 16 bytes = one 128-byte row segment; 8 rows per instruction
            const int rl = lane >> 3, ch = lane & 7;
            uint16_t *obase = reinterpret_cast<uint16_t *>(out) + (row0 + rl) * ld + col0 + ch * 8;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                v4i buf[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int r = (8 * h + u) * 8 + rl;
                    buf[u] = *reinterpret_cast<const v4i *>(epi + r * 128 + ((ch ^ ((r >> 1) & 7)) << 4));
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    __builtin_nontemporal_store(buf[u], reinterpret_cast<v4i *>(obase + (int64_t)((8 * h + u) * 8) * ld));
                __builtin_amdgcn_sched_barrier(0);
            }
        } else if constexpr (NJ == 2) {
            // Narrow tile, fp32: 128 rows x 256 bytes in two passes of 64 rows; chunk c (4 columns) of row r at
            // position c ^ (r & 15)
#pragma unroll
            for (int pass = 0; pass < 2; ++pass) {
#pragma unroll
                for (int ii = 0; ii < 2; ++ii)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
#pragma unroll
                        for (int qd = 0; qd < 4; ++qd) {
                            const int i = 2 * pass + ii;
                            const int r = ii * 32 + fr, c = j * 8 + qd * 2 + fh;
                            *reinterpret_cast<v4f *>(epi + r * 256 + ((c ^ (r & 15)) << 4)) =
                                (v4f){acc[i][j][4 * qd + 0], acc[i][j][4 * qd + 1], acc[i][j][4 * qd + 2],
                                      acc[i][j][4 * qd + 3]};
                            if (qd == 3) __builtin_amdgcn_sched_barrier(0);
                        }
                // 16 lanes x 16 bytes = one 256-byte row segment; 4 rows per instruction
                const int rl = lane >> 4, ch = lane & 15;
                float *obase = reinterpret_cast<float *>(out) + (row0 + pass * 64 + rl) * ld + col0 + ch * 4;
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    v4f buf[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const int r = (8 * h + u) * 4 + rl;
                        buf[u] = *reinterpret_cast<const v4f *>(epi + r * 256 + ((ch ^ (r & 15)) << 4));
                    }
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        v4f *o = reinterpret_cast<v4f *>(obase + (int64_t)((8 * h + u) * 4) * ld);
                        v4f v = buf[u];
                        if (ACC) v += *o;
                        __builtin_nontemporal_store(v, o);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        } else if constexpr (!OUT_FP32) {
#pragma unroll
            for (int pass = 0; pass < 2; ++pass) {
#pragma unroll
                for (int ii = 0; ii < 2; ++ii)
#pragma unroll
                    for (int j = 0; j < 4; ++j)
#pragma unroll
                        for (int qd = 0; qd < 4; ++qd) {
                            const int i = 2 * pass + ii;
                            const int r = ii * 32 + fr, c = j * 4 + qd;
                            uint2 pk;
                            pk.x = pack_bf16(acc[i][j][4 * qd + 0], acc[i][j][4 * qd + 1]);
                            pk.y = pack_bf16(acc[i][j][4 * qd + 2], acc[i][j][4 * qd + 3]);
                            *reinterpret_cast<uint2 *>(epi + r * 256 + ((c ^ (r & 15)) << 4) +
                                                       ((fh ^ ((r >> 4) & 1)) << 3)) = pk;
                            if (qd == 3) __builtin_amdgcn_sched_barrier(0);  // one 32x32 tile at a time
                        }
                // 16 lanes x 16 bytes = one 256-byte row segment; 4 rows per instruction.  Eight LDS reads are
                // issued before the first store needs its data, so their latencies overlap; the row pointer
                // is one per-lane base plus a scalar multiple of the leading dimension.
                const int rl = lane >> 4, ch = lane & 15;
                uint32_t roff[4];  // LDS offset of this lane's chunk in rows rl, 4 + rl, 8 + rl, 12 + rl
#pragma unroll
                for (int k = 0; k < 4; ++k) roff[k] = (uint32_t)((4 * k + rl) * 256 + ((ch ^ (4 * k + rl)) << 4));
                uint16_t *obase = reinterpret_cast<uint16_t *>(out) + (row0 + pass * 64 + rl) * ld + col0 + ch * 8;
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    v4i buf[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const int r4 = (8 * h + u) * 4;
                        buf[u] = *reinterpret_cast<const v4i *>(epi + (r4 & ~15) * 256 + roff[(r4 >> 2) & 3]);
                    }
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const int r4 = (8 * h + u) * 4;
                        v4i v = buf[u];
                        if ((r4 >> 4) & 1) v = (v4i){v.z, v.w, v.x, v.y};
                        __builtin_nontemporal_store(v, reinterpret_cast<v4i *>(obase + (int64_t)r4 * ld));
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        } else {
#pragma unroll
            for (int pass = 0; pass < 4; ++pass) {
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int qd = 0; qd < 4; ++qd) {
                        const int c = j * 8 + qd * 2 + fh;
                        *reinterpret_cast<v4f *>(epi + fr * 512 + ((c ^ fr) << 4)) =
                            (v4f){acc[pass][j][4 * qd + 0], acc[pass][j][4 * qd + 1], acc[pass][j][4 * qd + 2],
                                  acc[pass][j][4 * qd + 3]};
                        if (qd == 3) __builtin_amdgcn_sched_barrier(0);
                    }
                // 32 lanes x 16 bytes = one 512-byte row segment; 2 rows per instruction; reads batched by
                // eight as above
                const int rl = lane >> 5, ch = lane & 31;
                float *obase = reinterpret_cast<float *>(out) + (row0 + pass * 32 + rl) * ld + col0 + ch * 4;
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    v4f buf[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const int r = (8 * h + u) * 2 + rl;
                        buf[u] = *reinterpret_cast<const v4f *>(epi + r * 512 + ((ch ^ r) << 4));
                    }
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        v4f *o = reinterpret_cast<v4f *>(obase + (int64_t)((8 * h + u) * 2) * ld);
                        v4f v = buf[u];
                        if (ACC) v += *o;
                        __builtin_nontemporal_store(v, o);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
        // (the barrier at the top of the loop keeps the next tile's loads out of that buffer until
        // every wave is done reading its slice)
        cur = nxt;
        par = par_nxt;
        bp ^= nstages & 1;
    }
    // nothing may still be writing this workgroup's LDS when it retires
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#undef MXFP4_MMA
#undef MXFP8_MMA
#undef MXFP4_SLOT_MMA
#undef MXFP4_PIN
#undef MXFP4_16
#undef MXFP4_FRAG_SLOT
#undef MXFP4_FRAG_OF
#undef MXFP4_LOAD0_SLOT
#undef MXFP4_LOAD0_OF
#undef MXFP4_LOAD3_SLOT
#undef MXFP4_LOAD3_OF
}

struct TileGemm {
    const uint8_t *aq, *as, *bq, *bs;
    int64_t C;
    void *out;
    int64_t ld;
    int tiles_m, tiles_n;
};

template <bool OUT_FP32, bool ACC, int FMT, int NJ>
__global__ __launch_bounds__(256, 1) void gemm_tile_kernel(const TileGemm p)
{
    __shared__ __attribute__((aligned(1024))) uint8_t smem[LDS_BYTES];
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t *)smem;
    gemm_tile_body<OUT_FP32, ACC, FMT, NJ>(p.aq, p.as, p.bq, p.bs, p.C, p.out, p.ld, p.tiles_m, p.tiles_n,
                                           blockIdx.x, gridDim.x, smem, lds0);
}

// One launch for a product whose last round of 256 x 256 tiles is at most half full: every workgroup first walks
// the whole rounds (tiles 0 .. t_main-1 of the sequence) on 256 x 256 tiles, then the remaining tiles are worked on
// as twice as many 256 x 128 tiles, one per workgroup, so that the compute units that would idle in the last round
// take half of it.  (Nothing is prefetched across the two phases: the second one fills its pipeline again.)
template <bool OUT_FP32, bool ACC>
__global__ __launch_bounds__(256, 1) void gemm_tile_tail_kernel(const TileGemm p, const int t_main)
{
    __shared__ __attribute__((aligned(1024))) uint8_t smem[LDS_BYTES];
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t *)smem;
    gemm_tile_body<OUT_FP32, ACC, 0, 4>(p.aq, p.as, p.bq, p.bs, p.C, p.out, p.ld, p.tiles_m, p.tiles_n, blockIdx.x,
                                        gridDim.x, smem, lds0, 0, t_main);
    __syncthreads();  // (every wave is done with the LDS of the first phase)
    gemm_tile_body<OUT_FP32, ACC, 0, 2, true>(p.aq, p.as, p.bq, p.bs, p.C, p.out, p.ld, p.tiles_m, p.tiles_n,
                                              blockIdx.x, gridDim.x, smem, lds0, t_main, p.tiles_m * p.tiles_n);
}

// Two independent GEMMs in one launch of 256 workgroups (Dgrad and Wgrad of one layer): on every XCD the
// first n0 of its 32 workgroups work on p0, the others on p1, each set walking its own problem's tiles.
// The CUs are split in proportion to the work, so both problems end on full rounds of tiles.  Measured on
// the 8B shapes the launch takes about 5 % less than the two GEMMs one after the other (173-180 against
// 181-195 us): one dispatch gap and one pipeline fill less, no part-filled round, and the two problems' tiles
// have different lengths, so that their output bursts fall at different times.  It is not more: with half
// the chip idle in a partly filled last round the busy half clocks higher under the power cap, and here each
// XCD's L2 holds panels of two problems (22 % more traffic beyond L2).
// FMT0, FMT1: element format of each problem's operands (0 = E2M1, 1 = E4M3), as in gemm_tile_kernel.
template <bool OUT0, bool OUT1, bool ACC1, int FMT0, int FMT1>
__global__ __launch_bounds__(256, 1) void gemm_tile_pair_kernel(const TileGemm p0, const TileGemm p1, const int n0)
{
    __shared__ __attribute__((aligned(1024))) uint8_t smem[LDS_BYTES];
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t *)smem;
    const uint32_t xcd = blockIdx.x & 7, lw = blockIdx.x >> 3;
    if (lw < (uint32_t)n0)
        gemm_tile_body<OUT0, false, FMT0, 4>(p0.aq, p0.as, p0.bq, p0.bs, p0.C, p0.out, p0.ld, p0.tiles_m, p0.tiles_n,
                                             lw * 8 + xcd, (uint32_t)n0 * 8, smem, lds0);
    else
        gemm_tile_body<OUT1, ACC1, FMT1, 4>(p1.aq, p1.as, p1.bq, p1.bs, p1.C, p1.out, p1.ld, p1.tiles_m, p1.tiles_n,
                                            (lw - n0) * 8 + xcd, (uint32_t)(32 - n0) * 8, smem, lds0);
}

}  // namespace

// Compute units of the current device (MI355X: 256); asked once per process and device.
static int device_cus()
{
    static int cached[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return NUM_CUS;
    if (cached[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = NUM_CUS;
        cached[dev] = n;
    }
    return cached[dev];
}

// the tiled kernel wants whole 256 x 256 tiles, K in whole stages (128 bytes of codes per row: 256 E2M1
// or 128 E4M3 elements) and at least 1024 (scale bytes are fetched 32 per row), and 16-byte aligned
// code rows and output rows
// (tile_n: 256, or 128 for the narrow tile, which exists for E2M1 operands only)
static bool tile_eligible(const GemmArgs &g, int tile_n = TILE)
{
    if (g.a_fmt != g.b_fmt) return false;  // mixed formats: any-shape kernel
    if (tile_n != TILE && g.a_fmt != 0) return false;
    const bool k_ok = g.C >= 1024 && (g.C % (g.a_fmt ? 128 : 256)) == 0;
    return k_ok && (g.Ra % TILE) == 0 && (g.Rb % tile_n) == 0 && (g.ld % 8) == 0 &&
           (reinterpret_cast<uintptr_t>(g.as) % 16) == 0 && (reinterpret_cast<uintptr_t>(g.bs) % 16) == 0 &&
           (g.Ra / TILE) * (g.Rb / TILE) < (1 << 30) && g.C < (int64_t(1) << 26);  // (64 code rows: 32-bit lane offsets)
}

static TileGemm tile_args(const GemmArgs &g, int tile_n = TILE)
{
    return TileGemm{g.aq, g.as, g.bq, g.bs, g.C, g.out, g.ld, (int)(g.Ra / TILE), (int)(g.Rb / tile_n)};
}

template <int AF, int BF>
static hipError_t launch_any_f(const GemmArgs &g, hipStream_t st)
{
    dim3 grid((unsigned)((g.Ra + 63) / 64), (unsigned)((g.Rb + 63) / 64));
    if (g.out_fp32) {
        if (g.accumulate)
            hipLaunchKernelGGL((gemm_any_kernel<true, true, AF, BF>), grid, dim3(256), 0, st, g.aq, g.as, g.bq, g.bs,
                               g.Ra, g.Rb, g.C, g.out, g.ld);
        else
            hipLaunchKernelGGL((gemm_any_kernel<true, false, AF, BF>), grid, dim3(256), 0, st, g.aq, g.as, g.bq, g.bs,
                               g.Ra, g.Rb, g.C, g.out, g.ld);
    } else {
        hipLaunchKernelGGL((gemm_any_kernel<false, false, AF, BF>), grid, dim3(256), 0, st, g.aq, g.as, g.bq, g.bs,
                           g.Ra, g.Rb, g.C, g.out, g.ld);
    }
    return hipGetLastError();
}

static hipError_t launch_any(const GemmArgs &g, hipStream_t st)
{
    if (g.a_fmt == 0) return g.b_fmt == 0 ? launch_any_f<0, 0>(g, st) : launch_any_f<0, 1>(g, st);
    return g.b_fmt == 0 ? launch_any_f<1, 0>(g, st) : launch_any_f<1, 1>(g, st);
}

// rows r0.. (n of them) of A and columns c0.. (m of them) of B: the same problem on a sub-block of the output
static GemmArgs sub_block(const GemmArgs &g, int64_t r0, int64_t n, int64_t c0, int64_t m)
{
    GemmArgs h = g;
    const int64_t nkb = g.C / 32;
    h.aq = g.aq + r0 * (g.a_fmt ? g.C : g.C / 2);
    h.as = g.as + r0 * nkb;
    h.bq = g.bq + c0 * (g.b_fmt ? g.C : g.C / 2);
    h.bs = g.bs + c0 * nkb;
    h.Ra = n;
    h.Rb = m;
    h.out = static_cast<uint8_t *>(g.out) + (r0 * g.ld + c0) * (g.out_fp32 ? 4 : 2);
    return h;
}

template <int FMT, int NJ>
static hipError_t launch_tiled_f(const GemmArgs &g, hipStream_t st)
{
    const TileGemm p = tile_args(g, 64 * NJ);
    // persistent: one workgroup per CU (the kernel takes all of a CU's LDS) walks several tiles
    const int T = p.tiles_m * p.tiles_n;
    const int cus = device_cus();
    dim3 grid((unsigned)(T < cus ? T : cus));
    if (g.out_fp32) {
        if (g.accumulate)
            hipLaunchKernelGGL((gemm_tile_kernel<true, true, FMT, NJ>), grid, dim3(256), 0, st, p);
        else
            hipLaunchKernelGGL((gemm_tile_kernel<true, false, FMT, NJ>), grid, dim3(256), 0, st, p);
    } else {
        hipLaunchKernelGGL((gemm_tile_kernel<false, false, FMT, NJ>), grid, dim3(256), 0, st, p);
    }
    return hipGetLastError();
}

// whole rounds on 256 x 256 tiles, then the last round's tiles in halves (see gemm_tile_tail_kernel)
static hipError_t launch_tiled_tail(const GemmArgs &g, int64_t main_tiles, hipStream_t st)
{
    const TileGemm p = tile_args(g);
    dim3 grid((unsigned)device_cus());
    if (g.out_fp32) {
        if (g.accumulate)
            hipLaunchKernelGGL((gemm_tile_tail_kernel<true, true>), grid, dim3(256), 0, st, p, (int)main_tiles);
        else
            hipLaunchKernelGGL((gemm_tile_tail_kernel<true, false>), grid, dim3(256), 0, st, p, (int)main_tiles);
    } else {
        hipLaunchKernelGGL((gemm_tile_tail_kernel<false, false>), grid, dim3(256), 0, st, p, (int)main_tiles);
    }
    return hipGetLastError();
}

// Which kernels a GEMM is cut into (host logic only: no device is touched; cus = compute units of the device).
// Whole 256 x 256 tiles run on the tiled kernel, except where that would leave compute units idle (E2M1 operands):
//   * fewer tiles than compute units: 256 x 128 tiles (twice as many);
//   * a last round of tiles at most half full behind at most four whole rounds: the whole rounds run on 256 x 256
//     tiles and, in the same launch, the tiles of the last round as twice as many 256 x 128 tiles (GEMM_TILED_256_TAIL_128, main_tiles = the tiles of
//     the whole rounds);
//   * a column count in whole 128s but not 256s: 256 x 128 tiles throughout.
// Ragged row or column counts: the 256-aligned interior as above, the right and bottom edge strips (less than one
// tile wide) on the any-shape kernel; everything else on the any-shape kernel.
static void plan_tiled(const GemmArgs &g, int64_t r0, int64_t rows, int64_t cols, int64_t cus, GemmPlan &plan)
{
    auto add = [&](int kind, int64_t main_tiles) {
        plan.part[plan.n++] = GemmPart{kind, r0, rows, 0, cols, main_tiles};
    };
    if (g.a_fmt) return add(GEMM_TILED_256, 0);
    const int64_t T = (rows / TILE) * (cols / TILE);
    if (T < cus) return add(GEMM_TILED_128, 0);
    // (measured: 2 to 5 % on one to three and a half rounds; with more whole rounds in front the second pipeline fill
    // costs as much as the halves save)
    const int64_t rem = T % cus;
    if (rem != 0 && 2 * rem <= cus && T / cus <= 4) return add(GEMM_TILED_256_TAIL_128, T - rem);
    add(GEMM_TILED_256, 0);
}

GemmPlan plan_gemm(const GemmArgs &g, int cus)
{
    GemmPlan plan;
    plan.n = 0;
    if (tile_eligible(g)) {
        plan_tiled(g, 0, g.Ra, g.Rb, cus, plan);
    } else if (tile_eligible(g, TILE / 2)) {
        plan.part[plan.n++] = GemmPart{GEMM_TILED_128, 0, g.Ra, 0, g.Rb, 0};
    } else {
        const int64_t ra = g.Ra / TILE * TILE, rb = g.Rb / TILE * TILE;
        // (the interior starts at offset 0 of every array, so it keeps the alignment of the whole problem; the
        // any-shape kernel asks none of the strips' output pointers)
        if (ra > 0 && rb > 0 && tile_eligible(sub_block(g, 0, ra, 0, rb))) {
            plan_tiled(g, 0, ra, rb, cus, plan);
            if (g.Rb > rb) plan.part[plan.n++] = GemmPart{GEMM_ANY, 0, g.Ra, rb, g.Rb - rb, 0};
            if (g.Ra > ra) plan.part[plan.n++] = GemmPart{GEMM_ANY, ra, g.Ra - ra, 0, rb, 0};
        } else {
            plan.part[plan.n++] = GemmPart{GEMM_ANY, 0, g.Ra, 0, g.Rb, 0};
        }
    }
    return plan;
}

hipError_t launch_gemm(const GemmArgs &g, hipStream_t st)
{
    const GemmPlan plan = plan_gemm(g, device_cus());
    for (int i = 0; i < plan.n; ++i) {
        const GemmPart &p = plan.part[i];
        const GemmArgs h = sub_block(g, p.r0, p.rows, p.c0, p.cols);
        hipError_t e;
        if (p.kind == GEMM_ANY)
            e = launch_any(h, st);
        else if (p.kind == GEMM_TILED_128)
            e = launch_tiled_f<0, 2>(h, st);
        else if (p.kind == GEMM_TILED_256_TAIL_128)
            e = launch_tiled_tail(h, p.main_tiles, st);
        else
            e = g.a_fmt ? launch_tiled_f<1, 4>(h, st) : launch_tiled_f<0, 4>(h, st);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// g0 (no accumulation) and g1 on the same stream, no dependence between them.  Side by side in one launch
// when both fit the tiled kernel and together fill the chip; otherwise one after the other.
hipError_t launch_gemm_pair(const GemmArgs &g0, const GemmArgs &g1, hipStream_t st)
{
    // (the split below counts on 8 XCDs of 32 compute units each)
    // Formats: both problems MXFP4 (every combination of output types); or the second, or both, MXFP8 with the
    // output types of a backward pass (bf16 from problem 0, fp32 from problem 1): the stage-wise recipes of Table 1.
    const bool fmt_ok = g0.a_fmt == g0.b_fmt && g1.a_fmt == g1.b_fmt && (g0.a_fmt == 0 || g1.a_fmt == 1) &&
                        (g1.a_fmt == 0 || (!g0.out_fp32 && g1.out_fp32));
    const bool side_by_side = !g0.accumulate && fmt_ok && tile_eligible(g0) && tile_eligible(g1) &&
                              device_cus() == NUM_CUS;
    if (side_by_side) {
        const TileGemm p0 = tile_args(g0), p1 = tile_args(g1);
        const int64_t t0 = (int64_t)p0.tiles_m * p0.tiles_n, t1 = (int64_t)p1.tiles_m * p1.tiles_n;
        // (an E4M3 element costs the matrix unit twice the time of an E2M1 element)
        const double w0 = (double)t0 * (double)g0.C * (g0.a_fmt ? 2.0 : 1.0);
        const double w1 = (double)t1 * (double)g1.C * (g1.a_fmt ? 2.0 : 1.0);
        int n0 = (int)(32.0 * w0 / (w0 + w1) + 0.5);  // workgroups per XCD for g0, in proportion to the work
        n0 = n0 < 1 ? 1 : (n0 > 31 ? 31 : n0);
        // worth it only if both shares have enough tiles to keep their CUs busy
        if (t0 >= (int64_t)n0 * 8 && t1 >= (int64_t)(32 - n0) * 8) {
            dim3 grid(NUM_CUS);
#define MXFP4_PAIR(O0, O1, A1, F0, F1) \
    hipLaunchKernelGGL((gemm_tile_pair_kernel<O0, O1, A1, F0, F1>), grid, dim3(256), 0, st, p0, p1, n0)
            if (g1.a_fmt) {
                if (g0.a_fmt) {
                    if (g1.accumulate) MXFP4_PAIR(false, true, true, 1, 1); else MXFP4_PAIR(false, true, false, 1, 1);
                } else {
                    if (g1.accumulate) MXFP4_PAIR(false, true, true, 0, 1); else MXFP4_PAIR(false, true, false, 0, 1);
                }
            } else if (g0.out_fp32) {
                if (!g1.out_fp32) MXFP4_PAIR(true, false, false, 0, 0);
                else if (g1.accumulate) MXFP4_PAIR(true, true, true, 0, 0);
                else MXFP4_PAIR(true, true, false, 0, 0);
            } else {
                if (!g1.out_fp32) MXFP4_PAIR(false, false, false, 0, 0);
                else if (g1.accumulate) MXFP4_PAIR(false, true, true, 0, 0);
                else MXFP4_PAIR(false, true, false, 0, 0);
            }
#undef MXFP4_PAIR
            return hipGetLastError();
        }
    }
    hipError_t e = launch_gemm(g0, st);
    if (e != hipSuccess) return e;
    return launch_gemm(g1, st);
}

}  // namespace mxfp4
