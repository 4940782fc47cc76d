// Block-scaled FP4 GEMM for gfx950: out[i][j] (+)= sum_c A[i][c] * B[j][c] on MXFP4
// operands (the MXFP4 GEMM of the linear layers, Sec. 1 / App. A.2; operand axes per
// App. C.1-C.3), on the scaled matrix instruction V_MFMA_SCALE_F32_16X16X128_F8F6F4.
//
// Register layout of that instruction with FP4 operands (64 lanes, lane = l):
//   first operand  (16 x 128): lane l holds row  l%16, elements k = 32*(l/16) .. +31
//                  as 16 bytes (4 VGPRs), element k in nibble k%32 (low nibble first);
//                  its scale VGPR holds the E8M0 byte of exactly that 32-element block
//   second operand (128 x 16): the same with "row" = output column
//   result (16 x 16, 4 VGPRs): lane l holds column l%16, rows 4*(l/16) + {0,1,2,3}
// i.e. one lane's operand is precisely one MX block of the canonical layout, so the
// canonical q/s arrays feed the instruction without any repacking.
//
// The kernels pass B's rows as the first operand and A's rows as the second: a lane
// then owns 4 consecutive output columns of one output row (one 16- or 8-byte store).
#include <type_traits>

#include "mxfp4_internal.h"

namespace mxfp4 {
namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));

__device__ __forceinline__ v4f mfma_fp4(v4i first, v4i second, v4f acc, int scale_first, int scale_second)
{
    v8i a = {first.x, first.y, first.z, first.w, 0, 0, 0, 0};
    v8i b = {second.x, second.y, second.z, second.w, 0, 0, 0, 0};
    // cbsz = blgp = 4: both operands E2M1; scale byte 0 of each scale register
    return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, acc, 4, 4, 0, scale_first, 0, scale_second);
}

__device__ __forceinline__ uint16_t f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40u);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// ---- any-shape kernel --------------------------------------------------------------------
// 256 threads = 2x2 waves, each wave a 32x32 output tile (2x2 instruction tiles); operands
// come straight from global memory.  Rows beyond the matrix are clamped (their results
// are dropped), K blocks beyond C/32 are fed as zeros.
template <bool OUT_FP32, bool ACC>
__global__ __launch_bounds__(256) void gemm_any_kernel(const uint8_t *__restrict__ aq, const uint8_t *__restrict__ as,
                                                       const uint8_t *__restrict__ bq, const uint8_t *__restrict__ bs,
                                                       int64_t Ra, int64_t Rb, int64_t C, void *__restrict__ out,
                                                       int64_t ld)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l16 = lane & 15, kb = lane >> 4;
    const int64_t row0 = (int64_t)blockIdx.x * 64 + (wave >> 1) * 32;
    const int64_t col0 = (int64_t)blockIdx.y * 64 + (wave & 1) * 32;
    const int64_t nkb = C >> 5, rowbytes = C >> 1;

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
        const int64_t kk = k + kb;
        const bool kv = kk < nkb;
        v4i a[2], b[2];
        int sa[2], sb[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            a[t] = (v4i){0, 0, 0, 0};
            b[t] = (v4i){0, 0, 0, 0};
            sa[t] = 127;
            sb[t] = 127;
            if (kv) {
                a[t] = *reinterpret_cast<const v4i *>(aq + ar[t] * rowbytes + kk * 16);
                b[t] = *reinterpret_cast<const v4i *>(bq + br[t] * rowbytes + kk * 16);
                sa[t] = as[ar[t] * nkb + kk];
                sb[t] = bs[br[t] * nkb + kk];
            }
        }
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) acc[i][j] = mfma_fp4(b[j], a[i], acc[i][j], sb[j], sa[i]);
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
// (256 accumulator registers per lane).  With FP4 operands that instruction takes, per lane l,
// the 32 K-elements 32*(l/32).. of row l%32 of each operand (one MX block, 16 bytes) and the
// block's scale byte; the result holds, in register e of lane l, D[8*(e/4) + 4*(l/32) + e%4][l%32].
//
// Data path: packed codes go global -> LDS with the direct-to-LDS loads (no registers), one
// instruction per 8 rows x 128 bytes (whole cache lines).  A wave's 64 lanes land at
// consecutive 16-byte slots, so the lane -> (row, 16-byte chunk) choice on the global side fixes
// the LDS layout; chunk c of row r of an 8-row group g sits at slot r*8 + (c ^ r ^ (g&1)),
// which makes every 16-lane quarter of the later 16-byte fragment reads hit all 64 banks once.
// Scale bytes follow the same way (8 per row and stage) and are regrouped with one byte
// permute so that the instruction's byte selector picks the K-step.
// Two LDS stage buffers; fragments are double-buffered in registers across the 4 K-steps.
constexpr int TILE = 256;                       // output tile edge
constexpr int STAGE_K = 256;                    // K elements per stage = 128 bytes per row
constexpr int OP_BYTES = TILE * STAGE_K / 2;    // 32 KiB per operand and stage
constexpr int SC_BYTES = TILE * 8;              // 2 KiB of scale bytes per operand and stage
constexpr int OFF_A = 0, OFF_B = OP_BYTES, OFF_SA = 2 * OP_BYTES, OFF_SB = 2 * OP_BYTES + SC_BYTES;
constexpr int STAGE_BYTES = 2 * OP_BYTES + 2 * SC_BYTES;  // 69632
constexpr int GROUP_M = 4;                      // tile rows per rasterisation group

typedef float v16f __attribute__((ext_vector_type(16)));

__device__ __forceinline__ void dma16(uint32_t lds_addr, uint32_t voff, const uint8_t *sbase)
{
    // each lane: 16 bytes from sbase + voff to LDS[lds_addr + 16*lane]
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2\n\t" ::"s"(lds_addr), "v"(voff), "s"(sbase)
                 : "memory");
}
__device__ __forceinline__ void dma4(uint32_t lds_addr, uint32_t voff, const uint8_t *sbase)
{
    // each lane: 4 bytes from sbase + voff to LDS[lds_addr + 4*lane]
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dword %1, %2\n\t" ::"s"(lds_addr), "v"(voff), "s"(sbase)
                 : "memory");
}

template <bool OUT_FP32, bool ACC>
__global__ __launch_bounds__(256, 1) void gemm_tile_kernel(const uint8_t *__restrict__ aq,
                                                           const uint8_t *__restrict__ as,
                                                           const uint8_t *__restrict__ bq,
                                                           const uint8_t *__restrict__ bs, int64_t C,
                                                           void *__restrict__ out, int64_t ld, int tiles_m,
                                                           int tiles_n)
{
    __shared__ __attribute__((aligned(1024))) uint8_t smem[2 * STAGE_BYTES];
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t *)smem;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;

    // workgroup id -> tile.  Ids are dealt round-robin to the 8 XCDs (each with its own L2): give
    // every XCD a contiguous run of the tile sequence, and walk that sequence in groups of GROUP_M
    // tile rows so that the tiles in flight on one XCD share A and B panels.
    int tm, tn;
    {
        const int T = tiles_m * tiles_n, w = blockIdx.x;
        const int per = T >> 3, rem = T & 7, xcd = w & 7, local = w >> 3;
        const int L = xcd < rem ? xcd * (per + 1) + local : rem * (per + 1) + (xcd - rem) * per + local;
        const int span = GROUP_M * tiles_n, grp = L / span, first = grp * GROUP_M;
        const int gm = (tiles_m - first) < GROUP_M ? (tiles_m - first) : GROUP_M;
        const int in = L - grp * span;
        tm = first + in % gm;
        tn = in / gm;
    }
    const int64_t rowbytes = C >> 1, nkb = C >> 5;
    const int nstages = (int)(C / STAGE_K);
    const int64_t m0 = (int64_t)tm * TILE, n0 = (int64_t)tn * TILE;

    // ---- direct-to-LDS loads: per-lane offsets (fixed for the whole kernel) -----------------
    const int drr = lane >> 3, dcc = lane & 7;
    const uint32_t dvoff0 = (uint32_t)(drr * rowbytes) + (uint32_t)((dcc ^ drr) << 4);        // even 8-row groups
    const uint32_t dvoff1 = (uint32_t)(drr * rowbytes) + (uint32_t)((dcc ^ drr ^ 1) << 4);    // odd ones
    const uint32_t svoff = (uint32_t)(lane * nkb);
    const uint8_t *a_rows = aq + (m0 + wave * 64) * rowbytes;  // this wave loads rows wave*64 .. +63 of each tile
    const uint8_t *b_rows = bq + (n0 + wave * 64) * rowbytes;
    const uint8_t *as_rows = as + (m0 + wave * 64) * nkb;
    const uint8_t *bs_rows = bs + (n0 + wave * 64) * nkb;

    auto issue_stage = [&](int s, int buf) {
        const uint32_t base = lds0 + buf * STAGE_BYTES;
        const int64_t koff = (int64_t)s * (STAGE_K / 2);
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const uint32_t dst = (uint32_t)((wave * 8 + t) * 1024);
            const uint32_t vo = (t & 1) ? dvoff1 : dvoff0;
            dma16(base + OFF_A + dst, vo, a_rows + t * 8 * rowbytes + koff);
            dma16(base + OFF_B + dst, vo, b_rows + t * 8 * rowbytes + koff);
        }
#pragma unroll
        for (int d = 0; d < 2; ++d) {
            dma4(base + OFF_SA + d * 1024 + wave * 256, svoff, as_rows + s * 8 + d * 4);
            dma4(base + OFF_SB + d * 1024 + wave * 256, svoff, bs_rows + s * 8 + d * 4);
        }
    };

    // ---- fragment reads: per-lane offsets ---------------------------------------------------
    const int fr = lane & 31, fh = lane >> 5;
    const int fm = (fr & 7) ^ ((fr >> 3) & 1);
    const uint32_t fl0 = (uint32_t)((fr >> 3) * 1024 + (fr & 7) * 128);
    uint32_t foff[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) foff[kk] = fl0 + (uint32_t)((((kk << 1) | fh) ^ fm) << 4);
    const uint32_t a_frag0 = OFF_A + wm * 16 * 1024, b_frag0 = OFF_B + wn * 16 * 1024;
    const uint32_t sa_frag0 = OFF_SA + (wm * 128 + fr) * 4, sb_frag0 = OFF_SB + (wn * 128 + fr) * 4;
    const uint32_t perm_sel = fh ? 0x07050301u : 0x06040200u;

    v4i fa[2][4], fb[2][4];
    auto read_frags = [&](int buf, int kk, int set) {
        const uint8_t *p = smem + buf * STAGE_BYTES + foff[kk];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            fa[set][i] = *reinterpret_cast<const v4i *>(p + a_frag0 + i * 4096);
            fb[set][i] = *reinterpret_cast<const v4i *>(p + b_frag0 + i * 4096);
        }
    };
    auto read_scales = [&](int buf, int (&sa)[4], int (&sb)[4]) {
        const uint8_t *p = smem + buf * STAGE_BYTES;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t a0 = *reinterpret_cast<const uint32_t *>(p + sa_frag0 + i * 128);
            const uint32_t a1 = *reinterpret_cast<const uint32_t *>(p + sa_frag0 + 1024 + i * 128);
            const uint32_t b0 = *reinterpret_cast<const uint32_t *>(p + sb_frag0 + i * 128);
            const uint32_t b1 = *reinterpret_cast<const uint32_t *>(p + sb_frag0 + 1024 + i * 128);
            sa[i] = (int)__builtin_amdgcn_perm(a1, a0, perm_sel);  // bytes: K blocks fh, 2+fh, 4+fh, 6+fh
            sb[i] = (int)__builtin_amdgcn_perm(b1, b0, perm_sel);
        }
    };

    v16f acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

#define MXFP4_MMA_STEP(SET, KK, SA, SB)                                                                        \
    _Pragma("unroll") for (int i = 0; i < 4; ++i) _Pragma("unroll") for (int j = 0; j < 4; ++j)                \
    {                                                                                                          \
        v8i fb8 = {fb[SET][j].x, fb[SET][j].y, fb[SET][j].z, fb[SET][j].w, 0, 0, 0, 0};                        \
        v8i fa8 = {fa[SET][i].x, fa[SET][i].y, fa[SET][i].z, fa[SET][i].w, 0, 0, 0, 0};                        \
        acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fb8, fa8, acc[i][j], 4, 4, KK, SB[j], KK,  \
                                                                    SA[i]);                                    \
    }

    int sa_cur[4], sb_cur[4], sa_nxt[4], sb_nxt[4];
    issue_stage(0, 0);
    if (nstages > 1) issue_stage(1, 1);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    read_frags(0, 0, 0);
    read_scales(0, sa_cur, sb_cur);

    // One stage.  The loop body must stay one basic block (no data-dependent branches inside),
    // otherwise the matrix instructions get sunk behind the branches and stop overlapping the
    // fragment fetches; so the last two stages, which issue fewer loads, are peeled below.
    auto stage = [&](int s, auto refill, auto has_next) {
        const int buf = s & 1;
        // each K-step: fetch the next step's fragments into the other register set, then the 16
        // matrix instructions of this step; the scheduling barriers keep the compiler from
        // regrouping all fetches ahead of all matrix instructions
        read_frags(buf, 1, 1);
        MXFP4_MMA_STEP(0, 0, sa_cur, sb_cur)
        __builtin_amdgcn_sched_barrier(0);
        read_frags(buf, 2, 0);
        MXFP4_MMA_STEP(1, 1, sa_cur, sb_cur)
        __builtin_amdgcn_sched_barrier(0);
        read_frags(buf, 3, 1);
        MXFP4_MMA_STEP(0, 2, sa_cur, sb_cur)
        __builtin_amdgcn_sched_barrier(0);
        // every wave has fetched its last fragments of this buffer, and this wave's loads of the
        // next stage have landed: after the barrier the buffer may be refilled and the other read
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (decltype(refill)::value) issue_stage(s + 2, buf);
        if (decltype(has_next)::value) {
            read_frags(buf ^ 1, 0, 0);
            read_scales(buf ^ 1, sa_nxt, sb_nxt);
        }
        MXFP4_MMA_STEP(1, 3, sa_cur, sb_cur)
        __builtin_amdgcn_sched_barrier(0);
        if (decltype(has_next)::value) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                sa_cur[i] = sa_nxt[i];
                sb_cur[i] = sb_nxt[i];
            }
        }
    };
    using yes = std::integral_constant<bool, true>;
    using no = std::integral_constant<bool, false>;
    for (int s = 0; s + 2 < nstages; ++s) stage(s, yes{}, yes{});
    if (nstages >= 2) stage(nstages - 2, no{}, yes{});
    stage(nstages - 1, no{}, no{});
#undef MXFP4_MMA_STEP

    // ---- epilogue: lane owns row fr of each 32-row group and 4 x 4 consecutive columns ----------
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t row = m0 + wm * 128 + i * 32 + fr;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
#pragma unroll
            for (int qd = 0; qd < 4; ++qd) {
                const int64_t col = n0 + wn * 128 + j * 32 + 8 * qd + 4 * fh;
                float v0 = acc[i][j][4 * qd + 0], v1 = acc[i][j][4 * qd + 1], v2 = acc[i][j][4 * qd + 2],
                      v3 = acc[i][j][4 * qd + 3];
                if (OUT_FP32) {
                    v4f *o = reinterpret_cast<v4f *>(reinterpret_cast<float *>(out) + row * ld + col);
                    if (ACC) {
                        v4f old = *o;
                        v0 += old.x; v1 += old.y; v2 += old.z; v3 += old.w;
                    }
                    *o = (v4f){v0, v1, v2, v3};
                } else {
                    uint2 pk;
                    pk.x = (uint32_t)f32_to_bf16(v0) | ((uint32_t)f32_to_bf16(v1) << 16);
                    pk.y = (uint32_t)f32_to_bf16(v2) | ((uint32_t)f32_to_bf16(v3) << 16);
                    *reinterpret_cast<uint2 *>(reinterpret_cast<uint16_t *>(out) + row * ld + col) = pk;
                }
            }
        }
    }
}

}  // namespace

hipError_t launch_gemm(const GemmArgs &g, hipStream_t st)
{
    const bool tiled = g.C > 0 && (g.Ra % TILE) == 0 && (g.Rb % TILE) == 0 && (g.C % STAGE_K) == 0 &&
                       (g.ld % 4) == 0 && (reinterpret_cast<uintptr_t>(g.as) % 4) == 0 &&
                       (reinterpret_cast<uintptr_t>(g.bs) % 4) == 0 && (g.Ra / TILE) * (g.Rb / TILE) < (1 << 30) &&
                       g.C < (int64_t(1) << 31);
    if (tiled) {
        const int tiles_m = (int)(g.Ra / TILE), tiles_n = (int)(g.Rb / TILE);
        dim3 grid((unsigned)(tiles_m * tiles_n));
        if (g.out_fp32) {
            if (g.accumulate)
                hipLaunchKernelGGL((gemm_tile_kernel<true, true>), grid, dim3(256), 0, st, g.aq, g.as, g.bq, g.bs,
                                   g.C, g.out, g.ld, tiles_m, tiles_n);
            else
                hipLaunchKernelGGL((gemm_tile_kernel<true, false>), grid, dim3(256), 0, st, g.aq, g.as, g.bq, g.bs,
                                   g.C, g.out, g.ld, tiles_m, tiles_n);
        } else {
            hipLaunchKernelGGL((gemm_tile_kernel<false, false>), grid, dim3(256), 0, st, g.aq, g.as, g.bq, g.bs,
                               g.C, g.out, g.ld, tiles_m, tiles_n);
        }
        return hipGetLastError();
    }
    dim3 grid((unsigned)((g.Ra + 63) / 64), (unsigned)((g.Rb + 63) / 64));
    if (g.out_fp32) {
        if (g.accumulate)
            hipLaunchKernelGGL((gemm_any_kernel<true, true>), grid, dim3(256), 0, st, g.aq, g.as, g.bq, g.bs, g.Ra,
                               g.Rb, g.C, g.out, g.ld);
        else
            hipLaunchKernelGGL((gemm_any_kernel<true, false>), grid, dim3(256), 0, st, g.aq, g.as, g.bq, g.bs, g.Ra,
                               g.Rb, g.C, g.out, g.ld);
    } else {
        hipLaunchKernelGGL((gemm_any_kernel<false, false>), grid, dim3(256), 0, st, g.aq, g.as, g.bq, g.bs, g.Ra,
                           g.Rb, g.C, g.out, g.ld);
    }
    return hipGetLastError();
}

}  // namespace mxfp4
