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

}  // namespace

hipError_t launch_gemm(const GemmArgs &g, hipStream_t st)
{
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
