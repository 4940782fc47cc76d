// Device code shared by the quantiser kernels (MXFP4 in quantize.hip, MXFP8 in quantize_fp8.hip): the counter
// hash, one block's rotation and maximum in registers, bf16 widening, and the column-wise workgroup tile.
// Everything sits in an unnamed namespace: each translation unit gets its own copy.
#pragma once
#include "mxfp4_internal.h"

namespace mxfp4 {
namespace {

constexpr int HAD_NONE = 0, HAD_DET = 1, HAD_RANDSIGN = 2, HAD_DET16 = 3, HAD_RANDSIGN16 = 4;
constexpr int RND_RNE = 0, RND_SR = 1;

// ---- counter hash: stateless 32-bit mixer applied to (seed, index) -----------------
struct RngKey {
    uint32_t seed_lo_mul;  // low seed word times the odd constant
    uint32_t seed_hi_mix;  // mixed high seed word
};

__host__ __device__ __forceinline__ uint32_t mix32(uint32_t x)
{
    x ^= x >> 16;
    x *= 0x9E3779B9u;
    x ^= x >> 15;
    x *= 0xBB67AE85u;
    x ^= x >> 16;
    return x;
}

__host__ __device__ __forceinline__ uint32_t rand32(RngKey k, uint64_t idx)
{
    return mix32(mix32((uint32_t)idx + k.seed_lo_mul) ^ (uint32_t)(idx >> 32) ^ k.seed_hi_mix);
}

RngKey make_key(uint64_t seed)
{
    RngKey k;
    k.seed_lo_mul = (uint32_t)seed * 0x9E3779B9u;
    k.seed_hi_mix = mix32((uint32_t)(seed >> 32) ^ 0x6A09E667u);
    return k;
}

// the +-1 diagonal of the random-sign rotation: a function of the base seed alone
uint32_t sign_mask_of(uint64_t seed) { return rand32(make_key(seed & SEED_BASE_MASK), 0xFFFFFFFFFFFFFFFFull); }

// ---- one block in registers ---------------------------------------------------------
template <int N>
__device__ __forceinline__ void butterflies(float (&v)[32])
{
#pragma unroll
    for (int h = 1; h < N; h <<= 1) {
#pragma unroll
        for (int i = 0; i < 32; ++i) {
            if ((i & h) == 0) {
                float a = v[i], b = v[i + h];
                v[i] = a + b;
                v[i + h] = a - b;
            }
        }
    }
}

// Stochastic rounding of |t| (already divided by the block scale) to an E2M1 magnitude code.
__device__ __forceinline__ uint32_t sr_code(float t, uint32_t r)
{
    float a = fminf(fabsf(t), 6.0f);
    bool lo = a < 2.0f, mid = a < 4.0f;
    float inv_delta = lo ? 2.0f : (mid ? 1.0f : 0.5f);
    float q = a * inv_delta;  // exact: power-of-two factor
    float fl = floorf(q);
    float f = q - fl;  // exact
    float u = (float)(2u * (r >> 9) + 1u) * 0x1p-24f;  // odd multiple of 2^-24 below 1: exact
    uint32_t m = (uint32_t)fl + ((u < f) ? 1u : 0u);
    uint32_t code = m + (lo ? 0u : (mid ? 2u : 4u));
    return code | ((__float_as_uint(t) >> 28) & 8u);
}

// Optional sign flips and rotation of one block, in place (App. A.2).
template <int HAD>
__device__ __forceinline__ void rotate_block(float (&v)[32], uint32_t sign_mask)
{
    if (HAD == HAD_RANDSIGN || HAD == HAD_RANDSIGN16) {  // the block's 32-entry diagonal, whatever the rotation size
#pragma unroll
        for (int i = 0; i < 32; ++i)
            v[i] = __uint_as_float(__float_as_uint(v[i]) ^ (((sign_mask >> i) & 1u) << 31));
    }
    if (HAD == HAD_DET || HAD == HAD_RANDSIGN) {
        butterflies<32>(v);
        const float c = __uint_as_float(0x3E3504F3u);  // 2^-2.5 rounded to fp32
#pragma unroll
        for (int i = 0; i < 32; ++i) v[i] = v[i] * c;
    } else if (HAD == HAD_DET16 || HAD == HAD_RANDSIGN16) {
        butterflies<16>(v);
#pragma unroll
        for (int i = 0; i < 32; ++i) v[i] = v[i] * 0.25f;
    }
}

// Bit pattern of the block's largest magnitude.  V_MAXIMUM3_F32 (two new values per instruction, |.| as source
// modifiers) returns NaN if any input is NaN, so a NaN or an infinity anywhere in the block shows as an exponent
// field of 255, as in a comparison of the bit patterns.
__device__ __forceinline__ uint32_t amax_bits(const float (&v)[32])
{
    float m = 0.0f;
#pragma unroll
    for (int i = 0; i < 32; i += 2)
        m = __builtin_elementwise_maximum(
            __builtin_elementwise_maximum(__builtin_fabsf(v[i]), __builtin_fabsf(v[i + 1])), m);
    return __float_as_uint(m) & 0x7FFFFFFFu;
}

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// 32 contiguous bf16 (four 16-byte words) widened to fp32
__device__ __forceinline__ void widen(const uint4 (&raw)[4], float (&v)[32])
{
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        v[8 * j + 0] = bf16_lo(raw[j].x);
        v[8 * j + 1] = bf16_hi(raw[j].x);
        v[8 * j + 2] = bf16_lo(raw[j].y);
        v[8 * j + 3] = bf16_hi(raw[j].y);
        v[8 * j + 4] = bf16_lo(raw[j].z);
        v[8 * j + 5] = bf16_hi(raw[j].z);
        v[8 * j + 6] = bf16_lo(raw[j].w);
        v[8 * j + 7] = bf16_hi(raw[j].w);
    }
}

// FP4 codes of one rotated block under the scale that follows from the shared maximum `amax` (bit
// pattern): eq. (1) with the OCP scale rule.  idx0: linear index of element 0 in the quantised output
// (stochastic rounding counter).
template <int RND>
__device__ __forceinline__ void encode_scaled(const float (&v)[32], uint32_t amax, RngKey key, uint64_t idx0,
                                              uint4 &codes, uint32_t &scale_byte)
{
    uint32_t eb = amax >> 23;
    bool bad = (eb == 255u);
    uint32_t sb = eb > 2u ? eb - 2u : 0u;  // eb <= 254 here, so sb <= 252
    scale_byte = bad ? 0xFFu : sb;

    uint32_t w[4];
    if (RND == RND_RNE) {
        // The converter divides by 2^(exponent field of `scale` - 127), rounds to nearest
        // even on the E2M1 grid and saturates at 6; it writes one byte (two codes) per issue.
        float scale = __uint_as_float(sb << 23);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint32_t r = 0;
            r = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(r, v[8 * j + 0], v[8 * j + 1], scale, 0);
            r = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(r, v[8 * j + 2], v[8 * j + 3], scale, 1);
            r = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(r, v[8 * j + 4], v[8 * j + 5], scale, 2);
            r = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(r, v[8 * j + 6], v[8 * j + 7], scale, 3);
            w[j] = r;
        }
    } else {
        float inv = __uint_as_float((254u - sb) << 23);  // 2^-(sb-127); field in [2,254]
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint32_t r = 0;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                int i = 8 * j + e;
                uint32_t code = sr_code(v[i] * inv, rand32(key, idx0 + (uint64_t)i));
                r |= code << (4 * e);
            }
            w[j] = r;
        }
    }
    codes = bad ? make_uint4(0, 0, 0, 0) : make_uint4(w[0], w[1], w[2], w[3]);
}

// Code store.  streaming: for tensors larger than the 256 MB last-level cache the output cannot stay cached
// for the GEMM anyway, and marking the stores non-temporal is worth 3-8 % there (measured); smaller tensors
// keep ordinary stores so that the GEMM finds its operands in cache.
__device__ __forceinline__ void store_codes(uint4 *p, uint4 v, int streaming)
{
    if (streaming) {
        typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
        __builtin_nontemporal_store((u32x4){v.x, v.y, v.z, v.w}, reinterpret_cast<u32x4 *>(p));
    } else {
        *p = v;
    }
}

// ---- column-wise workgroup tile: 256 rows (8 row blocks, one per wave) x 128 columns (2 per lane) ----
constexpr int CT_COLS = 128, CT_RB = 8;
constexpr int RAW_PITCH = 272;  // bytes per parked row: 256 + 16, so that the 16-byte reads below (16 lanes =
                                // 4 rows x 4 blocks per issue) and the dword writes touch every bank once

// Orders the LDS accesses of one wave (which the hardware performs in program order) for the compiler too.
__device__ __forceinline__ void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

}  // namespace
}  // namespace mxfp4
