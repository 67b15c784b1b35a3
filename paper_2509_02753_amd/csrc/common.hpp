// Shared device helpers for the gfx950 MoE kernels (wave64, CDNA4).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lexi {

constexpr int kWave = 64;
constexpr int kRouterSegment = 128;  // the fixed fp32 logit order cuts d into segments of this length

typedef uint16_t bf16_t;  // bf16 bit pattern

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;  // MFMA A/B operand: 8 consecutive K elements
typedef __attribute__((ext_vector_type(4))) float f32x4_t;    // 16x16 MFMA accumulator
typedef __attribute__((ext_vector_type(16))) float f32x16_t;  // 32x32 MFMA accumulator
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;  // one 16-byte global/LDS transaction
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2_t;

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float((uint32_t)b << 16); }

// round-to-nearest-even fp32 -> bf16: the hardware conversion (v_cvt_pk_bf16_f32); a NaN stays a (quiet) NaN
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    typedef __attribute__((ext_vector_type(2))) float f32x2_t;
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
    const f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

__device__ __forceinline__ bf16_t f32_to_bf16(float f) { return (bf16_t)(pack_bf16x2(f, 0.0f) & 0xFFFFu); }

// silu(z) = z * sigmoid(z); hardware exp2 and reciprocal (about 1 ulp each), ample for a bf16 result
__device__ __forceinline__ float silu(float z) { return z * __builtin_amdgcn_rcpf(1.0f + __expf(-z)); }

// Element `i` of a tensor stored as fp32 (IS_BF16 = false) or bf16, widened exactly.
template <bool IS_BF16>
__device__ __forceinline__ float load_as_f32(const void* p, size_t i) {
    if (IS_BF16) return bf16_to_f32(((const bf16_t*)p)[i]);
    return ((const float*)p)[i];
}

// ---- wave-level reductions built on DPP (no LDS traffic) -------------------------------------------------
// dpp_ctrl encodings: quad_perm = 0x00..0xFF, row_shr:n = 0x110+n, row_mirror = 0x140, row_half_mirror = 0x141,
// row_bcast15 = 0x142, row_bcast31 = 0x143.
template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ float dpp_f32(float old, float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(old), __float_as_int(v), CTRL, ROW_MASK, 0xF, false));
}

// Maximum over the 64 lanes, returned to every lane (as a wave-uniform value).
__device__ __forceinline__ float wave_max(float v) {
    v = fmaxf(v, dpp_f32<0xB1>(v, v));   // quad_perm [1,0,3,2]
    v = fmaxf(v, dpp_f32<0x4E>(v, v));   // quad_perm [2,3,0,1]
    v = fmaxf(v, dpp_f32<0x141>(v, v));  // row_half_mirror
    v = fmaxf(v, dpp_f32<0x140>(v, v));  // row_mirror: every lane of a 16-lane row now holds the row maximum
    v = fmaxf(v, dpp_f32<0x142, 0xA>(v, v));  // row_bcast15 into rows 1 and 3
    v = fmaxf(v, dpp_f32<0x143, 0xC>(v, v));  // row_bcast31 into rows 2 and 3: lane 63 holds the wave maximum
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

// Sum over the 64 lanes in a fixed tree order, returned to every lane.
__device__ __forceinline__ float wave_sum(float v) {
    v += dpp_f32<0xB1>(0.0f, v);
    v += dpp_f32<0x4E>(0.0f, v);
    v += dpp_f32<0x141>(0.0f, v);
    v += dpp_f32<0x140>(0.0f, v);
    v += dpp_f32<0x142, 0xA>(0.0f, v);  // rows whose row_mask bit is clear receive `old` = 0
    v += dpp_f32<0x143, 0xC>(0.0f, v);
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

}  // namespace lexi
