// Device-side building blocks shared by the gfx950 kernels: element loads,
// the four format codecs, scale arithmetic and cross-lane reductions.
//
// Arithmetic contract (see include/mofq.h): every fp32 step is a single
// correctly rounded operation, so this file must be compiled with
// -ffp-contract=off and without fast-math.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "../../include/mofq.h"

namespace mofq {

#define MOFQ_DEV __device__ __forceinline__

MOFQ_DEV uint32_t f2u(float f) { return __builtin_bit_cast(uint32_t, f); }
MOFQ_DEV float u2f(uint32_t u) { return __builtin_bit_cast(float, u); }
MOFQ_DEV float med3(float x, float lo, float hi) { return __builtin_amdgcn_fmed3f(x, lo, hi); }

// ---- element loads: 8 consecutive elements, widened exactly to fp32 ---------

struct F32 { using type = float; };
struct F16 { using type = uint16_t; };
struct BF16 { using type = uint16_t; };

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

template <typename In> struct Load8;

template <> struct Load8<F32> {
  using elem = float;
  MOFQ_DEV static void load(const elem* p, float (&v)[8]) {
    const u32x4 a = *reinterpret_cast<const u32x4*>(p);
    const u32x4 b = *reinterpret_cast<const u32x4*>(p + 4);
#pragma unroll
    for (int i = 0; i < 4; ++i) { v[i] = u2f(a[i]); v[4 + i] = u2f(b[i]); }
  }
};

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

template <> struct Load8<F16> {
  using elem = uint16_t;
  MOFQ_DEV static void load(const elem* p, float (&v)[8]) {
    const f16x8 h = *reinterpret_cast<const f16x8*>(p);
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = static_cast<float>(h[i]);  // exact, subnormals included
  }
};

template <> struct Load8<BF16> {
  using elem = uint16_t;
  MOFQ_DEV static void load(const elem* p, float (&v)[8]) {
    const u32x4 a = *reinterpret_cast<const u32x4*>(p);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v[2 * i] = u2f(a[i] << 16);           // bf16 is the top half of an fp32
      v[2 * i + 1] = u2f(a[i] & 0xFFFF0000u);
    }
  }
};

// ---- codecs -------------------------------------------------------------------
//
// Each codec gives, for a scaled value t:
//   mag(|t|)  : magnitude of the nearest grid value (FP formats; sign-symmetric)
//   grid(t)   : signed nearest grid value
//   code(t)   : the bit pattern (4 or 8 bits)
// FP rounding adds and subtracts 1.5*2^23*q, q the grid spacing of the binade of
// max(|t|, smallest normal): the fp32 adder then rounds to a multiple of q with
// ties to the even multiple, which is the even code.

template <int FMT> struct Codec;

template <> struct Codec<MOFQ_INT4> {
  static constexpr float QMAX = 7.0f;
  static constexpr bool IS_INT = true;
  static constexpr int BITS = 4;
  MOFQ_DEV static float grid(float t) { return med3(__builtin_rintf(t), -8.0f, 7.0f); }
  MOFQ_DEV static uint32_t code(float t) { return static_cast<uint32_t>(static_cast<int>(grid(t))) & 0xFu; }
};

template <> struct Codec<MOFQ_INT8> {
  static constexpr float QMAX = 127.0f;
  static constexpr bool IS_INT = true;
  static constexpr int BITS = 8;
  MOFQ_DEV static float grid(float t) { return med3(__builtin_rintf(t), -128.0f, 127.0f); }
  MOFQ_DEV static uint32_t code(float t) { return static_cast<uint32_t>(static_cast<int>(grid(t))) & 0xFFu; }
};

template <> struct Codec<MOFQ_FP4_E2M1> {
  static constexpr float QMAX = 6.0f;
  static constexpr bool IS_INT = false;
  static constexpr int BITS = 4;
  // values 0 .5 1 1.5 | 2 3 | 4 6 : spacing .5 below 2, 1 in [2,4), 2 in [4,8)
  MOFQ_DEV static float mag(float at) {
    const float c = __builtin_fminf(at, 6.0f);
    const float a = __builtin_fmaxf(c, 1.0f);
    const float m = u2f((f2u(a) & 0x7F800000u) + 0x0B400000u);  // 1.5 * 2^(e+22)
    return (c + m) - m;
  }
  MOFQ_DEV static float grid(float t) { return __builtin_copysignf(mag(__builtin_fabsf(t)), t); }
  MOFQ_DEV static uint32_t code(float t) {
    const float g = mag(__builtin_fabsf(t));
    // g >= 1: code = 2*(exponent+1) + top mantissa bit; below: 0 or 1 (the subnormal .5)
    const uint32_t hi = (f2u(g) >> 22) - 252u;
    const uint32_t lo = (g == 0.5f) ? 1u : 0u;
    const uint32_t m = (g >= 1.0f) ? hi : lo;
    return m | ((f2u(t) >> 28) & 0x8u);
  }
};

template <> struct Codec<MOFQ_FP8_E4M3> {
  static constexpr float QMAX = 448.0f;
  static constexpr bool IS_INT = false;
  static constexpr int BITS = 8;
  // normal (1+m/8)*2^(e-7), e = 1..15 (max 1.75*2^8 = 448); subnormal m*2^-9
  MOFQ_DEV static float mag(float at) {
    const float c = __builtin_fminf(at, 448.0f);
    const float a = __builtin_fmaxf(c, 0x1p-6f);
    const float m = u2f((f2u(a) & 0x7F800000u) + 0x0A400000u);  // 1.5 * 2^(e+20)
    return (c + m) - m;
  }
  MOFQ_DEV static float grid(float t) { return __builtin_copysignf(mag(__builtin_fabsf(t)), t); }
  MOFQ_DEV static uint32_t code(float t) {
    const float g = mag(__builtin_fabsf(t));
    const uint32_t normal = (f2u(g) >> 20) - 960u;               // ((e+7) << 3) | mantissa
    const uint32_t sub = static_cast<uint32_t>(g * 512.0f);       // m of m*2^-9
    const uint32_t m = (g >= 0x1p-6f) ? normal : sub;
    return m | ((f2u(t) >> 24) & 0x80u);
  }
};

// Table 1, row "w/ NaN&Inf": the same grid up to 3, saturating there (codes 6 and 7 are
// Inf / NaN and never produced).
template <> struct Codec<MOFQ_FP4_E2M1_IEEE> {
  static constexpr float QMAX = 3.0f;
  static constexpr bool IS_INT = false;
  static constexpr int BITS = 4;
  MOFQ_DEV static float mag(float at) { return Codec<MOFQ_FP4_E2M1>::mag(__builtin_fminf(at, 3.0f)); }
  MOFQ_DEV static float grid(float t) { return __builtin_copysignf(mag(__builtin_fabsf(t)), t); }
  MOFQ_DEV static uint32_t code(float t) { return Codec<MOFQ_FP4_E2M1>::code(med3(t, -3.0f, 3.0f)); }
};

template <> struct Codec<MOFQ_FP8_E5M2> {
  static constexpr float QMAX = 57344.0f;
  static constexpr bool IS_INT = false;
  static constexpr int BITS = 8;
  // normal (1+m/4)*2^(e-15), e = 1..30 (max 1.75*2^15 = 57344); subnormal m*2^-16
  MOFQ_DEV static float mag(float at) {
    const float c = __builtin_fminf(at, 57344.0f);
    const float a = __builtin_fmaxf(c, 0x1p-14f);
    const float m = u2f((f2u(a) & 0x7F800000u) + 0x0AC00000u);  // 1.5 * 2^(e+21)
    return (c + m) - m;
  }
  MOFQ_DEV static float grid(float t) { return __builtin_copysignf(mag(__builtin_fabsf(t)), t); }
  MOFQ_DEV static uint32_t code(float t) {
    const float g = mag(__builtin_fabsf(t));
    const uint32_t normal = (f2u(g) >> 21) - 448u;                // ((e+15) << 2) | mantissa
    const uint32_t sub = static_cast<uint32_t>(g * 65536.0f);     // m of m*2^-16
    const uint32_t m = (g >= 0x1p-14f) ? normal : sub;
    return m | ((f2u(t) >> 24) & 0x80u);
  }
};

// ---- scale of a unit ----------------------------------------------------------

// Nearest fp16 (ties to even, fp16 subnormals kept) clamped to 65504, as fp32.
MOFQ_DEV float round_fp16_clamped(float s) {
  const float c = __builtin_fminf(s, 65504.0f);
  return __half2float(__float2half_rn(c));
}

MOFQ_DEV float unit_scale(float absmax, float ratio, float qmax, bool scale_f16) {
  const float ra = ratio * absmax;
  float s = ra / qmax;                // IEEE division
  if (scale_f16) s = round_fp16_clamped(s);
  if (!(s >= 0x1p-126f)) s = 1.0f;    // zero or degenerate unit
  return s;
}

// ---- cross-lane reductions (wave = 64 lanes) -------------------------------------

template <int CTRL> MOFQ_DEV double dpp_f64(double v) {
  const uint64_t u = __builtin_bit_cast(uint64_t, v);
  const int lo = __builtin_amdgcn_update_dpp(0, static_cast<int>(u), CTRL, 0xF, 0xF, true);
  const int hi = __builtin_amdgcn_update_dpp(0, static_cast<int>(u >> 32), CTRL, 0xF, 0xF, true);
  return __builtin_bit_cast(double, (static_cast<uint64_t>(static_cast<uint32_t>(hi)) << 32) |
                                        static_cast<uint32_t>(lo));
}
template <int CTRL> MOFQ_DEV float dpp_f32(float v) {
  return u2f(static_cast<uint32_t>(
      __builtin_amdgcn_update_dpp(0, static_cast<int>(f2u(v)), CTRL, 0xF, 0xF, true)));
}

constexpr int DPP_QUAD_XOR1 = 0xB1;   // quad_perm:[1,0,3,2]
constexpr int DPP_QUAD_XOR2 = 0x4E;   // quad_perm:[2,3,0,1]
constexpr int DPP_ROW_HALF_MIRROR = 0x141;
constexpr int DPP_ROW_MIRROR = 0x140;

MOFQ_DEV double readlane_f64(double v, int lane) {
  const uint64_t u = __builtin_bit_cast(uint64_t, v);
  const uint32_t lo = __builtin_amdgcn_readlane(static_cast<int>(u), lane);
  const uint32_t hi = __builtin_amdgcn_readlane(static_cast<int>(u >> 32), lane);
  return __builtin_bit_cast(double, (static_cast<uint64_t>(hi) << 32) | lo);
}

// Sum over 4 adjacent lanes; every lane of the quad gets it.
MOFQ_DEV double quad_sum(double v) {
  v += dpp_f64<DPP_QUAD_XOR1>(v);
  v += dpp_f64<DPP_QUAD_XOR2>(v);
  return v;
}
// Sum over each row of 16 lanes; every lane of the row gets it.
MOFQ_DEV double row16_sum(double v) {
  v = quad_sum(v);
  v += dpp_f64<DPP_ROW_HALF_MIRROR>(v);
  v += dpp_f64<DPP_ROW_MIRROR>(v);
  return v;
}
// Sum over the wave; uniform result (fixed order, so deterministic).
MOFQ_DEV double wave_sum(double v) {
  v = row16_sum(v);
  return (readlane_f64(v, 0) + readlane_f64(v, 16)) + (readlane_f64(v, 32) + readlane_f64(v, 48));
}

MOFQ_DEV float wave_max(float v) {
  v = __builtin_fmaxf(v, dpp_f32<DPP_QUAD_XOR1>(v));
  v = __builtin_fmaxf(v, dpp_f32<DPP_QUAD_XOR2>(v));
  v = __builtin_fmaxf(v, dpp_f32<DPP_ROW_HALF_MIRROR>(v));
  v = __builtin_fmaxf(v, dpp_f32<DPP_ROW_MIRROR>(v));
  const float a = u2f(__builtin_amdgcn_readlane(static_cast<int>(f2u(v)), 0));
  const float b = u2f(__builtin_amdgcn_readlane(static_cast<int>(f2u(v)), 16));
  const float c = u2f(__builtin_amdgcn_readlane(static_cast<int>(f2u(v)), 32));
  const float d = u2f(__builtin_amdgcn_readlane(static_cast<int>(f2u(v)), 48));
  return __builtin_fmaxf(__builtin_fmaxf(a, b), __builtin_fmaxf(c, d));
}

// Lexicographic minimum of (value, index) over the wave: smallest value, and
// among equal values the smallest index (the first candidate).  Uniform result.
MOFQ_DEV void wave_argmin(double& v, int& idx) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) {
    const double ov = __shfl_xor(v, m, 64);
    const int oi = __shfl_xor(idx, m, 64);
    const bool take = (ov < v) || (ov == v && oi < idx);
    v = take ? ov : v;
    idx = take ? oi : idx;
  }
}

}  // namespace mofq
