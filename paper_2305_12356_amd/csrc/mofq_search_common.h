// Shared by the two per-channel searches that do not score every (element, candidate) pair
// (mofq_sweep_sorted.hip: sort the row and search it; mofq_sweep_hist.hip: count the row's bit
// patterns): their kernel arguments and the device helpers both use.
#pragma once
#include <cmath>
#include <type_traits>

#include "mofq_device.h"
#include "mofq_internal.h"

namespace mofq {

// One launch searches up to kSweepGroupMax tensors of one row length, dtype and configuration:
// the rows of all tensors are numbered through, one workgroup per row.
struct SortedTensor {
  const void* w;
  int64_t ld;
  UnitRecords rec;
};
struct SortedArgs {
  SortedTensor t[kSweepGroupMax];
  uint32_t row0[kSweepGroupMax];   // number of the first row of tensor i (unused entries: 0xFFFFFFFF)
  int64_t cols;                    // of every tensor
  int32_t scale_f16, n_clip;
  int32_t nbin, ntbin;             // histogram kernel: counters of the row's histogram and of INT4's negative elements
  float clip[MOFQ_MAX_CLIP];
  // per format slot: level magnitudes 0 = m_0 < m_1 < ... < m_7;  |level|(t) <= m_b  <=>  t <= thr[b]
  // for b = 0..6.  Entry 7 is INT4's extra boundary (|t| below it: a negative element stays on -7)
  // with the weights of the step from 7 to 8; unused (zero weights) for E2M1.
  float thr[2][8];
  double dgd[2][8];   // m_b - m_{b+1};  entry 7: 8 - 7
  int32_t dg2q[2][8]; // 4 (m_b^2 - m_{b+1}^2): an integer for every 4-bit format;  entry 7: 4 (64 - 49)
  float g_last[2];    // m_7
  float g_absmax[2];  // largest |level|
};

constexpr int kHistMaxBins = 8192;      // histogram kernel: patterns with a counter at most (16 KB)
constexpr int kHistMaxTailBins = 2048;  // of INT4's negative elements

// The histogram kernel for arguments with nbin > 0 (mofq_sweep_hist.hip).
int launch_sweep_hist(const SweepParams& p, const SortedArgs& a, int64_t total_rows, hipStream_t st);

namespace {

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

// ---- sort keys ------------------------------------------------------------------------
// The key of an element is the low 15 bits of its own 16-bit pattern (the magnitude; fp16 and
// bf16 magnitudes order like their patterns); the sign bit rides along untouched.
typedef short i16x2 __attribute__((ext_vector_type(2)));
MOFQ_DEV uint32_t sign_fill2(uint32_t w) {   // each half: 0xFFFF where its top bit is set, else 0
  return __builtin_bit_cast(uint32_t, __builtin_bit_cast(i16x2, w) >> 15);
}

template <typename In> MOFQ_DEV float bits_to_float(uint32_t h);
template <> MOFQ_DEV float bits_to_float<F16>(uint32_t h) {
  return static_cast<float>(__builtin_bit_cast(_Float16, static_cast<uint16_t>(h)));
}
template <> MOFQ_DEV float bits_to_float<BF16>(uint32_t h) { return u2f(h << 16); }

// fl32(|x| * inv) for the element with bit pattern h.  For fp16 the widening and the product are
// one mixed-precision fused multiply-add with a zero addend: the same single rounding of the
// exact product.
template <typename In> MOFQ_DEV float scaled(uint32_t h, float inv);
template <> MOFQ_DEV float scaled<F16>(uint32_t h, float inv) {
  return __builtin_fmaf(__builtin_fabsf(static_cast<float>(__builtin_bit_cast(_Float16, static_cast<uint16_t>(h)))), inv, 0.0f);
}
template <> MOFQ_DEV float scaled<BF16>(uint32_t h, float inv) { return __builtin_fabsf(u2f(h << 16)) * inv; }

// x plus the value the data-parallel-primitive control CTRL brings from another lane (0 where
// the control has no source lane or ROW_MASK excludes the row)
template <int CTRL, int ROW_MASK> MOFQ_DEV uint32_t dpp_add_u32(uint32_t x) {
  return x + static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(x), CTRL, ROW_MASK, 0xf, false));
}
// exclusive prefix over the wave and the wave total: shifts by 1, 2, 4, 8 inside each row of
// 16 lanes, then lane 15 of a row into the next row, then lane 31 into the upper half
MOFQ_DEV uint32_t wave_excl_scan_u32(uint32_t v, uint32_t& total) {
  uint32_t inc = v;
  inc = dpp_add_u32<0x111, 0xf>(inc);   // row_shr:1
  inc = dpp_add_u32<0x112, 0xf>(inc);   // row_shr:2
  inc = dpp_add_u32<0x114, 0xf>(inc);   // row_shr:4
  inc = dpp_add_u32<0x118, 0xf>(inc);   // row_shr:8
  inc = dpp_add_u32<0x142, 0xa>(inc);   // row_bcast:15 into rows 1 and 3
  inc = dpp_add_u32<0x143, 0xc>(inc);   // row_bcast:31 into rows 2 and 3
  total = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(inc), 63));
  return inc - v;
}
// the same for doubles: each step moves the two halves of the running sum separately
template <int CTRL, int ROW_MASK> MOFQ_DEV double dpp_add_f64(double x) {
  const uint64_t u = __builtin_bit_cast(uint64_t, x);
  const uint32_t lo = static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(static_cast<uint32_t>(u)), CTRL, ROW_MASK, 0xf, false));
  const uint32_t hi = static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(static_cast<uint32_t>(u >> 32)), CTRL, ROW_MASK, 0xf, false));
  return x + __builtin_bit_cast(double, (static_cast<uint64_t>(hi) << 32) | lo);   // +0.0 where nothing arrives
}
MOFQ_DEV double wave_excl_scan_f64(double v, double& total) {
  double inc = v;
  inc = dpp_add_f64<0x111, 0xf>(inc);   // row_shr:1
  inc = dpp_add_f64<0x112, 0xf>(inc);   // row_shr:2
  inc = dpp_add_f64<0x114, 0xf>(inc);   // row_shr:4
  inc = dpp_add_f64<0x118, 0xf>(inc);   // row_shr:8
  inc = dpp_add_f64<0x142, 0xa>(inc);   // row_bcast:15 into rows 1 and 3
  inc = dpp_add_f64<0x143, 0xc>(inc);   // row_bcast:31 into rows 2 and 3
  total = __shfl(inc, 63, 64);
  return inc - v;
}

// sum over the wave in fp32 (uniform result)
MOFQ_DEV float wave_sum_f32(float v) {
  v += dpp_f32<DPP_QUAD_XOR1>(v);
  v += dpp_f32<DPP_QUAD_XOR2>(v);
  v += dpp_f32<DPP_ROW_HALF_MIRROR>(v);
  v += dpp_f32<DPP_ROW_MIRROR>(v);
  const float a = u2f(__builtin_amdgcn_readlane(static_cast<int>(f2u(v)), 0));
  const float b = u2f(__builtin_amdgcn_readlane(static_cast<int>(f2u(v)), 16));
  const float c = u2f(__builtin_amdgcn_readlane(static_cast<int>(f2u(v)), 32));
  const float d = u2f(__builtin_amdgcn_readlane(static_cast<int>(f2u(v)), 48));
  return (a + b) + (c + d);
}

// exact re-score of two elements (same arithmetic as the direct kernel's second phase)
template <int FMT> MOFQ_DEV void rescore2(double& acc, float x0, float x1, float inv_s, double sd, uint32_t& carry) {
  f32x2 g;
  if constexpr (FMT == MOFQ_FP4_E2M1) {
    carry = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(carry, x0 * inv_s, x1 * inv_s, 1.0f, 0);
    g = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(carry, 1.0f, 0);
  } else {
    g[0] = Codec<FMT>::grid(x0 * inv_s);
    g[1] = Codec<FMT>::grid(x1 * inv_s);
  }
  const double d0 = __builtin_fma(-static_cast<double>(g[0]), sd, static_cast<double>(x0));
  const double d1 = __builtin_fma(-static_cast<double>(g[1]), sd, static_cast<double>(x1));
  acc = __builtin_fma(d0, d0, acc);
  acc = __builtin_fma(d1, d1, acc);
}

}  // namespace

}  // namespace mofq
