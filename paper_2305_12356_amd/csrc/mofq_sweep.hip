// Scale search ("sweep"): for every unit of a tensor and every candidate format,
// evaluate all clip ratios and keep the first with the smallest error.
//
// This is the quantize_layer + compute_error pair of Algorithm 1 with the
// tensor-error metric (Section 4.1), evaluated for all scale candidates of a
// unit while the unit's elements sit in registers: the tensor is read from HBM
// once, however many candidates there are.
//
// Work per element and candidate (INT: multiply, round, clamp; FP: multiply,
// clamp, pick spacing, add/subtract rounding constant; then an fp64 residual and
// an fp64 fused multiply-add into the error) is plain vector ALU work: with the
// 100-candidate search the kernel is bound by the vector units, not by HBM.
#include <type_traits>

#include "mofq_device.h"
#include "mofq_internal.h"

namespace mofq {

namespace {

struct SweepArgs {
  const void* w;
  int64_t rows, cols, ld;
  int64_t units;
  int32_t group;
  int32_t scale_f16;
  int32_t n_clip;
  UnitRecords rec;
  float* absmax_part;
  double* sse_part;
  double* energy_part;
  int32_t n_blocks;  // per-tensor: blocks of the partial passes
  const float* ext_absmax;   // per-tensor: calibrated magnitude replacing the tensor's own, or nullptr
  int32_t k0;                // per-tensor: first clip candidate of this scoring pass
  uint8_t* emit_i8;          // per-tensor 8-bit pair: also write the codes (see SweepParams)
  void* emit_f8;
  int32_t emit_f8_as_bf16;
  uint16_t* emit_grid[kMaxFmt];   // per-channel single-candidate pair: grid values as bf16 (see SweepParams)
  float clip[MOFQ_MAX_CLIP];
};

// Squared error of one element at one scale: the grid value is chosen in fp32
// (the decision arithmetic), the residual and its square are fp64.
template <int FMT>
MOFQ_DEV void accumulate(double& acc, float x, double xd, float inv_s, double sd) {
  const float t = x * inv_s;
  if constexpr (Codec<FMT>::IS_INT) {
    const double g = static_cast<double>(Codec<FMT>::grid(t));
    const double d = __builtin_fma(-g, sd, xd);
    acc = __builtin_fma(d, d, acc);
  } else {
    // sign-symmetric grid: (|x| - |g| s)^2 == (x - g s)^2
    const double g = static_cast<double>(Codec<FMT>::mag(__builtin_fabsf(t)));
    const double d = __builtin_fma(-g, sd, __builtin_fabs(xd));
    acc = __builtin_fma(d, d, acc);
  }
}

// ---- grid value of a scaled element, two elements at a time ---------------------
//
// FP formats use the gfx950 pack-convert instructions (round to nearest even,
// subnormals, saturation); they agree with Codec<>::mag / code on every finite fp32
// bit pattern (checked exhaustively on the part), and cost about half the vector
// cycles of the add/subtract-constant form.
typedef float f32x2 __attribute__((ext_vector_type(2)));

// `carry` is the register the fp4 encode merges its byte into; its other bytes are
// never read, so it is simply handed from call to call (no clearing instruction).
template <int FMT> MOFQ_DEV f32x2 grid2(float t0, float t1, uint32_t& carry) {
  f32x2 g;
  if constexpr (FMT == MOFQ_FP4_E2M1) {
    carry = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(carry, t0, t1, 1.0f, 0);
    g = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(carry, 1.0f, 0);
  } else if constexpr (FMT == MOFQ_FP4_E2M1_IEEE) {
    // the same grid below 3: clamp, then the same convert
    carry = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(carry, med3(t0, -3.0f, 3.0f), med3(t1, -3.0f, 3.0f), 1.0f, 0);
    g = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(carry, 1.0f, 0);
  } else if constexpr (FMT == MOFQ_FP8_E4M3) {
    const int p = __builtin_amdgcn_cvt_pk_fp8_f32(med3(t0, -448.0f, 448.0f), med3(t1, -448.0f, 448.0f), 0, false);
    g = __builtin_amdgcn_cvt_pk_f32_fp8(p, false);
  } else {
    g[0] = Codec<FMT>::grid(t0);
    g[1] = Codec<FMT>::grid(t1);
  }
  return g;
}

// Phase 1 of the search: squared error of two elements in fp32 (fused residual and
// accumulation, relative error of a unit's sum below 60 * 2^-24).
template <int FMT> MOFQ_DEV void score2_f32(float& acc, float x0, float x1, float inv_s, float s, uint32_t& carry) {
  const f32x2 g = grid2<FMT>(x0 * inv_s, x1 * inv_s, carry);
  const float d0 = __builtin_fmaf(-g[0], s, x0);
  const float d1 = __builtin_fmaf(-g[1], s, x1);
  acc = __builtin_fmaf(d0, d0, acc);
  acc = __builtin_fmaf(d1, d1, acc);
}

// Phase 2: the same two elements with the residual and its square in fp64.
template <int FMT> MOFQ_DEV void score2_f64(double& acc, float x0, float x1, float inv_s, double sd, uint32_t& carry) {
  const f32x2 g = grid2<FMT>(x0 * inv_s, x1 * inv_s, carry);
  const double d0 = __builtin_fma(-static_cast<double>(g[0]), sd, static_cast<double>(x0));
  const double d1 = __builtin_fma(-static_cast<double>(g[1]), sd, static_cast<double>(x1));
  acc = __builtin_fma(d0, d0, acc);
  acc = __builtin_fma(d1, d1, acc);
}

// Sum over the wave in six DPP steps; the total is valid in lanes 48..63 only.
MOFQ_DEV float wave_sum_f32_hi(float v) {
  v += dpp_f32<DPP_QUAD_XOR1>(v);
  v += dpp_f32<DPP_QUAD_XOR2>(v);
  v += dpp_f32<DPP_ROW_HALF_MIRROR>(v);
  v += dpp_f32<DPP_ROW_MIRROR>(v);           // every lane: sum of its row of 16
  // rows 1 and 3 add the row before them, then rows 2 and 3 add lane 31 (rows 0+1)
  v += u2f(static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(f2u(v)), 0x142, 0xA, 0xF, false)));
  v += u2f(static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(f2u(v)), 0x143, 0xC, 0xF, false)));
  return v;
}

// Candidates whose fp32 error is within this factor of the smallest fp32 error are
// re-scored in fp64.  The fp32 sum of a unit is within (1 +- 60*2^-24) of the exact
// sum for the same grid choices, so the fp64 winner is always among them.
constexpr float kShortlistFactor = 1.0f + 1.0e-5f;
// Below this the fp32 sums may have lost terms to underflow: re-score everything.
constexpr float kTinySum = 0x1p-80f;

// ------------------------------------------------------------------------------
// Per-channel: one workgroup per row; the row lives in registers (CH chunks of 8
// elements per thread, chunk j of thread t = elements [(j*THREADS + t)*8, +8)).
//
// Phase 1 scores every (format, candidate) in fp32; phase 2 re-scores in fp64 the
// candidates that fp32 cannot separate from the best one and picks the first
// smallest of those, which is the first smallest of all.
// ------------------------------------------------------------------------------
template <typename In, int FA, int FB, int THREADS, int CH>
__global__ __launch_bounds__(THREADS) __attribute__((amdgpu_waves_per_eu(CH <= 4 ? 8 : 5))) void sweep_channel_kernel(const SweepArgs a) {
  using L = Load8<In>;
  constexpr int NF = (FB >= 0) ? 2 : 1;
  constexpr int FBX = (FB >= 0) ? FB : FA;
  constexpr int NW = THREADS / 64;
  constexpr int NE = CH * 8;
  constexpr int MAXL = NF * MOFQ_MAX_CLIP;

  __shared__ float s_scale[NF][MOFQ_MAX_CLIP];
  __shared__ float s_inv[NF][MOFQ_MAX_CLIP];
  __shared__ float s_p1[NW][MOFQ_MAX_CLIP][NF];   // phase-1 partial sums per wave
  __shared__ float s_tot[NF][MOFQ_MAX_CLIP];
  __shared__ float s_wmax[NW];
  __shared__ double s_wen[NW];
  __shared__ float s_thr[NF];
  __shared__ int s_list[MAXL];                    // shortlisted (format, candidate) pairs
  __shared__ int s_nlist;
  __shared__ double s_p2[NW];
  __shared__ double s_val[MAXL];                  // fp64 error of the shortlisted pairs

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int64_t row = blockIdx.x;
  const typename L::elem* src = static_cast<const typename L::elem*>(a.w) + row * a.ld;
  const int K = a.n_clip;

  float x[NE];
  float amax = 0.0f;
  double en = 0.0;
#pragma unroll
  for (int j = 0; j < CH; ++j) {
    const int64_t c0 = (static_cast<int64_t>(j) * THREADS + tid) * 8;
    float v[8];
    if (c0 < a.cols) {
      L::load(src + c0, v);
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] = 0.0f;
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      x[j * 8 + i] = v[i];
      amax = __builtin_fmaxf(amax, __builtin_fabsf(v[i]));
      const double xd = static_cast<double>(v[i]);
      en = __builtin_fma(xd, xd, en);
    }
  }

  // unit absmax and energy
  amax = wave_max(amax);
  en = wave_sum(en);
  if (lane == 0) { s_wmax[wave] = amax; s_wen[wave] = en; }
  __syncthreads();
  amax = s_wmax[0];
  en = s_wen[0];
#pragma unroll
  for (int w = 1; w < NW; ++w) { amax = __builtin_fmaxf(amax, s_wmax[w]); en += s_wen[w]; }

  // scales of every (format, candidate)
  for (int idx = tid; idx < NF * K; idx += THREADS) {
    const int f = idx / K, k = idx - f * K;
    const float qmax = (f == 0) ? Codec<FA>::QMAX : Codec<FBX>::QMAX;
    const float s = unit_scale(amax, a.clip[k], qmax, a.scale_f16 != 0);
    s_scale[f][k] = s;
    s_inv[f][k] = 1.0f / s;
  }
  __syncthreads();

  // which of this wave's chunks hold data (wave-uniform)
  bool live[CH];
#pragma unroll
  for (int j = 0; j < CH; ++j)
    live[j] = (static_cast<int64_t>(j) * THREADS + wave * 64) * 8 < a.cols;

  uint32_t carry = 0;
  // ---- phase 1: fp32 error of every candidate (nothing to filter with one candidate) --
  for (int k = 0; k < K && K > 1; ++k) {
    const float sA = u2f(__builtin_amdgcn_readfirstlane(f2u(s_scale[0][k])));
    const float iA = u2f(__builtin_amdgcn_readfirstlane(f2u(s_inv[0][k])));
    const float sB = u2f(__builtin_amdgcn_readfirstlane(f2u(s_scale[NF - 1][k])));
    const float iB = u2f(__builtin_amdgcn_readfirstlane(f2u(s_inv[NF - 1][k])));
    float accA = 0.0f, accB = 0.0f;
#pragma unroll
    for (int j = 0; j < CH; ++j) {
      if (live[j]) {
#pragma unroll
        for (int i = 0; i < 8; i += 2) {
          score2_f32<FA>(accA, x[j * 8 + i], x[j * 8 + i + 1], iA, sA, carry);
          if constexpr (NF == 2) score2_f32<FBX>(accB, x[j * 8 + i], x[j * 8 + i + 1], iB, sB, carry);
        }
      }
    }
    accA = wave_sum_f32_hi(accA);
    if constexpr (NF == 2) accB = wave_sum_f32_hi(accB);
    if (lane == 63) {
      s_p1[wave][k][0] = accA;
      if constexpr (NF == 2) s_p1[wave][k][1] = accB;
    }
  }
  __syncthreads();

  for (int idx = tid; idx < NF * K; idx += THREADS) {
    const int f = idx / K, k = idx - f * K;
    float t = 0.0f;
    if (K > 1) {
#pragma unroll
      for (int r = 0; r < NW; ++r) t += s_p1[r][k][f];
    }
    s_tot[f][k] = t;   // K == 1: zero, which shortlists the only candidate
  }
  __syncthreads();

  // ---- shortlist: candidates fp32 cannot tell from the best ----------------------
  for (int f = wave; f < NF; f += NW) {
    float m = __builtin_inff();
    for (int k = lane; k < K; k += 64) m = __builtin_fminf(m, s_tot[f][k]);
    m = -wave_max(-m);
    if (lane == 0) s_thr[f] = (m >= kTinySum && m < __builtin_inff()) ? m * kShortlistFactor : __builtin_inff();
  }
  __syncthreads();
  if (tid == 0) {
    int n = 0;
    for (int f = 0; f < NF; ++f)
      for (int k = 0; k < K; ++k)
        if (s_tot[f][k] <= s_thr[f] || !(s_tot[f][k] == s_tot[f][k])) s_list[n++] = f * MOFQ_MAX_CLIP + k;
    s_nlist = n;
  }
  __syncthreads();
  const int n_list = s_nlist;

  // ---- phase 2: fp64 error of the shortlisted candidates ---------------------------
  for (int e = 0; e < n_list; ++e) {
    const int fk = s_list[e];
    const int f = __builtin_amdgcn_readfirstlane(fk / MOFQ_MAX_CLIP);
    const int k = __builtin_amdgcn_readfirstlane(fk % MOFQ_MAX_CLIP);
    const float s = s_scale[f][k], inv = s_inv[f][k];
    const double sd = static_cast<double>(s);
    double acc = 0.0;
#pragma unroll
    for (int j = 0; j < CH; ++j) {
      if (live[j]) {
#pragma unroll
        for (int i = 0; i < 8; i += 2) {
          if (f == 0) score2_f64<FA>(acc, x[j * 8 + i], x[j * 8 + i + 1], inv, sd, carry);
          else score2_f64<FBX>(acc, x[j * 8 + i], x[j * 8 + i + 1], inv, sd, carry);
        }
      }
    }
    acc = wave_sum(acc);
    if (lane == 0) s_p2[wave] = acc;
    __syncthreads();
    if (tid == 0) {
      double t = s_p2[0];
#pragma unroll
      for (int w = 1; w < NW; ++w) t += s_p2[w];
      s_val[e] = t;
    }
    __syncthreads();
  }

  // first smallest fp64 error per format (the list is in candidate order)
  if (tid < NF) {
    const int f = tid;
    double best = __builtin_inf();
    int bk = -1;
    for (int e = 0; e < n_list; ++e) {
      const int fk = s_list[e];
      if (fk / MOFQ_MAX_CLIP != f) continue;
      if (s_val[e] < best) { best = s_val[e]; bk = fk % MOFQ_MAX_CLIP; }
    }
    if (bk < 0) { bk = 0; best = __builtin_nan(""); }   // only on non-finite input
    a.rec.scale[f][row] = s_scale[f][bk];
    a.rec.clip[f][row] = bk;
    a.rec.err[f][row] = best;
    if (f == 0 && a.rec.energy) a.rec.energy[row] = en;
  }
}

// ------------------------------------------------------------------------------
// Per-channel with a single candidate (absmax scale, no search): a memory-bound pass.
// Same register-resident row, but no candidate tables and two barriers in all; not
// held to the register budget of the search kernel.
// ------------------------------------------------------------------------------
#ifndef K1_WAVES
#define K1_WAVES 4
#endif
// GRID: the pass also writes the grid values of both formats as bf16 (dense rows), the operands
// of the weight-only layer-output products, so that they cost no further read of the tensor.
template <typename In, int FA, int FB, int THREADS, int CH, bool GRID = false>
__global__ __launch_bounds__(THREADS) __attribute__((amdgpu_waves_per_eu(GRID ? 2 : K1_WAVES))) void sweep_channel_single_kernel(const SweepArgs a) {
  using L = Load8<In>;
  constexpr int NF = (FB >= 0) ? 2 : 1;
  constexpr int FBX = (FB >= 0) ? FB : FA;
  constexpr int NW = THREADS / 64;
  constexpr int NE = CH * 8;
  __shared__ float s_wmax[NW];
  __shared__ double s_wen[NW];
  __shared__ double s_acc[2][NW];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int64_t row = blockIdx.x;
  const typename L::elem* src = static_cast<const typename L::elem*>(a.w) + row * a.ld;

  float x[NE];
  float amax = 0.0f;
  double en = 0.0;
#pragma unroll
  for (int j = 0; j < CH; ++j) {
    const int64_t c0 = (static_cast<int64_t>(j) * THREADS + tid) * 8;
    float v[8];
    if (c0 < a.cols) {
      L::load(src + c0, v);
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] = 0.0f;   // zeros past the row's end add nothing
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      x[j * 8 + i] = v[i];
      amax = __builtin_fmaxf(amax, __builtin_fabsf(v[i]));
      const double xd = static_cast<double>(v[i]);
      en = __builtin_fma(xd, xd, en);
    }
  }
  amax = wave_max(amax);
  en = wave_sum(en);
  if (lane == 0) { s_wmax[wave] = amax; s_wen[wave] = en; }
  __syncthreads();
  amax = s_wmax[0];
  en = s_wen[0];
#pragma unroll
  for (int w = 1; w < NW; ++w) { amax = __builtin_fmaxf(amax, s_wmax[w]); en += s_wen[w]; }

  const float sA = unit_scale(amax, a.clip[0], Codec<FA>::QMAX, a.scale_f16 != 0);
  const float sB = unit_scale(amax, a.clip[0], Codec<FBX>::QMAX, a.scale_f16 != 0);
  const float iA = 1.0f / sA, iB = 1.0f / sB;
  const double sAd = static_cast<double>(sA), sBd = static_cast<double>(sB);
  double accA = 0.0, accB = 0.0;
  uint32_t carry = 0;
#pragma unroll
  for (int j = 0; j < CH; ++j) {
    if constexpr (GRID) {
      // grid values have at most 7 significant bits: exact in bf16 (the top half of an fp32)
      u32x4 ga, gb;
#pragma unroll
      for (int i = 0; i < 8; i += 2) {
        const float x0 = x[j * 8 + i], x1 = x[j * 8 + i + 1];
        const f32x2 qa = grid2<FA>(x0 * iA, x1 * iA, carry);
        const f32x2 qb = grid2<FBX>(x0 * iB, x1 * iB, carry);
        ga[i >> 1] = (f2u(qa[0]) >> 16) | (f2u(qa[1]) & 0xFFFF0000u);
        gb[i >> 1] = (f2u(qb[0]) >> 16) | (f2u(qb[1]) & 0xFFFF0000u);
        const double a0 = __builtin_fma(-static_cast<double>(qa[0]), sAd, static_cast<double>(x0));
        const double a1 = __builtin_fma(-static_cast<double>(qa[1]), sAd, static_cast<double>(x1));
        accA = __builtin_fma(a0, a0, accA);
        accA = __builtin_fma(a1, a1, accA);
        const double b0 = __builtin_fma(-static_cast<double>(qb[0]), sBd, static_cast<double>(x0));
        const double b1 = __builtin_fma(-static_cast<double>(qb[1]), sBd, static_cast<double>(x1));
        accB = __builtin_fma(b0, b0, accB);
        accB = __builtin_fma(b1, b1, accB);
      }
      const int64_t c0 = (static_cast<int64_t>(j) * THREADS + tid) * 8;
      if (c0 < a.cols) {
        const int64_t e8 = (row * a.cols + c0) / 8;
        reinterpret_cast<u32x4*>(a.emit_grid[0])[e8] = ga;
        reinterpret_cast<u32x4*>(a.emit_grid[1])[e8] = gb;
      }
    } else {
#pragma unroll
      for (int i = 0; i < 8; i += 2) {
        score2_f64<FA>(accA, x[j * 8 + i], x[j * 8 + i + 1], iA, sAd, carry);
        if constexpr (NF == 2) score2_f64<FBX>(accB, x[j * 8 + i], x[j * 8 + i + 1], iB, sBd, carry);
      }
    }
  }
  accA = wave_sum(accA);
  if constexpr (NF == 2) accB = wave_sum(accB);
  if (lane == 0) { s_acc[0][wave] = accA; s_acc[1][wave] = accB; }
  __syncthreads();
  if (tid < NF) {
    double t = 0.0;
#pragma unroll
    for (int w = 0; w < NW; ++w) t += s_acc[tid][w];
    a.rec.scale[tid][row] = tid == 0 ? sA : sB;
    a.rec.clip[tid][row] = 0;
    a.rec.err[tid][row] = t;
    if (tid == 0 && a.rec.energy) a.rec.energy[row] = en;
  }
}

// ------------------------------------------------------------------------------
// Per-group: LPG lanes share one group of GROUP elements; each lane holds
// GROUP/LPG consecutive elements.  Scales differ per group, so they are per-lane
// values; the LPG lanes of a group split the scale computations of a batch of LPG
// candidates and hand them round with DPP.
// ------------------------------------------------------------------------------
template <int LPG> MOFQ_DEV double group_sum(double v);
template <> MOFQ_DEV double group_sum<4>(double v) { return quad_sum(v); }
template <> MOFQ_DEV double group_sum<16>(double v) { return row16_sum(v); }
template <int LPG> MOFQ_DEV float group_max(float v);
template <> MOFQ_DEV float group_max<4>(float v) {
  v = __builtin_fmaxf(v, dpp_f32<DPP_QUAD_XOR1>(v));
  return __builtin_fmaxf(v, dpp_f32<DPP_QUAD_XOR2>(v));
}
template <> MOFQ_DEV float group_max<16>(float v) {
  v = group_max<4>(v);
  v = __builtin_fmaxf(v, dpp_f32<DPP_ROW_HALF_MIRROR>(v));
  return __builtin_fmaxf(v, dpp_f32<DPP_ROW_MIRROR>(v));
}

// value held by lane `j` of the caller's quad
template <int J> MOFQ_DEV float quad_bcast(float v) { return dpp_f32<J * 0x55>(v); }

MOFQ_DEV float quad_sum_f32(float v) {
  v += dpp_f32<DPP_QUAD_XOR1>(v);
  return v + dpp_f32<DPP_QUAD_XOR2>(v);    // the same value in all four lanes
}
MOFQ_DEV uint32_t quad_or(uint32_t v) {
  v |= static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(v), DPP_QUAD_XOR1, 0xF, 0xF, false));
  return v | static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(v), DPP_QUAD_XOR2, 0xF, 0xF, false));
}

constexpr int kGroupQuads = 256 / 4;             // groups per workgroup
constexpr int kMaskWords = MOFQ_MAX_CLIP / 32;

// Phase 1 scores every candidate of a group in fp32 (hardware fp4/fp8 converts) and
// parks the sums in LDS; the candidates fp32 cannot tell from the group's best are
// collected in a bit mask per group and re-scored in fp64 in candidate order, the j-th
// survivor of all 16 groups of a wave at the same time.  The fp32 sum of a group (32
// terms per lane, two more additions across the quad) is within (1 +- 40*2^-24) of the
// exact sum for the same grid choices, so the fp64 winner is always among the survivors.
template <typename In, int FA, int FB, int GROUP>
__global__ __launch_bounds__(256) void sweep_group_kernel(const SweepArgs a) {
  using L = Load8<In>;
  constexpr int NF = (FB >= 0) ? 2 : 1;
  constexpr int FBX = (FB >= 0) ? FB : FA;
  constexpr int LPG = 4;
  constexpr int NE = GROUP / LPG;       // elements per lane
  constexpr int CH = NE / 8;
  static_assert(NE % 8 == 0, "group too small for 4 lanes");

  extern __shared__ float s_dyn[];      // clip[K], then p1[NF][K][kGroupQuads]
  const int K = a.n_clip;
  float* s_clip = s_dyn;
  float* s_p1 = s_dyn + MOFQ_MAX_CLIP;

  const int tid = threadIdx.x;
  const int q = tid & (LPG - 1);
  const int quad = tid >> 2;
  const int64_t gpr = a.cols / GROUP;   // groups per row
  int64_t unit = static_cast<int64_t>(blockIdx.x) * kGroupQuads + quad;
  const bool valid = unit < a.units;
  if (!valid) unit = a.units - 1;       // keep every lane active for the DPP exchanges
  const int64_t row = unit / gpr, gi = unit - row * gpr;
  const typename L::elem* src =
      static_cast<const typename L::elem*>(a.w) + row * a.ld + gi * GROUP + q * NE;
  const bool f16 = a.scale_f16 != 0;

  for (int k = tid; k < K; k += 256) s_clip[k] = a.clip[k];

  float x[NE];
  float amax = 0.0f;
  double en = 0.0;
#pragma unroll
  for (int j = 0; j < CH; ++j) {
    float v[8];
    L::load(src + j * 8, v);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      x[j * 8 + i] = v[i];
      amax = __builtin_fmaxf(amax, __builtin_fabsf(v[i]));
      const double xd = static_cast<double>(v[i]);
      en = __builtin_fma(xd, xd, en);
    }
  }
  amax = group_max<LPG>(amax);
  en = group_sum<LPG>(en);
  __syncthreads();                       // clip table in place

  uint32_t carry = 0;
  uint32_t maskA[kMaskWords], maskB[kMaskWords];
#pragma unroll
  for (int w = 0; w < kMaskWords; ++w) { maskA[w] = 0; maskB[w] = 0; }

  if (K > 1) {
    // ---- phase 1 ----------------------------------------------------------------
    float minA = __builtin_inff(), minB = __builtin_inff();
    for (int k0 = 0; k0 < K; k0 += LPG) {
      // lane q of the group prepares candidate k0+q (clamped; surplus ones are ignored)
      const int kq = (k0 + q < K) ? k0 + q : K - 1;
      const float r = s_clip[kq];
      const float mysA = unit_scale(amax, r, Codec<FA>::QMAX, f16);
      const float myiA = 1.0f / mysA;
      float mysB = 0.0f, myiB = 0.0f;
      if constexpr (NF == 2) {
        mysB = unit_scale(amax, r, Codec<FBX>::QMAX, f16);
        myiB = 1.0f / mysB;
      }
      auto one = [&](float sA, float iA, float sB, float iB, int k) {
        if (k < K) {   // uniform over the workgroup
          float accA = 0.0f, accB = 0.0f;
#pragma unroll
          for (int i = 0; i < NE; i += 2) {
            score2_f32<FA>(accA, x[i], x[i + 1], iA, sA, carry);
            if constexpr (NF == 2) score2_f32<FBX>(accB, x[i], x[i + 1], iB, sB, carry);
          }
          accA = quad_sum_f32(accA);
          minA = __builtin_fminf(minA, accA);
          if (q == 0) s_p1[k * kGroupQuads + quad] = accA;
          if constexpr (NF == 2) {
            accB = quad_sum_f32(accB);
            minB = __builtin_fminf(minB, accB);
            if (q == 1) s_p1[(K + k) * kGroupQuads + quad] = accB;
          }
        }
      };
      one(quad_bcast<0>(mysA), quad_bcast<0>(myiA), quad_bcast<0>(mysB), quad_bcast<0>(myiB), k0 + 0);
      one(quad_bcast<1>(mysA), quad_bcast<1>(myiA), quad_bcast<1>(mysB), quad_bcast<1>(myiB), k0 + 1);
      one(quad_bcast<2>(mysA), quad_bcast<2>(myiA), quad_bcast<2>(mysB), quad_bcast<2>(myiB), k0 + 2);
      one(quad_bcast<3>(mysA), quad_bcast<3>(myiA), quad_bcast<3>(mysB), quad_bcast<3>(myiB), k0 + 3);
    }
    __syncthreads();                     // the sums parked by lanes 0 and 1 are visible to the quad

    // ---- survivors: lane q tests candidates q, q+4, ... ----------------------------
    const float thrA = (minA >= kTinySum && minA < __builtin_inff()) ? minA * kShortlistFactor : __builtin_inff();
    const float thrB = (minB >= kTinySum && minB < __builtin_inff()) ? minB * kShortlistFactor : __builtin_inff();
    for (int k = q; k < K; k += LPG) {
      const float vA = s_p1[k * kGroupQuads + quad];
      const uint32_t bit = 1u << (k & 31);
      const bool keepA = vA <= thrA || !(vA == vA);
      bool keepB = false;
      if constexpr (NF == 2) {
        const float vB = s_p1[(K + k) * kGroupQuads + quad];
        keepB = vB <= thrB || !(vB == vB);
      }
#pragma unroll
      for (int w = 0; w < kMaskWords; ++w) {
        if ((k >> 5) == w) {
          if (keepA) maskA[w] |= bit;
          if (keepB) maskB[w] |= bit;
        }
      }
    }
#pragma unroll
    for (int w = 0; w < kMaskWords; ++w) {
      maskA[w] = quad_or(maskA[w]);
      if constexpr (NF == 2) maskB[w] = quad_or(maskB[w]);
    }
  } else {
    maskA[0] = 1u;
    if constexpr (NF == 2) maskB[0] = 1u;
  }

  // ---- phase 2: fp64 error of the survivors, first smallest wins -------------------
  double bestA = __builtin_inf(), bestB = __builtin_inf();
  int bkA = -1, bkB = -1;
  float bsA = 1.0f, bsB = 1.0f;
  auto rescore = [&](auto fmt_c, uint32_t (&mask)[kMaskWords], double& best, int& bk, float& bs) {
    constexpr int FMT = decltype(fmt_c)::value;
    for (;;) {
      int k = -1;                        // this group's next survivor, in candidate order
#pragma unroll
      for (int w = 0; w < kMaskWords; ++w) {
        if (k < 0 && mask[w] != 0) {
          k = w * 32 + __builtin_ctz(mask[w]);
          mask[w] &= mask[w] - 1;
        }
      }
      if (__builtin_amdgcn_ballot_w64(k >= 0) == 0) break;
      const float s = unit_scale(amax, s_clip[k >= 0 ? k : 0], Codec<FMT>::QMAX, f16);
      const float inv = 1.0f / s;
      const double sd = static_cast<double>(s);
      double acc = 0.0;
#pragma unroll
      for (int i = 0; i < NE; i += 2) score2_f64<FMT>(acc, x[i], x[i + 1], inv, sd, carry);
      acc = group_sum<LPG>(acc);
      if (k >= 0 && acc < best) { best = acc; bk = k; bs = s; }
    }
  };
  rescore(std::integral_constant<int, FA>{}, maskA, bestA, bkA, bsA);
  if constexpr (NF == 2) rescore(std::integral_constant<int, FBX>{}, maskB, bestB, bkB, bsB);

  if (valid && q == 0) {
    if (bkA < 0) { bkA = 0; bestA = __builtin_nan(""); bsA = unit_scale(amax, s_clip[0], Codec<FA>::QMAX, f16); }   // only on non-finite input
    a.rec.scale[0][unit] = bsA;
    a.rec.clip[0][unit] = bkA;
    a.rec.err[0][unit] = bestA;
    if constexpr (NF == 2) {
      if (bkB < 0) { bkB = 0; bestB = __builtin_nan(""); bsB = unit_scale(amax, s_clip[0], Codec<FBX>::QMAX, f16); }
      a.rec.scale[1][unit] = bsB;
      a.rec.clip[1][unit] = bkB;
      a.rec.err[1][unit] = bestB;
    }
    if (a.rec.energy) a.rec.energy[unit] = en;
  }
}

// ------------------------------------------------------------------------------
// Per-tensor: absmax pass, then a pass of per-block partial errors, then one
// block that adds the partials in block order and picks the candidate.
// ------------------------------------------------------------------------------
template <typename In>
__global__ __launch_bounds__(256) void tensor_absmax_kernel(const SweepArgs a) {
  using L = Load8<In>;
  __shared__ float s_wmax[4];
  __shared__ double s_wen[4];
  const int tid = threadIdx.x;
  const int64_t cpr = a.cols / 8;                 // chunks per row
  const int64_t n_chunks = a.rows * cpr;
  float amax = 0.0f;
  double en = 0.0;
  for (int64_t c = static_cast<int64_t>(blockIdx.x) * 256 + tid; c < n_chunks;
       c += static_cast<int64_t>(gridDim.x) * 256) {
    const int64_t row = c / cpr, col = (c - row * cpr) * 8;
    float v[8];
    L::load(static_cast<const typename L::elem*>(a.w) + row * a.ld + col, v);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      amax = __builtin_fmaxf(amax, __builtin_fabsf(v[i]));
      const double d = static_cast<double>(v[i]);
      en = __builtin_fma(d, d, en);
    }
  }
  amax = wave_max(amax);
  en = wave_sum(en);
  if ((tid & 63) == 0) { s_wmax[tid >> 6] = amax; s_wen[tid >> 6] = en; }
  __syncthreads();
  if (tid == 0) {
    a.absmax_part[blockIdx.x] =
        __builtin_fmaxf(__builtin_fmaxf(s_wmax[0], s_wmax[1]), __builtin_fmaxf(s_wmax[2], s_wmax[3]));
    a.energy_part[blockIdx.x] = (s_wen[0] + s_wen[1]) + (s_wen[2] + s_wen[3]);
  }
}

constexpr int kTensorMaxClip = 8;

MOFQ_DEV float tensor_absmax(const SweepArgs& a, float* s_tmp) {
  if (a.ext_absmax) return *a.ext_absmax;   // uniform over the grid
  const int tid = threadIdx.x;
  float m = 0.0f;
  for (int i = tid; i < a.n_blocks; i += 256) m = __builtin_fmaxf(m, a.absmax_part[i]);
  m = wave_max(m);
  if ((tid & 63) == 0) s_tmp[tid >> 6] = m;
  __syncthreads();
  return __builtin_fmaxf(__builtin_fmaxf(s_tmp[0], s_tmp[1]), __builtin_fmaxf(s_tmp[2], s_tmp[3]));
}

template <typename In, int FA, int FB>
__global__ __launch_bounds__(256) void tensor_score_kernel(const SweepArgs a) {
  using L = Load8<In>;
  constexpr int NF = (FB >= 0) ? 2 : 1;
  constexpr int FBX = (FB >= 0) ? FB : FA;
  __shared__ float s_tmp[4];
  __shared__ float s_scale[NF][kTensorMaxClip];
  __shared__ float s_inv[NF][kTensorMaxClip];
  __shared__ double s_part[4][NF][kTensorMaxClip];
  const int tid = threadIdx.x;
  // one pass scores up to kTensorMaxClip candidates, a.k0 onwards (more candidates: more passes)
  const int K = (a.n_clip - a.k0) < kTensorMaxClip ? (a.n_clip - a.k0) : kTensorMaxClip;
  const float amax = tensor_absmax(a, s_tmp);
  if (tid < NF * K) {
    const int f = tid / K, k = tid - f * K;
    const float s = unit_scale(amax, a.clip[a.k0 + k], f == 0 ? Codec<FA>::QMAX : Codec<FBX>::QMAX,
                               a.scale_f16 != 0);
    s_scale[f][k] = s;
    s_inv[f][k] = 1.0f / s;
  }
  __syncthreads();

  double acc[NF][kTensorMaxClip];
#pragma unroll
  for (int f = 0; f < NF; ++f)
#pragma unroll
    for (int k = 0; k < kTensorMaxClip; ++k) acc[f][k] = 0.0;

  const int64_t cpr = a.cols / 8;
  const int64_t n_chunks = a.rows * cpr;
  for (int64_t c = static_cast<int64_t>(blockIdx.x) * 256 + tid; c < n_chunks;
       c += static_cast<int64_t>(gridDim.x) * 256) {
    const int64_t row = c / cpr, col = (c - row * cpr) * 8;
    float v[8];
    L::load(static_cast<const typename L::elem*>(a.w) + row * a.ld + col, v);
#pragma unroll
    for (int k = 0; k < kTensorMaxClip; ++k) {
      if (k < K) {
        const float iA = s_inv[0][k], iB = s_inv[NF - 1][k];
        const double sAd = static_cast<double>(s_scale[0][k]);
        const double sBd = static_cast<double>(s_scale[NF - 1][k]);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const double xd = static_cast<double>(v[i]);
          accumulate<FA>(acc[0][k], v[i], xd, iA, sAd);
          if constexpr (NF == 2) accumulate<FBX>(acc[1][k], v[i], xd, iB, sBd);
        }
      }
    }
  }
#pragma unroll
  for (int f = 0; f < NF; ++f)
#pragma unroll
    for (int k = 0; k < kTensorMaxClip; ++k) {
      if (k < K) {
        const double t = wave_sum(acc[f][k]);
        if ((tid & 63) == 0) s_part[tid >> 6][f][k] = t;
      }
    }
  __syncthreads();
  if (tid < NF * K) {
    const int f = tid / K, k = tid - f * K;
    a.sse_part[(static_cast<int64_t>(blockIdx.x) * NF + f) * a.n_clip + a.k0 + k] =
        (s_part[0][f][k] + s_part[1][f][k]) + (s_part[2][f][k] + s_part[3][f][k]);
  }
}

// Per-tensor (INT8, FP8-E4M3) pair at one clip ratio, as the weight-activation path uses
// it: the same partial errors as tensor_score_kernel, and in the same pass the int8 codes
// and the E4M3 codes (or their grid values as bf16) of every element, so that the operands
// of the layer-output products cost one read of the tensor instead of three.
template <typename In>
__global__ __launch_bounds__(256) void tensor_score_emit8_kernel(const SweepArgs a) {
  using L = Load8<In>;
  __shared__ float s_tmp[4];
  __shared__ double s_part[4][2];
  const int tid = threadIdx.x;
  const float amax = tensor_absmax(a, s_tmp);
  const float sA = unit_scale(amax, a.clip[0], Codec<MOFQ_INT8>::QMAX, a.scale_f16 != 0);
  const float sB = unit_scale(amax, a.clip[0], Codec<MOFQ_FP8_E4M3>::QMAX, a.scale_f16 != 0);
  const float iA = 1.0f / sA, iB = 1.0f / sB;
  const double sAd = static_cast<double>(sA), sBd = static_cast<double>(sB);
  double accA = 0.0, accB = 0.0;
  const int64_t cpr = a.cols / 8;
  const int64_t n_chunks = a.rows * cpr;
  for (int64_t c = static_cast<int64_t>(blockIdx.x) * 256 + tid; c < n_chunks;
       c += static_cast<int64_t>(gridDim.x) * 256) {
    const int64_t row = c / cpr, col = (c - row * cpr) * 8;
    float v[8];
    L::load(static_cast<const typename L::elem*>(a.w) + row * a.ld + col, v);
    uint32_t wi[2] = {0u, 0u};
    int wf[2] = {0, 0};
    u32x4 gb;
#pragma unroll
    for (int i = 0; i < 8; i += 2) {
      // INT8
      const float q0 = Codec<MOFQ_INT8>::grid(v[i] * iA), q1 = Codec<MOFQ_INT8>::grid(v[i + 1] * iA);
      wi[i >> 2] |= (static_cast<uint32_t>(static_cast<int>(q0)) & 0xFFu) << (8 * (i & 3));
      wi[i >> 2] |= (static_cast<uint32_t>(static_cast<int>(q1)) & 0xFFu) << (8 * ((i & 3) + 1));
      const double d0 = __builtin_fma(-static_cast<double>(q0), sAd, static_cast<double>(v[i]));
      const double d1 = __builtin_fma(-static_cast<double>(q1), sAd, static_cast<double>(v[i + 1]));
      accA = __builtin_fma(d0, d0, accA);
      accA = __builtin_fma(d1, d1, accA);
      // E4M3: pack-convert (exact agreement with the codec, see grid2), decode for the error
      const int p = __builtin_amdgcn_cvt_pk_fp8_f32(med3(v[i] * iB, -448.0f, 448.0f),
                                                    med3(v[i + 1] * iB, -448.0f, 448.0f), 0, false);
      const f32x2 g = __builtin_amdgcn_cvt_pk_f32_fp8(p, false);
      wf[i >> 2] |= (p & 0xFFFF) << (16 * ((i >> 1) & 1));
      gb[i >> 1] = (f2u(g[0]) >> 16) | (f2u(g[1]) & 0xFFFF0000u);
      const double e0 = __builtin_fma(-static_cast<double>(g[0]), sBd, static_cast<double>(v[i]));
      const double e1 = __builtin_fma(-static_cast<double>(g[1]), sBd, static_cast<double>(v[i + 1]));
      accB = __builtin_fma(e0, e0, accB);
      accB = __builtin_fma(e1, e1, accB);
    }
    const int64_t e8 = (row * a.cols + col) / 8;   // dense output rows
    u32x2 oi;
    oi[0] = wi[0];
    oi[1] = wi[1];
    reinterpret_cast<u32x2*>(a.emit_i8)[e8] = oi;
    if (a.emit_f8_as_bf16) {
      reinterpret_cast<u32x4*>(a.emit_f8)[e8] = gb;
    } else {
      u32x2 of;
      of[0] = static_cast<uint32_t>(wf[0]);
      of[1] = static_cast<uint32_t>(wf[1]);
      reinterpret_cast<u32x2*>(a.emit_f8)[e8] = of;
    }
  }
  accA = wave_sum(accA);
  accB = wave_sum(accB);
  if ((tid & 63) == 0) { s_part[tid >> 6][0] = accA; s_part[tid >> 6][1] = accB; }
  __syncthreads();
  if (tid < 2)
    a.sse_part[static_cast<int64_t>(blockIdx.x) * 2 + tid] =
        (s_part[0][tid] + s_part[1][tid]) + (s_part[2][tid] + s_part[3][tid]);
}

template <int FA, int FB>
__global__ __launch_bounds__(256) void tensor_finalize_kernel(const SweepArgs a) {
  constexpr int NF = (FB >= 0) ? 2 : 1;
  constexpr int FBX = (FB >= 0) ? FB : FA;
  __shared__ float s_tmp[4];
  __shared__ double s_red[4];
  __shared__ double s_tot[NF][MOFQ_MAX_CLIP];
  const int tid = threadIdx.x;
  const int K = a.n_clip;
  const float amax = tensor_absmax(a, s_tmp);
  // Partials in a fixed order.  Few (format, candidate) pairs: the whole workgroup adds each
  // of them; many: one wave per pair.
  if (NF * K <= 4) {
    for (int idx = 0; idx < NF * K; ++idx) {
      const int f = idx / K, k = idx - f * K;
      double t = 0.0;
      for (int b = tid; b < a.n_blocks; b += 256)
        t += a.sse_part[(static_cast<int64_t>(b) * NF + f) * K + k];
      t = wave_sum(t);
      __syncthreads();
      if ((tid & 63) == 0) s_red[tid >> 6] = t;
      __syncthreads();
      if (tid == 0) s_tot[f][k] = (s_red[0] + s_red[1]) + (s_red[2] + s_red[3]);
    }
  } else {
    for (int idx = tid >> 6; idx < NF * K; idx += 4) {
      const int f = idx / K, k = idx - f * K;
      double t = 0.0;
      for (int b = tid & 63; b < a.n_blocks; b += 64)
        t += a.sse_part[(static_cast<int64_t>(b) * NF + f) * K + k];
      t = wave_sum(t);
      if ((tid & 63) == 0) s_tot[f][k] = t;
    }
  }
  double en = 0.0;
  for (int b = tid; b < a.n_blocks; b += 256) en += a.energy_part[b];
  en = wave_sum(en);
  __syncthreads();
  if ((tid & 63) == 0) s_red[tid >> 6] = en;
  __syncthreads();
  if (tid == 0) {
    for (int f = 0; f < NF; ++f) {
      double best = __builtin_inf();
      int bk = 0;
      for (int k = 0; k < K; ++k)
        if (s_tot[f][k] < best) { best = s_tot[f][k]; bk = k; }
      a.rec.scale[f][0] = unit_scale(amax, a.clip[bk], f == 0 ? Codec<FA>::QMAX : Codec<FBX>::QMAX,
                                     a.scale_f16 != 0);
      a.rec.clip[f][0] = bk;
      a.rec.err[f][0] = best;
    }
    if (a.rec.energy) a.rec.energy[0] = (s_red[0] + s_red[1]) + (s_red[2] + s_red[3]);
  }
}

// *dst = max(*dst, max of the partials): one workgroup.
__global__ __launch_bounds__(256) void absmax_fold_kernel(const float* part, int n, float* dst) {
  __shared__ float s_tmp[4];
  const int tid = threadIdx.x;
  float m = 0.0f;
  for (int i = tid; i < n; i += 256) m = __builtin_fmaxf(m, part[i]);
  m = wave_max(m);
  if ((tid & 63) == 0) s_tmp[tid >> 6] = m;
  __syncthreads();
  if (tid == 0) {
    m = __builtin_fmaxf(__builtin_fmaxf(s_tmp[0], s_tmp[1]), __builtin_fmaxf(s_tmp[2], s_tmp[3]));
    *dst = __builtin_fmaxf(*dst, m);
  }
}

// ---- dispatch ---------------------------------------------------------------------

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

template <typename In, int FA, int FB>
int launch_channel(const SweepArgs& a, hipStream_t st) {
  const dim3 grid(static_cast<unsigned>(a.rows));
  const int64_t chunks = a.cols / 8;
#define MOFQ_CH(THREADS, CH)                                                            \
  if (chunks <= static_cast<int64_t>(THREADS) * (CH)) {                                  \
    if (a.emit_grid[0]) {                                                                \
      if constexpr (std::is_same<In, BF16>::value && FB >= 0) {                          \
        if (a.n_clip != 1 || !a.emit_grid[1]) return MOFQ_ERR_UNSUPPORTED;               \
        hipLaunchKernelGGL((sweep_channel_single_kernel<In, FA, FB, THREADS, CH, true>), grid, dim3(THREADS), 0, st, a); \
      } else {                                                                           \
        return MOFQ_ERR_UNSUPPORTED;                                                     \
      }                                                                                  \
    } else if (a.n_clip == 1)                                                            \
      hipLaunchKernelGGL((sweep_channel_single_kernel<In, FA, FB, THREADS, CH>), grid, dim3(THREADS), 0, st, a); \
    else                                                                                 \
      hipLaunchKernelGGL((sweep_channel_kernel<In, FA, FB, THREADS, CH>), grid, dim3(THREADS), 0, st, a); \
    return hip_status(hipGetLastError());                                                \
  }
  // 32 to 48 elements per lane: enough work per candidate to amortise the cross-lane
  // reduction, few enough registers for many waves per SIMD
  MOFQ_CH(64, 1)     //   512 columns
  MOFQ_CH(64, 4)     //  2048
  MOFQ_CH(128, 4)    //  4096
  MOFQ_CH(256, 4)    //  8192
  MOFQ_CH(256, 6)    // 12288
  MOFQ_CH(512, 4)    // 16384
  MOFQ_CH(512, 6)    // 24576
  MOFQ_CH(1024, 4)   // 32768
#undef MOFQ_CH
  return MOFQ_ERR_UNSUPPORTED;
}

template <typename In, int FA, int FB>
int launch_group(const SweepArgs& a, hipStream_t st) {
  const dim3 grid(static_cast<unsigned>(ceil_div(a.units, kGroupQuads)));
  constexpr int NF = (FB >= 0) ? 2 : 1;
  const size_t lds = sizeof(float) * (MOFQ_MAX_CLIP + static_cast<size_t>(NF) * a.n_clip * kGroupQuads);
  switch (a.group) {
#define MOFQ_G(G)                                                                        \
  case G:                                                                                \
    hipLaunchKernelGGL((sweep_group_kernel<In, FA, FB, G>), grid, dim3(256), lds, st, a);  \
    return hip_status(hipGetLastError());
    MOFQ_G(32)
    MOFQ_G(64)
    MOFQ_G(128)
    MOFQ_G(256)
#undef MOFQ_G
  }
  return MOFQ_ERR_UNSUPPORTED;
}

template <typename In, int FA, int FB>
int launch_tensor(SweepArgs a, hipStream_t st) {
  const int64_t n_chunks = a.rows * (a.cols / 8);
  a.n_blocks = static_cast<int32_t>(std::min<int64_t>(kTensorBlocks, ceil_div(n_chunks, 256)));
  hipLaunchKernelGGL((tensor_absmax_kernel<In>), dim3(a.n_blocks), dim3(256), 0, st, a);
  if constexpr (FA == MOFQ_INT8 && FB == MOFQ_FP8_E4M3) {
    if (a.emit_i8 && a.emit_f8 && a.n_clip == 1) {
      hipLaunchKernelGGL((tensor_score_emit8_kernel<In>), dim3(a.n_blocks), dim3(256), 0, st, a);
      hipLaunchKernelGGL((tensor_finalize_kernel<FA, FB>), dim3(1), dim3(256), 0, st, a);
      return hip_status(hipGetLastError());
    }
  }
  if (a.emit_i8 || a.emit_f8) return MOFQ_ERR_UNSUPPORTED;
  for (a.k0 = 0; a.k0 < a.n_clip; a.k0 += kTensorMaxClip)
    hipLaunchKernelGGL((tensor_score_kernel<In, FA, FB>), dim3(a.n_blocks), dim3(256), 0, st, a);
  a.k0 = 0;
  hipLaunchKernelGGL((tensor_finalize_kernel<FA, FB>), dim3(1), dim3(256), 0, st, a);
  return hip_status(hipGetLastError());
}

template <typename In, int FA, int FB>
int launch_gran(const SweepParams& p, const SweepArgs& a, hipStream_t st) {
  switch (p.gran) {
    case MOFQ_PER_CHANNEL: return launch_channel<In, FA, FB>(a, st);
    case MOFQ_PER_GROUP: return launch_group<In, FA, FB>(a, st);
    case MOFQ_PER_TENSOR: return launch_tensor<In, FA, FB>(a, st);
  }
  return MOFQ_ERR_INVALID_ARG;
}

template <typename In>
int launch_fmt(const SweepParams& p, const SweepArgs& a, hipStream_t st) {
  const int fa = p.fmt[0], fb = p.n_fmt == 2 ? p.fmt[1] : -1;
#define MOFQ_F(A, B) \
  if (fa == (A) && fb == (B)) return launch_gran<In, A, B>(p, a, st);
  MOFQ_F(MOFQ_INT4, -1)
  MOFQ_F(MOFQ_FP4_E2M1, -1)
  MOFQ_F(MOFQ_INT8, -1)
  MOFQ_F(MOFQ_FP8_E4M3, -1)
  MOFQ_F(MOFQ_FP4_E2M1_IEEE, -1)
  MOFQ_F(MOFQ_FP8_E5M2, -1)
  MOFQ_F(MOFQ_INT4, MOFQ_FP4_E2M1)   // pairs come in (INT, FP) order; the caller maps slots
  MOFQ_F(MOFQ_INT8, MOFQ_FP8_E4M3)
#undef MOFQ_F
  return MOFQ_ERR_UNSUPPORTED;
}

}  // namespace

int launch_sweep(const SweepParams& p, hipStream_t st) {
  {
    const int rc = launch_sweep_sorted(p, st);
    if (rc != MOFQ_ERR_UNSUPPORTED) return rc;
  }
  SweepArgs a{};
  a.w = p.w;
  a.rows = p.rows;
  a.cols = p.cols;
  a.ld = p.ld;
  a.group = p.group;
  a.scale_f16 = p.scale_f16;
  a.n_clip = p.n_clip;
  a.rec = p.rec;
  a.absmax_part = p.absmax_part;
  a.sse_part = p.sse_part;
  a.energy_part = p.energy_part;
  a.ext_absmax = (p.gran == MOFQ_PER_TENSOR) ? p.ext_absmax : nullptr;
  if (p.emit_i8 || p.emit_f8) {
    if (p.gran != MOFQ_PER_TENSOR) return MOFQ_ERR_UNSUPPORTED;
    a.emit_i8 = p.emit_i8;
    a.emit_f8 = p.emit_f8;
    a.emit_f8_as_bf16 = p.emit_f8_as_bf16;
  }
  if (p.emit_grid[0] || p.emit_grid[1]) {
    if (p.gran != MOFQ_PER_CHANNEL || p.n_clip != 1 || p.n_fmt != 2) return MOFQ_ERR_UNSUPPORTED;
    a.emit_grid[0] = static_cast<uint16_t*>(p.emit_grid[0]);
    a.emit_grid[1] = static_cast<uint16_t*>(p.emit_grid[1]);
  }
  a.units = mofq_num_units(p.rows, p.cols, p.gran, p.group);
  for (int k = 0; k < p.n_clip; ++k) a.clip[k] = p.clip[k];
  if (a.units <= 0) return MOFQ_ERR_INVALID_ARG;
  // same format twice in one launch is handled as two single launches by the caller
  switch (p.dtype) {
    case MOFQ_F32: return launch_fmt<F32>(p, a, st);
    case MOFQ_F16: return launch_fmt<F16>(p, a, st);
    case MOFQ_BF16: return launch_fmt<BF16>(p, a, st);
  }
  return MOFQ_ERR_INVALID_ARG;
}

int launch_sweep_group(const SweepParams* p, int n, hipStream_t st) {
  if (n > 1) {
    const int rc = launch_sweep_sorted_group(p, n, st);
    if (rc != MOFQ_ERR_UNSUPPORTED) return rc;
  }
  for (int i = 0; i < n; ++i) {
    const int rc = launch_sweep(p[i], st);
    if (rc != MOFQ_OK) return rc;
  }
  return MOFQ_OK;
}

int launch_running_absmax(const SweepParams& p, float* running, hipStream_t st) {
  if (!running || !p.absmax_part || !p.energy_part) return MOFQ_ERR_INVALID_ARG;
  SweepArgs a{};
  a.w = p.w;
  a.rows = p.rows;
  a.cols = p.cols;
  a.ld = p.ld;
  a.absmax_part = p.absmax_part;
  a.energy_part = p.energy_part;
  const int64_t n_chunks = a.rows * (a.cols / 8);
  a.n_blocks = static_cast<int32_t>(std::min<int64_t>(kTensorBlocks, ceil_div(n_chunks, 256)));
  switch (p.dtype) {
    case MOFQ_F32: hipLaunchKernelGGL((tensor_absmax_kernel<F32>), dim3(a.n_blocks), dim3(256), 0, st, a); break;
    case MOFQ_F16: hipLaunchKernelGGL((tensor_absmax_kernel<F16>), dim3(a.n_blocks), dim3(256), 0, st, a); break;
    case MOFQ_BF16: hipLaunchKernelGGL((tensor_absmax_kernel<BF16>), dim3(a.n_blocks), dim3(256), 0, st, a); break;
    default: return MOFQ_ERR_INVALID_ARG;
  }
  hipLaunchKernelGGL(absmax_fold_kernel, dim3(1), dim3(256), 0, st, a.absmax_part, a.n_blocks, running);
  return hip_status(hipGetLastError());
}

}  // namespace mofq
