// Tensor-level reduce + format select (Algorithm 1's strict-less rule), and the
// second quantize_layer call of Algorithm 1: emit the codes of the winning format
// with the scales the search chose.  Both read the decision from device memory,
// so a whole model can be processed without a host synchronisation.
#include "mofq_device.h"
#include "mofq_internal.h"

namespace mofq {

namespace {

// ---- decide ---------------------------------------------------------------------

constexpr int kDecideThreads = 1024;

// Sum of v[0..n) over the block in a fixed order (thread-strided partials, then
// wave sums, then the waves in order); the result is valid on thread 0.
MOFQ_DEV double block_sum(const double* v, int64_t n, double* s_red, int64_t step = 1) {
  const int tid = threadIdx.x;
  double t = 0.0;
  for (int64_t i = tid; i < n; i += kDecideThreads) t += v[i * step];
  t = wave_sum(t);
  __syncthreads();
  if ((tid & 63) == 0) s_red[tid >> 6] = t;
  __syncthreads();
  double r = 0.0;
  if (tid == 0)
    for (int w = 0; w < kDecideThreads / 64; ++w) r += s_red[w];
  return r;
}

// First stage for tensors with many units: workgroup b adds units [b*chunk, (b+1)*chunk)
// of every candidate (and of the energies) in the same fixed order; the decide kernel
// then adds the kDecideBlocks partials.
struct PartialArgs {
  DecideParams p;
  int64_t chunk;
};
__global__ __launch_bounds__(kDecideThreads) void decide_partial_kernel(const PartialArgs a) {
  __shared__ double s_red[kDecideThreads / 64];
  const DecideParams& p = a.p;
  const int64_t lo = static_cast<int64_t>(blockIdx.x) * a.chunk;
  int64_t n = p.units - lo;
  n = n < 0 ? 0 : (n < a.chunk ? n : a.chunk);
#pragma unroll
  for (int c = 0; c <= MOFQ_MAX_CANDIDATES; ++c) {
    const double* v = (c < MOFQ_MAX_CANDIDATES) ? (c < p.n_cand ? p.err[c] : nullptr) : p.energy;
    if (!v) continue;    // uniform
    const double t = block_sum(v + lo, n, s_red);
    if (threadIdx.x == 0) p.part[c * kDecideBlocks + blockIdx.x] = t;
  }
}

// Fixed-order sums of the unit errors, Algorithm 1's select, result record.  Returns the
// chosen index on thread 0.
MOFQ_DEV int decide_body(const DecideParams& p, double* s_red);

struct FinishBatchArgs {
  FinishParams p[kFinishBatch];
};
__global__ __launch_bounds__(kDecideThreads) void finish_batch_kernel(const FinishBatchArgs a) {
  __shared__ double s_red[kDecideThreads / 64];
  __shared__ int s_best;
  const FinishParams& p = a.p[blockIdx.x];
  const int b = decide_body(p.d, s_red);
  if (threadIdx.x == 0) s_best = (b < 0 || b >= p.d.n_cand) ? 0 : b;   // no candidate beat infinity: keep the first
  __syncthreads();
  const int best = s_best;
  for (int64_t u = threadIdx.x; u < p.d.units; u += kDecideThreads) {
    const float s = p.scale[best][u];
    if (p.out_scales) {
      if (p.scale_f16_out)
        static_cast<uint16_t*>(p.out_scales)[u] = __half_as_ushort(__float2half_rn(s));  // exact: s is an fp16 value
      else
        static_cast<float*>(p.out_scales)[u] = s;
    }
    if (p.out_clip) p.out_clip[u] = p.clip[best][u];
    if (p.out_unit_err) p.out_unit_err[u] = p.d.err[best][u];
  }
}

__global__ __launch_bounds__(kDecideThreads) void decide_kernel(const DecideParams p) {
  __shared__ double s_red[kDecideThreads / 64];
  decide_body(p, s_red);
}

MOFQ_DEV int decide_body(const DecideParams& p, double* s_red) {
  double err[MOFQ_MAX_CANDIDATES];
#pragma unroll
  for (int c = 0; c < MOFQ_MAX_CANDIDATES; ++c)
    err[c] = (c < p.n_cand) ? block_sum(p.err[c], p.units, s_red) : 0.0;
  const double energy = p.energy ? block_sum(p.energy, p.units, s_red) : 0.0;
  int best = -1;
  if (threadIdx.x == 0) {
    // Algorithm 1: min_error starts at infinity, candidates in list order, a
    // candidate wins only if strictly smaller.
    double min_err = __builtin_inf();
#pragma unroll
    for (int c = 0; c < MOFQ_MAX_CANDIDATES; ++c)
      if (c < p.n_cand && err[c] < min_err) { min_err = err[c]; best = c; }
    if (p.result) {
      // no candidate below infinity (non-finite input): the first candidate, which is also what
      // the emission falls back to, so record and codes agree
      p.result->best = best < 0 ? 0 : best;
      p.result->n = p.n_cand;
#pragma unroll
      for (int c = 0; c < MOFQ_MAX_CANDIDATES; ++c) p.result->err[c] = (c < p.n_cand) ? err[c] : 0.0;
      p.result->ref_energy = energy;
    }
    if (p.tensor_err_out) *p.tensor_err_out = err[0];
    if (p.energy_out) *p.energy_out = energy;
  }
  return best;
}

// The weight-activation path after the matrix kernels of a group of layers, one workgroup per
// layer: select from the per-tile partials, then the one-unit outputs of the chosen format
// for X and W.
struct WaFinishArgs {
  WaFinishParams p[kWaGroup];
};
__global__ __launch_bounds__(kDecideThreads) void wa_finish_kernel(const WaFinishArgs args) {
  __shared__ double s_red[kDecideThreads / 64];
  __shared__ int s_best;
  const WaFinishParams& a = args.p[blockIdx.x];
  const int b = decide_body(a.d, s_red);
  if (threadIdx.x == 0) s_best = (b < 0 || b >= a.d.n_cand) ? 0 : b;   // no candidate beat infinity: keep the first
  __syncthreads();
  const int f = a.fmt_slot[s_best];
#pragma unroll
  for (int which = 0; which < 2; ++which) {
    const WaFinishTensor& t = a.t[which];
    if (t.n_segments < 1) continue;   // uniform
    double e = 0.0;
    if (t.out_unit_err) e = block_sum(t.sse_part + f, t.n_segments, s_red, 2);
    if (threadIdx.x == 0) {
      if (t.out_unit_err) *t.out_unit_err = e;
      if (t.out_scales) *static_cast<float*>(t.out_scales) = t.scale[f];
      if (t.out_clip) *t.out_clip = 0;
    }
  }
}

// Copy of the chosen format's codes (16-byte pieces, grid-stride, four in flight per lane) for
// the tensors of a group of layers.  Workgroups are dealt to the tensors in proportion to
// their sizes.
constexpr int kCopyTensors = 2 * kWaGroup;
struct WaCopyArgs {
  const mofq_result_t* result[kCopyTensors];
  int32_t n_cand[kCopyTensors];
  int32_t fmt_slot[kCopyTensors][MOFQ_MAX_CANDIDATES];
  WaCopyTensor t[kCopyTensors];
  int32_t first_block[kCopyTensors + 1];
  int32_t n;
};
__global__ __launch_bounds__(256) void wa_copy_kernel(const WaCopyArgs a) {
  int k = 0;
  while (k + 1 < a.n && static_cast<int>(blockIdx.x) >= a.first_block[k + 1]) ++k;   // uniform
  const int b = static_cast<int>(blockIdx.x) - a.first_block[k];
  const int nb = a.first_block[k + 1] - a.first_block[k];
  int best = a.result[k]->best;
  if (best < 0 || best >= a.n_cand[k]) best = 0;
  const int f = a.fmt_slot[k][__builtin_amdgcn_readfirstlane(best)];
  const WaCopyTensor& t = a.t[k];
  const uint8_t* src = f ? t.src[1] : t.src[0];
  if (src == t.dst) return;   // uniform: the codes are in place
  const u32x4* s4 = reinterpret_cast<const u32x4*>(src);
  u32x4* d4 = reinterpret_cast<u32x4*>(t.dst);
  const int64_t n = t.bytes / 16;
  const int64_t stride = static_cast<int64_t>(nb) * 256;
  int64_t i = static_cast<int64_t>(b) * 256 + threadIdx.x;
  for (; i + 3 * stride < n; i += 4 * stride) {
    const u32x4 v0 = s4[i], v1 = s4[i + stride], v2 = s4[i + 2 * stride], v3 = s4[i + 3 * stride];
    d4[i] = v0; d4[i + stride] = v1; d4[i + 2 * stride] = v2; d4[i + 3 * stride] = v3;
  }
  for (; i < n; i += stride) d4[i] = s4[i];
}

// ---- emit -------------------------------------------------------------------------

// Codes of 8 scaled elements.  4-bit: one word, element 2j in the low nibble of byte j;
// 8-bit: two words, one byte per element.  The FP formats use the gfx950 pack-convert
// instructions (round to nearest even, subnormals kept, saturating; the E4M3 convert
// needs its input clamped to +-448 first), which agree with Codec<>::code on every
// finite fp32 bit pattern.
template <int FMT>
MOFQ_DEV void encode8(const float (&v)[8], float inv_s, uint32_t (&words)[2]) {
  if constexpr (FMT == MOFQ_FP4_E2M1) {
    uint32_t w = 0;
    w = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w, v[0] * inv_s, v[1] * inv_s, 1.0f, 0);
    w = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w, v[2] * inv_s, v[3] * inv_s, 1.0f, 1);
    w = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w, v[4] * inv_s, v[5] * inv_s, 1.0f, 2);
    w = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w, v[6] * inv_s, v[7] * inv_s, 1.0f, 3);
    words[0] = w;
    words[1] = 0;
  } else if constexpr (FMT == MOFQ_FP8_E4M3) {
    float t[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) t[i] = med3(v[i] * inv_s, -448.0f, 448.0f);
    int w0 = 0, w1 = 0;
    w0 = __builtin_amdgcn_cvt_pk_fp8_f32(t[0], t[1], w0, false);
    w0 = __builtin_amdgcn_cvt_pk_fp8_f32(t[2], t[3], w0, true);
    w1 = __builtin_amdgcn_cvt_pk_fp8_f32(t[4], t[5], w1, false);
    w1 = __builtin_amdgcn_cvt_pk_fp8_f32(t[6], t[7], w1, true);
    words[0] = static_cast<uint32_t>(w0);
    words[1] = static_cast<uint32_t>(w1);
  } else if constexpr (Codec<FMT>::BITS == 4) {
    uint32_t w = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) w |= Codec<FMT>::code(v[i] * inv_s) << (4 * i);
    words[0] = w;
    words[1] = 0;
  } else {
    uint32_t w0 = 0, w1 = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      w0 |= Codec<FMT>::code(v[i] * inv_s) << (8 * i);
      w1 |= Codec<FMT>::code(v[4 + i] * inv_s) << (8 * i);
    }
    words[0] = w0;
    words[1] = w1;
  }
}

struct EmitArgs {
  const void* w;
  int64_t rows, cols, ld;
  int64_t units;
  int32_t gran, group;
  int32_t scale_f16_out;
  int32_t n_cand;
  int32_t fmt[MOFQ_MAX_CANDIDATES];
  const float* scale[MOFQ_MAX_CANDIDATES];
  const int32_t* clip[MOFQ_MAX_CANDIDATES];
  const double* err[MOFQ_MAX_CANDIDATES];
  const mofq_result_t* result;
  const uint8_t* unit_fmt;  // per-unit candidate index, or nullptr (then the tensor-level choice)
  mofq_qout_t out;
  int32_t as_bf16_values;   // write dequantised grid values (bf16, unscaled) instead of codes
};

MOFQ_DEV int chosen(const EmitArgs& a) {
  int best = a.result ? a.result->best : 0;
  if (best < 0 || best >= a.n_cand) best = 0;   // no candidate beat infinity: keep the first
  return __builtin_amdgcn_readfirstlane(best);
}

// One 8-element chunk: quantize with the unit's scale and store.
template <typename In>
MOFQ_DEV void emit_chunk(const EmitArgs& a, int best, int64_t cpr, int64_t c, const float (&v)[8]) {
  const int64_t row = c / cpr, col = (c - row * cpr) * 8;
  int64_t unit = 0;
  if (a.gran == MOFQ_PER_CHANNEL) unit = row;
  else if (a.gran == MOFQ_PER_GROUP) unit = row * (a.cols / a.group) + col / a.group;
  if (a.unit_fmt) {
    best = a.unit_fmt[unit];
    if (best >= a.n_cand) best = 0;
  }
  const int fmt = a.fmt[best];
  const float inv_s = 1.0f / a.scale[best][unit];
  uint32_t words[2];
  switch (fmt) {
    case MOFQ_INT4: encode8<MOFQ_INT4>(v, inv_s, words); break;
    case MOFQ_FP4_E2M1: encode8<MOFQ_FP4_E2M1>(v, inv_s, words); break;
    case MOFQ_INT8: encode8<MOFQ_INT8>(v, inv_s, words); break;
    case MOFQ_FP4_E2M1_IEEE: encode8<MOFQ_FP4_E2M1_IEEE>(v, inv_s, words); break;
    case MOFQ_FP8_E5M2: encode8<MOFQ_FP8_E5M2>(v, inv_s, words); break;
    default: encode8<MOFQ_FP8_E4M3>(v, inv_s, words); break;
  }
  const int64_t e0 = row * a.cols + col;   // dense output rows
  if (a.as_bf16_values) {
    // grid values have at most 7 significant bits: exact in bf16 (top half of fp32)
    u32x4 o;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float g0, g1;
      switch (fmt) {
        case MOFQ_INT4: g0 = Codec<MOFQ_INT4>::grid(v[2 * i] * inv_s); g1 = Codec<MOFQ_INT4>::grid(v[2 * i + 1] * inv_s); break;
        case MOFQ_FP4_E2M1: g0 = Codec<MOFQ_FP4_E2M1>::grid(v[2 * i] * inv_s); g1 = Codec<MOFQ_FP4_E2M1>::grid(v[2 * i + 1] * inv_s); break;
        case MOFQ_INT8: g0 = Codec<MOFQ_INT8>::grid(v[2 * i] * inv_s); g1 = Codec<MOFQ_INT8>::grid(v[2 * i + 1] * inv_s); break;
        case MOFQ_FP4_E2M1_IEEE: g0 = Codec<MOFQ_FP4_E2M1_IEEE>::grid(v[2 * i] * inv_s); g1 = Codec<MOFQ_FP4_E2M1_IEEE>::grid(v[2 * i + 1] * inv_s); break;
        case MOFQ_FP8_E5M2: g0 = Codec<MOFQ_FP8_E5M2>::grid(v[2 * i] * inv_s); g1 = Codec<MOFQ_FP8_E5M2>::grid(v[2 * i + 1] * inv_s); break;
        default: g0 = Codec<MOFQ_FP8_E4M3>::grid(v[2 * i] * inv_s); g1 = Codec<MOFQ_FP8_E4M3>::grid(v[2 * i + 1] * inv_s); break;
      }
      o[i] = (f2u(g0) >> 16) | (f2u(g1) & 0xFFFF0000u);
    }
    reinterpret_cast<u32x4*>(a.out.codes)[e0 / 8] = o;
  } else if (fmt == MOFQ_INT4 || fmt == MOFQ_FP4_E2M1 || fmt == MOFQ_FP4_E2M1_IEEE) {
    static_cast<uint32_t*>(a.out.codes)[e0 / 8] = words[0];
  } else {
    u32x2 o;
    o[0] = words[0];
    o[1] = words[1];
    reinterpret_cast<u32x2*>(a.out.codes)[e0 / 8] = o;
  }
}

// Grid-stride over 8-element chunks, kEmitUnroll chunks per thread and iteration so that
// several 16-byte loads are in flight per lane (the pass is HBM-bound).
constexpr int kEmitUnroll = 4;
template <typename In>
__global__ __launch_bounds__(256) void emit_codes_kernel(const EmitArgs a) {
  using L = Load8<In>;
  const int best = chosen(a);
  const int64_t cpr = a.cols / 8;
  const int64_t n_chunks = a.rows * cpr;
  const int64_t stride = static_cast<int64_t>(gridDim.x) * 256;
  int64_t c = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  for (; c + (kEmitUnroll - 1) * stride < n_chunks; c += kEmitUnroll * stride) {
    float v[kEmitUnroll][8];
#pragma unroll
    for (int u = 0; u < kEmitUnroll; ++u) {
      const int64_t cu = c + u * stride;
      const int64_t row = cu / cpr, col = (cu - row * cpr) * 8;
      L::load(static_cast<const typename L::elem*>(a.w) + row * a.ld + col, v[u]);
    }
#pragma unroll
    for (int u = 0; u < kEmitUnroll; ++u) emit_chunk<In>(a, best, cpr, c + u * stride, v[u]);
  }
  for (; c < n_chunks; c += stride) {
    float v[8];
    const int64_t row = c / cpr, col = (c - row * cpr) * 8;
    L::load(static_cast<const typename L::elem*>(a.w) + row * a.ld + col, v);
    emit_chunk<In>(a, best, cpr, c, v);
  }
}

__global__ __launch_bounds__(256) void emit_units_kernel(const EmitArgs a) {
  int best = chosen(a);
  const int64_t u = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (u >= a.units) return;
  if (a.unit_fmt) {
    best = a.unit_fmt[u];
    if (best >= a.n_cand) best = 0;
  }
  const float s = a.scale[best][u];
  if (a.out.scales) {
    if (a.scale_f16_out)
      static_cast<uint16_t*>(a.out.scales)[u] = __half_as_ushort(__float2half_rn(s));  // exact: s is an fp16 value
    else
      static_cast<float*>(a.out.scales)[u] = s;
  }
  if (a.out.clip_idx) a.out.clip_idx[u] = a.clip[best][u];
  if (a.out.unit_err) a.out.unit_err[u] = a.err[best][u];
}

__global__ __launch_bounds__(256) void pick_units_kernel(const PickUnitsParams p) {
  const int64_t u = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (u >= p.units) return;
  // Algorithm 1's rule for one unit: start at infinity, list order, strictly smaller wins
  double min_err = __builtin_inf();
  int best = 0;
#pragma unroll
  for (int c = 0; c < MOFQ_MAX_CANDIDATES; ++c)
    if (c < p.n_cand) {
      const double e = p.err[c][u];
      if (e < min_err) { min_err = e; best = c; }
    }
  p.unit_fmt[u] = static_cast<uint8_t>(best);
  p.picked_err[u] = p.err[best][u];
}

}  // namespace

int launch_finish_batch(const FinishParams* p, int n, hipStream_t st) {
  if (!p || n < 1 || n > kFinishBatch) return MOFQ_ERR_INVALID_ARG;
  FinishBatchArgs a{};
  for (int i = 0; i < n; ++i) {
    if (p[i].d.units < 1 || p[i].d.units > kFinishMaxUnits) return MOFQ_ERR_INVALID_ARG;
    a.p[i] = p[i];
  }
  hipLaunchKernelGGL(finish_batch_kernel, dim3(static_cast<unsigned>(n)), dim3(kDecideThreads), 0, st, a);
  return hip_status(hipGetLastError());
}

int launch_wa_finish(const WaFinishParams* p, int n, hipStream_t st) {
  if (!p || n < 1 || n > kWaGroup) return MOFQ_ERR_INVALID_ARG;
  WaFinishArgs a{};
  for (int i = 0; i < n; ++i) {
    const DecideParams& d = p[i].d;
    if (d.units < 1 || d.n_cand < 1 || d.n_cand > MOFQ_MAX_CANDIDATES || !d.result) return MOFQ_ERR_INVALID_ARG;
    for (int c = 0; c < d.n_cand; ++c)
      if (!d.err[c] || p[i].fmt_slot[c] < 0 || p[i].fmt_slot[c] > 1) return MOFQ_ERR_INVALID_ARG;
    a.p[i] = p[i];
  }
  hipLaunchKernelGGL(wa_finish_kernel, dim3(static_cast<unsigned>(n)), dim3(kDecideThreads), 0, st, a);
  return hip_status(hipGetLastError());
}

int launch_wa_copy(const WaCopyParams* p, int n, hipStream_t st) {
  if (!p || n < 1 || n > kWaGroup) return MOFQ_ERR_INVALID_ARG;
  WaCopyArgs a{};
  int64_t want[kCopyTensors];
  int64_t total = 0;
  for (int i = 0; i < n; ++i) {
    if (!p[i].result || p[i].n_cand < 1 || p[i].n_cand > MOFQ_MAX_CANDIDATES) return MOFQ_ERR_INVALID_ARG;
    for (int which = 0; which < 2; ++which) {
      const WaCopyTensor& t = p[i].t[which];
      if (!t.dst) continue;
      if (t.bytes < 16 || t.bytes % 16 != 0 || !t.src[0] || !t.src[1]) return MOFQ_ERR_INVALID_ARG;
      const int k = a.n++;
      a.result[k] = p[i].result;
      a.n_cand[k] = p[i].n_cand;
      for (int c = 0; c < MOFQ_MAX_CANDIDATES; ++c) a.fmt_slot[k][c] = p[i].fmt_slot[c];
      a.t[k] = t;
      want[k] = (t.bytes / 16 + 256 * 4 - 1) / (256 * 4);
      total += want[k];
    }
  }
  if (a.n < 1) return MOFQ_OK;
  const int64_t cap = 256 * 8;
  for (int k = 0; k < a.n; ++k) {
    const int64_t nb = total <= cap ? want[k] : std::max<int64_t>(1, want[k] * cap / total);
    a.first_block[k + 1] = a.first_block[k] + static_cast<int32_t>(nb);
  }
  hipLaunchKernelGGL(wa_copy_kernel, dim3(static_cast<unsigned>(a.first_block[a.n])), dim3(256), 0, st, a);
  return hip_status(hipGetLastError());
}

int launch_pick_units(const PickUnitsParams& p, hipStream_t st) {
  if (p.units <= 0 || p.n_cand < 1 || p.n_cand > MOFQ_MAX_CANDIDATES) return MOFQ_ERR_INVALID_ARG;
  hipLaunchKernelGGL(pick_units_kernel, dim3(static_cast<unsigned>((p.units + 255) / 256)), dim3(256), 0, st, p);
  return hip_status(hipGetLastError());
}

int launch_decide(const DecideParams& p, hipStream_t st) {
  if (p.part && p.units > 16 * 1024) {
    PartialArgs a{p, (p.units + kDecideBlocks - 1) / kDecideBlocks};
    hipLaunchKernelGGL(decide_partial_kernel, dim3(kDecideBlocks), dim3(kDecideThreads), 0, st, a);
    DecideParams d = p;
    d.units = kDecideBlocks;
    for (int c = 0; c < MOFQ_MAX_CANDIDATES; ++c) d.err[c] = c < p.n_cand ? p.part + c * kDecideBlocks : nullptr;
    d.energy = p.energy ? p.part + MOFQ_MAX_CANDIDATES * kDecideBlocks : nullptr;
    hipLaunchKernelGGL(decide_kernel, dim3(1), dim3(kDecideThreads), 0, st, d);
    return hip_status(hipGetLastError());
  }
  hipLaunchKernelGGL(decide_kernel, dim3(1), dim3(kDecideThreads), 0, st, p);
  return hip_status(hipGetLastError());
}

int launch_emit(const EmitParams& p, hipStream_t st) {
  EmitArgs a{};
  a.w = p.w;
  a.rows = p.rows;
  a.cols = p.cols;
  a.ld = p.ld;
  a.gran = p.gran;
  a.group = p.group;
  a.scale_f16_out = p.scale_f16_out;
  a.n_cand = p.n_cand;
  for (int c = 0; c < MOFQ_MAX_CANDIDATES; ++c) {
    a.fmt[c] = p.fmt[c];
    a.scale[c] = p.scale[c];
    a.clip[c] = p.clip[c];
    a.err[c] = p.err[c];
  }
  a.result = p.result;
  a.unit_fmt = p.unit_fmt;
  a.out = p.out;
  a.as_bf16_values = p.as_bf16_values;
  a.units = mofq_num_units(p.rows, p.cols, p.gran, p.group);
  if (a.units <= 0) return MOFQ_ERR_INVALID_ARG;
  const int64_t n_chunks = p.rows * (p.cols / 8);
  // full occupancy (8 workgroups of 256 on each of 256 compute units), several chunks per thread
  const int64_t cap = p.max_blocks > 0 ? p.max_blocks : 256 * 8;
  const unsigned blocks = static_cast<unsigned>(
      std::max<int64_t>(1, std::min<int64_t>((n_chunks + 256 * kEmitUnroll - 1) / (256 * kEmitUnroll), cap)));
  if (p.out.codes) {
    switch (p.dtype) {
      case MOFQ_F32: hipLaunchKernelGGL(emit_codes_kernel<F32>, dim3(blocks), dim3(256), 0, st, a); break;
      case MOFQ_F16: hipLaunchKernelGGL(emit_codes_kernel<F16>, dim3(blocks), dim3(256), 0, st, a); break;
      case MOFQ_BF16: hipLaunchKernelGGL(emit_codes_kernel<BF16>, dim3(blocks), dim3(256), 0, st, a); break;
      default: return MOFQ_ERR_INVALID_ARG;
    }
  }
  if (p.out.scales || p.out.clip_idx || p.out.unit_err)
    hipLaunchKernelGGL(emit_units_kernel, dim3(static_cast<unsigned>((a.units + 255) / 256)), dim3(256), 0, st, a);
  return hip_status(hipGetLastError());
}

}  // namespace mofq
