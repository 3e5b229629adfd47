// Per-tensor 8-bit quantization of the inputs of linear layers for the layer-output metric of
// the weight-activation case (Section 3.2: A_out = W * A_in with both inputs quantized;
// Section 5: INT8 against FP8-E4M3, activations per tensor).  The activations and weights of a
// group of layers go through every pass together, one launch per pass:
//
//   1. largest magnitude of each tensor (per-workgroup partial maxima);
//   2. both formats at once: the INT8 codes, the E4M3 codes and, where the exact E4M3
//      product is wanted, the E4M3 grid values as bf16, all from one read of the tensor,
//      with the tensor error of each format as partial sums in fp64.
//
// The small dependent steps (folding the partial maxima, the two scales) are redone by every
// workgroup of pass 2 from the partials, so no one-workgroup kernel sits between the passes.
// Nothing is accumulated atomically.  A tensor is cut into a fixed number of segments that
// depends only on its shape; a workgroup takes whole segments and leaves one partial error sum
// per segment, so the sums do not depend on how many workgroups a launch has (which varies
// with how many tensors share it).
#include <algorithm>
#include <type_traits>

#include "mofq_device.h"
#include "mofq_internal.h"

namespace mofq {

namespace {

typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr int kThreads = 256;
constexpr int kMaxTensors = 2 * kWaGroup;

struct PrepTensor {
  const uint16_t* data;
  int64_t n_chunks, cpr, ld;   // 8-element chunks in the tensor and per row; elements between rows
  int32_t n_seg;               // segments of the tensor
  int32_t seg_chunks;          // chunks per segment (the last one may be shorter)
  float ratio;                 // clip ratio of the scale
  float* absmax_part;
  int32_t n_absmax;            // partial maxima to fold; 0 = one per workgroup of the quantize pass
  double* sse_part;
  uint8_t* q_i8;
  uint8_t* q_f8;
  uint8_t* q_g;
  float* scale;
  // column split (fp8-unit product); null / 0 otherwise
  int32_t is_x;
  int32_t ld_i32;              // elements between rows (for the column passes)
  int32_t rows_i32, cols_i32;
  float* colmax;
  uint8_t* col_slot;
  int32_t* side_cols;
  uint8_t* q_f8_main;
  uint16_t* side;
};
struct PrepArgs {
  PrepTensor t[kMaxTensors];
  int32_t first_block[kMaxTensors + 1];   // workgroups [first_block[k], first_block[k + 1]) walk tensor k
  int32_t n;
};

// The workgroup's tensor, its index among the tensor's workgroups and their number.
MOFQ_DEV const PrepTensor& my_tensor(const PrepArgs& a, int& b, int& nb) {
  int k = 0;
  while (k + 1 < a.n && static_cast<int>(blockIdx.x) >= a.first_block[k + 1]) ++k;   // uniform
  b = static_cast<int>(blockIdx.x) - a.first_block[k];
  nb = a.first_block[k + 1] - a.first_block[k];
  return a.t[k];
}

// Address of chunk c: rows are dense in the outputs, `ld` apart in the input.
MOFQ_DEV const uint16_t* chunk_src(const PrepTensor& t, int64_t c) {
  if (t.ld == t.cpr * 8) return t.data + c * 8;   // uniform: dense input, no division
  const int64_t row = c / t.cpr;
  return t.data + row * t.ld + (c - row * t.cpr) * 8;
}

constexpr int kInFlight = 8;   // 16-byte loads in flight per lane (largest-magnitude pass)
constexpr int kQuantInFlight = 2;   // quantize pass: every further chunk in flight costs some 17 registers

__global__ __launch_bounds__(kThreads) void wa_absmax_kernel(const PrepArgs a) {
  using L = Load8<BF16>;
  __shared__ float s_wmax[kThreads / 64];
  int b, nb;
  const PrepTensor& t = my_tensor(a, b, nb);
  const int tid = threadIdx.x;
  const int64_t stride = static_cast<int64_t>(nb) * kThreads;
  float amax = 0.0f;
  int64_t c = static_cast<int64_t>(b) * kThreads + tid;
  for (; c + (kInFlight - 1) * stride < t.n_chunks; c += kInFlight * stride) {
    float v[kInFlight][8];
#pragma unroll
    for (int u = 0; u < kInFlight; ++u) L::load(chunk_src(t, c + u * stride), v[u]);
#pragma unroll
    for (int u = 0; u < kInFlight; ++u)
#pragma unroll
      for (int i = 0; i < 8; ++i) amax = __builtin_fmaxf(amax, __builtin_fabsf(v[u][i]));
  }
  for (; c < t.n_chunks; c += stride) {
    float v[8];
    L::load(chunk_src(t, c), v);
#pragma unroll
    for (int i = 0; i < 8; ++i) amax = __builtin_fmaxf(amax, __builtin_fabsf(v[i]));
  }
  amax = wave_max(amax);
  if ((tid & 63) == 0) s_wmax[tid >> 6] = amax;
  __syncthreads();
  if (tid == 0)
    t.absmax_part[b] = __builtin_fmaxf(__builtin_fmaxf(s_wmax[0], s_wmax[1]), __builtin_fmaxf(s_wmax[2], s_wmax[3]));
}

// One chunk in both formats: codes, optional grid values, squared differences.
MOFQ_DEV void quant_chunk(const PrepTensor& t, int64_t c, const u32x4 raw, float iA, float iB, double sAd,
                          double sBd, double& accA, double& accB) {
  float v[8];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    v[2 * i] = u2f(raw[i] << 16);           // bf16 is the top half of an fp32
    v[2 * i + 1] = u2f(raw[i] & 0xFFFF0000u);
  }
  uint32_t wi[2] = {0u, 0u};
  int wf[2] = {0, 0};
  u32x4 gb;
#pragma unroll
  for (int i = 0; i < 8; i += 2) {
    const float q0 = Codec<MOFQ_INT8>::grid(v[i] * iA), q1 = Codec<MOFQ_INT8>::grid(v[i + 1] * iA);
    wi[i >> 2] |= (static_cast<uint32_t>(static_cast<int>(q0)) & 0xFFu) << (8 * (i & 3));
    wi[i >> 2] |= (static_cast<uint32_t>(static_cast<int>(q1)) & 0xFFu) << (8 * ((i & 3) + 1));
    const double d0 = __builtin_fma(-static_cast<double>(q0), sAd, static_cast<double>(v[i]));
    const double d1 = __builtin_fma(-static_cast<double>(q1), sAd, static_cast<double>(v[i + 1]));
    accA = __builtin_fma(d0, d0, accA);
    accA = __builtin_fma(d1, d1, accA);
    // E4M3 through the pack-convert (round to nearest even, subnormals kept; saturating once
    // the input is clamped), which agrees with the codec on every finite fp32 pattern
    const int p = __builtin_amdgcn_cvt_pk_fp8_f32(med3(v[i] * iB, -448.0f, 448.0f),
                                                  med3(v[i + 1] * iB, -448.0f, 448.0f), 0, false);
    const f32x2 g = __builtin_amdgcn_cvt_pk_f32_fp8(p, false);
    wf[i >> 2] |= (p & 0xFFFF) << (16 * ((i >> 1) & 1));
    gb[i >> 1] = (f2u(g[0]) >> 16) | (f2u(g[1]) & 0xFFFF0000u);   // at most 4 significant bits: exact in bf16
    const double e0 = __builtin_fma(-static_cast<double>(g[0]), sBd, static_cast<double>(v[i]));
    const double e1 = __builtin_fma(-static_cast<double>(g[1]), sBd, static_cast<double>(v[i + 1]));
    accB = __builtin_fma(e0, e0, accB);
    accB = __builtin_fma(e1, e1, accB);
    // one pair at a time: the two fp64 chains are sequential anyway, and scheduling all eight
    // elements of a chunk together costs some 130 registers
    __builtin_amdgcn_sched_barrier(0);
  }
  u32x2 oi, of;
  oi[0] = wi[0];
  oi[1] = wi[1];
  of[0] = static_cast<uint32_t>(wf[0]);
  of[1] = static_cast<uint32_t>(wf[1]);
  reinterpret_cast<u32x2*>(t.q_i8)[c] = oi;
  reinterpret_cast<u32x2*>(t.q_f8)[c] = of;
  if (t.q_g) reinterpret_cast<u32x4*>(t.q_g)[c] = gb;
  if (t.q_f8_main) {   // uniform: the activation of an fp8-unit product
    // slot bytes of the chunk's 8 columns: bit 7 set = not split off = keep the code
    const uint32_t col8 = static_cast<uint32_t>(c) % static_cast<uint32_t>(t.cpr);   // fewer than 2^31 chunks (checked by the host)
    const u32x2 m = reinterpret_cast<const u32x2*>(t.col_slot)[col8];
    u32x2 om;
    om[0] = of[0] & (((m[0] >> 7) & 0x01010101u) * 0xFFu);
    om[1] = of[1] & (((m[1] >> 7) & 0x01010101u) * 0xFFu);
    reinterpret_cast<u32x2*>(t.q_f8_main)[c] = om;
  }
}

// ---- column split for the fp8-unit product ------------------------------------------------

// Largest magnitude of every column of an activation: a workgroup takes 64 columns, a thread 8
// of them (one 16-byte load per row) on every 32nd row.
__global__ __launch_bounds__(kThreads) void wa_colmax_kernel(const PrepArgs a) {
  __shared__ float s_max[32][65];
  int b, nb;
  const PrepTensor& t = my_tensor(a, b, nb);
  const int tid = threadIdx.x;
  const int cx = tid & 7, ry = tid >> 3;
  const int col0 = b * 64 + cx * 8;          // nb = cols / 64 workgroups
  float m[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) m[i] = 0.0f;
  int r = ry;
  for (; r + 7 * 32 < t.rows_i32; r += 8 * 32) {   // eight loads in flight per lane
    u32x4 raw[8];
#pragma unroll
    for (int u = 0; u < 8; ++u)
      raw[u] = *reinterpret_cast<const u32x4*>(t.data + static_cast<int64_t>(r + u * 32) * t.ld_i32 + col0);
#pragma unroll
    for (int u = 0; u < 8; ++u)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        m[2 * i] = __builtin_fmaxf(m[2 * i], __builtin_fabsf(u2f(raw[u][i] << 16)));
        m[2 * i + 1] = __builtin_fmaxf(m[2 * i + 1], __builtin_fabsf(u2f(raw[u][i] & 0xFFFF0000u)));
      }
  }
  for (; r < t.rows_i32; r += 32) {
    float v[8];
    Load8<BF16>::load(t.data + static_cast<int64_t>(r) * t.ld_i32 + col0, v);
#pragma unroll
    for (int i = 0; i < 8; ++i) m[i] = __builtin_fmaxf(m[i], __builtin_fabsf(v[i]));
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) s_max[ry][cx * 8 + i] = m[i];
  __syncthreads();
  if (tid < 64) {
    float r = 0.0f;
#pragma unroll
    for (int y = 0; y < 32; ++y) r = __builtin_fmaxf(r, s_max[y][tid]);
    t.colmax[b * 64 + tid] = r;
  }
}

// Which columns to split off: those whose largest magnitude exceeds kOutlierFactor times the
// typical one, in ascending order, at most kWaSideCols of them.  "Typical" is the mean over the
// columns that do not exceed kOutlierFactor times the mean over all columns, so that the
// outliers themselves do not hide each other where they are many.  One workgroup per
// activation.  (Any choice gives the same sum; the choice only decides how much the fp8 unit's
// alignment can lose.)
constexpr float kOutlierFactor = 4.0f;
constexpr int kPickCached = 12288;   // column maxima held in LDS up to this many columns
__global__ __launch_bounds__(kThreads) void wa_pick_kernel(const PrepArgs a) {
  __shared__ float s_col[kPickCached];
  __shared__ __attribute__((aligned(16))) uint8_t s_slot[kPickCached];
  __shared__ double s_sum[2][kThreads / 64];
  __shared__ uint32_t s_cnt[2][kThreads / 64];
  __shared__ float s_amax[kThreads / 64];
  const PrepTensor& t = a.t[blockIdx.x];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int K = t.cols_i32;
  const bool cached = K <= kPickCached;   // uniform
  if (cached) {
    // all of a thread's loads are issued before the first is used (K is a multiple of 64)
    constexpr int NV = kPickCached / (kThreads * 4);
    u32x4 v[NV];
#pragma unroll
    for (int u = 0; u < NV; ++u) {
      const int c = (u * kThreads + tid) * 4;
      if (c < K) v[u] = *reinterpret_cast<const u32x4*>(t.colmax + c);
    }
#pragma unroll
    for (int u = 0; u < NV; ++u) {
      const int c = (u * kThreads + tid) * 4;
      if (c < K) *reinterpret_cast<u32x4*>(&s_col[c]) = v[u];
    }
    __syncthreads();
  }
  // two copies of the rest, so that neither reads through a run-time choice of memory
  auto rest = [&](auto cached_c) {
    constexpr bool CACHED = decltype(cached_c)::value;
    auto col = [&](int c) {
      if constexpr (CACHED) return s_col[c];
      else return t.colmax[c];
    };
    double sum = 0.0;
    float amax = 0.0f;
    for (int c = tid; c < K; c += kThreads) {
      const float v = col(c);
      sum += static_cast<double>(v);
      amax = __builtin_fmaxf(amax, v);
    }
    sum = wave_sum(sum);
    amax = wave_max(amax);
    if (lane == 0) { s_sum[0][wave] = sum; s_amax[wave] = amax; }
    __syncthreads();
    // the tensor's largest magnitude is the largest column maximum: the first pass skips it
    if (tid == 0) t.absmax_part[0] = __builtin_fmaxf(__builtin_fmaxf(s_amax[0], s_amax[1]), __builtin_fmaxf(s_amax[2], s_amax[3]));
    const float thr0 = kOutlierFactor * static_cast<float>(((s_sum[0][0] + s_sum[0][1]) + (s_sum[0][2] + s_sum[0][3])) / K);
    double sum1 = 0.0;
    uint32_t n1 = 0;
    for (int c = tid; c < K; c += kThreads) {
      const float v = col(c);
      if (!(v > thr0)) { sum1 += static_cast<double>(v); ++n1; }
    }
    sum1 = wave_sum(sum1);
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) n1 += static_cast<uint32_t>(__shfl_xor(static_cast<int>(n1), d, 64));
    if (lane == 0) { s_sum[1][wave] = sum1; s_cnt[1][wave] = n1; }
    __syncthreads();
    const uint32_t n_typ = (s_cnt[1][0] + s_cnt[1][1]) + (s_cnt[1][2] + s_cnt[1][3]);
    const double typ = ((s_sum[1][0] + s_sum[1][1]) + (s_sum[1][2] + s_sum[1][3])) / (n_typ > 0 ? n_typ : 1);
    const float thr = n_typ > 0 ? kOutlierFactor * static_cast<float>(typ) : thr0;
    // thread t owns the columns [t * per, (t + 1) * per): count, scan over the threads, assign slots
    const int per = (K + kThreads - 1) / kThreads;
    const int lo = tid * per, hi = (lo + per < K) ? lo + per : K;
    uint32_t n = 0;
    for (int c = lo; c < hi; ++c) n += (col(c) > thr) ? 1u : 0u;
    uint32_t incl = n;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const uint32_t o = static_cast<uint32_t>(__shfl_up(static_cast<int>(incl), d, 64));
      if (lane >= d) incl += o;
    }
    if (lane == 63) s_cnt[0][wave] = incl;
    __syncthreads();
    uint32_t base = incl - n;
    for (int w = 0; w < wave; ++w) base += s_cnt[0][w];
    for (int c = lo; c < hi; ++c) {
      uint8_t slot = 0xFFu;
      if (col(c) > thr) {
        if (base < static_cast<uint32_t>(kWaSideCols)) { slot = static_cast<uint8_t>(base); t.side_cols[base] = c; }
        ++base;
      }
      if constexpr (CACHED) s_slot[c] = slot;
      else t.col_slot[c] = slot;
    }
    if constexpr (CACHED) {   // the slot bytes leave in 16-byte pieces
      __syncthreads();
      for (int c = tid * 16; c < K; c += kThreads * 16)
        *reinterpret_cast<u32x4*>(t.col_slot + c) = *reinterpret_cast<const u32x4*>(&s_slot[c]);
    }
    if (tid == kThreads - 1) t.side_cols[kWaSideCols] = static_cast<int32_t>(base < static_cast<uint32_t>(kWaSideCols) ? base : kWaSideCols);
  };
  if (cached) rest(std::true_type{});
  else rest(std::false_type{});
}

// The side operand of a tensor: the E4M3 grid values of its split-off columns as bf16, dense
// [rows][kWaSideCols], zero in the slots beyond the number of split-off columns.  Runs after the
// quantize pass (which leaves the E4M3 scale in t.scale[1]).
__global__ __launch_bounds__(kThreads) void wa_side_kernel(const PrepArgs a) {
  int b, nb;
  const PrepTensor& t = my_tensor(a, b, nb);
  const int count = t.side_cols[kWaSideCols];
  const float inv = 1.0f / t.scale[1];
  const int64_t n = static_cast<int64_t>(t.rows_i32) * kWaSideCols;
  for (int64_t e = static_cast<int64_t>(b) * kThreads + threadIdx.x; e < n; e += static_cast<int64_t>(nb) * kThreads) {
    const int slot = static_cast<int>(e % kWaSideCols);
    const int64_t row = e / kWaSideCols;
    uint16_t out = 0;
    if (slot < count) {
      const float x = u2f(static_cast<uint32_t>(t.data[row * t.ld_i32 + t.side_cols[slot]]) << 16);
      const int p = __builtin_amdgcn_cvt_pk_fp8_f32(med3(x * inv, -448.0f, 448.0f), 0.0f, 0, false);
      const f32x2 g = __builtin_amdgcn_cvt_pk_f32_fp8(p, false);
      out = static_cast<uint16_t>(f2u(g[0]) >> 16);   // exact: at most 4 significant bits
    }
    t.side[e] = out;
  }
}

__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(5))) void wa_quant_kernel(const PrepArgs a) {
  __shared__ float s_tmp[kThreads / 64];
  __shared__ double s_part[kThreads / 64][2];
  int b, nb;
  const PrepTensor& t = my_tensor(a, b, nb);
  const int tid = threadIdx.x;
  // the tensor's largest magnitude from the partials of the first pass (same launch shape) or
  // from the one the column pass left
  float amax = 0.0f;
  const int na = t.n_absmax ? t.n_absmax : nb;
  for (int i = tid; i < na; i += kThreads) amax = __builtin_fmaxf(amax, t.absmax_part[i]);
  amax = wave_max(amax);
  if ((tid & 63) == 0) s_tmp[tid >> 6] = amax;
  __syncthreads();
  amax = __builtin_fmaxf(__builtin_fmaxf(s_tmp[0], s_tmp[1]), __builtin_fmaxf(s_tmp[2], s_tmp[3]));
  const float sA = unit_scale(amax, t.ratio, Codec<MOFQ_INT8>::QMAX, false);
  const float sB = unit_scale(amax, t.ratio, Codec<MOFQ_FP8_E4M3>::QMAX, false);
  if (b == 0 && tid == 0) { t.scale[0] = sA; t.scale[1] = sB; }
  const float iA = 1.0f / sA, iB = 1.0f / sB;
  const double sAd = static_cast<double>(sA), sBd = static_cast<double>(sB);
  const bool dense = t.ld == t.cpr * 8;
  for (int seg = b; seg < t.n_seg; seg += nb) {
    const int64_t lo = static_cast<int64_t>(seg) * t.seg_chunks;
    const int64_t hi = (lo + t.seg_chunks < t.n_chunks) ? lo + t.seg_chunks : t.n_chunks;
    double accA = 0.0, accB = 0.0;
    int64_t c = lo + tid;
    // dense input (uniform): several loads in flight; rows apart: one chunk at a time
    for (; dense && c + (kQuantInFlight - 1) * kThreads < hi; c += kQuantInFlight * kThreads) {
      u32x4 raw[kQuantInFlight];
#pragma unroll
      for (int u = 0; u < kQuantInFlight; ++u) raw[u] = *reinterpret_cast<const u32x4*>(t.data + (c + u * kThreads) * 8);
#pragma unroll
      for (int u = 0; u < kQuantInFlight; ++u) {
        quant_chunk(t, c + u * kThreads, raw[u], iA, iB, sAd, sBd, accA, accB);
        __builtin_amdgcn_sched_barrier(0);   // one chunk at a time: keeps the register count low
      }
    }
    for (; c < hi; c += kThreads) {
      const u32x4 raw = *reinterpret_cast<const u32x4*>(chunk_src(t, c));
      quant_chunk(t, c, raw, iA, iB, sAd, sBd, accA, accB);
    }
    accA = wave_sum(accA);
    accB = wave_sum(accB);
    __syncthreads();   // the previous segment's partials have been read
    if ((tid & 63) == 0) { s_part[tid >> 6][0] = accA; s_part[tid >> 6][1] = accB; }
    __syncthreads();
    if (tid < 2)
      t.sse_part[static_cast<int64_t>(seg) * 2 + tid] = (s_part[0][tid] + s_part[1][tid]) + (s_part[2][tid] + s_part[3][tid]);
  }
}

bool fill(const WaPrepTensor& p, PrepTensor* t) {
  *t = PrepTensor{};
  if (p.rows < 1 || p.cols < 8 || p.cols % 8 != 0 || p.ld < p.cols || p.ld % 8 != 0) return false;
  if (!p.absmax_part || !p.sse_part || !p.q_i8 || !p.q_f8 || !p.scale) return false;
  t->data = static_cast<const uint16_t*>(p.data);
  t->cpr = p.cols / 8;
  t->n_chunks = p.rows * t->cpr;
  t->ld = p.ld;
  t->n_seg = wa_prep_segments(p.rows, p.cols);
  t->seg_chunks = static_cast<int32_t>((t->n_chunks + t->n_seg - 1) / t->n_seg);
  t->ratio = p.ratio;
  t->absmax_part = p.absmax_part;
  t->sse_part = p.sse_part;
  t->q_i8 = p.q_i8;
  t->q_f8 = p.q_f8;
  t->q_g = p.q_g;
  t->scale = p.scale;
  if (p.side) {
    if (!p.col_slot || !p.side_cols || p.cols % 64 != 0 || p.rows > (1 << 30) || p.cols > (1 << 20) ||
        p.ld > (int64_t{1} << 30))
      return false;
    if (p.is_x && (!p.colmax || !p.q_f8_main || t->n_chunks >= (int64_t{1} << 31))) return false;
    t->is_x = p.is_x;
    t->ld_i32 = static_cast<int32_t>(p.ld);
    t->rows_i32 = static_cast<int32_t>(p.rows);
    t->cols_i32 = static_cast<int32_t>(p.cols);
    t->colmax = p.colmax;
    t->col_slot = p.col_slot;
    t->side_cols = p.side_cols;
    t->q_f8_main = p.is_x ? p.q_f8_main : nullptr;
    t->side = p.side;
  }
  return true;
}

}  // namespace

int wa_prep_segments(int64_t rows, int64_t cols) {
  const int64_t n_chunks = rows * (cols / 8);
  const int64_t b = (n_chunks + kThreads - 1) / kThreads;
  return static_cast<int>(b < 1 ? 1 : (b > kTensorBlocks ? kTensorBlocks : b));
}

int launch_wa_prep(const WaPrepTensor* p, int n, hipStream_t st) {
  if (!p || n < 1 || n > kMaxTensors) return MOFQ_ERR_INVALID_ARG;
  PrepArgs a{};
  int64_t total_seg = 0;
  for (int i = 0; i < n; ++i) {
    if (!p[i].data) continue;   // skipped
    if (!fill(p[i], &a.t[a.n])) return MOFQ_ERR_INVALID_ARG;
    if (a.t[a.n].n_chunks > (int64_t{1} << 40)) return MOFQ_ERR_UNSUPPORTED;
    total_seg += a.t[a.n].n_seg;
    ++a.n;
  }
  if (a.n < 1) return MOFQ_OK;
  // One workgroup per segment while the launch stays within 16 workgroups per compute unit's
  // worth (4096); beyond that every tensor gets its share and workgroups take several segments.
  constexpr int64_t kMaxBlocks = 4096;
  for (int k = 0; k < a.n; ++k) {
    int64_t nb = a.t[k].n_seg;
    if (total_seg > kMaxBlocks) nb = std::max<int64_t>(1, nb * kMaxBlocks / total_seg);
    a.first_block[k + 1] = a.first_block[k] + static_cast<int32_t>(nb);
  }
  const int blocks = a.first_block[a.n];
  // first pass: every tensor but the activations of a column split, whose largest magnitude
  // comes out of the column maxima
  PrepArgs am{};
  for (int k = 0; k < a.n; ++k) {
    if (a.t[k].side && a.t[k].is_x) { a.t[k].n_absmax = 1; continue; }
    am.t[am.n] = a.t[k];
    am.first_block[am.n + 1] = am.first_block[am.n] + (a.first_block[k + 1] - a.first_block[k]);
    ++am.n;
  }
  if (am.n) hipLaunchKernelGGL(wa_absmax_kernel, dim3(am.first_block[am.n]), dim3(kThreads), 0, st, am);
  // column split: the activations' column maxima and the pick come before the quantize pass
  // (which zeroes the picked columns in the fp8 operand), the side operands after it (they
  // use the scale it leaves)
  PrepArgs xs{}, sd{};
  for (int k = 0; k < a.n; ++k) {
    if (!a.t[k].side) continue;
    if (a.t[k].is_x) {
      xs.t[xs.n] = a.t[k];
      xs.first_block[xs.n + 1] = xs.first_block[xs.n] + a.t[k].cols_i32 / 64;
      ++xs.n;
    }
    sd.t[sd.n] = a.t[k];
    const int64_t nb = (static_cast<int64_t>(a.t[k].rows_i32) * kWaSideCols + kThreads * 4 - 1) / (kThreads * 4);
    sd.first_block[sd.n + 1] = sd.first_block[sd.n] + static_cast<int32_t>(std::min<int64_t>(nb, 1024));
    ++sd.n;
  }
  if (xs.n) {
    hipLaunchKernelGGL(wa_colmax_kernel, dim3(xs.first_block[xs.n]), dim3(kThreads), 0, st, xs);
    hipLaunchKernelGGL(wa_pick_kernel, dim3(xs.n), dim3(kThreads), 0, st, xs);
  }
  hipLaunchKernelGGL(wa_quant_kernel, dim3(blocks), dim3(kThreads), 0, st, a);
  if (sd.n) hipLaunchKernelGGL(wa_side_kernel, dim3(sd.first_block[sd.n]), dim3(kThreads), 0, st, sd);
  return hip_status(hipGetLastError());
}

}  // namespace mofq
